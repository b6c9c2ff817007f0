// Exact attention at the kept positions (paper section 3.4 / 5.1): SDDMM (equation 2 sampled at
// the mask), softmax over the kept entries (equation 4) and SpMM (equation 3).
//
// Row kernel.  One 64-lane wavefront owns one query row.  A key / value row of d elements is
// d*e bytes; it is read as 16-byte pieces by LPR = d*e/16 neighbouring lanes, so one wavefront
// load instruction fetches 64/LPR complete, fully coalesced rows of the gather list.  The
// kernel is bound by those gathers (about 1 flop per byte), so everything else stays on chip:
// the row's scores go to LDS, the softmax statistics live in registers, and the weights are
// recomputed from the LDS scores while the value rows stream in.  S and P never reach HBM in
// the fused mode.
#include "dsa_internal.h"
#include "attention_api.h"

#include <type_traits>

namespace dsa {
namespace {

constexpr int kRowWaves = 4;          // query rows (wavefronts) per workgroup
constexpr int kRowPad = 8;            // the row kernel pads a key list to a multiple of this
constexpr int kMaxKeep = 4096;        // list and scores of a row in LDS: 4 waves * 4096 * 8 B = 128 KB

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// 16 bytes of a row: how to load them, to take a dot product of two of them and to add p times one
// of them to fp32 accumulators.
template <typename T> struct Piece;
template <> struct Piece<float> {
    static constexpr int N = 4;
    typedef float4 raw_t;
    static __device__ __forceinline__ raw_t load(const float *p) { return *reinterpret_cast<const float4 *>(p); }
    static __device__ __forceinline__ float dot(raw_t a, raw_t b)
    {
        return fmaf(a.w, b.w, fmaf(a.z, b.z, fmaf(a.y, b.y, a.x * b.x)));
    }
    // A weight as the word that is kept in LDS, the sum of weights, o += weight * b, and -a.
    static __device__ __forceinline__ unsigned weight(float p) { return __float_as_uint(p); }
    static __device__ __forceinline__ float wsum(float z, unsigned w) { return z + __uint_as_float(w); }
    static __device__ __forceinline__ void axpy(float (&o)[4], unsigned w, raw_t b)
    {
        const float p = __uint_as_float(w);
        o[0] = fmaf(p, b.x, o[0]); o[1] = fmaf(p, b.y, o[1]); o[2] = fmaf(p, b.z, o[2]); o[3] = fmaf(p, b.w, o[3]);
    }
    static __device__ __forceinline__ raw_t negate(raw_t a) { return make_float4(-a.x, -a.y, -a.z, -a.w); }
};
// bfloat16: v_dot2_f32_bf16 multiplies two packed pairs and accumulates in fp32, so no element is
// ever unpacked.  For the weighted sum the weight is rounded to bfloat16 (relative 2^-9, inside the
// 2e-2 budget of bfloat16 inputs) and paired with a zero: (v0, v1) . (p, 0) = p v0, (v0, v1) . (0, p) = p v1.
template <> struct Piece<uint16_t> {
    static constexpr int N = 8;
    typedef uint4 raw_t;
    static __device__ __forceinline__ raw_t load(const uint16_t *p) { return *reinterpret_cast<const uint4 *>(p); }
    static __device__ __forceinline__ float dot2(unsigned a, unsigned b, float acc)
    {
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), acc, false);
    }
    static __device__ __forceinline__ float dot(raw_t a, raw_t b)
    {
        return dot2(a.w, b.w, dot2(a.z, b.z, dot2(a.y, b.y, dot2(a.x, b.x, 0.f))));
    }
    // The weight kept in LDS is the pair (p rounded to bfloat16, 0); the sum takes the rounded weights, the
    // ones the products use.
    static __device__ __forceinline__ unsigned weight(float p) { return __builtin_bit_cast(unsigned short, (__bf16)p); }
    static __device__ __forceinline__ float wsum(float z, unsigned w) { return dot2(w, 0x3f803f80u, z); }
    static __device__ __forceinline__ raw_t negate(raw_t a)
    {
        return make_uint4(a.x ^ 0x80008000u, a.y ^ 0x80008000u, a.z ^ 0x80008000u, a.w ^ 0x80008000u);
    }
    static __device__ __forceinline__ void axpy(float (&o)[8], unsigned lo, raw_t b)
    {
        const unsigned hi = lo << 16;
        o[0] = dot2(b.x, lo, o[0]); o[1] = dot2(b.x, hi, o[1]);
        o[2] = dot2(b.y, lo, o[2]); o[3] = dot2(b.y, hi, o[3]);
        o[4] = dot2(b.z, lo, o[4]); o[5] = dot2(b.z, hi, o[5]);
        o[6] = dot2(b.w, lo, o[6]); o[7] = dot2(b.w, hi, o[7]);
    }
};

// Cross-lane moves inside a row of 16 lanes without LDS traffic (DPP).
template <int CTRL> __device__ __forceinline__ float dpp_f(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true));
}
// Sum over the LPR neighbouring lanes that hold one row (LPR = 8, 16 or 32); every one of them gets it.
template <int LPR> __device__ __forceinline__ float piece_sum(float x)
{
    x += dpp_f<0xB1>(x);                          // lane ^ 1 (quad permute 1,0,3,2)
    x += dpp_f<0x4E>(x);                          // lane ^ 2 (quad permute 2,3,0,1)
    x += dpp_f<0x141>(x);                         // the other quad of the 8 (half-row mirror)
    if (LPR >= 16) x += dpp_f<0x140>(x);          // the other half of the 16 (row mirror)
    if (LPR >= 32) x += __shfl_xor(x, 16, kWave);
    return x;
}
// Combine the 64/LPR row groups of a wavefront: lane (group, piece) with every (group', piece).
template <int LPR> __device__ __forceinline__ float groups_sum(float x)
{
    if (LPR <= 8) x += dpp_f<0x128>(x);           // lane ^ 8 (row rotate by 8)
#pragma unroll
    for (int off = (LPR <= 8 ? 16 : LPR); off < kWave; off <<= 1) x += __shfl_xor(x, off, kWave);
    return x;
}
template <int LPR> __device__ __forceinline__ float groups_max(float x)
{
    if (LPR <= 8) x = fmaxf(x, dpp_f<0x128>(x));
#pragma unroll
    for (int off = (LPR <= 8 ? 16 : LPR); off < kWave; off <<= 1) x = fmaxf(x, __shfl_xor(x, off, kWave));
    return x;
}

// Reductions over all 64 lanes.
__device__ __forceinline__ float wave_all_sum(float x)
{
    x = piece_sum<16>(x);
    x += __shfl_xor(x, 16, kWave);
    x += __shfl_xor(x, 32, kWave);
    return x;
}
__device__ __forceinline__ float wave_all_max(float x)
{
    x = fmaxf(x, dpp_f<0xB1>(x));
    x = fmaxf(x, dpp_f<0x4E>(x));
    x = fmaxf(x, dpp_f<0x141>(x));
    x = fmaxf(x, dpp_f<0x140>(x));
    x = fmaxf(x, __shfl_xor(x, 16, kWave));
    x = fmaxf(x, __shfl_xor(x, 32, kWave));
    return x;
}

// Makes LDS writes of some lanes of a wavefront visible to reads of its other lanes.  Every LDS
// region below belongs to one wavefront, so no workgroup barrier is ever needed.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// MODE kFused: Q,K,V,idx -> O.  kSddmm: Q,K,idx -> S.  kSpmm: Pin,V,idx -> O.
template <typename T, int D, int MODE>
__global__ __launch_bounds__(kRowWaves *kWave) void attention_rows(
    const T *__restrict__ Q, const T *__restrict__ K, const T *__restrict__ V,
    const int32_t *__restrict__ idx, const float *__restrict__ Pin, float *__restrict__ S,
    float *__restrict__ O, int L, int keep, int keep_pad, int vec, float scale, unsigned total_rows)
{
    typedef Piece<T> P;
    constexpr int E = P::N;               // elements per lane
    constexpr int LPR = D / E;            // lanes per row
    constexpr int RPI = kWave / LPR;      // gathered rows per wavefront instruction
    extern __shared__ float lds_scores[];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int sub = lane % LPR, grp = lane / LPR;
    const unsigned vblock = xcd_contiguous(blockIdx.x, gridDim.x);
    const unsigned row = vblock * kRowWaves + wave;                 // wavefront-uniform from here on
    const bool live = row < total_rows;
    const unsigned r = live ? row : total_rows - 1;      // dead waves shadow a real row, write nothing
    const unsigned n = r / (unsigned)L, i = r % (unsigned)L;
    const int32_t *list = idx + ((size_t)n * (L / vec) + i / vec) * keep;
    // per wavefront in LDS: the row's key list, as the byte offset of every key row inside its head
    // (keys clamped into [0, L), so that no idx can send a gather outside K / V), and its scores, later
    // (or from the start, when the weights are given) its weights.  The list is padded to keep_pad, a multiple of the keys one
    // trip of the loops below takes, with its last key: a padded entry has the score of a real one (no
    // effect on the maximum) and gets the weight 0, so the loops test nothing.
    constexpr unsigned kRowBytes = D * sizeof(T), kPieceBytes = E * sizeof(T);
    unsigned *sl = reinterpret_cast<unsigned *>(lds_scores) + wave * 2 * keep_pad;
    float *sc = reinterpret_cast<float *>(sl + keep_pad);
    unsigned *sw = reinterpret_cast<unsigned *>(sc);      // the same words once they hold weights
    for (int t = lane; t < keep_pad; t += kWave) sl[t] = (unsigned)min(max(list[min(t, keep - 1)], 0), L - 1) * kRowBytes;
    wave_lds_fence();
    constexpr int U = 4;                  // independent gathers in flight per lane
    static_assert(kRowPad % RPI == 0, "keep_pad is a whole number of single trips");
    const unsigned piece_at = sub * kPieceBytes;
    auto piece_of = [&](const T *head, unsigned row_at) {
        return P::load(reinterpret_cast<const T *>(reinterpret_cast<const char *>(head) + (size_t)(row_at + piece_at)));
    };

    float m = -INFINITY;
    // fused mode: the scores are kept as sign(scale) * q.k and the factor |scale| waits for the exponential
    const bool flip = MODE == kFused && scale < 0.f;
    const float factor = MODE == kFused ? fabsf(scale) : scale;
    if (MODE != kSpmm) {
        typename P::raw_t q = P::load(Q + (size_t)r * D + sub * E);
        if (flip) q = P::negate(q);
        const T *Kh = K + (size_t)n * L * D;
        // UU gathers in flight per lane: trips of U while they fit, single ones for the rest
        auto scores_of = [&](int t0, auto uu) {
            constexpr int UU = decltype(uu)::value;
            typename P::raw_t kv[UU];
#pragma unroll
            for (int u = 0; u < UU; ++u) kv[u] = piece_of(Kh, sl[t0 + u * RPI + grp]);
            float acc[UU];
#pragma unroll
            for (int u = 0; u < UU; ++u) acc[u] = piece_sum<LPR>(P::dot(q, kv[u]));
#pragma unroll
            for (int u = 0; u < UU; ++u) {
                const int t = t0 + u * RPI + grp;
                if (MODE != kSddmm) m = fmaxf(m, acc[u]);
                sc[t] = acc[u];               // every lane of the group writes the same value
            }
        };
        int t0 = 0;
        for (; t0 + U * RPI <= keep_pad; t0 += U * RPI) scores_of(t0, std::integral_constant<int, U>{});
        for (; t0 < keep_pad; t0 += RPI) scores_of(t0, std::integral_constant<int, 1>{});
        if (MODE == kSddmm) {
            // the row of scores leaves in one piece: consecutive lanes, consecutive entries
            wave_lds_fence();
            if (live)
                for (int t = lane; t < keep; t += kWave) S[(size_t)r * keep + t] = sc[t] * factor;
            return;
        }
        m = groups_max<LPR>(m);
        wave_lds_fence();
        // unnormalised weights, computed once per kept key (the lanes that share a value row would
        // otherwise each repeat the exponential), in the form the products take them
        for (int t = lane; t < keep_pad; t += kWave) sw[t] = t < keep ? P::weight(__expf(factor * (sc[t] - m))) : 0u;
        wave_lds_fence();
    }

    if (MODE == kSpmm) {
        // the given weights come in the same way and wait in LDS in the form the products take them
        for (int t = lane; t < keep_pad; t += kWave) sw[t] = t < keep ? P::weight(Pin[(size_t)r * keep + t]) : 0u;
        wave_lds_fence();
    }
    float o[E], z = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) o[e] = 0.f;
    const T *Vh = V + (size_t)n * L * D;
    auto values_of = [&](int t0, auto uu) {
        constexpr int UU = decltype(uu)::value;
        typename P::raw_t vv[UU];
        unsigned w[UU];
#pragma unroll
        for (int u = 0; u < UU; ++u) {
            const int t = t0 + u * RPI + grp;
            vv[u] = piece_of(Vh, sl[t]);
            w[u] = sw[t];
        }
#pragma unroll
        for (int u = 0; u < UU; ++u) {
            z = P::wsum(z, w[u]);
            P::axpy(o, w[u], vv[u]);
        }
    };
    {
        int t0 = 0;
        for (; t0 + U * RPI <= keep_pad; t0 += U * RPI) values_of(t0, std::integral_constant<int, U>{});
        for (; t0 < keep_pad; t0 += RPI) values_of(t0, std::integral_constant<int, 1>{});
    }
#pragma unroll
    for (int e = 0; e < E; ++e) o[e] = groups_sum<LPR>(o[e]);
    if (MODE == kFused) {
        z = groups_sum<LPR>(z);
        const float inv = 1.f / z;
#pragma unroll
        for (int e = 0; e < E; ++e) o[e] *= inv;
    }
    if (live && grp == 0) {
        float *out = O + (size_t)r * D + sub * E;
#pragma unroll
        for (int e = 0; e < E; e += 4)
            *reinterpret_cast<float4 *>(out + e) = make_float4(o[e], o[e + 1], o[e + 2], o[e + 3]);
    }
}

// Row kernel for masks in CSR form (threshold masks, section 3.1: the count per row varies).  Same
// wavefront-per-row scheme as attention_rows, fused only; a row's list is taken in chunks of
// kCsrChunk keys with a running maximum, so that any count fits the same LDS: when a later chunk
// raises the maximum, the sums so far are rescaled by exp(m_old - m_new).
constexpr int kCsrChunk = 1024;

template <typename T, int D>
__global__ __launch_bounds__(kRowWaves *kWave) void attention_rows_csr(
    const T *__restrict__ Q, const T *__restrict__ K, const T *__restrict__ V,
    const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col, float *__restrict__ O, int L, int vec,
    float scale, unsigned total_rows)
{
    typedef Piece<T> P;
    constexpr int E = P::N, LPR = D / E, RPI = kWave / LPR, U = 4;
    __shared__ int lists[kRowWaves][kCsrChunk];
    __shared__ float scores[kRowWaves][kCsrChunk];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int sub = lane % LPR, grp = lane / LPR;
    const unsigned row = xcd_contiguous(blockIdx.x, gridDim.x) * kRowWaves + wave;
    if (row >= total_rows) return;                        // the whole wavefront: nothing below is shared
    const unsigned n = row / (unsigned)L, i = row % (unsigned)L;
    const size_t u = (size_t)n * (L / vec) + i / vec;
    const int beg = row_ptr[u];
    const int cnt = max(row_ptr[u + 1] - beg, 0);
    int *sl = lists[wave];
    float *sc = scores[wave];
    const typename P::raw_t q = P::load(Q + (size_t)row * D + sub * E);
    const T *Kh = K + (size_t)n * L * D, *Vh = V + (size_t)n * L * D;

    float m = -INFINITY, z = 0.f, o[E];
#pragma unroll
    for (int e = 0; e < E; ++e) o[e] = 0.f;
    for (int c0 = 0; c0 < cnt; c0 += kCsrChunk) {
        const int nk = min(kCsrChunk, cnt - c0);
        for (int t = lane; t < nk; t += kWave) sl[t] = min(max(col[beg + c0 + t], 0), L - 1);
        wave_lds_fence();
        float mc = -INFINITY;
        for (int t0 = 0; t0 < nk; t0 += U * RPI) {
            typename P::raw_t kv[U];
#pragma unroll
            for (int x = 0; x < U; ++x) kv[x] = P::load(Kh + (unsigned)(sl[min(t0 + x * RPI + grp, nk - 1)] * D + sub * E));
#pragma unroll
            for (int x = 0; x < U; ++x) {
                const int t = t0 + x * RPI + grp;
                const float acc = piece_sum<LPR>(P::dot(q, kv[x])) * scale;
                if (t < nk) {
                    mc = fmaxf(mc, acc);
                    if (sub == 0) sc[t] = acc;
                }
            }
        }
        mc = groups_max<LPR>(mc);
        const float m_new = fmaxf(m, mc);
        const float f = __expf(m - m_new);               // 0 for the first chunk (m = -inf)
        z *= f;
#pragma unroll
        for (int e = 0; e < E; ++e) o[e] *= f;
        m = m_new;
        wave_lds_fence();
        for (int t = lane; t < nk; t += kWave) sc[t] = __expf(sc[t] - m);
        wave_lds_fence();
        for (int t0 = 0; t0 < nk; t0 += U * RPI) {
            typename P::raw_t vv[U];
            float p[U];
#pragma unroll
            for (int x = 0; x < U; ++x) {
                const int t = t0 + x * RPI + grp;
                const int tt = min(t, nk - 1);
                vv[x] = P::load(Vh + (unsigned)(sl[tt] * D + sub * E));
                p[x] = t < nk ? sc[tt] : 0.f;
            }
#pragma unroll
            for (int x = 0; x < U; ++x) {
                z += p[x];
                P::axpy(o, P::weight(p[x]), vv[x]);
            }
        }
        wave_lds_fence();                                  // the next chunk overwrites list and scores
    }
#pragma unroll
    for (int e = 0; e < E; ++e) o[e] = groups_sum<LPR>(o[e]);
    z = groups_sum<LPR>(z);
    const float inv = cnt > 0 ? 1.f / z : 0.f;            // a row without keys (not made by the predictor) gives 0
    if (grp == 0) {
        float *out = O + (size_t)row * D + sub * E;
#pragma unroll
        for (int e = 0; e < E; e += 4)
            *reinterpret_cast<float4 *>(out + e) = make_float4(o[e] * inv, o[e + 1] * inv, o[e + 2] * inv, o[e + 3] * inv);
    }
}

// Measurement aid: the gathers of attention_rows and nothing else.  Same launch shape, same key list
// staged in LDS, same 16-byte pieces with four gathers in flight per lane, first over K and then over V;
// the pieces are only folded into one word per row so that the loads cannot be dropped.  Its rate, in
// gathered bytes per second, is the roof the memory hierarchy (L1 / L2, where K and V of a head live)
// sets for this access pattern: the yardstick for attention_rows.
template <typename T, int D>
__global__ __launch_bounds__(kRowWaves *kWave) void gather_probe(const T *__restrict__ K, const T *__restrict__ V,
                                                                 const int32_t *__restrict__ idx,
                                                                 unsigned *__restrict__ sink, int L, int keep,
                                                                 int keep_pad, int vec, unsigned total_rows)
{
    typedef Piece<T> P;
    constexpr int E = P::N, LPR = D / E, RPI = kWave / LPR, U = 4;
    constexpr unsigned kRowBytes = D * sizeof(T), kPieceBytes = E * sizeof(T);
    extern __shared__ float lds_scores[];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int sub = lane % LPR, grp = lane / LPR;
    const unsigned row = xcd_contiguous(blockIdx.x, gridDim.x) * kRowWaves + wave;
    const bool live = row < total_rows;
    const unsigned r = live ? row : total_rows - 1;
    const unsigned n = r / (unsigned)L, i = r % (unsigned)L;
    const int32_t *list = idx + ((size_t)n * (L / vec) + i / vec) * keep;
    // the same padded list of byte offsets as in attention_rows, the same address arithmetic
    unsigned *sl = reinterpret_cast<unsigned *>(lds_scores) + wave * keep_pad;
    for (int t = lane; t < keep_pad; t += kWave) sl[t] = (unsigned)min(max(list[min(t, keep - 1)], 0), L - 1) * kRowBytes;
    wave_lds_fence();
    const unsigned piece_at = sub * kPieceBytes;
    unsigned acc = 0;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const T *Xh = (pass ? V : K) + (size_t)n * L * D;
        auto gather = [&](int t0, auto uu) {
            constexpr int UU = decltype(uu)::value;
            typename P::raw_t x[UU];
#pragma unroll
            for (int u = 0; u < UU; ++u)
                x[u] = P::load(reinterpret_cast<const T *>(reinterpret_cast<const char *>(Xh) +
                                                           (size_t)(sl[t0 + u * RPI + grp] + piece_at)));
#pragma unroll
            for (int u = 0; u < UU; ++u) {
                const uint4 w = __builtin_bit_cast(uint4, x[u]);
                acc ^= (w.x ^ w.y) ^ (w.z ^ w.w);
            }
        };
        int t0 = 0;
        for (; t0 + U * RPI <= keep_pad; t0 += U * RPI) gather(t0, std::integral_constant<int, U>{});
        for (; t0 < keep_pad; t0 += RPI) gather(t0, std::integral_constant<int, 1>{});
    }
    if (live) sink[(size_t)r * kWave + lane] = acc;
}

// Group kernel for the vector-wise mask with bfloat16 inputs.  The 8 query rows of a group share
// one key list, so each gathered key / value row serves 8 rows and the products become small
// dense contractions for the bf16 matrix cores (v_mfma_f32_16x16x32_bf16, fp32 accumulate).  One
// wavefront owns one group.
//   Scores: the gathered key rows are the A operand (16 keys per tile, loaded straight from
//   global memory as 16-byte pieces: lane (r = lane%16, g = lane/16) holds key r, elements
//   [8g, 8g+8) of each 32-element step), the 8 query rows (padded to 16) the B operand.  Lane
//   (c, g) then owns, for query c, keys 4g..4g+3 of the tile.  Scaled scores go to LDS.
//   Output: weights stay in the lane that owns them.  Over a 32-key step lane group g owns keys
//   {4g+i} of the first tile and {16+4g+i} of the second: these 8 are its slots of the step's
//   contraction index, so its packed bf16 weights ARE the A operand (query c, slots of g).  The
//   32 gathered value rows go through LDS once and come back transposed as the B operand with
//   the same slot order (lane (c, g): column c of the rows that are g's slots).
// The weights are rounded to bfloat16 for the second product (relative 2^-9, inside the 2e-2
// budget of bfloat16 inputs); scores, softmax statistics and accumulation are fp32.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));

constexpr int kGroupWaves = 4;


// (The launch bound is twice the launched size: with at most 256 registers per lane the compiler
// gives the matrix core plain VGPR destinations instead of accumulation registers that every
// other instruction would have to copy from.)
// MODE kFused: Q,K,V,idx -> O.  kSddmm: Q,K,idx -> S (scaled scores of the 8 rows).  kSpmm: Pin,V,idx -> O.
template <int D, int MODE>
__global__ __launch_bounds__(2 * kGroupWaves *kWave) void attention_groups_bf16(
    const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K, const uint16_t *__restrict__ V,
    const int32_t *__restrict__ idx, const float *__restrict__ Pin, float *__restrict__ S, float *__restrict__ O,
    int L, int keep, int keep_pad, float scale, unsigned total_groups)
{
    constexpr int KS = D / 32;             // contraction steps of Q K^T
    constexpr int CT = D / 16;             // 16-column tiles of the output
    constexpr int VROW = D * 2 + 16;       // bytes of one value row in LDS (padded against bank conflicts)
    constexpr int LPR = D / 8;             // lanes that load one row as 16-byte pieces
    constexpr int RPI = kWave / LPR;       // rows per load instruction
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int c = lane & 15, g = lane >> 4;
    const size_t per_wave = (size_t)9 * keep_pad * sizeof(float) + 32 * VROW;
    float *sS = reinterpret_cast<float *>(lds_raw + wave * per_wave);          // [8][keep_pad]
    int *sl = reinterpret_cast<int *>(sS + 8 * keep_pad);                      // [keep_pad] key list
    char *sV = reinterpret_cast<char *>(sl + keep_pad);                        // [32][VROW]

    const unsigned vblock = xcd_contiguous(blockIdx.x, gridDim.x);
    const unsigned grp = vblock * kGroupWaves + wave;
    const bool live = grp < total_groups;
    const unsigned gi = live ? grp : total_groups - 1;     // dead waves shadow a real group, write nothing
    const unsigned G = L / 8, n = gi / G, u = gi % G;
    const int32_t *list = idx + (size_t)gi * keep;
    const uint16_t *Kh = K + (size_t)n * L * D, *Vh = V + (size_t)n * L * D;

    bf16x8 qop[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        const uint4 raw = (MODE != kSpmm && c < 8) ? *reinterpret_cast<const uint4 *>(Q + ((size_t)n * L + u * 8 + c) * D + 32 * s + 8 * g)
                                : make_uint4(0, 0, 0, 0);
        qop[s] = __builtin_bit_cast(bf16x8, raw);
    }

    // the group's key list once into LDS, clamped into [0, L) (no idx can send a gather outside K / V)
    // and padded with its last entry
    for (int t = lane; t < keep_pad; t += kWave) sl[t] = min(max(list[min(t, keep - 1)], 0), L - 1);
    wave_lds_fence();

    // scores of all kept keys -> LDS, running maximum per query.  The key rows of a step (32 keys) are
    // gathered the way the value rows are below: D / 8 neighbouring lanes fetch one row as 16-byte pieces
    // (whole cache lines per row, which is what the vector memory path serves best; fetched straight
    // into the operand layout, 16 lanes take 16 bytes of 16 different rows each and the same bytes come
    // at a third of the rate), pass through the value tile's LDS and come back as the first operand of
    // the matrix instruction.  The rows of step t + 1 are requested before step t is consumed.
    float mx = -INFINITY;
    constexpr int VP = 32 / RPI;           // load instructions per step of 32 rows
    const int vrow = lane / LPR, vpiece = lane % LPR;
    if (MODE != kSpmm) {
        v4u kring[VP];
#pragma unroll
        for (int rr = 0; rr < VP; ++rr)
            kring[rr] = *reinterpret_cast<const v4u *>(Kh + (size_t)sl[rr * RPI + vrow] * D + vpiece * 8);
        for (int t0 = 0; t0 < keep_pad; t0 += 32) {
#pragma unroll
            for (int rr = 0; rr < VP; ++rr) *reinterpret_cast<v4u *>(sV + (rr * RPI + vrow) * VROW + vpiece * 16) = kring[rr];
            const int tn = min(t0 + 32, keep_pad - 32);
#pragma unroll
            for (int rr = 0; rr < VP; ++rr)
                kring[rr] = *reinterpret_cast<const v4u *>(Kh + (size_t)sl[tn + rr * RPI + vrow] * D + vpiece * 8);
            wave_lds_fence();
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int tile = t0 + 16 * half;
                v4f acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < KS; ++s) {
                    const bf16x8 ka = *reinterpret_cast<const bf16x8 *>(sV + (16 * half + c) * VROW + (32 * s + 8 * g) * 2);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qop[s], acc, 0, 0, 0);
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    acc[i] = tile + 4 * g + i < keep ? acc[i] * scale : -INFINITY;
                    mx = fmaxf(mx, acc[i]);
                }
                if (c < 8) *reinterpret_cast<v4f *>(sS + c * keep_pad + tile + 4 * g) = acc;
            }
            wave_lds_fence();       // the next step overwrites the tile
        }
    }
    if (MODE == kSddmm) {
        // the 8 rows of scores leave through LDS: consecutive lanes write consecutive entries of a row
        wave_lds_fence();
        if (live) {
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                float *dst = S + ((size_t)n * L + u * 8 + r) * keep;
                for (int t = lane; t < keep; t += kWave) dst[t] = sS[r * keep_pad + t];
            }
        }
        return;
    }
    if (MODE == kSpmm) {
        // the given weights come in the same way (0 beyond the list)
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const float *src = Pin + ((size_t)n * L + u * 8 + r) * keep;
            for (int t = lane; t < keep_pad; t += kWave) sS[r * keep_pad + t] = t < keep ? src[t] : 0.f;
        }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
    mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
    wave_lds_fence();

    v4f o[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) o[ct] = v4f{0.f, 0.f, 0.f, 0.f};
    float z = 0.f;
    const float *srow = sS + (c & 7) * keep_pad + 4 * g;
    // value rows of a step: 32 / RPI pieces of 16 bytes per lane; a ring of VF steps is kept in flight
    constexpr int VF = 1;
    v4u vring[VF][VP];
#pragma unroll
    for (int f = 0; f < VF; ++f)
#pragma unroll
        for (int rr = 0; rr < VP; ++rr)
            vring[f][rr] = *reinterpret_cast<const v4u *>(
                Vh + (size_t)sl[min(32 * f, keep_pad - 32) + rr * RPI + vrow] * D + vpiece * 8);
    for (int t1 = 0; t1 < keep_pad; t1 += 32 * VF) {
#pragma unroll
        for (int f = 0; f < VF; ++f) {
            const int t0 = t1 + 32 * f;
            if (t0 < keep_pad) {
                // 32 gathered value rows -> LDS, and the request for the rows of step t0 + VF
#pragma unroll
                for (int rr = 0; rr < VP; ++rr)
                    *reinterpret_cast<v4u *>(sV + (rr * RPI + vrow) * VROW + vpiece * 16) = vring[f][rr];
                const int tn = min(t0 + 32 * VF, keep_pad - 32);
#pragma unroll
                for (int rr = 0; rr < VP; ++rr)
                    vring[f][rr] = *reinterpret_cast<const v4u *>(
                        Vh + (size_t)sl[tn + rr * RPI + vrow] * D + vpiece * 8);
                // weights of this lane's 8 slots
                const v4f s0 = *reinterpret_cast<const v4f *>(srow + t0);
                const v4f s1 = *reinterpret_cast<const v4f *>(srow + t0 + 16);
                bf16x8 pa;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float p0 = MODE == kSpmm ? s0[i] : __expf(s0[i] - mx);
                    const float p1 = MODE == kSpmm ? s1[i] : __expf(s1[i] - mx);
                    z += p0 + p1;
                    pa[i] = (__bf16)p0;
                    pa[4 + i] = (__bf16)p1;
                }
                wave_lds_fence();
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) {
                    bf16x8 vb;
                    const char *col = sV + (16 * ct + c) * 2;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        vb[i] = *reinterpret_cast<const __bf16 *>(col + (4 * g + i) * VROW);
                        vb[4 + i] = *reinterpret_cast<const __bf16 *>(col + (16 + 4 * g + i) * VROW);
                    }
                    o[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa, vb, o[ct], 0, 0, 0);
                }
                wave_lds_fence();       // the next step overwrites the value tile
            }
        }
    }
    z += __shfl_xor(z, 16, kWave);
    z += __shfl_xor(z, 32, kWave);
    // lane (c, g) holds O[query 4g+i][16 ct + c]; the sum of query q sits in the lanes with column q
    if (live) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float inv = MODE == kSpmm ? 1.f : 1.f / __shfl(z, (4 * g + i) & 7, kWave);
            if (g < 2) {
                float *out = O + ((size_t)n * L + u * 8 + 4 * g + i) * D + c;
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) out[16 * ct] = o[ct][i] * inv;
            }
        }
    }
}

// Softmax over the `keep` scores of each row: one wavefront per row.
__global__ __launch_bounds__(kRowWaves *kWave) void softmax_rows(const float *S, float *P, int keep,
                                                                  unsigned total_rows)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const unsigned row = blockIdx.x * kRowWaves + wave;
    if (row >= total_rows) return;
    const float *s = S + (size_t)row * keep;
    float *p = P + (size_t)row * keep;
    constexpr int R = 8;                   // rows of up to 64 R entries stay in registers: read once, one exponential each
    if (keep <= R * kWave) {
        float v[R];
        float m = -INFINITY;
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const int t = lane + i * kWave;
            v[i] = t < keep ? s[t] : -INFINITY;
            m = fmaxf(m, v[i]);
        }
        m = wave_all_max(m);
        float z = 0.f;
#pragma unroll
        for (int i = 0; i < R; ++i) {
            v[i] = __expf(v[i] - m);      // exp(-inf) = 0 beyond the row
            z += v[i];
        }
        z = wave_all_sum(z);
        const float inv = 1.f / z;
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const int t = lane + i * kWave;
            if (t < keep) p[t] = v[i] * inv;
        }
        return;
    }
    float m = -INFINITY;
    for (int t = lane; t < keep; t += kWave) m = fmaxf(m, s[t]);
    m = wave_all_max(m);
    float z = 0.f;
    for (int t = lane; t < keep; t += kWave) z += __expf(s[t] - m);
    z = wave_all_sum(z);
    const float inv = 1.f / z;
    for (int t = lane; t < keep; t += kWave) p[t] = __expf(s[t] - m) * inv;
}

template <typename T, int D>
hipError_t launch_rows(AttnMode mode, const dsa_shape &sh, const void *Q, const void *K, const void *V,
                       const int32_t *idx, const float *Pin, float *S, float *O, hipStream_t st)
{
    const unsigned rows = (unsigned)sh.B * sh.H * sh.L;
    const dim3 grid((rows + kRowWaves - 1) / kRowWaves), block(kRowWaves * kWave);
    // per wavefront: the padded key list and the scores / weights
    const int keep_pad = (sh.keep + kRowPad - 1) / kRowPad * kRowPad;
    const size_t lds = (size_t)kRowWaves * keep_pad * sizeof(float) * 2;
    const T *q = static_cast<const T *>(Q), *k = static_cast<const T *>(K), *v = static_cast<const T *>(V);
    if (mode == kFused) {
        auto kern = attention_rows<T, D, kFused>;
        if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds)) return e;
        hipLaunchKernelGGL(kern, grid, block, lds, st, q, k, v, idx, Pin, S, O, sh.L, sh.keep, keep_pad, sh.vec,
                           sh.scale, rows);
    } else if (mode == kSddmm) {
        auto kern = attention_rows<T, D, kSddmm>;
        if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds)) return e;
        hipLaunchKernelGGL(kern, grid, block, lds, st, q, k, v, idx, Pin, S, O, sh.L, sh.keep, keep_pad, sh.vec,
                           sh.scale, rows);
    } else {
        auto kern = attention_rows<T, D, kSpmm>;
        if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds)) return e;
        hipLaunchKernelGGL(kern, grid, block, lds, st, q, k, v, idx, Pin, S, O, sh.L, sh.keep, keep_pad, sh.vec,
                           sh.scale, rows);
    }
    return hipGetLastError();
}

// LDS of one workgroup of the group kernel: per wavefront 8 rows of scores and a 32-row value tile.
size_t groups_lds_bytes(const dsa_shape &sh)
{
    const size_t keep_pad = (size_t)(sh.keep + 31) / 32 * 32;
    return kGroupWaves * (9 * keep_pad * sizeof(float) + 32 * ((size_t)sh.d * 2 + 16));
}

template <int D, int MODE>
hipError_t launch_groups(const dsa_shape &sh, const void *Q, const void *K, const void *V, const int32_t *idx,
                         const float *Pin, float *S, float *O, hipStream_t st)
{
    const unsigned groups = (unsigned)sh.B * sh.H * (sh.L / 8);
    const int keep_pad = (sh.keep + 31) / 32 * 32;
    const size_t lds = groups_lds_bytes(sh);
    auto kern = attention_groups_bf16<D, MODE>;
    if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds)) return e;
    hipLaunchKernelGGL(kern, dim3((groups + kGroupWaves - 1) / kGroupWaves), dim3(kGroupWaves * kWave), lds, st,
                       static_cast<const uint16_t *>(Q), static_cast<const uint16_t *>(K),
                       static_cast<const uint16_t *>(V), idx, Pin, S, O, sh.L, sh.keep, keep_pad, sh.scale, groups);
    return hipGetLastError();
}

template <int D>
hipError_t launch_groups_d(AttnMode mode, const dsa_shape &sh, const void *Q, const void *K, const void *V,
                           const int32_t *idx, const float *Pin, float *S, float *O, hipStream_t st)
{
    if (mode == kSddmm) return launch_groups<D, kSddmm>(sh, Q, K, V, idx, Pin, S, O, st);
    if (mode == kSpmm) return launch_groups<D, kSpmm>(sh, Q, K, V, idx, Pin, S, O, st);
    return launch_groups<D, kFused>(sh, Q, K, V, idx, Pin, S, O, st);
}

}  // namespace

int attention_max_keep() { return kMaxKeep; }

// The row kernel forms byte offsets inside one head (key index * bytes of a row, at most 512) in 32-bit arithmetic.
int attention_max_L() { return 1 << 22; }

hipError_t launch_attention(AttnMode mode, const dsa_shape &sh, const void *Q, const void *K,
                            const void *V, const int32_t *idx, const float *Pin, float *S, float *O,
                            hipStream_t st)
{
    if (sh.dtype == DSA_F32) {
        if (sh.d == 64) return launch_rows<float, 64>(mode, sh, Q, K, V, idx, Pin, S, O, st);
        return launch_rows<float, 128>(mode, sh, Q, K, V, idx, Pin, S, O, st);
    }
    if (sh.vec == 8 && groups_lds_bytes(sh) <= 144 * 1024) {
        if (sh.d == 64) return launch_groups_d<64>(mode, sh, Q, K, V, idx, Pin, S, O, st);
        return launch_groups_d<128>(mode, sh, Q, K, V, idx, Pin, S, O, st);
    }
    if (sh.d == 64) return launch_rows<uint16_t, 64>(mode, sh, Q, K, V, idx, Pin, S, O, st);
    return launch_rows<uint16_t, 128>(mode, sh, Q, K, V, idx, Pin, S, O, st);
}

hipError_t launch_attention_csr(const dsa_shape &sh, const void *Q, const void *K, const void *V,
                                const int32_t *row_ptr, const int32_t *col, float *O, hipStream_t st)
{
    const unsigned rows = (unsigned)sh.B * sh.H * sh.L;
    const dim3 grid((rows + kRowWaves - 1) / kRowWaves), block(kRowWaves * kWave);
    auto go = [&](auto kern, auto *q, auto *k, auto *v) -> hipError_t {
        hipLaunchKernelGGL(kern, grid, block, 0, st, q, k, v, row_ptr, col, O, sh.L, sh.vec, sh.scale, rows);
        return hipGetLastError();
    };
    if (sh.dtype == DSA_F32) {
        const float *q = static_cast<const float *>(Q), *k = static_cast<const float *>(K), *v = static_cast<const float *>(V);
        return sh.d == 64 ? go(attention_rows_csr<float, 64>, q, k, v) : go(attention_rows_csr<float, 128>, q, k, v);
    }
    const uint16_t *q = static_cast<const uint16_t *>(Q), *k = static_cast<const uint16_t *>(K),
                   *v = static_cast<const uint16_t *>(V);
    return sh.d == 64 ? go(attention_rows_csr<uint16_t, 64>, q, k, v) : go(attention_rows_csr<uint16_t, 128>, q, k, v);
}

hipError_t launch_gather_probe(const dsa_shape &sh, const void *K, const void *V, const int32_t *idx, unsigned *sink,
                               hipStream_t st)
{
    const unsigned rows = (unsigned)sh.B * sh.H * sh.L;
    const dim3 grid((rows + kRowWaves - 1) / kRowWaves), block(kRowWaves * kWave);
    const int keep_pad = (sh.keep + kRowPad - 1) / kRowPad * kRowPad;
    const size_t lds = (size_t)kRowWaves * keep_pad * sizeof(int);
    auto go = [&](auto kern, auto *k, auto *v) -> hipError_t {
        if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds)) return e;
        hipLaunchKernelGGL(kern, grid, block, lds, st, k, v, idx, sink, sh.L, sh.keep, keep_pad, sh.vec, rows);
        return hipGetLastError();
    };
    if (sh.dtype == DSA_F32) {
        const float *k = static_cast<const float *>(K), *v = static_cast<const float *>(V);
        return sh.d == 64 ? go(gather_probe<float, 64>, k, v) : go(gather_probe<float, 128>, k, v);
    }
    const uint16_t *k = static_cast<const uint16_t *>(K), *v = static_cast<const uint16_t *>(V);
    return sh.d == 64 ? go(gather_probe<uint16_t, 64>, k, v) : go(gather_probe<uint16_t, 128>, k, v);
}

hipError_t launch_softmax(const dsa_shape &sh, const float *S, float *P, hipStream_t st)
{
    const unsigned rows = (unsigned)sh.B * sh.H * sh.L;
    hipLaunchKernelGGL(softmax_rows, dim3((rows + kRowWaves - 1) / kRowWaves), dim3(kRowWaves * kWave),
                       0, st, S, P, sh.keep, rows);
    return hipGetLastError();
}

}  // namespace dsa
