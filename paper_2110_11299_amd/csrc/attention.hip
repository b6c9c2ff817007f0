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

namespace dsa {
namespace {

constexpr int kRowWaves = 4;          // query rows (wavefronts) per workgroup
constexpr int kMaxKeep = 8192;        // scores of a row in LDS: 4 waves * 8192 * 4 B = 128 KB

template <typename T> struct Piece;   // 16 bytes of a row as floats
template <> struct Piece<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void load(const float *p, float (&v)[4])
    {
        const float4 x = *reinterpret_cast<const float4 *>(p);
        v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
    }
};
template <> struct Piece<uint16_t> {  // bfloat16: the upper half of a float
    static constexpr int N = 8;
    static __device__ __forceinline__ void load(const uint16_t *p, float (&v)[8])
    {
        const uint4 x = *reinterpret_cast<const uint4 *>(p);
        const unsigned w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
};

// Sum over the LPR lanes that hold one row (LPR is a power of two <= 32).
template <int LPR> __device__ __forceinline__ float piece_sum(float x)
{
#pragma unroll
    for (int off = 1; off < LPR; off <<= 1) x += __shfl_xor(x, off, kWave);
    return x;
}
// Combine the 64/LPR row groups of a wavefront.
template <int LPR> __device__ __forceinline__ float groups_sum(float x)
{
#pragma unroll
    for (int off = LPR; off < kWave; off <<= 1) x += __shfl_xor(x, off, kWave);
    return x;
}
template <int LPR> __device__ __forceinline__ float groups_max(float x)
{
#pragma unroll
    for (int off = LPR; off < kWave; off <<= 1) x = fmaxf(x, __shfl_xor(x, off, kWave));
    return x;
}

// MODE kFused: Q,K,V,idx -> O.  kSddmm: Q,K,idx -> S.  kSpmm: Pin,V,idx -> O.
template <typename T, int D, int MODE>
__global__ __launch_bounds__(kRowWaves *kWave) void attention_rows(
    const T *__restrict__ Q, const T *__restrict__ K, const T *__restrict__ V,
    const int32_t *__restrict__ idx, const float *__restrict__ Pin, float *__restrict__ S,
    float *__restrict__ O, int L, int keep, int vec, float scale, unsigned total_rows)
{
    constexpr int E = Piece<T>::N;        // elements per lane
    constexpr int LPR = D / E;            // lanes per row
    constexpr int RPI = kWave / LPR;      // gathered rows per wavefront instruction
    extern __shared__ float lds_scores[];

    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int sub = lane % LPR, grp = lane / LPR;
    const unsigned vblock = xcd_contiguous(blockIdx.x, gridDim.x);
    const unsigned row = vblock * kRowWaves + wave;
    const bool live = row < total_rows;
    const unsigned r = live ? row : total_rows - 1;      // dead waves shadow a real row, write nothing
    const unsigned n = r / (unsigned)L, i = r % (unsigned)L;
    const int32_t *list = idx + ((size_t)n * (L / vec) + i / vec) * keep;
    float *sc = lds_scores + wave * keep;

    float m = -INFINITY;
    if (MODE != kSpmm) {
        float q[E];
        Piece<T>::load(Q + (size_t)r * D + sub * E, q);
#pragma unroll
        for (int e = 0; e < E; ++e) q[e] *= scale;
        const T *Kh = K + (size_t)n * L * D + sub * E;
        for (int t0 = 0; t0 < keep; t0 += RPI) {
            const int t = t0 + grp;
            const bool valid = t < keep;
            const int j = min(max(list[valid ? t : keep - 1], 0), L - 1);   // stay inside K for any idx
            float kv[E];
            Piece<T>::load(Kh + (size_t)j * D, kv);
            float acc = 0.f;
#pragma unroll
            for (int e = 0; e < E; ++e) acc = fmaf(q[e], kv[e], acc);
            acc = piece_sum<LPR>(acc);
            if (valid) {
                m = fmaxf(m, acc);
                if (sub == 0) {
                    if (MODE == kSddmm) { if (live) S[(size_t)r * keep + t] = acc; }
                    else sc[t] = acc;
                }
            }
        }
        if (MODE == kSddmm) return;
        m = groups_max<LPR>(m);
        __syncthreads();
    }

    float o[E], z = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) o[e] = 0.f;
    const T *Vh = V + (size_t)n * L * D + sub * E;
    for (int t0 = 0; t0 < keep; t0 += RPI) {
        const int t = t0 + grp;
        const bool valid = t < keep;
        const int tt = valid ? t : keep - 1;
        const int j = min(max(list[tt], 0), L - 1);
        float p;
        if (MODE == kSpmm) p = Pin[(size_t)r * keep + tt];
        else p = __expf(sc[tt] - m);
        p = valid ? p : 0.f;
        float vv[E];
        Piece<T>::load(Vh + (size_t)j * D, vv);
        z += p;
#pragma unroll
        for (int e = 0; e < E; ++e) o[e] = fmaf(p, vv[e], o[e]);
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

// Softmax over the `keep` scores of each row: one wavefront per row.
__global__ __launch_bounds__(kRowWaves *kWave) void softmax_rows(const float *S, float *P, int keep,
                                                                  unsigned total_rows)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const unsigned row = blockIdx.x * kRowWaves + wave;
    if (row >= total_rows) return;
    const float *s = S + (size_t)row * keep;
    float *p = P + (size_t)row * keep;
    float m = -INFINITY;
    for (int t = lane; t < keep; t += kWave) m = fmaxf(m, s[t]);
    m = groups_max<1>(m);
    float z = 0.f;
    for (int t = lane; t < keep; t += kWave) z += __expf(s[t] - m);
    z = groups_sum<1>(z);
    const float inv = 1.f / z;
    for (int t = lane; t < keep; t += kWave) p[t] = __expf(s[t] - m) * inv;
}

template <typename T, int D>
hipError_t launch_rows(AttnMode mode, const dsa_shape &sh, const void *Q, const void *K, const void *V,
                       const int32_t *idx, const float *Pin, float *S, float *O, hipStream_t st)
{
    const unsigned rows = (unsigned)sh.B * sh.H * sh.L;
    const dim3 grid((rows + kRowWaves - 1) / kRowWaves), block(kRowWaves * kWave);
    const size_t lds = mode == kFused ? (size_t)kRowWaves * sh.keep * sizeof(float) : 0;
    const T *q = static_cast<const T *>(Q), *k = static_cast<const T *>(K), *v = static_cast<const T *>(V);
    if (mode == kFused) {
        auto kern = attention_rows<T, D, kFused>;
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kern, grid, block, lds, st, q, k, v, idx, Pin, S, O, sh.L, sh.keep, sh.vec,
                           sh.scale, rows);
    } else if (mode == kSddmm) {
        hipLaunchKernelGGL((attention_rows<T, D, kSddmm>), grid, block, 0, st, q, k, v, idx, Pin, S, O,
                           sh.L, sh.keep, sh.vec, sh.scale, rows);
    } else {
        hipLaunchKernelGGL((attention_rows<T, D, kSpmm>), grid, block, 0, st, q, k, v, idx, Pin, S, O,
                           sh.L, sh.keep, sh.vec, sh.scale, rows);
    }
    return hipGetLastError();
}

}  // namespace

int attention_max_keep() { return kMaxKeep; }

hipError_t launch_attention(AttnMode mode, const dsa_shape &sh, const void *Q, const void *K,
                            const void *V, const int32_t *idx, const float *Pin, float *S, float *O,
                            hipStream_t st)
{
    if (sh.dtype == DSA_F32) {
        if (sh.d == 64) return launch_rows<float, 64>(mode, sh, Q, K, V, idx, Pin, S, O, st);
        return launch_rows<float, 128>(mode, sh, Q, K, V, idx, Pin, S, O, st);
    }
    if (sh.d == 64) return launch_rows<uint16_t, 64>(mode, sh, Q, K, V, idx, Pin, S, O, st);
    return launch_rows<uint16_t, 128>(mode, sh, Q, K, V, idx, Pin, S, O, st);
}

hipError_t launch_softmax(const dsa_shape &sh, const float *S, float *P, hipStream_t st)
{
    const unsigned rows = (unsigned)sh.B * sh.H * sh.L;
    hipLaunchKernelGGL(softmax_rows, dim3((rows + kRowWaves - 1) / kRowWaves), dim3(kRowWaves * kWave),
                       0, st, S, P, sh.keep, rows);
    return hipGetLastError();
}

}  // namespace dsa
