// Prediction path of Dynamic Sparse Attention (paper section 3.1): approximate scores
// S~ = Q~ K~^T from int8 projections, optional sum over the 8 rows of a column vector
// (section 5.1), and the per-unit top-k that becomes the mask.  Scores are exact integers, so
// the selection is exact: larger score first, lower key index among equals, list ascending.
#include "dsa_internal.h"
#include "predict_api.h"
#include "predict_stream_api.h"
#include "wave_select.h"

namespace dsa {
namespace {

constexpr int kUnitThreads = 256;
constexpr int kUnitMaxL = 32768;     // one unit's scores in LDS: 128 KB

// One workgroup per selection unit.  All L scores of the unit are computed with packed int8
// dot products into LDS; the keep-th largest value T is found by bisection on the value (the
// count of scores >= T is monotone in T); then the keys with score > T, and the first
// keep - count(> T) keys with score == T, are written in ascending key order.
template <int VEC>
__global__ __launch_bounds__(kUnitThreads) void predict_unit(const int8_t *__restrict__ Qt,
                                                             const int8_t *__restrict__ Kt,
                                                             int32_t *__restrict__ idx, int L, int k,
                                                             int keep)
{
    extern __shared__ int lds[];
    int *score = lds;                       // [L]
    int *qrows = lds + L;                   // [VEC * k/4] packed int8x4
    int *red = qrows + VEC * (k / 4);       // [8]
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    constexpr int kWaves = kUnitThreads / kWave;
    const unsigned u = blockIdx.x;
    const unsigned G = L / VEC, n = u / G, g = u % G;
    const int k4 = k / 4;

    const int *qsrc = reinterpret_cast<const int *>(Qt + ((size_t)n * L + (size_t)g * VEC) * k);
    for (int c = tid; c < VEC * k4; c += kUnitThreads) qrows[c] = qsrc[c];
    __syncthreads();

    const int8_t *Kh = Kt + (size_t)n * L * k;
    int vmax = INT32_MIN, vmin = INT32_MAX;
    for (int j = tid; j < L; j += kUnitThreads) {
        const v4i *kr = reinterpret_cast<const v4i *>(Kh + (size_t)j * k);
        int s = 0;
        for (int c4 = 0; c4 < k4; c4 += 4) {
            const v4i kk = kr[c4 / 4];
#pragma unroll
            for (int r = 0; r < VEC; ++r) {
                s = __builtin_amdgcn_sdot4(qrows[r * k4 + c4 + 0], kk.x, s, false);
                s = __builtin_amdgcn_sdot4(qrows[r * k4 + c4 + 1], kk.y, s, false);
                s = __builtin_amdgcn_sdot4(qrows[r * k4 + c4 + 2], kk.z, s, false);
                s = __builtin_amdgcn_sdot4(qrows[r * k4 + c4 + 3], kk.w, s, false);
            }
        }
        score[j] = s;
        vmax = max(vmax, s);
        vmin = min(vmin, s);
    }
    vmax = wave_max(vmax);
    vmin = wave_min(vmin);
    if (lane == 0) { red[wave] = vmax; red[kWaves + wave] = vmin; }
    __syncthreads();
    int hi = red[0], lo = red[kWaves];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) { hi = max(hi, red[w]); lo = min(lo, red[kWaves + w]); }
    __syncthreads();

    // Invariant: count(score >= lo) >= keep; count(score >= hi + 1) < keep.  Ends with lo == hi.
    int *cnt = red;   // cnt[0]
    while (lo < hi) {
        const int mid = lo + (int)(((long long)hi - lo + 1) / 2);
        if (tid == 0) cnt[0] = 0;
        __syncthreads();
        int c = 0;
        for (int j = tid; j < L; j += kUnitThreads) c += score[j] >= mid;
        c = wave_sum(c);
        if (lane == 0) atomicAdd(&cnt[0], c);
        __syncthreads();
        const int total = cnt[0];
        __syncthreads();
        if (total >= keep) lo = mid; else hi = mid - 1;
    }
    const int T = lo;

    if (wave == 0) {
        int c = 0;
        for (int j = lane; j < L; j += kWave) c += score[j] > T;
        const int need_eq = keep - wave_sum(c);
        int32_t *out = idx + (size_t)u * keep;
        int out_base = 0, eq_base = 0;
        const unsigned long long below = (1ull << lane) - 1ull;
        for (int j0 = 0; j0 < L; j0 += kWave) {
            const int j = j0 + lane;
            const int s = j < L ? score[j] : INT32_MIN;
            const bool gt = j < L && s > T, eq = j < L && s == T;
            const unsigned long long meq = __ballot(eq);
            const bool sel = gt || (eq && eq_base + __popcll(meq & below) < need_eq);
            const unsigned long long msel = __ballot(sel);
            if (sel) out[out_base + __popcll(msel & below)] = j;
            out_base += __popcll(msel);
            eq_base += __popcll(meq);
        }
    }
}


// ---------------------------------------------------------------------------------------------
// Tiled predictor.  One workgroup of W wavefronts owns 16 selection units of one head and sweeps
// the keys in chunks of 16*W*TC.  Matrix-core orientation: keys are the rows (A operand), units
// the columns (B operand) of v_mfma_i32_16x16x{32,64}_i8, so lane (c = lane%16, g = lane/16)
// ends up holding, for unit c, the scores of 4 keys per tile.  The 4*W "holders" (wave, g) of a
// unit each own 4*TC consecutive keys of the chunk, which makes every lane's score stream
// contiguous in key order.  For vec = 8 the unit's 8 query rows are simply concatenated along
// the contraction (length 8k, the key operand repeating with period k): the matrix core
// produces the group sum itself.
//
// Selection never sorts and never re-reads a score from memory.  Scores stay in registers.
//  (A) each lane keeps NB bucket maxima of its stream;
//  (B) the keep-th largest of a unit's bucket maxima is a lower bound T0 of its keep-th largest
//      score (the buckets are disjoint, so that many distinct scores reach T0);
//  (C) each lane compares its scores with T0: the outcomes, shifted into 32-bit words, ARE the
//      unit's bitmap over keys, and the scores that pass are appended to the lane's own small
//      LDS segment (every score is written at the current end of the segment, and the end only
//      moves past it if it passed) -- 5 VALU operations and one LDS write per score, no branch;
//  (D) one wavefront per unit walks the bitmap in key order, pairs each candidate key with its
//      score from the segments, bisects for the exact threshold in registers and writes the kept
//      keys in ascending order, breaking ties by key index through ballot prefix counts.
// A unit whose candidates do not fit is almost always one where very many keys share the score
// T0 (codes with few levels).  In a single-chunk plan its lanes run (C) once more with T0 + 1:
// the bits that drop out of the bitmap are the ties, and if fewer than keep scores lie above T0
// the answer is those keys plus the first ties in key order, with no score involved.  What still
// does not fit (very large keep, plateaus above T0, multi-chunk plans) takes a slower path that
// recomputes scores from Q~, K~ with packed dot products.
// When a compute unit holds one workgroup, one workgroup per compute unit is launched and each
// loops over its tiles.
// ---------------------------------------------------------------------------------------------
constexpr int kTileUnits = 16;

constexpr int kCompactCap = 512;      // candidates of one unit that the register path handles
constexpr int kSegSlots = 1024;       // segment slots per unit (all holders, all chunks)
constexpr size_t kLdsBudget = 150 * 1024;       // of the 160 KB a gfx950 workgroup may use
constexpr int kAllCandidates = INT32_MIN + 1;   // T0 when no bound is known; padding scores are INT32_MIN

template <int KSTEP> struct Mfma;
template <> struct Mfma<32> {
    typedef long op_t;
    static constexpr int kBytes = 8;
    static __device__ __forceinline__ op_t load(const int8_t *p) { return *reinterpret_cast<const long *>(p); }
    static __device__ __forceinline__ op_t zero() { return 0; }
    static __device__ __forceinline__ v4i run(op_t a, op_t b, v4i c)
    {
        return __builtin_amdgcn_mfma_i32_16x16x32_i8(a, b, c, 0, 0, 0);
    }
};
template <> struct Mfma<64> {
    typedef v4i op_t;
    static constexpr int kBytes = 16;
    static __device__ __forceinline__ op_t load(const int8_t *p) { return *reinterpret_cast<const v4i *>(p); }
    static __device__ __forceinline__ op_t zero() { return v4i{0, 0, 0, 0}; }
    static __device__ __forceinline__ v4i run(op_t a, op_t b, v4i c)
    {
        return __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0);
    }
};

// (A) for one wavefront and one chunk: scores of TC tiles into registers plus bucket maxima.
// Key rows are loaded unconditionally from clamped addresses: a key beyond L only feeds output
// rows that TAIL overwrites with INT32_MIN, and a contraction piece beyond Ka meets a zero unit
// operand, so neither needs a zeroed key operand.
template <int TC, int NB, int KSTEP, int MAXSTEPS, bool TAIL>
__device__ __forceinline__ void score_chunk(v4i (&acc)[TC], int (&bmax)[NB], const int8_t *__restrict__ Kh,
                                            int k, int L, int op_lo, int out_lo, int nsteps, bool same_kop,
                                            const typename Mfma<KSTEP>::op_t (&qop)[MAXSTEPS],
                                            const int (&koff)[MAXSTEPS])
{
    typedef Mfma<KSTEP> M;
    constexpr int BATCH = 8;
    // Byte offsets inside the head (L * k <= 4 MB) on top of the wavefront-uniform base pointer: one
    // 32-bit add per key row instead of a 64-bit multiply.
    const unsigned off0 = (unsigned)op_lo * (unsigned)k;
    const unsigned tile_step = 4u * (unsigned)k;
    const unsigned off_last = (unsigned)(L - 1) * (unsigned)k;
#pragma unroll
    for (int t0 = 0; t0 < TC; t0 += BATCH) {
        typename M::op_t kop[BATCH];
        unsigned krow[BATCH];
#pragma unroll
        for (int b = 0; b < BATCH; ++b) {
            unsigned off = off0 + (unsigned)(t0 + b) * tile_step;
            if (TAIL) off = min(off, off_last);
            krow[b] = off;
            kop[b] = M::load(Kh + (size_t)(off + (unsigned)koff[0]));
        }
#pragma unroll
        for (int b = 0; b < BATCH; ++b) {
            const int t = t0 + b;
            v4i a = {0, 0, 0, 0};
            a = M::run(kop[b], qop[0], a);
#pragma unroll
            for (int s = 1; s < MAXSTEPS; ++s) {
                if (s < nsteps) {
                    if (!same_kop) kop[b] = M::load(Kh + (size_t)(krow[b] + (unsigned)koff[s]));
                    a = M::run(kop[b], qop[s], a);
                }
            }
            if (TAIL) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (out_lo + 4 * t + i >= L) a[i] = INT32_MIN;
            }
            acc[t] = a;
            const int bk = t * NB / TC;
            bmax[bk] = max(bmax[bk], max(max(a[0], a[1]), max(a[2], a[3])));
        }
    }
}

template <int TC, int NB, int KSTEP, int MAXSTEPS, int MAXW>
__global__ __launch_bounds__(MAXW *kWave) void predict_tiles(const int8_t *__restrict__ Qt,
                                                     const int8_t *__restrict__ Kt,
                                                     int32_t *__restrict__ idx, int L, int k, int keep,
                                                     int vec, int nchunks, int tiles_per_head, int hc_log2,
                                                     unsigned total_tiles)
{
    typedef Mfma<KSTEP> M;
    static_assert(TC % 8 == 0 && TC % NB == 0, "tile counts");
    constexpr int WPH = TC / 8;                  // bitmap words per holder and chunk
    extern __shared__ int smem[];
    const int W = blockDim.x >> 6;
    const int lane = threadIdx.x & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wavefront index, scalar
    const int c = lane & 15, g = lane >> 4;
    const int NBT = 4 * W * NB;                  // bucket maxima per unit and chunk
    const int chunk_keys = kTileUnits * W * TC;
    const int NW = nchunks * (chunk_keys / 32);  // bitmap words per unit
    const int HC = 1 << hc_log2;                 // slots of one holder's segment
    const int NHT = nchunks * 4 * W;             // holders per unit over all chunks
    const int SL = NHT << hc_log2;               // segment slots per unit
    // Per-unit arrays use odd strides (length + 1) so that the 16 units of a wavefront instruction
    // fall into different LDS banks.
    const int NBTp = NBT + 1, NWp = NW + 1, NHTp = NHT + 1;
    int *T0s = smem;                                                            // [16]
    int *strict = T0s + kTileUnits;                                             // [16] unit redone with score > T0
    int *wrapf = strict + kTileUnits;                                           // [16] some holder wrapped
    int *ncand = wrapf + kTileUnits;                                            // [16][4] candidates (single chunk),
                                                                                // one counter per lane group
    int *seg = ncand + 4 * kTileUnits;                                          // [16][NHT][HC]
    unsigned *bitmap = reinterpret_cast<unsigned *>(seg + kTileUnits * SL);     // [16][NW+1]
    int *cnts = reinterpret_cast<int *>(bitmap + kTileUnits * NWp);             // [16][NHT+1]
    int *bm = cnts + kTileUnits * NHTp;                                         // [16][NBT+1], phases A-B
    int2 *compact = reinterpret_cast<int2 *>(bm) + w * kCompactCap;             // per wavefront, phase D:
                                                                                // reuses the bm storage
    // [16][NW+1] keys whose score equals T0, single-chunk plans only
    unsigned *eqmap = reinterpret_cast<unsigned *>(bm + max(kTileUnits * NBTp, W * kCompactCap * 2));

    // A workgroup works through tiles blockIdx.x, blockIdx.x + gridDim.x, ...: with one workgroup
    // resident per compute unit the stores of one tile then drain while the next tile's keys load.
    // gridDim.x is a multiple of the XCD count whenever it is smaller than total_tiles, so all tiles
    // of a workgroup map to the XCD it runs on.
    for (unsigned vt = blockIdx.x; vt < total_tiles; vt += gridDim.x) {
    const unsigned tile = xcd_contiguous(vt, total_tiles);
    const unsigned n = tile / (unsigned)tiles_per_head;
    const int u0 = (int)(tile % (unsigned)tiles_per_head) * kTileUnits;
    const int G = L / vec;
    const int Ka = vec * k;
    const int nsteps = (Ka + KSTEP - 1) / KSTEP;
    const int8_t *Kh = Kt + (size_t)n * L * k;
    const int8_t *Qh = Qt + (size_t)n * L * k;   // unit u occupies bytes [u*Ka, u*Ka + Ka)

    // B operand: unit u0+c, piece g of every contraction step.  Key operand offsets per step.  The
    // 16-wavefront plans (128 registers a lane) load them per chunk, so that the registers are free
    // again in the selection phases; the 8-wavefront plans keep them.
    typename M::op_t qop[MAXSTEPS];
    int koff[MAXSTEPS];
    auto load_unit_operands = [&]() {
        const bool unit_live = u0 + c < G;
#pragma unroll
        for (int s = 0; s < MAXSTEPS; ++s) {
            const int m = KSTEP * s + M::kBytes * g;
            const bool ok = s < nsteps && m < Ka;
            qop[s] = (ok && unit_live) ? M::load(Qh + (size_t)(u0 + c) * Ka + m) : M::zero();
            koff[s] = ok ? m % k : 0;
        }
    };
    if (MAXW != 16) load_unit_operands();
    // the key operand repeats from step to step when k divides the step width
    const bool same_kop = (KSTEP % k) == 0;

    if (threadIdx.x < kTileUnits) {
        T0s[threadIdx.x] = kAllCandidates;
        strict[threadIdx.x] = 0;
        wrapf[threadIdx.x] = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) ncand[4 * threadIdx.x + i] = 0;
    }
    __syncthreads();

    for (int chunk = 0; chunk < nchunks; ++chunk) {
        const int chunk_base = chunk * chunk_keys;
        const int wave_lo = chunk_base + w * kTileUnits * TC;          // first key of this wavefront
        const int out_lo = wave_lo + g * 4 * TC;                        // first key of this lane's stream
        const int op_lo = wave_lo + (c >> 2) * 4 * TC + (c & 3);        // operand row c of tile 0
        if (MAXW == 16) load_unit_operands();
        v4i acc[TC];
        int bmax[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) bmax[b] = INT32_MIN;

        if (wave_lo < L) {
            if (wave_lo + kTileUnits * TC > L)
                score_chunk<TC, NB, KSTEP, MAXSTEPS, true>(acc, bmax, Kh, k, L, op_lo, out_lo, nsteps, same_kop,
                                                          qop, koff);
            else
                score_chunk<TC, NB, KSTEP, MAXSTEPS, false>(acc, bmax, Kh, k, L, op_lo, out_lo, nsteps,
                                                           same_kop, qop, koff);
        } else {
#pragma unroll
            for (int t = 0; t < TC; ++t) acc[t] = v4i{INT32_MIN, INT32_MIN, INT32_MIN, INT32_MIN};
        }

        // (B) lower bound T0 per unit from the bucket maxima
#pragma unroll
        for (int b = 0; b < NB; ++b) bm[c * NBTp + (4 * w + g) * NB + b] = bmax[b];
        __syncthreads();
        // Buckets follow key order inside the chunk, so the ones that hold a real key are the first
        // `real` of them; the others keep INT32_MIN.
        const int bucket_keys = 4 * TC / NB;
        const int real = min(NBT, max(0, (L - chunk_base + bucket_keys - 1) / bucket_keys));
        constexpr int VB = NB * MAXW / 16;  // NBT <= 4 * MAXW * NB values over 64 lanes
        const bool dense = real == NBT && NBT == VB * kWave;
        for (int uu = w; uu < kTileUnits; uu += W) {
            const int *v = bm + uu * NBTp;
            int vb[VB];
            int T = INT32_MIN;
            if (dense) {
#pragma unroll
                for (int i = 0; i < VB; ++i) vb[i] = v[i * kWave + lane];
                int lo = vb[0], hi = vb[0];
#pragma unroll
                for (int i = 1; i < VB; ++i) {
                    lo = min(lo, vb[i]);
                    hi = max(hi, vb[i]);
                }
                if (real >= keep) T = kth_largest<VB>(vb, keep, wave_min(lo), wave_max(hi), keep >> 4);
            } else {
#pragma unroll
                for (int i = 0; i < VB; ++i) vb[i] = v[min(i * kWave + lane, NBT - 1)];
                int lo = INT32_MAX, hi = INT32_MIN;
#pragma unroll
                for (int i = 0; i < VB; ++i) {
                    if (i * kWave + lane >= real) vb[i] = INT32_MIN;
                    else lo = min(lo, vb[i]);
                    hi = max(hi, vb[i]);
                }
                if (real >= keep)
                    T = kth_largest_of<VB>(vb, (NBT + kWave - 1) / kWave, keep, wave_min(lo), wave_max(hi), keep >> 4);
            }
            if (lane == 0) T0s[uu] = max(T0s[uu], T);
        }
        __syncthreads();

        // (C) candidates: bit j of a unit's bitmap = score(unit, key j) >= thr; passing scores are
        // appended, in key order, to this holder's segment.  thr is T0.
        // (C') Ties.  When a unit's candidates do not fit (more than the compact list holds, or a
        // holder with HC or more) it is nearly always because very many keys share the score T0, as
        // with few-level codes.  Such a unit goes through the same code once more with thr = T0 + 1:
        // bitmap and segments then take score > T0, and the bits that drop out of the bitmap are the
        // keys with score == T0, kept in a second bitmap.  If fewer than keep scores lie above T0 the
        // answer is those plus the first ties in key order and needs no score at all.  Only plans
        // with a single chunk still hold every score in registers at that point.
        const int holder = chunk * 4 * W + 4 * w + g;
        int *myseg = seg + c * SL + (holder << hc_log2);
        // entry o sits in slot (o + rot) % HC; the rotation spreads the lanes of this instruction, and
        // the lanes that later read one unit's segments, over the LDS banks
        const int rot = lane + (holder >> 2);
        unsigned *words = bitmap + c * NWp + out_lo / 32;
        int thr = T0s[c];
        bool mine = true;             // this lane's unit takes part in the current pass
        for (int pass = 0; pass < 2; ++pass) {
            if (mine) {
                int pos0 = 0;
#pragma unroll
                for (int q = 0; q < WPH; ++q) {
                    unsigned word = 0;
                    int pos = pos0;
#pragma unroll
                    for (int e = 0; e < 32; ++e) {
                        const int s = acc[8 * q + e / 4][e % 4];
                        myseg[(pos + rot) & (HC - 1)] = s;      // kept only if the end moves past it
                        // word = 2*word + (s >= thr): compare into the carry, add with carry
                        asm("v_cmp_ge_i32 vcc, %1, %2\n\tv_addc_co_u32 %0, vcc, %0, %0, vcc"
                            : "+v"(word)
                            : "v"(s), "v"(thr)
                            : "vcc");
                        pos = pos0 + __popc(word);
                    }
                    word = __brev(word);                // the first key of the word was shifted in first
                    if (pass) eqmap[c * NWp + out_lo / 32 + q] = words[q] & ~word;
                    words[q] = word;
                    pos0 = pos;
                }
                cnts[c * NHTp + holder] = pos0;         // HC or more means the segment wrapped
                if (pass == 0 && nchunks == 1 && thr != kAllCandidates) {
                    atomicAdd(&ncand[4 * c + g], pos0);     // 64 different addresses per instruction
                    if (pos0 >= HC) wrapf[c] = 1;
                }
            }
            if (nchunks != 1) break;
            __syncthreads();              // also the barrier in front of (D)
            if (pass) break;
            const int4 part = *reinterpret_cast<const int4 *>(ncand + 4 * c);
            mine = ((part.x + part.y) + (part.z + part.w) > kCompactCap || wrapf[c] != 0) && u0 + c < G;
            // lanes c = 0..15 of every wavefront see all units: the same outcome everywhere
            if (__ballot(mine) == 0) break;
            strict[c] = mine;
            thr += 1;
        }
        // bm / T0s are rewritten only after the next chunk's first barrier
    }
    if (nchunks != 1) __syncthreads();

    // (D) exact selection among the candidates, one wavefront per unit
    const int k4 = k / 4;
    const unsigned long long below = (1ull << lane) - 1ull;
    for (int uu = w; uu < kTileUnits; uu += W) {
        const int u = u0 + uu;
        if (u >= G) break;
        const unsigned *bw = bitmap + uu * NWp;
        const int *cu = cnts + uu * NHTp;
        const int *sg = seg + uu * SL;
        const int *qu = reinterpret_cast<const int *>(Qh + (size_t)u * Ka);
        int32_t *out = idx + ((size_t)n * G + u) * keep;
        // candidates have score >= lo0: T0, or T0 + 1 for a unit redone with the strict threshold
        const int lo0 = T0s[uu] + strict[uu];

        int nc = 0;
        for (int h = lane; h < NHT; h += kWave) nc += cu[h];
        nc = wave_sum(nc);
        const bool fits = nc <= kCompactCap;

        if (strict[uu] && nc < keep) {
            // fewer than keep scores above T0 and at least keep at or above it: the keep-th largest is
            // T0, and the answer is every key above it plus the first keep - nc keys equal to it
            const unsigned *ew = eqmap + uu * NWp;
            int need = keep - nc, out_base = 0;
            for (int w0 = 0; w0 < NW; w0 += 2 * kWave) {
                const int wi = w0 + 2 * lane;
                const bool live = wi < NW;
                const int wic = min(wi, NW - 2);
                const unsigned g0 = live ? bw[wic] : 0u, g1 = live ? bw[wic + 1] : 0u;
                const unsigned e0 = live ? ew[wic] : 0u, e1 = live ? ew[wic + 1] : 0u;
                const int ce0 = __popc(e0), ce = ce0 + __popc(e1);
                int ties_round;
                const int ties_incl = wave_incl_scan(ce, lane, &ties_round);
                const int room = need - (ties_incl - ce);        // ties this lane may still take
                need -= ties_round;
                const unsigned s0 = g0 | lowest_set_bits(e0, room);
                const unsigned s1 = g1 | lowest_set_bits(e1, room - ce0);
                const int cs = __popc(s0) + __popc(s1);
                int sel_round;
                const int sel_incl = wave_incl_scan(cs, lane, &sel_round);
                int32_t *dst = out + out_base + sel_incl - cs;
                out_base += sel_round;
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    unsigned m = half ? s1 : s0;
                    while (m) {
                        *dst++ = (wic + half) * 32 + __ffs(m) - 1;
                        m &= m - 1;
                    }
                }
            }
        } else if (fits) {
            // candidates in key order as (score, key) pairs; a lane takes two bitmap words per round
            int rank_base = 0;
            for (int w0 = 0; w0 < NW; w0 += 2 * kWave) {
                const int wi = w0 + 2 * lane;           // even; NW is a multiple of 4
                const bool live = wi < NW;
                const int wic = min(wi, NW - 2);
                const unsigned m0 = live ? bw[wic] : 0u;
                const unsigned m1 = live ? bw[wic + 1] : 0u;
                const int c0 = __popc(m0), c1 = __popc(m1);
                int round_total;
                const int incl = wave_incl_scan(c0 + c1, lane, &round_total);
                const int r = rank_base + incl - (c0 + c1);
                rank_base += round_total;
                // holder of each word and the slot of the word's first entry in the holder's segment
                // (the writer's rotation plus the entries of the holder's earlier words)
                const int hold0 = wic / WPH;
                const int hold1 = WPH == 1 ? wic + 1 : hold0;
                int o0 = uu + 16 * (hold0 & 3) + (hold0 >> 2);
                if (WPH == 4 && (wic & 2)) o0 += __popc(bw[wic - 1]) + __popc(bw[wic - 2]);
                const int o1 = WPH == 1 ? uu + 16 * (hold1 & 3) + (hold1 >> 2) : o0 + c0;
                // HC or more hits in a holder: its segment wrapped and a later non-candidate overwrote
                // the first entry; such a holder's few scores are recomputed instead
                const bool wrapped = (c0 && cu[hold0] >= HC) || (c1 && cu[hold1] >= HC);
                if (__ballot(wrapped) == 0) {
#pragma unroll
                    for (int half = 0; half < 2; ++half) {
                        unsigned m = half ? m1 : m0;
                        const int cw = half ? c1 : c0;
                        const int o = half ? o1 : o0;
                        const int *src = sg + ((half ? hold1 : hold0) << hc_log2);
                        int2 *dst = compact + r + (half ? c0 : 0);
                        const int key0 = (wic + half) * 32;
                        // the same trip count for every lane, two entries a trip: both segment reads
                        // are in flight before the first write
                        for (int t = 0; __ballot(t < cw) != 0; t += 2) {
                            const int v0 = src[(o + t) & (HC - 1)];
                            const int v1 = src[(o + t + 1) & (HC - 1)];
                            const int b0 = __ffs(m) - 1;
                            m &= m - 1;
                            const int b1 = __ffs(m) - 1;
                            m &= m - 1;
                            if (t < cw) dst[t] = make_int2(v0, key0 + b0);
                            if (t + 1 < cw) dst[t + 1] = make_int2(v1, key0 + b1);
                        }
                    }
                } else {
                    int rr = r;
#pragma unroll
                    for (int half = 0; half < 2; ++half) {
                        unsigned m = half ? m1 : m0;
                        const int hold = half ? hold1 : hold0;
                        int o = half ? o1 : o0;
                        const int *src = sg + (hold << hc_log2);
                        const bool redo = m && cu[hold] >= HC;
                        while (m) {
                            const int bit = __ffs(m) - 1;
                            m &= m - 1;
                            const int key = (wic + half) * 32 + bit;
                            const int sc1 = redo ? unit_key_score(qu, Kh + (size_t)key * k, vec, k4)
                                                 : src[o & (HC - 1)];
                            ++o;
                            compact[rr++] = make_int2(sc1, key);
                        }
                    }
                }
            }
            wave_lds_sync();
            constexpr int NR = kCompactCap / kWave;
            const int groups = (nc + kWave - 1) / kWave;
            int sc[NR], ck[NR];
#pragma unroll
            for (int b = 0; b < NR; ++b) {      // unconditional loads; slots past nc are blanked below
                const int2 e = compact[b * kWave + lane];
                sc[b] = e.x;
                ck[b] = e.y;
            }
            int hi = INT32_MIN;
#pragma unroll
            for (int b = 0; b < NR; ++b) {
                if (b * kWave + lane >= nc) sc[b] = INT32_MIN;
                hi = max(hi, sc[b]);
            }
            // every candidate reaches T0 and there are at least keep of them
            const int T = kth_largest_of<NR>(sc, groups, keep, lo0, wave_max(hi));
            int gt = 0;
#pragma unroll
            for (int b = 0; b < NR; ++b)
                if (b < groups) gt += __popcll(__ballot(sc[b] > T));
            const int need_eq = keep - gt;
            int out_base = 0, eq_base = 0;
#pragma unroll
            for (int b = 0; b < NR; ++b) {
                if (b < groups) {
                    const bool eq = sc[b] == T;       // T >= T0 > INT32_MIN: empty slots never match
                    const unsigned long long meq = __ballot(eq);
                    const bool sel = sc[b] > T || (eq && eq_base + __popcll(meq & below) < need_eq);
                    const unsigned long long msel = __ballot(sel);
                    if (sel) out[out_base + __popcll(msel & below)] = ck[b];
                    out_base += __popcll(msel);
                    eq_base += __popcll(meq);
                }
            }
            wave_lds_sync();      // the next unit reuses `compact`
        } else {
            // Too many candidates (massive ties or a very large keep): the same steps over all keys,
            // recomputing the score of every flagged key in every pass.
            auto flagged_score = [&](int j) -> int {
                if (j >= L || !((bw[j >> 5] >> (j & 31)) & 1u)) return INT32_MIN;
                return unit_key_score(qu, Kh + (size_t)j * k, vec, k4);
            };
            int hi = INT32_MIN;
            for (int j = lane; j < L; j += kWave) hi = max(hi, flagged_score(j));
            hi = wave_max(hi);
            int lo = lo0;
            while (lo < hi) {
                const int mid = (int)(lo + ((long long)hi - lo + 1) / 2);
                int ge = 0;
                for (int j0 = 0; j0 < L; j0 += kWave) ge += __popcll(__ballot(flagged_score(j0 + lane) >= mid));
                if (ge >= keep) lo = mid; else hi = mid - 1;
            }
            const int T = lo;
            int gt = 0;
            for (int j0 = 0; j0 < L; j0 += kWave) gt += __popcll(__ballot(flagged_score(j0 + lane) > T));
            const int need_eq = keep - gt;
            int out_base = 0, eq_base = 0;
            for (int j0 = 0; j0 < L; j0 += kWave) {
                const int j = j0 + lane;
                const int s = flagged_score(j);
                const bool eq = s == T;          // T >= T0 > INT32_MIN, so unflagged keys never match
                const unsigned long long meq = __ballot(eq);
                const bool sel = s > T || (eq && eq_base + __popcll(meq & below) < need_eq);
                const unsigned long long msel = __ballot(sel);
                if (sel) out[out_base + __popcll(msel & below)] = j;
                out_base += __popcll(msel);
                eq_base += __popcll(meq);
            }
        }
    }
    __syncthreads();      // the next tile reuses every LDS array
    }
}

struct TilePlan {
    int W, TC, NB, nchunks, kstep, maxsteps, maxw, tiles_per_head, hc_log2;
    size_t lds;
    bool ok;
};

TilePlan plan_tiles(const dsa_shape &sh)
{
    TilePlan p{};
    const int L = sh.L;
    const int Ka = sh.vec * sh.k;
    p.kstep = Ka <= 32 ? 32 : 64;
    const int nsteps = (Ka + p.kstep - 1) / p.kstep;
    p.maxsteps = nsteps <= 1 ? 1 : nsteps <= 4 ? 4 : nsteps <= 8 ? 8 : 16;
    // Short contractions leave room for 16 wavefronts of <= 128 registers (one unit each in the
    // selection phases); long ones keep their unit operands in registers and run 8 wavefronts.
    p.maxw = p.maxsteps <= 4 ? 16 : 8;
    if (L <= 128 * p.maxw) { p.TC = 8; p.W = (L + 127) / 128; }
    else if (L <= 256 * p.maxw) { p.TC = 16; p.W = p.maxw; }
    else if (p.maxw == 16) { p.TC = 16; p.W = 16; }
    else { p.TC = 32; p.W = 8; }
    const int chunk_keys = kTileUnits * p.W * p.TC;
    p.nchunks = (L + chunk_keys - 1) / chunk_keys;
    // enough buckets that the bound is tight: about twice as many as kept keys
    p.NB = 8;
    while (p.NB < p.TC && 4 * p.W * p.NB < 2 * sh.keep) p.NB *= 2;
    p.tiles_per_head = (L / sh.vec + kTileUnits - 1) / kTileUnits;
    const int NHT = p.nchunks * 4 * p.W;
    p.hc_log2 = 5;                                   // at most 32 slots per holder ...
    while (p.hc_log2 > 0 && (NHT << p.hc_log2) > kSegSlots) --p.hc_log2;   // ... and kSegSlots per unit
    const size_t NW = (size_t)p.nchunks * chunk_keys / 32;
    auto lds_bytes = [&](int nb, int hcl) {
        const size_t bm_bytes = sizeof(int) * (size_t)kTileUnits * (4 * p.W * nb + 1);
        const size_t compact_bytes = sizeof(int2) * (size_t)p.W * kCompactCap;      // shares bm's storage
        const size_t eq_bytes = p.nchunks == 1 ? sizeof(int) * kTileUnits * (NW + 1) : 0;   // ties bitmap
        return sizeof(int) * (7 * kTileUnits + kTileUnits * (NW + 1) + ((size_t)kTileUnits * NHT << hcl) +
                              (size_t)kTileUnits * (NHT + 1)) +
               (bm_bytes > compact_bytes ? bm_bytes : compact_bytes) + eq_bytes;
    };
    while (lds_bytes(p.NB, p.hc_log2) > kLdsBudget && (p.NB > 8 || p.hc_log2 > 0)) {
        if (p.NB > 8) p.NB /= 2; else --p.hc_log2;
    }
    p.lds = lds_bytes(p.NB, p.hc_log2);
    p.ok = p.lds <= kLdsBudget;
    return p;
}

// Workgroups to launch when each is to loop over tiles: the number of compute units if a compute
// unit holds exactly one workgroup of this kernel (nothing else hides the start and the end of a
// tile then), rounded down to a multiple of the XCD count; 0 when several fit (the hardware
// already overlaps them) and the launch should be one workgroup per tile.  The answer is kept per
// (kernel, block size, LDS size, device) and thread: the occupancy query costs microseconds that
// a launch-bound call would feel.
hipError_t looping_grid(const void *kern, int threads, size_t lds, unsigned *out)
{
    struct Entry { const void *kern; int threads; size_t lds; int dev; unsigned grid; };
    static thread_local Entry cache[8];
    static thread_local int used = 0;
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev)) return e;
    for (int i = 0; i < used; ++i)
        if (cache[i].kern == kern && cache[i].threads == threads && cache[i].lds == lds && cache[i].dev == dev) {
            *out = cache[i].grid;
            return hipSuccess;
        }
    int cus = 0, per_cu = 0;
    if (hipError_t e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) return e;
    if (hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, threads, lds)) return e;
    unsigned grid = per_cu == 1 && cus > 0 ? (unsigned)cus : 0u;
    grid -= grid % kXcds;
    const int slot = used < 8 ? used++ : 7;
    cache[slot] = Entry{kern, threads, lds, dev, grid};
    *out = grid;
    return hipSuccess;
}

template <int TC, int NB, int KSTEP, int MAXSTEPS, int MAXW>
hipError_t launch_tiles_t(const TilePlan &p, const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt,
                          int32_t *idx, hipStream_t st)
{
    auto kern = predict_tiles<TC, NB, KSTEP, MAXSTEPS, MAXW>;
    if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), p.lds)) return e;
    const unsigned tiles = (unsigned)sh.B * sh.H * p.tiles_per_head;
    // one workgroup per compute unit (a multiple of the XCD count), each looping over tiles
    unsigned resident = 0;
    if (hipError_t e = looping_grid(reinterpret_cast<const void *>(kern), p.W * kWave, p.lds, &resident)) return e;
    const unsigned grid = (resident == 0 || tiles <= resident) ? tiles : resident;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(p.W * kWave), p.lds, st, Qt, Kt, idx, sh.L, sh.k, sh.keep,
                       sh.vec, p.nchunks, p.tiles_per_head, p.hc_log2, tiles);
    return hipGetLastError();
}

template <int TC, int NB>
hipError_t launch_tiles_k(const TilePlan &p, const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt,
                          int32_t *idx, hipStream_t st)
{
    if constexpr (TC <= 16) {
        if (p.kstep == 32) return launch_tiles_t<TC, NB, 32, 1, 16>(p, sh, Qt, Kt, idx, st);
        if (p.maxsteps == 1) return launch_tiles_t<TC, NB, 64, 1, 16>(p, sh, Qt, Kt, idx, st);
        if (p.maxsteps == 4) return launch_tiles_t<TC, NB, 64, 4, 16>(p, sh, Qt, Kt, idx, st);
    }
    if (p.maxsteps == 8) return launch_tiles_t<TC, NB, 64, 8, 8>(p, sh, Qt, Kt, idx, st);
    return launch_tiles_t<TC, NB, 64, 16, 8>(p, sh, Qt, Kt, idx, st);
}

hipError_t launch_tiles(const TilePlan &p, const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt,
                        int32_t *idx, hipStream_t st)
{
    if (p.TC == 8) return launch_tiles_k<8, 8>(p, sh, Qt, Kt, idx, st);
    if (p.TC == 16) return p.NB == 8 ? launch_tiles_k<16, 8>(p, sh, Qt, Kt, idx, st)
                                     : launch_tiles_k<16, 16>(p, sh, Qt, Kt, idx, st);
    if (p.NB == 8) return launch_tiles_k<32, 8>(p, sh, Qt, Kt, idx, st);
    if (p.NB == 16) return launch_tiles_k<32, 16>(p, sh, Qt, Kt, idx, st);
    return launch_tiles_k<32, 32>(p, sh, Qt, Kt, idx, st);
}

// Row maximum of the approximate scores with the int8 matrix cores: the contraction with the
// smallest consumer that still looks at every score.  A wavefront keeps 64 query rows as two B
// operands of v_mfma_i32_32x32x32_i8 and sweeps its share of the keys 32 at a time as the A
// operand, so each lane ends up with one query column per operand and 16 key rows per tile: the
// running maximum is a per-lane scalar.  Key tiles are prefetched several tiles ahead into a
// register ring, and the maxima of tile t are taken (two scores per v_max3) while the matrix
// core works on tile t+1.  KSPLIT wavefronts share one 64-row query tile and split the keys, so
// that a SIMD holds several wavefronts and one's v_max3 stream fills the other's matrix-core
// time; they combine through LDS at the end.  A workgroup is always 8 wavefronts: 8 / KSPLIT
// query tiles times KSPLIT key shares.
// (With 512 threads, at most 256 registers per lane, the compiler gives the matrix core plain
// VGPR destinations that v_max3 can read directly.)
template <int KSTEPS, int KSPLIT, int NQ>   // k padded to 32 * KSTEPS; NQ blocks of 32 query rows per wavefront
__global__ __launch_bounds__(512) void rowmax_mfma(
    const int8_t *__restrict__ Qt, const int8_t *__restrict__ Kt, int32_t *__restrict__ rowmax, int L, int k,
    unsigned N)
{
    constexpr int PD = 8 / KSTEPS;                       // prefetch depth in tiles (KSTEPS <= 4)
    constexpr int QR = 32 * NQ;                          // query rows per wavefront
    constexpr int QSLOTS = 8 / KSPLIT;                   // query tiles per workgroup of 8 wavefronts
    __shared__ int part[8][QR];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int col = lane & 31, half = lane >> 5;
    const int qslot = wave / KSPLIT, ks = wave % KSPLIT;
    const unsigned qtiles_per_head = (L + QR - 1) / QR;
    const unsigned qtile = xcd_contiguous(blockIdx.x, gridDim.x) * QSLOTS + qslot;
    const bool live = qtile < N * qtiles_per_head;
    const unsigned n = live ? qtile / qtiles_per_head : 0;
    const int i0 = live ? (int)(qtile % qtiles_per_head) * QR : 0;
    const int8_t *Qh = Qt + (size_t)n * L * k, *Kh = Kt + (size_t)n * L * k;

    // operand piece of this lane: 16 consecutive c at 32*step + 16*half.  Beyond k (and, for
    // queries, beyond L) the query piece is zero, so the key piece there may hold anything and is
    // read from offset 0.  Key rows beyond L are read from row L-1 and masked at the end.
    int coff[KSTEPS];
    v4i qop[NQ][KSTEPS];
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) {
        const int c = 32 * s + 16 * half;
        coff[s] = c < k ? c : 0;
#pragma unroll
        for (int h = 0; h < NQ; ++h) {
            const int qi = i0 + 32 * h + col;
            qop[h][s] = (qi < L && c < k) ? *reinterpret_cast<const v4i *>(Qh + (size_t)qi * k + c) : v4i{0, 0, 0, 0};
        }
    }
    const int T = (L + 31) / 32;                       // key tiles in all
    const int Tper = (T + KSPLIT - 1) / KSPLIT;
    const int ta = ks * Tper, tb = min(T, ta + Tper);  // this wavefront's tiles
    auto load_tile = [&](int t, v4i (&dst)[KSTEPS]) {
        const int8_t *row = Kh + (size_t)min(32 * t + col, L - 1) * k;
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) dst[s] = *reinterpret_cast<const v4i *>(row + coff[s]);
    };
    v4i ring[PD][KSTEPS];
#pragma unroll
    for (int p = 0; p < PD; ++p) load_tile(min(ta + p, T - 1), ring[p]);

    int m[NQ];
    v16i prev[NQ];         // scores of the previous tile, reduced while the next one is computed
#pragma unroll
    for (int h = 0; h < NQ; ++h) {
        m[h] = INT32_MIN;
#pragma unroll
        for (int r = 0; r < 16; ++r) prev[h][r] = INT32_MIN;
    }
    auto step = [&](v4i (&kop)[KSTEPS]) {
        v16i cur[NQ];
#pragma unroll
        for (int h = 0; h < NQ; ++h) {
            cur[h] = v16i{0};
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s)
                cur[h] = __builtin_amdgcn_mfma_i32_32x32x32_i8(kop[s], qop[h][s], cur[h], 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
#pragma unroll
            for (int h = 0; h < NQ; ++h) m[h] = max(max(prev[h][r], prev[h][r + 1]), m[h]);
        }
#pragma unroll
        for (int h = 0; h < NQ; ++h) prev[h] = cur[h];
    };
    // all tiles but the last of the sweep hold only real keys; the ring slot of tile t is (t - ta) % PD
    int t = ta;
    for (; t + PD <= tb - 1; t += PD) {
#pragma unroll
        for (int p = 0; p < PD; ++p) {
            step(ring[p]);
            load_tile(min(t + p + PD, T - 1), ring[p]);
            // keep the refill of slot p here, PD tiles ahead of its use: left alone, the scheduler
            // gathers all refills at the end of the unrolled body, right before they are needed
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int p = 0; p < PD; ++p)
        if (t + p < tb) step(ring[p]);      // the rest; prev ends up as tile tb-1
    // that tile may reach past L: register r of this lane is key row 8*(r/4) + 4*half + r%4 of it
    if (ta < tb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            if (32 * (tb - 1) + 8 * (r / 4) + 4 * half + (r % 4) < L) {
#pragma unroll
                for (int h = 0; h < NQ; ++h) m[h] = max(m[h], prev[h][r]);
            }
        }
    }
#pragma unroll
    for (int h = 0; h < NQ; ++h) {
        m[h] = max(m[h], __shfl_xor(m[h], 32, kWave));
        if (half == 0) part[wave][32 * h + col] = m[h];
    }
    __syncthreads();
    if (ks == 0 && live) {
        for (int r = lane; r < QR; r += kWave) {
            int best = part[wave][r];
#pragma unroll
            for (int j = 1; j < KSPLIT; ++j) best = max(best, part[wave + j][r]);
            if (i0 + r < L) rowmax[(size_t)n * L + i0 + r] = best;
        }
    }
}

}  // namespace

int predict_max_L() { return kUnitMaxL; }

size_t predict_workspace_bytes(const dsa_shape &) { return 0; }

hipError_t launch_predict(const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt, int32_t *idx, void *,
                          hipStream_t st)
{
    if (stream_predict_fits(sh)) return launch_predict_stream(sh, Qt, Kt, idx, st);
    const TilePlan plan = plan_tiles(sh);
    if (plan.ok) return launch_tiles(plan, sh, Qt, Kt, idx, st);
    const unsigned units = (unsigned)sh.B * sh.H * (sh.L / sh.vec);
    const size_t lds = ((size_t)sh.L + sh.vec * (sh.k / 4) + 8) * sizeof(int);
    auto go = [&](auto kern) -> hipError_t {
        if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds)) return e;
        hipLaunchKernelGGL(kern, dim3(units), dim3(kUnitThreads), lds, st, Qt, Kt, idx, sh.L, sh.k, sh.keep);
        return hipGetLastError();
    };
    if (sh.vec == 1) return go(predict_unit<1>);
    if (sh.vec == 4) return go(predict_unit<4>);
    return go(predict_unit<8>);
}

// Nothing but v_mfma_i32_32x32x32_i8: four independent accumulation chains per wavefront, no memory
// traffic inside the loop.  Measures the int8 matrix-core rate the chip sustains at its own clocks,
// the yardstick for rowmax_mfma next to the published peak.
__global__ __launch_bounds__(256) void mfma_i8_stream(int iters, int32_t *__restrict__ sink)
{
    v4i a, b;
#pragma unroll
    for (int i = 0; i < 4; ++i) { a[i] = 0x01020304 * (i + 1) + (int)threadIdx.x; b[i] = 0x04030201 * (i + 1) - (int)threadIdx.x; }
    v16i c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    for (int i = 0; i < iters; ++i) {
        c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c3, 0, 0, 0);
    }
    sink[blockIdx.x * 256 + threadIdx.x] = c0[0] + c1[1] + c2[2] + c3[3];
}

template <int KSTEPS, int NQ>
hipError_t launch_rowmax_q(const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt, int32_t *rowmax, hipStream_t st)
{
    const unsigned N = (unsigned)sh.B * sh.H;
    const unsigned qtiles = N * ((sh.L + 32 * NQ - 1) / (32 * NQ));
    // enough wavefronts for a few per SIMD (1024 SIMDs), but at least 8 key tiles each
    const int tiles = (sh.L + 31) / 32;
    int ksplit = 1;
    while (ksplit < 8 && (size_t)qtiles * ksplit < 2048 && tiles / (2 * ksplit) >= 8) ksplit *= 2;
    const unsigned slots = 8 / ksplit;
    const dim3 grid((qtiles + slots - 1) / slots), block(512);
    switch (ksplit) {
    case 1: hipLaunchKernelGGL((rowmax_mfma<KSTEPS, 1, NQ>), grid, block, 0, st, Qt, Kt, rowmax, sh.L, sh.k, N); break;
    case 2: hipLaunchKernelGGL((rowmax_mfma<KSTEPS, 2, NQ>), grid, block, 0, st, Qt, Kt, rowmax, sh.L, sh.k, N); break;
    case 4: hipLaunchKernelGGL((rowmax_mfma<KSTEPS, 4, NQ>), grid, block, 0, st, Qt, Kt, rowmax, sh.L, sh.k, N); break;
    default: hipLaunchKernelGGL((rowmax_mfma<KSTEPS, 8, NQ>), grid, block, 0, st, Qt, Kt, rowmax, sh.L, sh.k, N); break;
    }
    return hipGetLastError();
}

template <int KSTEPS>
hipError_t launch_rowmax_k(const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt, int32_t *rowmax, hipStream_t st)
{
    // 128 query rows per wavefront (one key operand feeds four MFMAs) when that still leaves enough
    // wavefronts to fill the chip and k is short enough for the registers; else 64
    const size_t rows = (size_t)sh.B * sh.H * sh.L;
    if (KSTEPS <= 2 && rows >= 65536) return launch_rowmax_q<KSTEPS, 4>(sh, Qt, Kt, rowmax, st);
    return launch_rowmax_q<KSTEPS, 2>(sh, Qt, Kt, rowmax, st);
}

hipError_t launch_rowmax(const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt, int32_t *rowmax,
                         hipStream_t st)
{
    switch ((sh.k + 31) / 32) {
    case 1: return launch_rowmax_k<1>(sh, Qt, Kt, rowmax, st);
    case 2: return launch_rowmax_k<2>(sh, Qt, Kt, rowmax, st);
    case 3: return launch_rowmax_k<3>(sh, Qt, Kt, rowmax, st);
    default: return launch_rowmax_k<4>(sh, Qt, Kt, rowmax, st);
    }
}

hipError_t launch_mfma_i8_stream(int blocks, int iters, int32_t *sink, hipStream_t st)
{
    hipLaunchKernelGGL(mfma_i8_stream, dim3(blocks), dim3(256), 0, st, iters, sink);
    return hipGetLastError();
}

}  // namespace dsa
