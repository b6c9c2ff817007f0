// Prediction path of Dynamic Sparse Attention (paper section 3.1): approximate scores
// S~ = Q~ K~^T from int8 projections, optional sum over the 8 rows of a column vector
// (section 5.1), and the per-unit top-k that becomes the mask.  Scores are exact integers, so
// the selection is exact: larger score first, lower key index among equals, list ascending.
#include "dsa_internal.h"

namespace dsa {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kUnitThreads = 256;
constexpr int kUnitMaxL = 32768;     // one unit's scores in LDS: 128 KB

__device__ __forceinline__ int wave_sum(int x)
{
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) x += __shfl_xor(x, off, kWave);
    return x;
}
__device__ __forceinline__ int wave_max(int x)
{
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) x = max(x, __shfl_xor(x, off, kWave));
    return x;
}
__device__ __forceinline__ int wave_min(int x)
{
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) x = min(x, __shfl_xor(x, off, kWave));
    return x;
}

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

// Row maximum of the approximate scores with the int8 matrix cores.  A wavefront keeps 32 query
// rows as the B operand of v_mfma_i32_32x32x32_i8 and sweeps the keys 32 at a time as the A
// operand, so each lane ends up with one query column and 16 key rows per tile: the running
// maximum is a per-lane scalar, reduced across the two lane halves at the end.
template <int KSTEPS>   // k padded to 32 * KSTEPS
__global__ __launch_bounds__(256) void rowmax_mfma(const int8_t *__restrict__ Qt,
                                                   const int8_t *__restrict__ Kt,
                                                   int32_t *__restrict__ rowmax, int L, int k,
                                                   unsigned N)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int col = lane & 31, half = lane >> 5;
    const unsigned tiles_per_head = (L + 31) / 32;
    const unsigned qtile = blockIdx.x * 4 + wave;
    const unsigned n = qtile / tiles_per_head, i0 = (qtile % tiles_per_head) * 32;
    if (n >= N) return;
    const int8_t *Qh = Qt + (size_t)n * L * k, *Kh = Kt + (size_t)n * L * k;

    // operand piece of this lane: 16 consecutive c at 32*step + 16*half; zero beyond k or L
    v4i qop[KSTEPS];
    const int qi = i0 + col;
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) {
        const int c = 32 * s + 16 * half;
        qop[s] = (qi < L && c < k) ? *reinterpret_cast<const v4i *>(Qh + (size_t)qi * k + c) : v4i{0, 0, 0, 0};
    }
    int m = INT32_MIN;
    for (int j0 = 0; j0 < L; j0 += 32) {
        const int j = j0 + col;
        v16i acc = {0};
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {
            const int c = 32 * s + 16 * half;
            const v4i kop = (j < L && c < k) ? *reinterpret_cast<const v4i *>(Kh + (size_t)j * k + c)
                                             : v4i{0, 0, 0, 0};
            acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(kop, qop[s], acc, 0, 0, 0);
        }
        // register r of this lane is key row 8*(r/4) + 4*half + r%4 of the tile
        if (j0 + 32 <= L) {
#pragma unroll
            for (int r = 0; r < 16; ++r) m = max(m, acc[r]);
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int jr = j0 + 8 * (r / 4) + 4 * half + (r % 4);
                if (jr < L) m = max(m, acc[r]);
            }
        }
    }
    m = max(m, __shfl_xor(m, 32, kWave));
    if (half == 0 && qi < L) rowmax[(size_t)n * L + qi] = m;
}

}  // namespace

int predict_max_L() { return kUnitMaxL; }

size_t predict_workspace_bytes(const dsa_shape &) { return 0; }

hipError_t launch_predict(const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt, int32_t *idx, void *,
                          hipStream_t st)
{
    const unsigned units = (unsigned)sh.B * sh.H * (sh.L / sh.vec);
    const size_t lds = ((size_t)sh.L + sh.vec * (sh.k / 4) + 8) * sizeof(int);
    if (sh.vec == 1) {
        auto kern = predict_unit<1>;
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kern, dim3(units), dim3(kUnitThreads), lds, st, Qt, Kt, idx, sh.L, sh.k, sh.keep);
    } else {
        auto kern = predict_unit<8>;
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kern, dim3(units), dim3(kUnitThreads), lds, st, Qt, Kt, idx, sh.L, sh.k, sh.keep);
    }
    return hipGetLastError();
}

hipError_t launch_rowmax(const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt, int32_t *rowmax,
                         hipStream_t st)
{
    const unsigned N = (unsigned)sh.B * sh.H;
    const unsigned qtiles = N * ((sh.L + 31) / 32);
    const dim3 grid((qtiles + 3) / 4), block(256);
    const int ksteps = (sh.k + 31) / 32;
    switch (ksteps) {
    case 1: hipLaunchKernelGGL(rowmax_mfma<1>, grid, block, 0, st, Qt, Kt, rowmax, sh.L, sh.k, N); break;
    case 2: hipLaunchKernelGGL(rowmax_mfma<2>, grid, block, 0, st, Qt, Kt, rowmax, sh.L, sh.k, N); break;
    case 3: hipLaunchKernelGGL(rowmax_mfma<3>, grid, block, 0, st, Qt, Kt, rowmax, sh.L, sh.k, N); break;
    default: hipLaunchKernelGGL(rowmax_mfma<4>, grid, block, 0, st, Qt, Kt, rowmax, sh.L, sh.k, N); break;
    }
    return hipGetLastError();
}

}  // namespace dsa
