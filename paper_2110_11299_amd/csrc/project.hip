// The step in front of the prediction path (paper section 3.1, equation 5): reduce a [B,H,L,d]
// tensor to k dimensions with a projection matrix and quantise to int8.  With no trained
// predictor weights the projection is one matrix R [d,k]; the quantiser is symmetric per tensor.
// The arithmetic is fixed so that the int8 codes are reproducible bit for bit:
//   Y[r,j] = fma(X[r,d-1], R[d-1,j], ... fma(X[r,1], R[1,j], fma(X[r,0], R[0,j], 0)))   in fp32
//   amax   = max |Y|,   s = qmax / amax  (fp32 division),   code = clip(rint(Y * s), -qmax, qmax)
// with qmax = 127 (int8), 7 (INT4, the paper's default prediction precision, section 3.3) or 1 (INT2).
// Two launches: the maximum of |Y| (per-workgroup maxima), then projection again + quantiser: Y is
// never stored.
#include "dsa_internal.h"
#include "project_api.h"

#include <algorithm>
#include <type_traits>

namespace dsa {
namespace {

constexpr int kProjThreads = 256;

// 16 bytes of a row widened to fp32.
template <typename T> struct Chunk;
template <> struct Chunk<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void load(const float *p, float (&v)[4])
    {
        const float4 x = *reinterpret_cast<const float4 *>(p);
        v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
    }
};
template <> struct Chunk<uint16_t> {
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

// One lane per row and 16 output columns; a wavefront covers 64 consecutive rows and one chunk of 16
// columns.  The projection matrix sits in LDS as floats; all lanes of a wavefront read the same 16
// floats of it (one broadcast read per four multiply-adds), so neither LDS nor memory limits the
// pass: it runs at the fused multiply-add rate.  Each of the 16 chains takes its terms in
// increasing c, which fixes the result bit for bit.  A ternary matrix (entries -1, 0, 1: the sparse
// random projection of equation 5, up to its positive constant sqrt(3/k), which the quantiser's
// scale absorbs) becomes the floats -1, 0, 1: fma(x, +-1, y) is the exact sum or difference and
// fma(x, 0, y) leaves y alone, so the chain is the sequence of additions and subtractions itself.
// PASS 0: per-workgroup maximum of |Y| to block_max[blockIdx.x].  PASS 1: reduce block_max (the grid
// of pass 0 is at most kProjMaxBlocks), scale, round to nearest even, clip, pack BITS-wide codes.
constexpr int kProjCols = 16;
constexpr int kProjMaxBlocks = 1024;

template <typename T, int PASS, int BITS, bool TERNARY>
__global__ __launch_bounds__(kProjThreads) void project_lanes(const T *__restrict__ X, const float *__restrict__ R,
                                                              const int8_t *__restrict__ P3,
                                                              float *__restrict__ block_max, int n_block_max,
                                                              uint8_t *__restrict__ Xt, float *__restrict__ amax_out,
                                                              unsigned rows, int d, int k, unsigned items)
{
    constexpr int E = Chunk<T>::N;
    extern __shared__ float sR[];                  // [d][k], then one float per wavefront
    float *red = sR + d * k;
    // a dense matrix is read straight from memory through the scalar cache (the address is the same for
    // all lanes); only the ternary one is widened to floats in LDS
    if (TERNARY)
        for (int i = threadIdx.x; i < d * k; i += kProjThreads) sR[i] = (float)P3[i];
    float amax = 0.f;
    if (PASS == 1) {
        float m = 0.f;
        for (int i = threadIdx.x; i < n_block_max; i += kProjThreads) m = fmaxf(m, block_max[i]);
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) m = fmaxf(m, __shfl_xor(m, off, kWave));
        if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = m;
    }
    __syncthreads();
    if (PASS == 1) {
#pragma unroll
        for (int w = 0; w < kProjThreads / kWave; ++w) amax = fmaxf(amax, red[w]);
        if (amax_out && blockIdx.x == 0 && threadIdx.x == 0) *amax_out = amax;
    }
    constexpr float kQmax = (float)((1 << (BITS - 1)) - 1);
    const float scale = amax > 0.f ? __fdiv_rn(kQmax, amax) : 0.f;
    const int chunks = k / kProjCols;
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    float seen = 0.f;
    // work item = (tile of 64 rows, chunk of 16 columns); a wavefront takes items wave, wave + stride, ...
    for (unsigned item = blockIdx.x * (kProjThreads / kWave) + wave; item < items;
         item += gridDim.x * (kProjThreads / kWave)) {
        const unsigned tile = item / chunks;
        const int j0 = (int)(item % chunks) * kProjCols;
        const unsigned r = tile * kWave + lane;
        const bool live = r < rows;
        const T *x = X + (size_t)(live ? r : rows - 1) * d;
        float y[kProjCols];
#pragma unroll
        for (int j = 0; j < kProjCols; ++j) y[j] = 0.f;
        for (int c0 = 0; c0 < d; c0 += E) {
            float xv[E];
            Chunk<T>::load(x + c0, xv);
#pragma unroll
            for (int e = 0; e < E; ++e) {
                if (TERNARY) {
                    const float *rc = sR + (c0 + e) * k + j0;
#pragma unroll
                    for (int j = 0; j < kProjCols; ++j) y[j] = __fmaf_rn(xv[e], rc[j], y[j]);
                } else {
                    const float *rc = R + (c0 + e) * k + j0;     // wavefront-uniform: scalar loads
#pragma unroll
                    for (int j = 0; j < kProjCols; ++j) y[j] = __fmaf_rn(xv[e], rc[j], y[j]);
                }
            }
        }
        if (PASS == 0) {
            if (live) {
#pragma unroll
                for (int j = 0; j < kProjCols; ++j) seen = fmaxf(seen, fabsf(y[j]));
            }
        } else if (live) {
            unsigned packed[kProjCols * BITS / 32 > 0 ? kProjCols * BITS / 32 : 1];
#pragma unroll
            for (int i = 0; i < (int)(sizeof(packed) / sizeof(unsigned)); ++i) packed[i] = 0;
#pragma unroll
            for (int j = 0; j < kProjCols; ++j) {
                const float v = fminf(fmaxf(rintf(__fmul_rn(y[j], scale)), -kQmax), kQmax);
                packed[j * BITS / 32] |= ((unsigned)(int)v & ((1u << BITS) - 1u)) << ((j * BITS) % 32);
            }
            // codes j0 .. j0+15 of row r: 16, 8 or 4 bytes at byte (r * k + j0) * BITS / 8
            uint8_t *dst = Xt + ((size_t)r * k + j0) * BITS / 8;
            if (BITS == 8) *reinterpret_cast<uint4 *>(dst) = make_uint4(packed[0], packed[1], packed[2], packed[3]);
            else if (BITS == 4) *reinterpret_cast<uint2 *>(dst) = make_uint2(packed[0], packed[1]);
            else *reinterpret_cast<unsigned *>(dst) = packed[0];
        }
    }
    if (PASS == 0) {
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) seen = fmaxf(seen, __shfl_xor(seen, off, kWave));
        __syncthreads();
        if (lane == 0) red[wave] = seen;
        __syncthreads();
        if (threadIdx.x == 0) {
            float m = 0.f;
#pragma unroll
            for (int w = 0; w < kProjThreads / kWave; ++w) m = fmaxf(m, red[w]);
            block_max[blockIdx.x] = m;
        }
    }
}

// Packed codes back to one int8 per code: a thread expands 4 packed bytes.
template <int BITS>
__global__ __launch_bounds__(kProjThreads) void unpack_codes(const unsigned *__restrict__ packed,
                                                             int8_t *__restrict__ codes, size_t words)
{
    constexpr int PER = 32 / BITS;                  // codes in one 32-bit word
    const size_t i = (size_t)blockIdx.x * kProjThreads + threadIdx.x;
    if (i >= words) return;
    const unsigned w = packed[i];
    unsigned out[PER / 4];
#pragma unroll
    for (int o = 0; o < PER / 4; ++o) {
        unsigned v = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int f = 4 * o + e;
            // field f to the top of the word, then an arithmetic shift back: sign extension
            const int c = (int)(w << (32 - BITS * (f + 1))) >> (32 - BITS);
            v |= ((unsigned)c & 0xffu) << (8 * e);
        }
        out[o] = v;
    }
    unsigned *dst = reinterpret_cast<unsigned *>(codes) + i * (PER / 4);
#pragma unroll
    for (int o = 0; o < PER / 4; ++o) dst[o] = out[o];
}

}  // namespace

size_t project_workspace_bytes(const dsa_shape &) { return kProjMaxBlocks * sizeof(float); }

template <typename T>
hipError_t launch_project_t(const dsa_shape &sh, int bits, const T *X, const float *R, const int8_t *P3, void *Xt,
                            float *amax_out, void *ws, hipStream_t st)
{
    const unsigned rows = (unsigned)sh.B * sh.H * sh.L;
    const unsigned items = ((rows + kWave - 1) / kWave) * (unsigned)(sh.k / kProjCols);
    const unsigned per_block = kProjThreads / kWave;
    const unsigned grid = std::min<unsigned>((items + per_block - 1) / per_block, kProjMaxBlocks);
    const size_t lds = ((size_t)sh.d * sh.k + kProjThreads / kWave) * sizeof(float);
    float *block_max = static_cast<float *>(ws);
    uint8_t *out = static_cast<uint8_t *>(Xt);
    auto go = [&](auto kern) -> hipError_t {
        if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds)) return e;
        hipLaunchKernelGGL(kern, dim3(grid), dim3(kProjThreads), lds, st, X, R, P3, block_max, (int)grid, out, amax_out,
                           rows, sh.d, sh.k, items);
        return hipGetLastError();
    };
    auto both = [&](auto ternary_tag) -> hipError_t {
        constexpr bool TERNARY = decltype(ternary_tag)::value;
        if (hipError_t e = go(project_lanes<T, 0, 8, TERNARY>)) return e;
        if (bits == 8) return go(project_lanes<T, 1, 8, TERNARY>);
        if (bits == 4) return go(project_lanes<T, 1, 4, TERNARY>);
        return go(project_lanes<T, 1, 2, TERNARY>);
    };
    return P3 ? both(std::true_type{}) : both(std::false_type{});
}

hipError_t launch_project_quantize(const dsa_shape &sh, int bits, const void *X, const float *R, const int8_t *P3,
                                   void *Xt, float *amax_out, void *ws, hipStream_t st)
{
    if (sh.dtype == DSA_F32)
        return launch_project_t<float>(sh, bits, static_cast<const float *>(X), R, P3, Xt, amax_out, ws, st);
    return launch_project_t<uint16_t>(sh, bits, static_cast<const uint16_t *>(X), R, P3, Xt, amax_out, ws, st);
}

hipError_t launch_unpack_codes(int bits, const void *packed, int8_t *codes, size_t n_codes, hipStream_t st)
{
    const size_t words = n_codes * bits / 32;      // n_codes is a multiple of 16
    const dim3 grid((unsigned)((words + kProjThreads - 1) / kProjThreads)), block(kProjThreads);
    const unsigned *src = static_cast<const unsigned *>(packed);
    if (bits == 4) hipLaunchKernelGGL(unpack_codes<4>, grid, block, 0, st, src, codes, words);
    else hipLaunchKernelGGL(unpack_codes<2>, grid, block, 0, st, src, codes, words);
    return hipGetLastError();
}

}  // namespace dsa
