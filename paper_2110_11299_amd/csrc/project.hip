// The step in front of the prediction path (paper section 3.1, equation 5): reduce a [B,H,L,d]
// tensor to k dimensions with a projection matrix and quantise to int8.  With no trained
// predictor weights the projection is one matrix R [d,k]; the quantiser is symmetric per tensor.
// The arithmetic is fixed so that the int8 codes are reproducible bit for bit:
//   Y[r,j] = fma(X[r,d-1], R[d-1,j], ... fma(X[r,1], R[1,j], fma(X[r,0], R[0,j], 0)))   in fp32
//   amax   = max |Y|,   s = qmax / amax  (fp32 division),   code = clip(rint(Y * s), -qmax, qmax)
// with qmax = 127 (int8), 7 (INT4, the paper's default prediction precision, section 3.3) or 1 (INT2).
// Three launches: clear the maximum, project (Y to scratch, maximum by atomic max on the bit
// pattern of |Y|, which orders like the value for non-negative floats), quantise.
#include "dsa_internal.h"

namespace dsa {
namespace {

constexpr int kProjThreads = 256;

__global__ void clear_word(unsigned *w) { *w = 0u; }

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

// One thread per (row, four consecutive output columns).  The row is read 16 bytes at a time; the
// four chains still take their terms in increasing c.
template <typename T>
__global__ __launch_bounds__(kProjThreads) void project_rows(const T *__restrict__ X, const float *__restrict__ R,
                                                             float *__restrict__ Y, unsigned *__restrict__ amax_bits,
                                                             unsigned rows, int d, int k)
{
    constexpr int E = Chunk<T>::N;
    extern __shared__ float sR[];                  // [d][k]
    for (int i = threadIdx.x; i < d * k; i += kProjThreads) sR[i] = R[i];
    __syncthreads();
    const int k4 = k / 4;
    const unsigned item = blockIdx.x * kProjThreads + threadIdx.x;
    const unsigned r = item / k4;
    const int j = (item % k4) * 4;
    float y0 = 0.f, y1 = 0.f, y2 = 0.f, y3 = 0.f;
    if (r < rows) {
        const T *x = X + (size_t)r * d;
        for (int c0 = 0; c0 < d; c0 += E) {
            float xv[E];
            Chunk<T>::load(x + c0, xv);
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const float4 rc = *reinterpret_cast<const float4 *>(sR + (c0 + e) * k + j);
                y0 = __fmaf_rn(xv[e], rc.x, y0);
                y1 = __fmaf_rn(xv[e], rc.y, y1);
                y2 = __fmaf_rn(xv[e], rc.z, y2);
                y3 = __fmaf_rn(xv[e], rc.w, y3);
            }
        }
        *reinterpret_cast<float4 *>(Y + (size_t)r * k + j) = make_float4(y0, y1, y2, y3);
    }
    float m = fmaxf(fmaxf(fabsf(y0), fabsf(y1)), fmaxf(fabsf(y2), fabsf(y3)));
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) m = fmaxf(m, __shfl_xor(m, off, kWave));
    // the atomic only when it can still raise the maximum: after the first few wavefronts almost
    // none can, and the one hot address stops being a bottleneck
    if ((threadIdx.x & (kWave - 1)) == 0 && __float_as_uint(m) > __atomic_load_n(amax_bits, __ATOMIC_RELAXED))
        atomicMax(amax_bits, __float_as_uint(m));
}

// Four codes per thread, BITS wide each, stored two's complement with 8/BITS codes per byte (code j
// of a row in bits [BITS * (j mod 8/BITS), + BITS) of byte j / (8/BITS)): 4, 2 or 1 byte per thread.
template <int BITS>
__global__ __launch_bounds__(kProjThreads) void quantize_codes(const float *__restrict__ Y,
                                                               const unsigned *__restrict__ amax_bits,
                                                               uint8_t *__restrict__ Xt, float *__restrict__ amax_out,
                                                               size_t n4)
{
    constexpr float kQmax = (float)((1 << (BITS - 1)) - 1);
    const float amax = __uint_as_float(*amax_bits);
    if (amax_out && blockIdx.x == 0 && threadIdx.x == 0) *amax_out = amax;
    const float s = amax > 0.f ? __fdiv_rn(kQmax, amax) : 0.f;
    const size_t i = (size_t)blockIdx.x * kProjThreads + threadIdx.x;
    if (i >= n4) return;
    const float4 y = reinterpret_cast<const float4 *>(Y)[i];
    const float q[4] = {y.x, y.y, y.z, y.w};
    unsigned packed = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float v = fminf(fmaxf(rintf(__fmul_rn(q[e], s)), -kQmax), kQmax);
        packed |= ((unsigned)(int)v & ((1u << BITS) - 1u)) << (BITS * e);
    }
    if (BITS == 8) reinterpret_cast<unsigned *>(Xt)[i] = packed;
    else if (BITS == 4) reinterpret_cast<uint16_t *>(Xt)[i] = (uint16_t)packed;
    else Xt[i] = (uint8_t)packed;
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

size_t project_workspace_bytes(const dsa_shape &sh)
{
    return (size_t)sh.B * sh.H * sh.L * sh.k * sizeof(float) + 256;
}

hipError_t launch_project_quantize(const dsa_shape &sh, int bits, const void *X, const float *R, void *Xt,
                                   float *amax_out, void *ws, hipStream_t st)
{
    const unsigned rows = (unsigned)sh.B * sh.H * sh.L;
    const size_t n = (size_t)rows * sh.k;
    float *Y = static_cast<float *>(ws);
    unsigned *amax_bits = reinterpret_cast<unsigned *>(static_cast<char *>(ws) + n * sizeof(float));
    hipLaunchKernelGGL(clear_word, dim3(1), dim3(1), 0, st, amax_bits);
    const size_t items = n / 4;
    const dim3 grid((unsigned)((items + kProjThreads - 1) / kProjThreads)), block(kProjThreads);
    const size_t lds = (size_t)sh.d * sh.k * sizeof(float);
    const void *kern = sh.dtype == DSA_F32 ? reinterpret_cast<const void *>(project_rows<float>)
                                           : reinterpret_cast<const void *>(project_rows<uint16_t>);
    if (hipError_t e = allow_dynamic_lds(kern, lds)) return e;
    if (sh.dtype == DSA_F32)
        hipLaunchKernelGGL(project_rows<float>, grid, block, lds, st, static_cast<const float *>(X), R, Y, amax_bits,
                           rows, sh.d, sh.k);
    else
        hipLaunchKernelGGL(project_rows<uint16_t>, grid, block, lds, st, static_cast<const uint16_t *>(X), R, Y,
                           amax_bits, rows, sh.d, sh.k);
    uint8_t *out = static_cast<uint8_t *>(Xt);
    if (bits == 8) hipLaunchKernelGGL(quantize_codes<8>, grid, block, 0, st, Y, amax_bits, out, amax_out, items);
    else if (bits == 4) hipLaunchKernelGGL(quantize_codes<4>, grid, block, 0, st, Y, amax_bits, out, amax_out, items);
    else hipLaunchKernelGGL(quantize_codes<2>, grid, block, 0, st, Y, amax_bits, out, amax_out, items);
    return hipGetLastError();
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
