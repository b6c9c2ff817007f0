// Wavefront-level selection primitives shared by the predictor kernels: DPP reductions and scans,
// counting of register-resident values against a threshold, the k-th largest by bisection on the
// value, and the exact int8 score of one (unit, key) pair.  Device code only; everything is
// internal to the translation unit that includes it.
#pragma once

#include "dsa_internal.h"

namespace dsa {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Wavefront reductions without LDS traffic: butterfly inside each row of 16 lanes with DPP
// (quad permutes, then the two mirrors), then the four row results through v_readlane into
// scalar registers.  The result is wavefront-uniform and lives in an SGPR.
template <int CTRL> __device__ __forceinline__ int dpp_move(int x)
{
    return __builtin_amdgcn_update_dpp(x, x, CTRL, 0xF, 0xF, false);
}
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140;

__device__ __forceinline__ int wave_sum(int x)
{
    x += dpp_move<kDppXor1>(x);
    x += dpp_move<kDppXor2>(x);
    x += dpp_move<kDppHalfMirror>(x);
    x += dpp_move<kDppMirror>(x);
    return __builtin_amdgcn_readlane(x, 0) + __builtin_amdgcn_readlane(x, 16) +
           __builtin_amdgcn_readlane(x, 32) + __builtin_amdgcn_readlane(x, 48);
}
__device__ __forceinline__ int wave_max(int x)
{
    x = max(x, dpp_move<kDppXor1>(x));
    x = max(x, dpp_move<kDppXor2>(x));
    x = max(x, dpp_move<kDppHalfMirror>(x));
    x = max(x, dpp_move<kDppMirror>(x));
    return max(max(__builtin_amdgcn_readlane(x, 0), __builtin_amdgcn_readlane(x, 16)),
               max(__builtin_amdgcn_readlane(x, 32), __builtin_amdgcn_readlane(x, 48)));
}
__device__ __forceinline__ int wave_min(int x)
{
    x = min(x, dpp_move<kDppXor1>(x));
    x = min(x, dpp_move<kDppXor2>(x));
    x = min(x, dpp_move<kDppHalfMirror>(x));
    x = min(x, dpp_move<kDppMirror>(x));
    return min(min(__builtin_amdgcn_readlane(x, 0), __builtin_amdgcn_readlane(x, 16)),
               min(__builtin_amdgcn_readlane(x, 32), __builtin_amdgcn_readlane(x, 48)));
}

// Inclusive prefix sum over the 64 lanes: Hillis-Steele inside each row of 16 lanes with DPP row
// shifts (zero fill), then the totals of the lower rows through v_readlane.  *total = wavefront sum.
__device__ __forceinline__ int wave_incl_scan(int x, int lane, int *total)
{
    x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xF, 0xF, true);   // row_shr:1
    x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xF, 0xF, true);   // row_shr:2
    x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xF, 0xF, true);   // row_shr:4
    x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xF, 0xF, true);   // row_shr:8
    const int t0 = __builtin_amdgcn_readlane(x, 15), t1 = __builtin_amdgcn_readlane(x, 31),
              t2 = __builtin_amdgcn_readlane(x, 47), t3 = __builtin_amdgcn_readlane(x, 63);
    const int row = lane >> 4;
    x += (row >= 1 ? t0 : 0) + (row >= 2 ? t1 : 0) + (row >= 3 ? t2 : 0);
    *total = t0 + t1 + t2 + t3;
    return x;
}

// Makes LDS writes of some lanes of a wavefront visible to reads of its other lanes.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Exact score of (unit, key): sum over the unit's vec rows of the int8 dot product.
__device__ __forceinline__ int unit_key_score(const int *__restrict__ qu, const int8_t *__restrict__ krow,
                                              int vec, int k4)
{
    int s = 0;
    for (int c4 = 0; c4 < k4; c4 += 4) {
        const v4i kk = *reinterpret_cast<const v4i *>(krow + 4 * c4);
        for (int r = 0; r < vec; ++r) {
            const int *q = qu + r * k4 + c4;
            s = __builtin_amdgcn_sdot4(q[0], kk.x, s, false);
            s = __builtin_amdgcn_sdot4(q[1], kk.y, s, false);
            s = __builtin_amdgcn_sdot4(q[2], kk.z, s, false);
            s = __builtin_amdgcn_sdot4(q[3], kk.w, s, false);
        }
    }
    return s;
}

// Number of (register, lane) pairs with v >= t for a wavefront-uniform t.  The compares are issued
// back to back into separate mask registers and counted afterwards: with one shared mask register
// every compare would wait for the scalar count of the one before it.
__device__ __forceinline__ int count_ge4(int a, int b, int c, int d, int t)
{
    unsigned long long m0, m1, m2, m3;
    asm("v_cmp_ge_i32_e64 %0, %4, %8\n\tv_cmp_ge_i32_e64 %1, %5, %8\n\t"
        "v_cmp_ge_i32_e64 %2, %6, %8\n\tv_cmp_ge_i32_e64 %3, %7, %8"
        : "=&s"(m0), "=&s"(m1), "=&s"(m2), "=&s"(m3)
        : "v"(a), "v"(b), "v"(c), "v"(d), "s"(t));
    return (__popcll(m0) + __popcll(m1)) + (__popcll(m2) + __popcll(m3));
}
__device__ __forceinline__ int count_ge8(int a, int b, int c, int d, int e, int f, int g, int h, int t)
{
    unsigned long long m0, m1, m2, m3, m4, m5, m6, m7;
    asm("v_cmp_ge_i32_e64 %0, %8, %16\n\tv_cmp_ge_i32_e64 %1, %9, %16\n\t"
        "v_cmp_ge_i32_e64 %2, %10, %16\n\tv_cmp_ge_i32_e64 %3, %11, %16\n\t"
        "v_cmp_ge_i32_e64 %4, %12, %16\n\tv_cmp_ge_i32_e64 %5, %13, %16\n\t"
        "v_cmp_ge_i32_e64 %6, %14, %16\n\tv_cmp_ge_i32_e64 %7, %15, %16"
        : "=&s"(m0), "=&s"(m1), "=&s"(m2), "=&s"(m3), "=&s"(m4), "=&s"(m5), "=&s"(m6), "=&s"(m7)
        : "v"(a), "v"(b), "v"(c), "v"(d), "v"(e), "v"(f), "v"(g), "v"(h), "s"(t));
    return ((__popcll(m0) + __popcll(m1)) + (__popcll(m2) + __popcll(m3))) +
           ((__popcll(m4) + __popcll(m5)) + (__popcll(m6) + __popcll(m7)));
}
__device__ __forceinline__ int count_ge2(int a, int b, int t)
{
    unsigned long long m0, m1;
    asm("v_cmp_ge_i32_e64 %0, %2, %4\n\tv_cmp_ge_i32_e64 %1, %3, %4"
        : "=&s"(m0), "=&s"(m1)
        : "v"(a), "v"(b), "s"(t));
    return __popcll(m0) + __popcll(m1);
}
template <int NR, int USED>
__device__ __forceinline__ int count_ge(const int (&v)[NR], int t)
{
    int cnt = 0;
    int i = 0;
#pragma unroll
    for (; i + 8 <= USED; i += 8)
        cnt += count_ge8(v[i], v[i + 1], v[i + 2], v[i + 3], v[i + 4], v[i + 5], v[i + 6], v[i + 7], t);
    if (USED - i >= 4) { cnt += count_ge4(v[i], v[i + 1], v[i + 2], v[i + 3], t); i += 4; }
    if (USED - i >= 2) { cnt += count_ge2(v[i], v[i + 1], t); i += 2; }
    if (USED - i >= 1) cnt += __popcll(__ballot(v[i] >= t));
    return cnt;
}

// The keep-th largest of the values a wavefront holds in registers (NR per lane, unused slots
// INT32_MIN): the largest T with count(v >= T) >= keep, by bisection on the value.  lo and hi are
// wavefront-uniform; needs count(v >= lo) >= keep and hi >= every value.  Every probe is above
// INT32_MIN, so unused slots never count.  With slack > 0 the search stops at the first T whose
// count lies in [keep, keep + slack]: still a lower bound of the keep-th largest, found sooner.
template <int NR, int USED = NR>
__device__ __forceinline__ int kth_largest(const int (&v)[NR], int keep, int lo, int hi, int slack = 0)
{
    lo = __builtin_amdgcn_readfirstlane(lo);
    hi = __builtin_amdgcn_readfirstlane(hi);
    // One exit test per round keeps the loop a handful of scalar instructions around the compares;
    // the scalar unit is shared by all wavefronts of the compute unit and they all sit in this loop
    // at the same time.  |values| < 2^30, so lo + hi cannot overflow.
    bool more = lo < hi;
    while (more) {
        const int mid = (lo + hi + 1) >> 1;
        const int cnt = count_ge<NR, USED>(v, mid);
        const bool ge = cnt >= keep;
        lo = ge ? mid : lo;
        hi = ge ? hi : mid - 1;
        // slack > 0: any T with keep <= count(v >= T) <= keep + slack will do
        more = lo < hi && (unsigned)(cnt - keep) > (unsigned)slack;
    }
    return lo;
}

// kth_largest over the first `used` (wavefront-uniform) registers only.
template <int NR>
__device__ __forceinline__ int kth_largest_of(const int (&v)[NR], int used, int keep, int lo, int hi, int slack = 0)
{
    switch (used) {
    case 1: return kth_largest<NR, 1>(v, keep, lo, hi, slack);
    case 2: return kth_largest<NR, (NR >= 2 ? 2 : NR)>(v, keep, lo, hi, slack);
    case 3: return kth_largest<NR, (NR >= 3 ? 3 : NR)>(v, keep, lo, hi, slack);
    case 4: return kth_largest<NR, (NR >= 4 ? 4 : NR)>(v, keep, lo, hi, slack);
    case 5: return kth_largest<NR, (NR >= 5 ? 5 : NR)>(v, keep, lo, hi, slack);
    case 6: return kth_largest<NR, (NR >= 6 ? 6 : NR)>(v, keep, lo, hi, slack);
    default: return kth_largest<NR>(v, keep, lo, hi, slack);
    }
}

// m with all but its r lowest set bits cleared (r <= 0: none kept).
__device__ __forceinline__ unsigned lowest_set_bits(unsigned m, int r)
{
    if (r <= 0) return 0u;
    if (r >= __popc(m)) return m;
    unsigned rest = m;
    for (int i = 0; i < r; ++i) rest &= rest - 1;
    return m & ~rest;
}

}  // namespace
}  // namespace dsa
