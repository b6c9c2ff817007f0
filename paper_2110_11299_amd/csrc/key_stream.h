// The key stream shared by the fine-grained predictor kernels: approximate scores S~ = Q~ K~^T
// (paper section 3.1) of 16 query rows against all keys of their head, 16 keys at a time, from the
// int8 matrix cores, plus the two hand-written instruction pairs that consume a score.  Device code
// only; everything is internal to the translation unit that includes it.
#pragma once

#include "dsa_internal.h"
#include "wave_select.h"

namespace dsa {
namespace {

constexpr int kStreamPrefetch = 8;      // key tiles requested ahead of their use

// Geometry shared by the kernel and the host: the key range is cut into four quarters of Lq keys
// (a multiple of 32, so that a quarter is a whole number of bitmap words), quarter g = lane / 16.
__host__ __device__ inline int stream_quarter(int L) { return (L + 127) / 128 * 32; }

// sum[e] += byte e of w (signed), e = 0..3.
__device__ __forceinline__ void add_bytes(int (&sum)[4], int w)
{
#pragma unroll
    for (int e = 0; e < 4; ++e) sum[e] += (int)(int8_t)(w >> (8 * e));
}
// Four sums of up to 8 int8 values as two words of packed int8: sum = 128 * hi + lo, lo in [-64, 63].
__device__ __forceinline__ void split_sums(const int (&sum)[4], int &lo, int &hi)
{
    unsigned l = 0, h = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int top = (sum[e] + 64) >> 7;          // floor((sum + 64) / 128), |top| <= 8
        l |= ((unsigned)(sum[e] - 128 * top) & 0xffu) << (8 * e);
        h |= ((unsigned)top & 0xffu) << (8 * e);
    }
    lo = (int)l;
    hi = (int)h;
}

// The key stream of one wavefront: scores of tile t (16 keys x 16 units) from v_mfma_i32_16x16x64_i8.
// A matrix row is 64 bytes of contraction, i.e. R = 64 / K keys side by side: every lane loads 16
// bytes (a quarter, half or all of one key row, the widest load there is, which is what the vector
// memory path delivers best), and tile i of the R tiles that share a row operand is obtained with a
// unit operand that holds Q~ in the lanes of key i and zero in the others.  Row r of tile t is key
// (r / 4) * Lq + 4 t + r % 4, so lane (c, g) receives keys g * Lq + 4 t + {0..3} of unit c.
// Row operands sit in a ring and are requested 8 tiles before their use; the matrix core runs two
// tiles ahead of the consumer.  That distance is not only for speed: the consumers of a score include
// hand-written instruction pairs, for which the compiler inserts no wait for a matrix result, so a
// whole tile of vector work always lies between a matrix instruction and the first read of its result
// (in-order issue, pinned by the scheduling barriers of the callers).
// Vector-wise masks (VEC = 4 or 8 query rows per unit, the group score being the sum over the rows):
// the score is linear in the query, so the unit's rows are summed first (exact in integers) and the
// sum, which needs 11 bits, is split as sum = 128 * hi + lo with lo in [-64, 63]: both parts are int8
// operands, every tile takes two matrix instructions on the same row operand, and the consumer gets
// lo_scores + 128 * hi_scores, formed two tiles after the instructions were issued.
template <int K, int VEC = 1> struct KeyStream {
    static constexpr int R = 64 / K;            // keys per matrix row = tiles per ring slot
    static constexpr int LPK = K / 16;          // lanes (16-byte parts) per key row
    static constexpr int NS = 8 / R;            // ring slots: 8 tiles in flight
    static constexpr unsigned kSlotStep = 4u * R * K;   // bytes between the rows of consecutive slots
    const int8_t *Kh;
    unsigned off0, off_last;
    v4i qv[R], qh[VEC == 1 ? 1 : R], ring[NS], p0, p1, h0, h1;     // qh, h0, h1: the hi part (VEC > 1 only)
    v4i bias;                                   // added to every score (the matrix instruction's accumulator input)

    static __device__ __forceinline__ v4i load16(const int8_t *p) { return *reinterpret_cast<const v4i *>(p); }

    template <bool SAFE> __device__ __forceinline__ void issue(int t8, int jn, unsigned next)
    {
        const int slot = (jn % 8) / R;
        p1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(ring[slot], qv[jn % R], bias, 0, 0, 0);
        if (VEC != 1) h1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(ring[slot], qh[jn % R], v4i{0, 0, 0, 0}, 0, 0, 0);
        if (jn % R == R - 1) {                  // the slot's last tile is on its way: request what comes 8 tiles later
            unsigned off = next + (unsigned)(jn / R) * kSlotStep;
            if (SAFE) off = min(off, off_last);
            ring[slot] = load16(Kh + off);
        }
    }
    // Byte offset of the row operand that holds tile t8 + 8 (t8 a multiple of 8).
    __device__ __forceinline__ unsigned next_of(int t8) const { return off0 + (unsigned)(t8 / R + NS) * kSlotStep; }

    // Starts the stream: operands of tiles 0..7, tiles 0 and 1 issued.  Rows beyond L read row L - 1.
    // Qunit: the unit's first (or only) row of Q~; its VEC rows are contiguous.
    __device__ __forceinline__ void start(const int8_t *Kh_, const int8_t *Qunit, bool unit_live, int lane, int Lq, int L)
    {
        Kh = Kh_;
        const int r = lane & 15, kb = lane >> 4, sub = kb / LPK, part = kb % LPK;
        off0 = (unsigned)((r >> 2) * Lq + 4 * sub + (r & 3)) * (unsigned)K + 16u * part;
        off_last = (unsigned)(L - 1) * (unsigned)K + 16u * part;
        v4i lo = load16(Qunit + 16 * part), hi = {0, 0, 0, 0};
        if (VEC != 1) {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                int sum[4] = {0, 0, 0, 0};
#pragma unroll
                for (int row = 0; row < VEC; ++row) add_bytes(sum, reinterpret_cast<const int *>(Qunit + row * K + 16 * part)[w]);
                int l, h;
                split_sums(sum, l, h);
                lo[w] = l;
                hi[w] = h;
            }
        }
#pragma unroll
        for (int i = 0; i < R; ++i) {
            qv[i] = (unit_live && sub == i) ? lo : v4i{0, 0, 0, 0};
            if (VEC != 1) qh[i] = (unit_live && sub == i) ? hi : v4i{0, 0, 0, 0};
        }
        restart(0);
    }
    // Rewinds to tile 0; from here on every score comes out as score + b.
    __device__ __forceinline__ void restart(int b)
    {
        bias = v4i{b, b, b, b};
#pragma unroll
        for (int sl = 0; sl < NS; ++sl) ring[sl] = load16(Kh + min(off0 + (unsigned)sl * kSlotStep, off_last));
        const unsigned next = next_of(0);
        issue<true>(0, 0, next);
        p0 = p1;
        if (VEC != 1) h0 = h1;
        issue<true>(0, 1, next);
    }
    // Scores of tile t8 + j (j = 0..7, a constant after unrolling); issues tile t8 + j + 2.
    template <bool SAFE> __device__ __forceinline__ v4i next_tile(int t8, int j, unsigned next)
    {
        v4i cur = p0;
        if (VEC != 1) cur += h0 << 7;
        p0 = p1;
        if (VEC != 1) h0 = h1;
        issue<SAFE>(t8, j + 2, next);          // tile t8 + j + 2 (for j > 5 a tile of the next group)
        return cur;
    }
};

// cnt += (v >= t), per lane: compare into the carry, add with carry.
__device__ __forceinline__ void count_if_ge(int &cnt, int v, int t)
{
    asm("v_cmp_ge_i32 vcc, %1, %2\n\tv_addc_co_u32 %0, vcc, 0, %0, vcc" : "+v"(cnt) : "v"(v), "v"(t) : "vcc");
}
// word = 2 * word + (v < 0) for the four scores of a tile in turn, per lane: one funnel shift each.
// Hand-written so that the shifts stay where they are written, between the matrix instructions of their
// tile (the compiler gathers the plain form of a whole group of tiles behind the group's matrix
// instructions), and as one statement so that nothing is put between them.
__device__ __forceinline__ void shift_in_signs(unsigned &word, v4i v)
{
    asm("v_alignbit_b32 %0, %0, %1, 31\n\tv_alignbit_b32 %0, %0, %2, 31\n\t"
        "v_alignbit_b32 %0, %0, %3, 31\n\tv_alignbit_b32 %0, %0, %4, 31"
        : "+v"(word)
        : "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]));
}

// v = (key < L) ? v : INT32_MIN, per lane, as one inseparable pair (a plain compare per score of an
// unrolled round would be hoisted by the hundreds and exhaust the scalar registers).
__device__ __forceinline__ int mask_beyond(int v, int key, int L)
{
    asm("v_cmp_lt_i32 vcc, %1, %2\n\tv_cndmask_b32 %0, %3, %0, vcc" : "+v"(v) : "v"(key), "v"(L), "v"(INT32_MIN) : "vcc");
    return v;
}

// One bitmap word of a threshold sweep: 8 tiles, 32 consecutive keys of this lane's quarter, bit = score
// reaches the threshold.  The stream was restarted with bias = -threshold, so a score misses the
// threshold iff its sign bit is set, and one funnel shift per score moves that bit into the word.
template <bool SAFE, int K, int VEC>
__device__ __forceinline__ unsigned pass2_word(KeyStream<K, VEC> &ks, int t8)
{
    const unsigned next = ks.next_of(t8);
    unsigned word = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const v4i cur = ks.template next_tile<SAFE>(t8, j, next);
        shift_in_signs(word, cur);
        __builtin_amdgcn_sched_barrier(0);
    }
    return ~__brev(word);         // the first key of the word was shifted in first
}

// Largest magnitude a sweep threshold may have: score - threshold must not overflow (|score| < 2^27).
constexpr int kSweepLimit = 1 << 30;

}  // namespace
}  // namespace dsa
