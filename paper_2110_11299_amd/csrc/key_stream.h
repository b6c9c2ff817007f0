// The key streams of the streaming predictor and the threshold sweep: approximate scores
// S~ = Q~ K~^T (paper section 3.1) of 16 selection units (query rows, or groups of rows whose scores
// are summed: section 5.1) against all keys of their head, 16 keys at a time, from the int8 matrix
// cores, in two forms (a wavefront on its own, straight from memory; four wavefronts of a workgroup
// sharing the keys through LDS), plus the few hand-written instructions that consume a score.
// Device code only; everything is internal to the translation unit that includes it.
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

// Unit operands of the matrix instruction for lane (c = lane % 16, kb = lane / 16): the 16 bytes of
// the unit's query side that face part kb % (K / 16) of a key row, in the operand of the tile
// kb / (K / 16) that shares a row operand, zero in the other operands of the lane.  For VEC > 1 the
// query side is the sum of the unit's rows, split into the parts lo (qv) and hi (qh).
template <int K, int VEC>
__device__ __forceinline__ void unit_operands(const int8_t *Qunit, bool unit_live, int lane, v4i (&qv)[64 / K],
                                              v4i (&qh)[VEC == 1 ? 1 : 64 / K])
{
    constexpr int R = 64 / K, LPK = K / 16;
    const int kb = lane >> 4, sub = kb / LPK, part = kb % LPK;
    v4i lo = *reinterpret_cast<const v4i *>(Qunit + 16 * part), hi = {0, 0, 0, 0};
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
}

// The key stream of one wavefront: scores of tile t (16 keys x 16 units) from v_mfma_i32_16x16x64_i8.
// A matrix row is 64 bytes of contraction, i.e. R = 64 / K keys side by side: every lane loads 16
// bytes (a quarter, half or all of one key row, the widest load there is, which is what the vector
// memory path delivers best), and tile i of the R tiles that share a row operand is obtained with a
// unit operand that holds Q~ in the lanes of key i and zero in the others.  Row r of tile t is key
// (r / 4) * Lq + 4 t + r % 4, so lane (c, g) receives keys g * Lq + 4 t + {0..3} of unit c.
// Row operands sit in a ring and are requested 8 tiles before their use; the matrix core runs two
// tiles ahead of the consumer, so that the wait states between a matrix instruction and the first read
// of its result are mostly filled with work.  Whatever reads a score first must be plain code, not a
// hand-written instruction: the compiler keeps those wait states only for instructions it knows.
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
    // tiles beyond a group's own that it touches (issues, requests): a group is plain (not SAFE) when
    // these too hold only real keys
    static constexpr int kLookahead = 2 + kStreamPrefetch;
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
    // A group of 8 tiles starts (t8, its first tile, a multiple of 8): byte offset of the row operand
    // that holds tile t8 + 8.  PAR, the group's index modulo 4, means nothing to this stream.
    template <int PAR> __device__ __forceinline__ unsigned begin_group(int t8) const { return off0 + (unsigned)(t8 / R + NS) * kSlotStep; }
    __device__ __forceinline__ void end_group() const {}
    __device__ __forceinline__ void finish() const {}

    // Starts the stream: operands of tiles 0..7, tiles 0 and 1 issued.  Rows beyond L read row L - 1.
    // Qunit: the unit's first (or only) row of Q~; its VEC rows are contiguous.
    // Every score comes out as score + b.
    __device__ __forceinline__ void start(const int8_t *Kh_, const int8_t *Qunit, bool unit_live, int lane, int Lq, int L, int b = 0)
    {
        Kh = Kh_;
        const int r = lane & 15, kb = lane >> 4, sub = kb / LPK, part = kb % LPK;
        off0 = (unsigned)((r >> 2) * Lq + 4 * sub + (r & 3)) * (unsigned)K + 16u * part;
        off_last = (unsigned)(L - 1) * (unsigned)K + 16u * part;
        unit_operands<K, VEC>(Qunit, unit_live, lane, qv, qh);
        restart(b);
    }
    // Rewinds to tile 0; from here on every score comes out as score + b.
    __device__ __forceinline__ void restart(int b)
    {
        bias = v4i{b, b, b, b};
#pragma unroll
        for (int sl = 0; sl < NS; ++sl) ring[sl] = load16(Kh + min(off0 + (unsigned)sl * kSlotStep, off_last));
        const unsigned next = begin_group<0>(0);
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

// Dynamic LDS of the workgroup, as bytes (every dynamic array of a kernel starts at the same address).
extern __shared__ __align__(16) unsigned char stream_lds[];

constexpr int kStageWaves = 4;          // wavefronts of a workgroup that share staged keys

// The same stream for kStageWaves wavefronts that sweep the keys of one head together: the vector
// memory path delivers about 40 bytes per clock and compute unit whatever the pattern, and four
// wavefronts that each fetch every key row spend their sweep waiting for it.  Here the workgroup
// fetches every row once: the keys of a group of 8 tiles (a "chunk": 32 keys of each quarter) are
// copied by all 256 threads, 16 bytes each, through registers into one of four LDS buffers, and the
// wavefronts take their row operands from there.  Schedule, in groups:
//   group i, start   the chunk of group i + 3 (in registers since group i - kDepth) is written to buffer
//                    (i + 3) % 4, whose last reads (chunk i - 1) were issued in group i - 2; the chunk of
//                    group i + 3 + kDepth is requested (memory answers after several groups' time);
//   group i          row operands of tiles up to 8 ahead are read: chunks i + 1 and i + 2;
//   group i, end     every wavefront waits until its write has landed (not for the reads it has just
//                    issued: LDS answers in order) and meets the others at a barrier.
// Every wavefront of the workgroup must run the same groups (the sweeps depend on L only), and a sweep
// ends with finish().
// Buffer layout: quarter q at q * kRun, key j of the chunk's 32 at j * K, 16-byte part p at 16 * p',
// with kRun padded (K = 16, 32) or p' = p ^ f(j, q) (K = 64) so that the eight lanes that read
// together (rows r .. r + 7 of one part) fall into eight different 16-byte bank groups.
template <int K, int VEC = 1> struct StagedKeyStream {
    static constexpr int R = 64 / K, LPK = K / 16, NS = 8 / R;
    static constexpr unsigned kRun = 32u * K + (K == 16 ? 64u : K == 32 ? 16u : 0u);
    static constexpr unsigned kBufBytes = 4u * kRun;
    static constexpr int PER = K == 64 ? 2 : 1;         // 16-byte pieces a thread copies per chunk
    static constexpr int kDepth = K == 64 ? 2 : 4;      // chunks on their way from memory, per thread
    static constexpr int kLookahead = 0;                // the copies clamp their rows: SAFE is about the scores only
    const int8_t *Kh;
    int L, chunks;                              // chunks = groups per sweep
    unsigned stage0, stage_stride;              // byte offset of buffer 0 in LDS, distance to the next buffer (multiples of 16)
    unsigned rd_off, rd_next, rd_next2;         // this lane's read offset in a buffer; the same in the next two chunks' buffers
    unsigned wr_off[PER], part16[PER];
    int key0[PER];                              // copied key of chunk 0
    v4i g[kDepth][PER];                         // chunks on their way from memory
    v4i qv[R], qh[VEC == 1 ? 1 : R], ring[NS], p0, p1, h0, h1, bias;

    static __device__ __forceinline__ unsigned swizzle(int j, int q) { return K == 64 ? (unsigned)(((j >> 1) & 1) | ((q & 1) << 1)) : 0u; }

    __device__ __forceinline__ void fetch(v4i (&dst)[PER], int chunk)
    {
        const int first = 32 * min(chunk, chunks - 1);
#pragma unroll
        for (int e = 0; e < PER; ++e) {
            const unsigned key = (unsigned)min(key0[e] + first, L - 1);        // rows beyond L: the last row
            dst[e] = *reinterpret_cast<const v4i *>(Kh + key * (unsigned)K + part16[e]);
        }
    }
    __device__ __forceinline__ void put(const v4i (&src)[PER], unsigned buffer)
    {
#pragma unroll
        for (int e = 0; e < PER; ++e) *reinterpret_cast<v4i *>(stream_lds + stage0 + buffer * stage_stride + wr_off[e]) = src[e];
    }
    // Own LDS traffic done but for the N most recent operations, then the barrier; nothing moves across.
    template <int N> static __device__ __forceinline__ void meet()
    {
        asm volatile("s_waitcnt lgkmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
    }
    __device__ __forceinline__ v4i row_operand(unsigned at) const { return *reinterpret_cast<const v4i *>(stream_lds + at); }

    template <bool SAFE> __device__ __forceinline__ void issue(int, int jn, unsigned)
    {
        const int slot = (jn % 8) / R;
        p1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(ring[slot], qv[jn % R], bias, 0, 0, 0);
        if (VEC != 1) h1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(ring[slot], qh[jn % R], v4i{0, 0, 0, 0}, 0, 0, 0);
        if (jn % R == R - 1)                    // the slot's last tile is on its way: what comes 8 tiles later
            ring[slot] = row_operand((jn < 8 ? rd_next : rd_next2) + 256u * (unsigned)slot);
    }

    // tid: thread of the workgroup (0 .. 64 * kStageWaves - 1); stage0_16, stride_16: where the four
    // buffers are, in units of 16 bytes.
    __device__ __forceinline__ void start(const int8_t *Kh_, const int8_t *Qunit, bool unit_live, int tid, int Lq, int L_,
                                          unsigned stage0_16, unsigned stride_16)
    {
        Kh = Kh_;
        L = L_;
        chunks = Lq / 32;
        stage0 = 16u * stage0_16;               // in units of 16 bytes: the accesses are known to be aligned
        stage_stride = 16u * stride_16;
        const int lane = tid & (kWave - 1);
        const int r = lane & 15, kb = lane >> 4, sub = kb / LPK, part = kb % LPK, q = r >> 2;
        rd_off = stage0 + (unsigned)q * kRun + (unsigned)(4 * sub + (r & 3)) * K + 16u * ((unsigned)part ^ swizzle(r & 3, q));
#pragma unroll
        for (int e = 0; e < PER; ++e) {
            // byte of the unpadded chunk (K = 16: the chunk is copied twice, no thread stands aside)
            const unsigned o = (unsigned)(tid + 64 * kStageWaves * e) * 16u % (128u * K);
            const int cq = o / (32u * K), j = o % (32u * K) / K, p = o % K / 16;
            key0[e] = cq * Lq + j;
            part16[e] = 16u * p;
            wr_off[e] = (unsigned)cq * kRun + (unsigned)j * K + 16u * ((unsigned)p ^ swizzle(j, cq));
        }
        unit_operands<K, VEC>(Qunit, unit_live, lane, qv, qh);
        restart(0);
    }
    // Rewinds to tile 0; from here on every score comes out as score + b.  The buffers are free: a sweep
    // ends with the barrier of its last group.
    __device__ __forceinline__ void restart(int b)
    {
        bias = v4i{b, b, b, b};
        if (kDepth >= 3) {                      // the first three chunks in one round trip to memory
            fetch(g[0], 0);
            fetch(g[1], 1);
            fetch(g[2 % kDepth], 2);
            put(g[0], 0);
            put(g[1], 1);
            put(g[2 % kDepth], 2);
        } else {
            fetch(g[0], 0);
            fetch(g[1], 1);
            put(g[0], 0);
            fetch(g[0], 2);
            put(g[1], 1);
            put(g[0], 2);
        }
#pragma unroll
        for (int d = 0; d < kDepth; ++d) fetch(g[d], 3 + d);
        meet<0>();
#pragma unroll
        for (int sl = 0; sl < NS; ++sl) ring[sl] = row_operand(rd_off + 256u * sl);
        rd_next = rd_off + stage_stride;        // chunk 1 is in buffer 1, chunk 2 in buffer 2
        rd_next2 = rd_off + 2 * stage_stride;
        issue<true>(0, 0, 0u);
        p0 = p1;
        if (VEC != 1) h0 = h1;
        issue<true>(0, 1, 0u);
    }
    // Group i = t8 / 8 starts; PAR = i % 4.
    template <int PAR> __device__ __forceinline__ unsigned begin_group(int t8)
    {
        const unsigned i = (unsigned)t8 / 8u;                    // chunk i sits in buffer i % 4
        put(g[PAR % kDepth], (i + 3u) & 3u);
        fetch(g[PAR % kDepth], (int)i + 3 + kDepth);
        rd_next = rd_off + ((i + 1u) & 3u) * stage_stride;
        rd_next2 = rd_off + ((i + 2u) & 3u) * stage_stride;
        return 0u;
    }
    // The group's NS reads may still be on their way; the write before them has landed.
    __device__ __forceinline__ void end_group() { meet<NS>(); }
    // End of a sweep: every wavefront's reads are done, the buffers may be used for anything.
    __device__ __forceinline__ void finish() { meet<0>(); }

    template <bool SAFE> __device__ __forceinline__ v4i next_tile(int t8, int j, unsigned next)
    {
        v4i cur = p0;
        if (VEC != 1) cur += h0 << 7;
        p0 = p1;
        if (VEC != 1) h0 = h1;
        issue<SAFE>(t8, j + 2, next);
        return cur;
    }
};

// cnt += (v >= t), per lane: compare into the carry, add with carry.
__device__ __forceinline__ void count_if_ge(int &cnt, int v, int t)
{
    asm("v_cmp_ge_i32 vcc, %1, %2\n\tv_addc_co_u32 %0, vcc, 0, %0, vcc" : "+v"(cnt) : "v"(v), "v"(t) : "vcc");
}
// word = 2 * word + (v < 0) for the four scores of a tile in turn, per lane: one funnel shift each, in
// plain code, so that the compiler sees a vector instruction reading a matrix result and keeps the wait
// states that takes.  The empty statement behind them pins the shifts to their tile: without it the
// compiler gathers the shifts of a whole group of tiles behind the group's matrix instructions.
__device__ __forceinline__ void shift_in_signs(unsigned &word, v4i v)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) word = __builtin_amdgcn_alignbit(word, (unsigned)v[i], 31);
    asm volatile("" : "+v"(word));
}

// v = (key < L) ? v : INT32_MIN, per lane, as one inseparable pair (a plain compare per score of an
// unrolled round would be hoisted by the hundreds and exhaust the scalar registers).
__device__ __forceinline__ int mask_beyond(int v, int key, int L)
{
    // v may come straight from a matrix instruction, and a hand-written instruction gets no wait states
    // from the compiler: pass it through a plain vector move first (identity lane permutation)
    v = __builtin_amdgcn_update_dpp(0, v, 0xE4, 0xF, 0xF, false);
    asm("v_cmp_lt_i32 vcc, %1, %2\n\tv_cndmask_b32 %0, %3, %0, vcc" : "+v"(v) : "v"(key), "v"(L), "v"(INT32_MIN) : "vcc");
    return v;
}

// One bitmap word of a threshold sweep: 8 tiles, 32 consecutive keys of this lane's quarter, bit = score
// reaches the threshold.  The stream was restarted with bias = -threshold, so a score misses the
// threshold iff its sign bit is set, and one funnel shift per score moves that bit into the word.
template <bool SAFE, int PAR, class Stream>
__device__ __forceinline__ unsigned pass2_word(Stream &ks, int t8)
{
    const unsigned next = ks.template begin_group<PAR>(t8);
    unsigned word = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const v4i cur = ks.template next_tile<SAFE>(t8, j, next);
        shift_in_signs(word, cur);
        __builtin_amdgcn_sched_barrier(0);
    }
    ks.end_group();
    return ~__brev(word);         // the first key of the word was shifted in first
}

// Largest magnitude a sweep threshold may have: score - threshold must not overflow (|score| < 2^27).
constexpr int kSweepLimit = 1 << 30;

}  // namespace
}  // namespace dsa
