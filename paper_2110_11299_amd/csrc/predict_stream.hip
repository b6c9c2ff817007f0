// Predictor in streaming form (paper section 3.1: approximate scores S~ = Q~ K~^T and the per-unit
// top-k that becomes the mask; section 3.4: the score contraction is cheap, "a low-precision GEMM";
// section 5.1: a unit is a query row or a group of 4 / 8 rows whose scores are summed).  The
// contraction is so cheap on the int8 matrix cores (7 us for all of L = 4096, 16 heads) that it pays
// to compute it twice and never keep a score:
//
//   One wavefront owns 16 selection units of one head and sweeps all L keys.  Four wavefronts with
//   consecutive units of the same head form a workgroup and share the two sweeps: the keys are
//   fetched once per workgroup and handed round through LDS (key_stream.h), one barrier per group
//   of 8 tiles; everything between and after the sweeps is a wavefront's own business.
//   Matrix-core orientation: keys are the rows (A operand), the 16 units the columns (B operand) of
//   v_mfma_i32_16x16x64_i8.  Lane (c = lane % 16, g = lane / 16) receives, per tile, the scores of
//   unit c against 4 consecutive keys of quarter g of the key range.  Every phase keeps that
//   layout: the four lanes (c, 0..3) work for unit c, so all 16 units advance together in plain
//   vector instructions, with no scalar bookkeeping and no serial chain per unit.
//
//   pass 1  sweep the keys; every lane keeps NB maxima over disjoint key sets ("buckets", tile
//           t of a quarter belongs to bucket t % NB): half a vector operation per score.
//   bound   T0 = the keep-th largest of a unit's 4*NB bucket maxima (a few more are accepted): at
//           least keep keys reach T0, so T0 is a lower bound of the keep-th largest score.  A
//           histogram of the maxima in LDS narrows the range to one bin, a bisection on the value
//           (each lane counting its own maxima) finishes inside it.
//   pass 2  sweep the keys again with -T0 as the accumulator input: the sign of what comes out
//           says whether the score reaches T0, and one funnel shift per score collects the signs
//           in 32-bit words: the unit's bitmap of candidate keys, in key order.
//   ties    units with too many candidates (plateaus of equal scores) are swept once more with
//           T0 + 1; the bits that drop out are the ties, of which the first in key order are kept.
//   list    every lane turns its words into key indices, appended to its unit's list in LDS at the
//           offset its quarter starts at: the list is in key order.
//   scores  the list is dealt out again in four equal runs, one per lane of the unit (whatever the
//           distribution of the candidates over the key range); each lane recomputes the scores of
//           its run with packed dot products (about 1.25 * keep per unit) into registers.
//   select  exact threshold T = keep-th largest candidate score by bisection on the value, again all
//           units at once; then keys with score > T, and the first keys with score == T in key
//           order, are placed through running counts into an LDS image of the 16 index rows,
//           which leaves as one contiguous block.
#include "dsa_internal.h"
#include "predict_stream_api.h"
#include "wave_select.h"
#include "key_stream.h"

#include <algorithm>
#include <type_traits>

namespace dsa {
namespace {

constexpr int kStreamUnits = 16;        // units per wavefront: the columns of one matrix instruction
constexpr int kStreamSlots = 88;        // candidate scores a lane holds in registers
constexpr int kStreamCap = 4 * kStreamSlots;   // candidates of one unit (its four lanes)
constexpr int kStreamStride = kStreamCap + 2;  // list entries per unit in LDS: one spare slot, kept even
constexpr int kStreamMaxL = 8192;       // bitmap of 16 units in LDS: 2 * L bytes per wavefront
constexpr int kStreamWaves = kStageWaves;      // wavefronts (tasks) per workgroup: same head, the key sweeps are shared
constexpr int kStreamLongNB = 128;      // bucket maxima per lane for long sequences

// Words at the start of a wavefront's LDS: the bitmap of its 16 units (word w of lane l at w * 64 + l),
// later the image of the 16 index rows (one spare slot); a multiple of 16 bytes.
__host__ __device__ inline int stream_head_words(int L, int keep)
{
    const int bitmap = stream_quarter(L) / 32 * kWave, rows = (kStreamUnits * keep + 2) / 2;
    return ((bitmap > rows ? bitmap : rows) + 3) & ~3;
}

// Sum / minimum / maximum over the four lanes (c, 0..3) that share a unit; every one of them gets it.
__device__ __forceinline__ int unit_sum(int x)
{
    x += __shfl_xor(x, 16, kWave);
    return x + __shfl_xor(x, 32, kWave);
}
__device__ __forceinline__ int unit_min(int x)
{
    x = min(x, __shfl_xor(x, 16, kWave));
    return min(x, __shfl_xor(x, 32, kWave));
}
__device__ __forceinline__ int unit_max(int x)
{
    x = max(x, __shfl_xor(x, 16, kWave));
    return max(x, __shfl_xor(x, 32, kWave));
}

// One group of 8 tiles of pass 1 (t8, the group's first tile, is a multiple of 8).  SAFE: the group may
// touch keys beyond L or tiles beyond the quarter: requests are clamped to the last key row and such
// scores become INT32_MIN.
template <bool SAFE, int PAR, class Stream, int NB>
__device__ __forceinline__ void pass1_group(int (&bmax)[NB], Stream &ks, int t8, int b0, int key_lo, int key_lim)
{
    const unsigned next = ks.template begin_group<PAR>(t8);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        v4i cur = ks.template next_tile<SAFE>(t8, j, next);
        if (SAFE) {
#pragma unroll
            for (int i = 0; i < 4; ++i) cur[i] = mask_beyond(cur[i], key_lo + 4 * (t8 + j) + i, key_lim);
        }
        bmax[b0 + j] = max(max(bmax[b0 + j], cur[0]), max(max(cur[1], cur[2]), cur[3]));
        __builtin_amdgcn_sched_barrier(0);                           // keep the stream in order
    }
    ks.end_group();
}

// Exclusive prefix and total of a per-lane count over the four lanes (c, 0..3) of a unit, in lane
// order g = 0..3.
__device__ __forceinline__ int unit_excl_scan(int x, int g, int *total)
{
    const int s1 = __shfl_xor(x, 16, kWave);      // lane g ^ 1
    const int s2 = __shfl_xor(x, 32, kWave);      // lane g ^ 2
    const int s3 = __shfl_xor(s1, 32, kWave);     // lane g ^ 3
    *total = x + s1 + s2 + s3;
    // g ^ 1 < g iff bit 0 of g is set; g ^ 2 < g and g ^ 3 < g iff bit 1 is set
    return ((g & 1) ? s1 : 0) + ((g & 2) ? s2 + s3 : 0);
}

// K is the projection dimension k (a template argument, so that the byte offsets of the key stream
// are constants).
template <int K, int VEC, int NB>
__global__ __launch_bounds__(kStreamWaves *kWave, 2) void predict_stream(const int8_t *__restrict__ Qt,
                                                           const int8_t *__restrict__ Kt,
                                                           int32_t *__restrict__ idx, int L, int keep,
                                                           int tasks_per_head, int wgs_per_head,
                                                           int lds_words_per_wave)
{
    constexpr int k = K;
    static_assert(kStreamPrefetch == 8 && NB % 32 == 0, "groups of 8 tiles: one trip of the ring, one bitmap word; runs of 4 groups");
    extern __shared__ unsigned smem_all[];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int c = lane & 15, g = lane >> 4;
    unsigned *smem = smem_all + wave * lds_words_per_wave;
    // The wavefronts of a workgroup take consecutive tasks of one head: each has its own units and its
    // own LDS, the key sweeps they make together.  A wavefront without a task mirrors the head's last
    // one and writes nothing.
    const unsigned wg = xcd_contiguous(blockIdx.x, gridDim.x);
    const unsigned n = wg / (unsigned)wgs_per_head;
    const int slot = (int)(wg % (unsigned)wgs_per_head) * kStreamWaves + wave;
    const bool task_live = slot < tasks_per_head;
    const int u0 = min(slot, tasks_per_head - 1) * kStreamUnits;
    const int G = L / VEC;                       // units of a head (rows, or groups of VEC rows)
    const int nu = min(kStreamUnits, G - u0);    // real units of this wavefront
    const int Lq = stream_quarter(L);
    const int NT = Lq / 4;                       // tiles of 4 keys per quarter: a multiple of 8
    const int NWL = Lq / 32;                     // bitmap words per lane
    // LDS: [bitmap: word w of lane l at w * 64 + l | later the image of the 16 index rows][lists]
    unsigned *bitmap = smem;
    const int head_words = stream_head_words(L, keep);
    uint16_t *rows = reinterpret_cast<uint16_t *>(smem);                       // [16][keep]
    uint16_t *list = reinterpret_cast<uint16_t *>(smem + head_words) + c * kStreamStride;   // this unit's list

    const int8_t *Kh = Kt + (size_t)n * L * k;
    const int8_t *Qh = Qt + (size_t)n * L * k;
    const bool unit_live = u0 + c < G;
    const int8_t *Qunit = Qh + (size_t)min(u0 + c, G - 1) * (VEC * k);     // the unit's VEC rows are contiguous

    // tiles [0, tfull) hold only real keys in all four quarters
    int tfull = NT;
#pragma unroll
    for (int q = 0; q < 4; ++q) tfull = min(tfull, max(0, min(L - q * Lq, Lq)) / 4);
    const int key_lo = g * Lq;                   // first key of this lane's quarter
    const int key_lim = min(L, key_lo + Lq);     // its keys are below key_lim

    // the four staging buffers of the sweeps lie where the lists of the four wavefronts will be
    StagedKeyStream<K, VEC> ks;
    static_assert(StagedKeyStream<K, VEC>::kBufBytes <= kStreamUnits * kStreamStride * sizeof(uint16_t), "a buffer fits a list area");
    ks.start(Kh, Qunit, unit_live, (int)threadIdx.x, Lq, L, (unsigned)head_words / 4u, (unsigned)lds_words_per_wave / 4u);

    // ---- pass 1: bucket maxima -----------------------------------------------------------------
    int bmax[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) bmax[b] = INT32_MIN;
    {
        // A group is plain when every tile it touches holds only real keys.  Whole rounds of NB tiles that
        // are plain run without a test per group.
        constexpr int LA = decltype(ks)::kLookahead;
        auto group = [&](int t8, int b0, auto par, auto checked) {
            constexpr int PAR = decltype(par)::value;
            if (!decltype(checked)::value) {
                pass1_group<false, PAR>(bmax, ks, t8, b0, key_lo, key_lim);
            } else if (t8 < NT) {
                if (t8 + 8 + LA <= tfull)
                    pass1_group<false, PAR>(bmax, ks, t8, b0, key_lo, key_lim);
                else
                    pass1_group<true, PAR>(bmax, ks, t8, b0, key_lo, key_lim);
            }
        };
        auto round = [&](int t0, auto checked) {
#pragma unroll
            for (int b0 = 0; b0 < NB; b0 += 32) {
                group(t0 + b0, b0, std::integral_constant<int, 0>{}, checked);
                group(t0 + b0 + 8, b0 + 8, std::integral_constant<int, 1>{}, checked);
                group(t0 + b0 + 16, b0 + 16, std::integral_constant<int, 2>{}, checked);
                group(t0 + b0 + 24, b0 + 24, std::integral_constant<int, 3>{}, checked);
            }
        };
        int t0 = 0;
        for (; t0 + NB + LA <= tfull; t0 += NB) round(t0, std::false_type{});
        for (; t0 < NT; t0 += NB) round(t0, std::true_type{});
        ks.finish();
    }

    // ---- bound: T0 per unit, 16 units at once ---------------------------------------------------
    int T0;
    {
        int lo = INT32_MAX, hi = INT32_MIN;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            lo = min(lo, bmax[b]);
            hi = max(hi, bmax[b]);
        }
        // an empty bucket holds INT32_MIN: start below every possible score instead (the host only
        // takes this kernel when at least keep buckets of a unit hold a key)
        lo = max(unit_min(lo), -(VEC * k * 128 * 128) - 1);
        hi = max(unit_max(hi), lo);
        // Invariant: count(maxima >= lo) >= keep, count(maxima >= hi + 1) < keep.  A unit is done when
        // lo == hi, or as soon as a probe lands within `slack` of keep.
        const int slack = keep >> 4;
        // First a histogram: the unit's range [lo, hi] is cut into at most 128 equal bins, every lane adds
        // its maxima with LDS atomics (5 operations per value, where a round of the bisection takes 2 per
        // value and about ten rounds are needed), and the bin in which the count from the top reaches
        // keep becomes the new range: usually narrow enough to end the search at once.  The bins lie where
        // the lists will be (the sweeps' staging buffers, idle between the two sweeps).
        {
            constexpr int HB = 128;                      // bins per unit
            constexpr int HS = HB + 4;                   // words from unit to unit: the units' bins start in different banks
            static_assert(kStreamUnits * HS <= kStreamUnits * kStreamStride / 2, "the bins fit the list area");
            unsigned *hist = smem + head_words;          // [16 units][HS]
            const unsigned range = (unsigned)(hi - lo);
            const int shift = max(0, 25 - (int)__clz((int)(range | 1u)));        // range >> shift < HB
#pragma unroll
            for (int i = 0; i < (kStreamUnits * HS / 4 + kWave - 1) / kWave; ++i)
                if (i * kWave + lane < kStreamUnits * HS / 4) reinterpret_cast<v4i *>(hist)[i * kWave + lane] = v4i{0, 0, 0, 0};
            wave_lds_sync();
            unsigned *unit_hist = hist + c * HS;
#pragma unroll
            for (int b = 0; b < NB; ++b) atomicAdd(&unit_hist[(unsigned)(max(bmax[b], lo) - lo) >> shift], 1u);
            wave_lds_sync();
            // lane (c, g) walks bins 32 g + 31 .. 32 g of its unit from the top
            v4i part[HB / 16];
            int total = 0;
#pragma unroll
            for (int i = 0; i < HB / 16; ++i) {
                part[i] = reinterpret_cast<const v4i *>(unit_hist + (HB / 4) * g)[i];
                total += part[i][0] + part[i][1] + part[i][2] + part[i][3];
            }
            // maxima in the bins of the lanes above this one
            const int t1 = __shfl_xor(total, 16, kWave), t2 = __shfl_xor(total, 32, kWave), t3 = __shfl_xor(t1, 32, kWave);
            int cum = ((g & 1) ? 0 : t1) + ((g & 2) ? 0 : t2 + t3);       // lanes g ^ 1, g ^ 2, g ^ 3 that lie above g
            int found = -1, at = 0, before = 0;          // highest bin of this lane at which the count reaches keep
#pragma unroll
            for (int j = HB / 4 - 1; j >= 0; --j) {
                const int next = cum + part[j / 4][j % 4];
                const bool here = found < 0 && next >= keep;
                found = here ? (HB / 4) * g + j : found;
                at = here ? next : at;
                before = here ? cum : before;
                cum = next;
            }
            const int best = unit_max(found);            // >= 0: all maxima lie at or above lo
            const bool owner = found == best;            // one lane of the unit
            const int count_at = unit_sum(owner ? at : 0), count_above = unit_sum(owner ? before : 0);
            (void)count_above;                           // < keep by construction: the invariant of hi
            const int new_lo = lo + (best << shift);
            hi = min(hi, new_lo + (1 << shift) - 1);
            lo = new_lo;
            if (count_at - keep <= slack) hi = lo;
            wave_lds_sync();
        }
        while (__ballot(lo < hi) != 0) {
            const int mid = (lo + hi + 1) >> 1;     // == lo for a finished unit
            int cnt = 0;
#pragma unroll
            for (int b = 0; b < NB; ++b) count_if_ge(cnt, bmax[b], mid);
            cnt = unit_sum(cnt);
            const bool ge = cnt >= keep;
            lo = ge ? mid : lo;
            hi = ge ? hi : mid - 1;
            if (ge && cnt - keep <= slack) hi = lo;
        }
        T0 = lo;
    }

    // ---- pass 2: bitmap of candidates (score >= T0) ----------------------------------------------
    int mine = 0;                                // candidates in this lane's quarter
    {
        ks.finish();            // every wavefront is through with its bins: the buffers are the sweeps' again
        ks.restart(-T0);
        constexpr int LA = decltype(ks)::kLookahead;
        auto sweep_word = [&](int w, auto par, auto checked) {
            constexpr int PAR = decltype(par)::value;
            unsigned word;
            if (!decltype(checked)::value) {
                word = pass2_word<false, PAR>(ks, 8 * w);
            } else if (w >= NWL) {
                return;
            } else if (8 * w + 8 + LA <= tfull) {
                word = pass2_word<false, PAR>(ks, 8 * w);
            } else {
                word = pass2_word<true, PAR>(ks, 8 * w);
                const int nv = key_lim - (key_lo + 32 * w);      // real keys in this word
                word = nv >= 32 ? word : nv <= 0 ? 0u : word & ((1u << nv) - 1u);
            }
            bitmap[w * kWave + lane] = word;
            mine += __popc(word);
        };
        auto sweep4 = [&](int w, auto checked) {
            sweep_word(w, std::integral_constant<int, 0>{}, checked);
            sweep_word(w + 1, std::integral_constant<int, 1>{}, checked);
            sweep_word(w + 2, std::integral_constant<int, 2>{}, checked);
            sweep_word(w + 3, std::integral_constant<int, 3>{}, checked);
        };
        int w = 0;
        for (; 8 * (w + 4) + LA <= tfull; w += 4) sweep4(w, std::false_type{});
        for (; w < NWL; w += 4) sweep4(w, std::true_type{});
        ks.finish();
    }

    // ---- ties: units whose candidates do not fit ---------------------------------------------------
    // That is nearly always a plateau: very many keys share the score T0 (codes with few levels).  Such
    // units are swept once more with the threshold T0 + 1; the words of that sweep (score > T0) go
    // where the lists will be, and the bits that dropped out are the keys with score == T0.  If fewer
    // than keep scores lie above T0 the answer is those keys plus the first ties in key order: the
    // lane rewrites its words to exactly that set, and the unit goes on as one with keep candidates.
    // If the strict candidates fit, the unit goes on with them and the bound T0 + 1.
    int nc;
    int pos0 = unit_excl_scan(mine, g, &nc);
    unsigned *gtmap = smem + head_words;         // [NWL][64], in the (still unused) list storage
    const bool gt_fits = NWL * kWave * (int)sizeof(unsigned) <= kStreamUnits * kStreamStride * (int)sizeof(uint16_t);
    if (gt_fits && __ballot(nc > kStreamCap && unit_live) != 0) {
        const bool over = nc > kStreamCap && unit_live;
        const int thr = over ? T0 + 1 : kSweepLimit;       // above every score: no bit for the other units
        int above = 0;
        // a sweep of this wavefront alone: the keys come straight from memory
        KeyStream<K, VEC> alone;
        alone.start(Kh, Qunit, unit_live, lane, Lq, L, -thr);
        for (int w = 0; w < NWL; ++w) {
            unsigned word;
            if (8 * w + 8 + decltype(alone)::kLookahead <= tfull) {
                word = pass2_word<false, 0>(alone, 8 * w);
            } else {
                word = pass2_word<true, 0>(alone, 8 * w);
                const int nv = key_lim - (key_lo + 32 * w);
                word = nv >= 32 ? word : nv <= 0 ? 0u : word & ((1u << nv) - 1u);
            }
            gtmap[w * kWave + lane] = word;
            above += __popc(word);
        }
        int ngt;
        unit_excl_scan(above, g, &ngt);
        const bool ties = over && ngt < keep;
        const bool strict = over && !ties && ngt <= kStreamCap;
        int eq_unit;
        const int eq_before = unit_excl_scan(mine - above, g, &eq_unit);
        int quota = ties ? min(max(keep - ngt - eq_before, 0), mine - above) : 0;   // ties this lane keeps
        if (ties || strict) {
            mine = 0;
            for (int w = 0; w < NWL; ++w) {
                const unsigned gt = gtmap[w * kWave + lane];
                const unsigned eq = bitmap[w * kWave + lane] & ~gt;
                const unsigned kept_ties = lowest_set_bits(eq, quota);      // none for a strict unit
                quota -= __popc(kept_ties);
                const unsigned word = gt | kept_ties;
                bitmap[w * kWave + lane] = word;
                mine += __popc(word);
            }
            if (strict) T0 += 1;
        }
        pos0 = unit_excl_scan(mine, g, &nc);
    }

    // ---- list: candidate keys of every unit in key order ----------------------------------------
    {
        int pos = pos0;
        for (int w = 0; w < NWL; ++w) {
            unsigned m = bitmap[w * kWave + lane];          // this lane's own word: no fence needed
            // the wait for this read belongs here, once per word: left to the first use of m it would sit in
            // the loop below and also wait, on every trip, for the list write of the trip before
            asm volatile("" : "+v"(m));
            const int key1 = key_lo + 32 * w - 1;
            // one bit per trip and lane, no branch inside: a lane with nothing left (or no room) writes
            // to the spare slot behind its unit's list
            while (__ballot(m != 0u) != 0) {
#pragma unroll
                for (int twice = 0; twice < 2; ++twice) {       // two bits per test of the wavefront
                    const bool put = m != 0u && pos < kStreamCap;
                    list[put ? pos : kStreamCap] = (uint16_t)(key1 + __ffs(m));
                    pos += m != 0u;
                    m &= m - 1u;
                }
            }
        }
    }
    wave_lds_sync();
    const bool fits = nc <= kStreamCap;
    const unsigned long long below = (1ull << lane) - 1ull;

    // Units whose candidates do not fit (a plateau of equal scores at T0, or a bound that is not tight):
    // the whole wavefront works on one such unit, recomputing the score of every flagged key in
    // every pass, and writes its row straight to memory.
    for (unsigned long long todo = __ballot(!fits && unit_live && g == 0); todo != 0; todo &= todo - 1) {
        const int uu = __ffsll((long long)todo) - 1;             // lane index = unit index for g == 0
        const int lo0 = __builtin_amdgcn_readlane(T0, uu);
        const int *qu = reinterpret_cast<const int *>(Qh + (size_t)(u0 + uu) * (VEC * k));
        int32_t *out = idx + ((size_t)n * G + u0 + uu) * keep;
        auto flagged_score = [&](int j) -> int {
            if (j >= L) return INT32_MIN;
            const int q = j / Lq, r = j - q * Lq;               // quarter, key inside it
            if (!((bitmap[(r >> 5) * kWave + 16 * q + uu] >> (r & 31)) & 1u)) return INT32_MIN;
            return unit_key_score(qu, Kh + (size_t)j * k, VEC, k / 4);
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
            if (sel && task_live) out[out_base + __popcll(msel & below)] = j;
            out_base += __popcll(msel);
            eq_base += __popcll(meq);
        }
    }

    // ---- scores: lane (c, g) takes run g of its unit's list --------------------------------------
    const bool active = fits && unit_live;
    const int run = active ? (nc + 3) >> 2 : 0;          // candidates per lane, <= kStreamSlots
    const int first = g * run;
    const int run_max = wave_max(run);                   // wavefront-uniform
    // The unit's query side as packed int8: its row (VEC = 1), or the sum of its VEC rows in the two
    // parts of the key stream (the score is linear in the query).
    int qrow[K / 4], qhi[VEC == 1 ? 1 : K / 4];
#pragma unroll
    for (int i = 0; i < K / 4; ++i) {
        if (VEC == 1) {
            qrow[i] = reinterpret_cast<const int *>(Qunit)[i];
        } else {
            int sum[4] = {0, 0, 0, 0};
#pragma unroll
            for (int r = 0; r < VEC; ++r) add_bytes(sum, reinterpret_cast<const int *>(Qunit + r * K)[i]);
            split_sums(sum, qrow[i], qhi[i]);
        }
    }
    int sc[kStreamSlots];
    int top = INT32_MIN;
#pragma unroll
    for (int j0 = 0; j0 < kStreamSlots; j0 += 8) {
        if (j0 < run_max) {
            // eight candidates at a time: their keys, then all their key rows in flight, then the dots
            int key[8];
#pragma unroll
            for (int j = 0; j < 8; ++j)
                key[j] = min((int)list[min(first + j0 + j, kStreamCap - 1)], L - 1);      // never outside K~
            v4i kk[8][K / 16];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const v4i *kr = reinterpret_cast<const v4i *>(Kh + (size_t)((unsigned)key[j] * (unsigned)k));
#pragma unroll
                for (int q4 = 0; q4 < K / 16; ++q4) kk[j][q4] = kr[q4];
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                int s = 0, sh = 0;
#pragma unroll
                for (int q4 = 0; q4 < K / 16; ++q4) {
                    s = __builtin_amdgcn_sdot4(qrow[4 * q4 + 0], kk[j][q4].x, s, false);
                    s = __builtin_amdgcn_sdot4(qrow[4 * q4 + 1], kk[j][q4].y, s, false);
                    s = __builtin_amdgcn_sdot4(qrow[4 * q4 + 2], kk[j][q4].z, s, false);
                    s = __builtin_amdgcn_sdot4(qrow[4 * q4 + 3], kk[j][q4].w, s, false);
                    if (VEC != 1) {
                        sh = __builtin_amdgcn_sdot4(qhi[4 * q4 + 0], kk[j][q4].x, sh, false);
                        sh = __builtin_amdgcn_sdot4(qhi[4 * q4 + 1], kk[j][q4].y, sh, false);
                        sh = __builtin_amdgcn_sdot4(qhi[4 * q4 + 2], kk[j][q4].z, sh, false);
                        sh = __builtin_amdgcn_sdot4(qhi[4 * q4 + 3], kk[j][q4].w, sh, false);
                    }
                }
                s += 128 * sh;
                const bool valid = j0 + j < run && first + j0 + j < nc;
                sc[j0 + j] = valid ? s : INT32_MIN;
                top = max(top, sc[j0 + j]);
            }
        } else {
#pragma unroll
            for (int j = j0; j < j0 + 8; ++j) sc[j] = INT32_MIN;
        }
    }

    // ---- select: exact threshold, all units at once ---------------------------------------------
    int T;
    {
        // every candidate reaches T0 and there are at least keep of them
        int lo = T0, hi = active ? max(unit_max(top), T0) : T0;
        while (__ballot(lo < hi) != 0) {
            const int mid = (lo + hi + 1) >> 1;
            int cnt = 0;
#pragma unroll
            for (int j0 = 0; j0 < kStreamSlots; j0 += 8) {
                if (j0 < run_max) {
#pragma unroll
                    for (int j = j0; j < j0 + 8; ++j) count_if_ge(cnt, sc[j], mid);
                }
            }
            cnt = unit_sum(cnt);
            const bool ge = cnt >= keep;
            lo = ge ? mid : lo;
            hi = ge ? hi : mid - 1;
        }
        T = lo;
    }
    // kept keys into the image of the index rows: position = kept candidates before this one
    wave_lds_sync();          // the bitmap is dead from here on: `rows` takes its place
    {
        int gt = 0, eq = 0;
#pragma unroll
        for (int j0 = 0; j0 < kStreamSlots; j0 += 8) {
            if (j0 < run_max) {
#pragma unroll
                for (int j = j0; j < j0 + 8; ++j) {
                    gt += sc[j] > T;
                    eq += sc[j] == T;
                }
            }
        }
        int gt_unit, eq_unit;
        const int gt_before = unit_excl_scan(gt, g, &gt_unit);
        int eq_run = unit_excl_scan(eq, g, &eq_unit);            // ties before this lane's run
        const int need_eq = keep - gt_unit;                      // ties to keep, in key order
        // kept before this lane's run: every greater score, and the ties that still fit
        int pos = gt_before + min(eq_run, need_eq);
#pragma unroll
        for (int j0 = 0; j0 < kStreamSlots; j0 += 8) {
            if (j0 < run_max) {
                uint16_t key[8];           // all eight reads before the first write: one wait per group
#pragma unroll
                for (int j = 0; j < 8; ++j) key[j] = list[min(first + j0 + j, kStreamCap - 1)];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int s = sc[j0 + j];
                    const bool is_eq = s == T;                   // T >= T0 > INT32_MIN: empty slots never match
                    const bool take = s > T || (is_eq && eq_run < need_eq);
                    // a slot that is not kept writes to the spare slot behind the rows
                    rows[take && active ? c * keep + min(pos, keep - 1) : kStreamUnits * keep] = key[j];
                    pos += take;
                    eq_run += is_eq;
                }
            }
        }
    }
    wave_lds_sync();
    // the rows of this wavefront's units are contiguous in memory; rows of units that took the slow path
    // were written there and are skipped
    {
        int32_t *out = idx + ((size_t)n * G + u0) * keep;
        const unsigned fit_units = (unsigned)__ballot(fits && g == 0);      // bit = unit
        const unsigned all_units = nu >= 32 ? ~0u : (1u << nu) - 1u;
        if ((fit_units & all_units) == all_units) {
            // the usual case: one block of nu * keep indices, four per lane and store
            const int total = nu * keep;
            if (task_live) {
                for (int e = 4 * lane; e < total; e += 4 * kWave) {
                    const uint2 four = *reinterpret_cast<const uint2 *>(rows + e);      // the image has slack behind it
                    const int v[4] = {(int)(four.x & 0xffffu), (int)(four.x >> 16), (int)(four.y & 0xffffu), (int)(four.y >> 16)};
                    if (e + 4 <= total) {
                        *reinterpret_cast<int4 *>(out + e) = make_int4(v[0], v[1], v[2], v[3]);
                    } else {
                        for (int i = 0; e + i < total; ++i) out[e + i] = v[i];
                    }
                }
            }
        } else {
            for (int uu = 0; uu < nu; ++uu) {
                if (!((fit_units >> uu) & 1u) || !task_live) continue;
                for (int e = lane; e < keep; e += kWave) out[uu * keep + e] = (int)rows[uu * keep + e];
            }
        }
    }
}

// LDS of one workgroup: per wavefront the bitmap (later the image of the index rows) and the lists.
size_t stream_words_per_wave(const dsa_shape &sh)
{
    static_assert(kStreamUnits * kStreamStride % 8 == 0, "every wavefront's part starts on a 16-byte boundary");
    return (size_t)stream_head_words(sh.L, sh.keep) + (size_t)kStreamUnits * kStreamStride / 2;
}
size_t stream_lds_bytes(const dsa_shape &sh) { return sizeof(unsigned) * stream_words_per_wave(sh) * kStreamWaves; }

template <int K, int VEC, int NB>
hipError_t launch_stream_t(const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt, int32_t *idx, hipStream_t st)
{
    const size_t words_per_wave = stream_words_per_wave(sh);
    const size_t lds = stream_lds_bytes(sh);
    auto kern = predict_stream<K, VEC, NB>;
    if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds)) return e;
    const int tasks_per_head = (sh.L / VEC + kStreamUnits - 1) / kStreamUnits;
    const int wgs_per_head = (tasks_per_head + kStreamWaves - 1) / kStreamWaves;
    hipLaunchKernelGGL(kern, dim3((unsigned)sh.B * sh.H * wgs_per_head), dim3(kStreamWaves * kWave), lds, st, Qt, Kt, idx,
                       sh.L, sh.keep, tasks_per_head, wgs_per_head, (int)words_per_wave);
    return hipGetLastError();
}

// Buckets of a unit that hold at least one key, for NB maxima per lane.
int stream_buckets(int L, int nb)
{
    const int Lq = stream_quarter(L);
    int total = 0;
    for (int q = 0; q < 4; ++q) {
        const int nvalid = L - q * Lq < 0 ? 0 : (L - q * Lq > Lq ? Lq : L - q * Lq);
        const int tiles = (nvalid + 3) / 4;
        total += tiles < nb ? tiles : nb;
    }
    return total;
}

}  // namespace

// Bucket maxima per lane for a sequence length: one round of buckets for short sequences, the
// long-sequence count otherwise.
int stream_nb(int L)
{
    const int tiles = stream_quarter(L) / 4;
    return tiles <= 32 ? 32 : tiles <= 64 ? 64 : kStreamLongNB;
}

// The streaming kernel serves fine-grained masks whose bound can be tight: enough buckets for keep
// (so that about 1.25 * keep candidates survive) and a candidate list that fits the register path.
bool stream_predict_fits(const dsa_shape &sh)
{
    if ((sh.vec != 1 && sh.vec != 4 && sh.vec != 8) || (sh.k != 16 && sh.k != 32 && sh.k != 64)) return false;
    if (sh.L > kStreamMaxL) return false;
    // Vector-wise masks have few units: with less than one workgroup per compute unit the tiled
    // kernel, which spreads the keys of a unit over a whole workgroup, is faster (measured).
    const long long tasks = (long long)sh.B * sh.H * ((sh.L / sh.vec + kStreamUnits - 1) / kStreamUnits);
    if (sh.vec != 1 && tasks < 4 * 256) return false;
    if (sh.keep > kStreamCap * 5 / 8) return false;     // about 1.25 * keep candidates, with room to spare
    if (4 * stream_buckets(sh.L, stream_nb(sh.L)) < 5 * sh.keep) return false;
    return stream_lds_bytes(sh) <= 160 * 1024;
}

template <int K, int VEC>
hipError_t launch_stream_kv(const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt, int32_t *idx, hipStream_t st)
{
    switch (stream_nb(sh.L)) {
    case 32: return launch_stream_t<K, VEC, 32>(sh, Qt, Kt, idx, st);
    case 64: return launch_stream_t<K, VEC, 64>(sh, Qt, Kt, idx, st);
    default: return launch_stream_t<K, VEC, kStreamLongNB>(sh, Qt, Kt, idx, st);
    }
}

template <int K>
hipError_t launch_stream_k(const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt, int32_t *idx, hipStream_t st)
{
    if (sh.vec == 1) return launch_stream_kv<K, 1>(sh, Qt, Kt, idx, st);
    if (sh.vec == 4) return launch_stream_kv<K, 4>(sh, Qt, Kt, idx, st);
    return launch_stream_kv<K, 8>(sh, Qt, Kt, idx, st);
}

hipError_t launch_predict_stream(const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt, int32_t *idx,
                                 hipStream_t st)
{
    if (sh.k == 16) return launch_stream_k<16>(sh, Qt, Kt, idx, st);
    if (sh.k == 32) return launch_stream_k<32>(sh, Qt, Kt, idx, st);
    return launch_stream_k<64>(sh, Qt, Kt, idx, st);
}

}  // namespace dsa
