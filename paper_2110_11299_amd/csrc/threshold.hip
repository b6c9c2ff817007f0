// Threshold masks (paper section 3.1: the mask may be predicted "using thresholds" instead of a
// top-k search).  Unit u keeps every key whose approximate score reaches theta; a unit with none
// keeps its single best key (largest score, lower index among equals).  A unit is a query row or a
// group of vec rows whose scores are summed (section 3.3).  The count per unit varies,
// which is what the paper's equal-count constraint avoids (section 5.2), so the mask is CSR:
// row_ptr [units + 1], col [nnz], keys ascending per unit.
//
//   sweep   one wavefront per 16 units streams the keys once (the key stream of the fine-grained
//           predictor): every score is compared with theta, the outcomes are the unit's bitmap,
//           which goes to the workspace together with the unit's count.
//   scan    exclusive prefix sum of the counts: blocks of 1024 units, then the block totals.
//   fill    one wavefront per unit turns its bitmap into keys at row_ptr[u]; a unit without a key
//           finds its best key with packed dot products.
#include "dsa_internal.h"
#include "threshold_api.h"
#include "key_stream.h"

namespace dsa {
namespace {

constexpr int kScanBlock = 1024;        // units per block of the prefix sum

// Bitmap in the workspace: word w of lane l of task t at (t * NWL + w) * 64 + l (what a wavefront
// stores with one instruction is contiguous).
template <int K, int VEC>
__global__ __launch_bounds__(kWave, 4) void threshold_sweep(const int8_t *__restrict__ Qt, const int8_t *__restrict__ Kt,
                                                           unsigned *__restrict__ bitmap, int32_t *__restrict__ cnt,
                                                           int L, int theta, int tasks_per_head)
{
    const int lane = threadIdx.x;
    const int c = lane & 15, g = lane >> 4;
    const unsigned task = xcd_contiguous(blockIdx.x, gridDim.x);
    const unsigned n = task / (unsigned)tasks_per_head;
    const int u0 = (int)(task % (unsigned)tasks_per_head) * 16;
    const int Lq = stream_quarter(L), NT = Lq / 4, NWL = Lq / 32;
    const int8_t *Kh = Kt + (size_t)n * L * K;
    const int8_t *Qh = Qt + (size_t)n * L * K;
    const int G = L / VEC;                  // units of a head
    const bool unit_live = u0 + c < G;
    int tfull = NT;
#pragma unroll
    for (int q = 0; q < 4; ++q) tfull = min(tfull, max(0, min(L - q * Lq, Lq)) / 4);
    const int key_lo = g * Lq, key_lim = min(L, key_lo + Lq);

    KeyStream<K, VEC> ks;
    // no score lies beyond the limits
    ks.start(Kh, Qh + (size_t)min(u0 + c, G - 1) * (VEC * K), unit_live, lane, Lq, L,
             -max(-kSweepLimit, min(theta, kSweepLimit)));
    unsigned *words = bitmap + (size_t)task * NWL * kWave + lane;
    int mine = 0;
    for (int w = 0; w < NWL; ++w) {
        unsigned word;
        if (8 * w + 8 + decltype(ks)::kLookahead <= tfull) {
            word = pass2_word<false, 0>(ks, 8 * w);
        } else {
            word = pass2_word<true, 0>(ks, 8 * w);
            const int nv = key_lim - (key_lo + 32 * w);      // real keys in this word
            word = nv >= 32 ? word : nv <= 0 ? 0u : word & ((1u << nv) - 1u);
        }
        words[(size_t)w * kWave] = word;
        mine += __popc(word);
    }
    mine += __shfl_xor(mine, 16, kWave);
    mine += __shfl_xor(mine, 32, kWave);
    if (g == 0 && unit_live) cnt[(size_t)n * G + u0 + c] = max(mine, 1);      // an empty unit keeps one key
}

// Exclusive prefix sums inside blocks of kScanBlock counts (into row_ptr) and the block totals.
__global__ __launch_bounds__(256) void scan_blocks(const int32_t *__restrict__ cnt, int32_t *__restrict__ row_ptr,
                                                   int32_t *__restrict__ block_total, unsigned units)
{
    __shared__ int part[256];
    const unsigned base = blockIdx.x * kScanBlock + threadIdx.x * 4;
    int v[4], s = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[i] = base + i < units ? cnt[base + i] : 0;
        s += v[i];
    }
    part[threadIdx.x] = s;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {            // Hillis-Steele over the 256 partial sums
        const int add = threadIdx.x >= (unsigned)off ? part[threadIdx.x - off] : 0;
        __syncthreads();
        part[threadIdx.x] += add;
        __syncthreads();
    }
    int run = part[threadIdx.x] - s;                     // exclusive
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (base + i < units) row_ptr[base + i] = run;
        run += v[i];
    }
    if (threadIdx.x == 255) block_total[blockIdx.x] = part[255];
}

// Exclusive prefix sum of the block totals, in place: one workgroup walks them 256 at a time.
__global__ __launch_bounds__(256) void scan_totals(int32_t *__restrict__ block_total, unsigned blocks,
                                                   int32_t *__restrict__ row_ptr, unsigned units)
{
    __shared__ int part[256];
    __shared__ int carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (unsigned b0 = 0; b0 < blocks; b0 += 256) {
        const unsigned b = b0 + threadIdx.x;
        const int v = b < blocks ? block_total[b] : 0;
        part[threadIdx.x] = v;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {
            const int add = threadIdx.x >= (unsigned)off ? part[threadIdx.x - off] : 0;
            __syncthreads();
            part[threadIdx.x] += add;
            __syncthreads();
        }
        if (b < blocks) block_total[b] = carry + part[threadIdx.x] - v;
        __syncthreads();
        if (threadIdx.x == 255) carry += part[255];
        __syncthreads();
    }
    if (threadIdx.x == 0) row_ptr[units] = carry;        // nnz
}

// One wavefront per unit: final row_ptr[u] and the unit's keys.
template <int K>
__global__ __launch_bounds__(256) void threshold_fill(const int8_t *__restrict__ Qt, const int8_t *__restrict__ Kt,
                                                      const unsigned *__restrict__ bitmap,
                                                      const int32_t *__restrict__ block_total,
                                                      int32_t *__restrict__ row_ptr, int32_t *__restrict__ col,
                                                      long long col_capacity, int L, int vec, int tasks_per_head,
                                                      unsigned units)
{
    const int lane = threadIdx.x & (kWave - 1);
    const unsigned u = xcd_contiguous(blockIdx.x, gridDim.x) * 4 + (threadIdx.x >> 6);
    if (u >= units) return;
    const int G = L / vec;
    const unsigned n = u / (unsigned)G;
    const int i = (int)(u % (unsigned)G);
    const int Lq = stream_quarter(L), NWL = Lq / 32, NW = 4 * NWL;
    const unsigned task = n * (unsigned)tasks_per_head + (unsigned)(i >> 4);
    const int c = i & 15;
    const unsigned *words = bitmap + (size_t)task * NWL * kWave + c;
    const long long start = (long long)row_ptr[u] + block_total[u / kScanBlock];
    if (lane == 0) row_ptr[u] = (int32_t)start;
    int32_t *out = col + start;
    int base = 0;
    // word W of the unit in key order: quarter W / NWL, word W % NWL of lane 16 * quarter + c
    for (int W0 = 0; W0 < NW; W0 += kWave) {
        const int W = W0 + lane;
        const int q = W / NWL, w = W - q * NWL;
        unsigned m = W < NW ? words[(size_t)w * kWave + 16 * q] : 0u;
        const int cc = __popc(m);
        int total;
        int rank = base + wave_incl_scan(cc, lane, &total) - cc;
        base += total;
        const int key1 = q * Lq + 32 * w - 1;
        while (m) {
            if (start + rank < col_capacity) out[rank] = key1 + __ffs(m);
            ++rank;
            m &= m - 1u;
        }
    }
    if (base == 0) {
        // no key reached theta: the unit keeps its best key (largest score, lower index among equals)
        const int *qu = reinterpret_cast<const int *>(Qt + ((size_t)n * L + (size_t)i * vec) * K);
        const int8_t *Kh = Kt + (size_t)n * L * K;
        int best = INT32_MIN, at = 0;
        for (int j = lane; j < L; j += kWave) {
            const int s = unit_key_score(qu, Kh + (size_t)j * K, vec, K / 4);
            if (s > best) { best = s; at = j; }          // ascending j per lane: the first maximum stays
        }
        const int top = wave_max(best);
        const int first = wave_min(best == top ? at : INT32_MAX);
        if (lane == 0 && start < col_capacity) out[0] = first;
    }
}

template <int K, int VEC>
hipError_t launch_threshold_kv(const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt, int theta, int32_t *row_ptr,
                              int32_t *col, long long col_capacity, void *ws, hipStream_t st)
{
    const int tasks_per_head = (sh.L / VEC + 15) / 16;
    const unsigned tasks = (unsigned)sh.B * sh.H * tasks_per_head;
    const unsigned units = (unsigned)sh.B * sh.H * (sh.L / VEC);
    const unsigned blocks = (units + kScanBlock - 1) / kScanBlock;
    const size_t bitmap_words = (size_t)tasks * (stream_quarter(sh.L) / 32) * kWave;
    unsigned *bitmap = static_cast<unsigned *>(ws);
    int32_t *cnt = reinterpret_cast<int32_t *>(bitmap + bitmap_words);
    int32_t *block_total = cnt + units;
    hipLaunchKernelGGL((threshold_sweep<K, VEC>), dim3(tasks), dim3(kWave), 0, st, Qt, Kt, bitmap, cnt, sh.L, theta,
                       tasks_per_head);
    hipLaunchKernelGGL(scan_blocks, dim3(blocks), dim3(256), 0, st, cnt, row_ptr, block_total, units);
    hipLaunchKernelGGL(scan_totals, dim3(1), dim3(256), 0, st, block_total, blocks, row_ptr, units);
    hipLaunchKernelGGL(threshold_fill<K>, dim3((units + 3) / 4), dim3(256), 0, st, Qt, Kt, bitmap, block_total, row_ptr,
                       col, col_capacity, sh.L, VEC, tasks_per_head, units);
    return hipGetLastError();
}

template <int K>
hipError_t launch_threshold_k(const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt, int theta, int32_t *row_ptr,
                              int32_t *col, long long col_capacity, void *ws, hipStream_t st)
{
    if (sh.vec == 1) return launch_threshold_kv<K, 1>(sh, Qt, Kt, theta, row_ptr, col, col_capacity, ws, st);
    if (sh.vec == 4) return launch_threshold_kv<K, 4>(sh, Qt, Kt, theta, row_ptr, col, col_capacity, ws, st);
    return launch_threshold_kv<K, 8>(sh, Qt, Kt, theta, row_ptr, col, col_capacity, ws, st);
}

}  // namespace

bool threshold_supported(const dsa_shape &sh)
{
    return (sh.vec == 1 || sh.vec == 4 || sh.vec == 8) && (sh.k == 16 || sh.k == 32 || sh.k == 64);
}

size_t threshold_workspace_bytes(const dsa_shape &sh)
{
    const size_t tasks = (size_t)sh.B * sh.H * ((sh.L / sh.vec + 15) / 16);
    const size_t units = (size_t)sh.B * sh.H * (sh.L / sh.vec);
    const size_t blocks = (units + kScanBlock - 1) / kScanBlock;
    return sizeof(unsigned) * tasks * (stream_quarter(sh.L) / 32) * kWave + sizeof(int32_t) * (units + blocks);
}

hipError_t launch_predict_threshold(const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt, int theta,
                                    int32_t *row_ptr, int32_t *col, long long col_capacity, void *ws, hipStream_t st)
{
    if (sh.k == 16) return launch_threshold_k<16>(sh, Qt, Kt, theta, row_ptr, col, col_capacity, ws, st);
    if (sh.k == 32) return launch_threshold_k<32>(sh, Qt, Kt, theta, row_ptr, col, col_capacity, ws, st);
    return launch_threshold_k<64>(sh, Qt, Kt, theta, row_ptr, col, col_capacity, ws, st);
}

}  // namespace dsa
