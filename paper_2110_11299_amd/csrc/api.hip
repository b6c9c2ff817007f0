// C ABI of libdsa_hip.so: argument checking on the host, then dispatch to the launchers.
// Nothing here touches the device before every check has passed.
#include "dsa_internal.h"
#include "attention_api.h"
#include "predict_api.h"
#include "predict_stream_api.h"
#include "project_api.h"
#include "threshold_api.h"

#include <math.h>

#include <atomic>

// Mask storage for dsa_attention_fwd_noalloc: one array per GPU, held until the process ends.  In
// host code this name is only a handle for hipGetSymbolAddress; kernels get the resolved address.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device, resolved once per device (two threads racing
// on the first call both resolve the same address).
hipError_t static_scratch(void **out)
{
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev)) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return hipSuccess;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Checks that do not depend on which entry point is called.
dsa_status check_common(const dsa_shape *sh)
{
    if (!sh) return DSA_ERR_NULL;
    if (sh->B < 1 || sh->H < 1 || sh->L < 1) return DSA_ERR_SHAPE;
    if ((int64_t)sh->B * sh->H > (1 << 24)) return DSA_ERR_SHAPE;
    if (sh->vec != 1 && sh->vec != 4 && sh->vec != 8) return DSA_ERR_UNSUPPORTED;
    if (sh->L % sh->vec) return DSA_ERR_SHAPE;
    if (sh->keep < 1 || sh->keep > sh->L) return DSA_ERR_SHAPE;
    if ((int64_t)sh->B * sh->H * sh->L > (int64_t)1 << 31) return DSA_ERR_UNSUPPORTED;
    return DSA_OK;
}

dsa_status check_predict(const dsa_shape *sh)
{
    if (dsa_status s = check_common(sh)) return s;
    if (sh->k < 16 || sh->k > 128 || sh->k % 16) return DSA_ERR_UNSUPPORTED;
    if (sh->L > dsa::predict_max_L()) return DSA_ERR_UNSUPPORTED;
    return DSA_OK;
}

dsa_status check_attention(const dsa_shape *sh)
{
    if (dsa_status s = check_common(sh)) return s;
    if (sh->d != 64 && sh->d != 128) return DSA_ERR_UNSUPPORTED;
    if (sh->dtype != DSA_F32 && sh->dtype != DSA_BF16) return DSA_ERR_UNSUPPORTED;
    if (sh->keep > dsa::attention_max_keep()) return DSA_ERR_UNSUPPORTED;
    if (sh->L > dsa::attention_max_L()) return DSA_ERR_UNSUPPORTED;
    if (!isfinite(sh->scale)) return DSA_ERR_SHAPE;
    return DSA_OK;
}

size_t idx_bytes(const dsa_shape &sh)
{
    return (size_t)sh.B * sh.H * (sh.L / sh.vec) * sh.keep * sizeof(int32_t);
}

size_t round_up_256(size_t x) { return (x + 255) & ~(size_t)255; }

dsa_status from_hip(hipError_t e) { return e == hipSuccess ? DSA_OK : DSA_ERR_HIP; }

}  // namespace

extern "C" {

int32_t dsa_keep_from_ratio(int32_t L, double ratio)
{
    if (L < 1) return 0;
    double x = floor(ratio * (double)L + 0.5);
    if (!(x >= 1.0)) x = 1.0;
    if (x > (double)L) x = (double)L;
    return (int32_t)x;
}

size_t dsa_workspace_bytes(const dsa_shape *sh)
{
    if (check_predict(sh) != DSA_OK) return 0;
    // [mask for dsa_attention_fwd when the caller does not want it back][predict scratch]
    return round_up_256(idx_bytes(*sh)) + round_up_256(dsa::predict_workspace_bytes(*sh));
}

dsa_status dsa_predict_mask(const dsa_shape *sh, const int8_t *Qt, const int8_t *Kt, int32_t *idx,
                            void *ws, size_t ws_bytes, void *stream)
{
    if (!sh || !Qt || !Kt || !idx) return DSA_ERR_NULL;
    if (dsa_status s = check_predict(sh)) return s;
    if (!aligned16(Qt) || !aligned16(Kt) || !aligned16(idx) || !aligned16(ws)) return DSA_ERR_ALIGN;
    const size_t need = round_up_256(dsa::predict_workspace_bytes(*sh));
    if (need && (!ws || ws_bytes < need)) return DSA_ERR_WORKSPACE;
    return from_hip(dsa::launch_predict(*sh, Qt, Kt, idx, ws, (hipStream_t)stream));
}

dsa_status dsa_sddmm(const dsa_shape *sh, const void *Q, const void *K, const int32_t *idx, float *S,
                     void *stream)
{
    if (!sh || !Q || !K || !idx || !S) return DSA_ERR_NULL;
    if (dsa_status s = check_attention(sh)) return s;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(idx) || !aligned16(S)) return DSA_ERR_ALIGN;
    return from_hip(dsa::launch_attention(dsa::kSddmm, *sh, Q, K, nullptr, idx, nullptr, S, nullptr,
                                          (hipStream_t)stream));
}

dsa_status dsa_sparse_softmax(const dsa_shape *sh, const float *S, float *P, void *stream)
{
    if (!sh || !S || !P) return DSA_ERR_NULL;
    if (dsa_status s = check_common(sh)) return s;
    if (!aligned16(S) || !aligned16(P)) return DSA_ERR_ALIGN;
    return from_hip(dsa::launch_softmax(*sh, S, P, (hipStream_t)stream));
}

dsa_status dsa_spmm(const dsa_shape *sh, const float *P, const int32_t *idx, const void *V, float *O,
                    void *stream)
{
    if (!sh || !P || !idx || !V || !O) return DSA_ERR_NULL;
    if (dsa_status s = check_attention(sh)) return s;
    if (!aligned16(P) || !aligned16(idx) || !aligned16(V) || !aligned16(O)) return DSA_ERR_ALIGN;
    return from_hip(dsa::launch_attention(dsa::kSpmm, *sh, nullptr, nullptr, V, idx, P, nullptr, O,
                                          (hipStream_t)stream));
}

dsa_status dsa_masked_attention(const dsa_shape *sh, const void *Q, const void *K, const void *V,
                                const int32_t *idx, float *O, void *stream)
{
    if (!sh || !Q || !K || !V || !idx || !O) return DSA_ERR_NULL;
    if (dsa_status s = check_attention(sh)) return s;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(idx) || !aligned16(O))
        return DSA_ERR_ALIGN;
    return from_hip(dsa::launch_attention(dsa::kFused, *sh, Q, K, V, idx, nullptr, nullptr, O,
                                          (hipStream_t)stream));
}

dsa_status dsa_attention_fwd(const dsa_shape *sh, const void *Q, const void *K, const void *V,
                             const int8_t *Qt, const int8_t *Kt, float *O, int32_t *idx_out, void *ws,
                             size_t ws_bytes, void *stream)
{
    if (!sh || !Q || !K || !V || !Qt || !Kt || !O) return DSA_ERR_NULL;
    if (dsa_status s = check_predict(sh)) return s;
    if (dsa_status s = check_attention(sh)) return s;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(Qt) || !aligned16(Kt) ||
        !aligned16(O) || !aligned16(idx_out) || !aligned16(ws))
        return DSA_ERR_ALIGN;
    const size_t mask_bytes = round_up_256(idx_bytes(*sh));
    const size_t scratch = round_up_256(dsa::predict_workspace_bytes(*sh));
    const size_t need = (idx_out ? 0 : mask_bytes) + scratch;
    if (need && (!ws || ws_bytes < need)) return DSA_ERR_WORKSPACE;
    int32_t *idx = idx_out ? idx_out : static_cast<int32_t *>(ws);
    void *pws = idx_out ? ws : static_cast<void *>(static_cast<char *>(ws) + mask_bytes);
    hipStream_t st = (hipStream_t)stream;
    if (hipError_t e = dsa::launch_predict(*sh, Qt, Kt, idx, pws, st)) return from_hip(e);
    return from_hip(dsa::launch_attention(dsa::kFused, *sh, Q, K, V, idx, nullptr, nullptr, O, st));
}

size_t dsa_noalloc_max_mask_bytes(void) { return kStaticScratchBytes; }

dsa_status dsa_attention_fwd_noalloc(const dsa_shape *sh, const void *Q, const void *K, const void *V,
                                     const int8_t *Qt, const int8_t *Kt, float *O, void *stream)
{
    if (!sh || !Q || !K || !V || !Qt || !Kt || !O) return DSA_ERR_NULL;
    if (dsa_status s = check_predict(sh)) return s;
    if (dsa_status s = check_attention(sh)) return s;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(Qt) || !aligned16(Kt) || !aligned16(O))
        return DSA_ERR_ALIGN;
    const size_t mask_bytes = round_up_256(idx_bytes(*sh));
    const size_t need = mask_bytes + round_up_256(dsa::predict_workspace_bytes(*sh));
    if (need > kStaticScratchBytes) return DSA_ERR_WORKSPACE;
    void *base = nullptr;
    if (static_scratch(&base) != hipSuccess) return DSA_ERR_HIP;
    int32_t *idx = static_cast<int32_t *>(base);
    void *pws = static_cast<char *>(base) + mask_bytes;
    hipStream_t st = (hipStream_t)stream;
    if (hipError_t e = dsa::launch_predict(*sh, Qt, Kt, idx, pws, st)) return from_hip(e);
    return from_hip(dsa::launch_attention(dsa::kFused, *sh, Q, K, V, idx, nullptr, nullptr, O, st));
}

dsa_status dsa_approx_rowmax(const dsa_shape *sh, const int8_t *Qt, const int8_t *Kt, int32_t *rowmax,
                             void *stream)
{
    if (!sh || !Qt || !Kt || !rowmax) return DSA_ERR_NULL;
    if (sh->B < 1 || sh->H < 1 || sh->L < 1) return DSA_ERR_SHAPE;
    if ((int64_t)sh->B * sh->H * sh->L > (int64_t)1 << 31) return DSA_ERR_UNSUPPORTED;
    if (sh->k < 16 || sh->k > 128 || sh->k % 16) return DSA_ERR_UNSUPPORTED;
    if (!aligned16(Qt) || !aligned16(Kt) || !aligned16(rowmax)) return DSA_ERR_ALIGN;
    return from_hip(dsa::launch_rowmax(*sh, Qt, Kt, rowmax, (hipStream_t)stream));
}

size_t dsa_project_workspace_bytes(const dsa_shape *sh)
{
    if (check_predict(sh) != DSA_OK || check_attention(sh) != DSA_OK) return 0;
    return round_up_256(dsa::project_workspace_bytes(*sh));
}

dsa_status dsa_project_quantize_bits(const dsa_shape *sh, int32_t bits, const void *X, const float *R, void *Xt,
                                     float *amax_out, void *ws, size_t ws_bytes, void *stream)
{
    if (!sh || !X || !R || !Xt || !ws) return DSA_ERR_NULL;
    if (bits != 8 && bits != 4 && bits != 2) return DSA_ERR_UNSUPPORTED;
    if (dsa_status s = check_predict(sh)) return s;
    if (dsa_status s = check_attention(sh)) return s;
    if (!aligned16(X) || !aligned16(R) || !aligned16(Xt) || !aligned16(ws) ||
        (reinterpret_cast<uintptr_t>(amax_out) & 3u))
        return DSA_ERR_ALIGN;
    if (ws_bytes < round_up_256(dsa::project_workspace_bytes(*sh))) return DSA_ERR_WORKSPACE;
    return from_hip(dsa::launch_project_quantize(*sh, bits, X, R, nullptr, Xt, amax_out, ws, (hipStream_t)stream));
}

dsa_status dsa_project_quantize_ternary(const dsa_shape *sh, int32_t bits, const void *X, const int8_t *P3, void *Xt,
                                        float *amax_out, void *ws, size_t ws_bytes, void *stream)
{
    if (!sh || !X || !P3 || !Xt || !ws) return DSA_ERR_NULL;
    if (bits != 8 && bits != 4 && bits != 2) return DSA_ERR_UNSUPPORTED;
    if (dsa_status s = check_predict(sh)) return s;
    if (dsa_status s = check_attention(sh)) return s;
    if (!aligned16(X) || !aligned16(P3) || !aligned16(Xt) || !aligned16(ws) ||
        (reinterpret_cast<uintptr_t>(amax_out) & 3u))
        return DSA_ERR_ALIGN;
    if (ws_bytes < round_up_256(dsa::project_workspace_bytes(*sh))) return DSA_ERR_WORKSPACE;
    return from_hip(dsa::launch_project_quantize(*sh, bits, X, nullptr, P3, Xt, amax_out, ws, (hipStream_t)stream));
}

dsa_status dsa_project_quantize(const dsa_shape *sh, const void *X, const float *R, int8_t *Xt, float *amax_out,
                                void *ws, size_t ws_bytes, void *stream)
{
    return dsa_project_quantize_bits(sh, 8, X, R, Xt, amax_out, ws, ws_bytes, stream);
}

size_t dsa_predict_workspace_bytes_bits(const dsa_shape *sh, int32_t bits)
{
    if (check_predict(sh) != DSA_OK || (bits != 8 && bits != 4 && bits != 2)) return 0;
    const size_t codes = bits == 8 ? 0 : round_up_256((size_t)sh->B * sh->H * sh->L * sh->k);
    return 2 * codes + round_up_256(dsa::predict_workspace_bytes(*sh));
}

dsa_status dsa_predict_mask_bits(const dsa_shape *sh, int32_t bits, const void *Qt, const void *Kt, int32_t *idx,
                                 void *ws, size_t ws_bytes, void *stream)
{
    if (!sh || !Qt || !Kt || !idx) return DSA_ERR_NULL;
    if (bits != 8 && bits != 4 && bits != 2) return DSA_ERR_UNSUPPORTED;
    if (bits == 8)
        return dsa_predict_mask(sh, static_cast<const int8_t *>(Qt), static_cast<const int8_t *>(Kt), idx, ws, ws_bytes,
                                stream);
    if (dsa_status s = check_predict(sh)) return s;
    if (!aligned16(Qt) || !aligned16(Kt) || !aligned16(idx) || !aligned16(ws)) return DSA_ERR_ALIGN;
    const size_t need = dsa_predict_workspace_bytes_bits(sh, bits);
    if (!ws || ws_bytes < need) return DSA_ERR_WORKSPACE;
    const size_t n_codes = (size_t)sh->B * sh->H * sh->L * sh->k;
    const size_t codes = round_up_256(n_codes);
    int8_t *q8 = static_cast<int8_t *>(ws), *k8 = q8 + codes;
    void *pws = k8 + codes;
    hipStream_t st = (hipStream_t)stream;
    if (hipError_t e = dsa::launch_unpack_codes(bits, Qt, q8, n_codes, st)) return from_hip(e);
    if (hipError_t e = dsa::launch_unpack_codes(bits, Kt, k8, n_codes, st)) return from_hip(e);
    return from_hip(dsa::launch_predict(*sh, q8, k8, idx, pws, st));
}

size_t dsa_workspace_bytes_bits(const dsa_shape *sh, int32_t bits)
{
    if (check_predict(sh) != DSA_OK || (bits != 8 && bits != 4 && bits != 2)) return 0;
    return round_up_256(idx_bytes(*sh)) + dsa_predict_workspace_bytes_bits(sh, bits);
}

dsa_status dsa_attention_fwd_bits(const dsa_shape *sh, int32_t bits, const void *Q, const void *K, const void *V,
                                  const void *Qt, const void *Kt, float *O, int32_t *idx_out, void *ws,
                                  size_t ws_bytes, void *stream)
{
    if (!sh || !Q || !K || !V || !Qt || !Kt || !O) return DSA_ERR_NULL;
    if (bits != 8 && bits != 4 && bits != 2) return DSA_ERR_UNSUPPORTED;
    if (dsa_status s = check_predict(sh)) return s;
    if (dsa_status s = check_attention(sh)) return s;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(idx_out) || !aligned16(ws))
        return DSA_ERR_ALIGN;
    const size_t mask_bytes = round_up_256(idx_bytes(*sh));
    const size_t need = (idx_out ? 0 : mask_bytes) + dsa_predict_workspace_bytes_bits(sh, bits);
    if (need && (!ws || ws_bytes < need)) return DSA_ERR_WORKSPACE;
    int32_t *idx = idx_out ? idx_out : static_cast<int32_t *>(ws);
    void *pws = idx_out ? ws : static_cast<void *>(static_cast<char *>(ws) + mask_bytes);
    if (dsa_status s = dsa_predict_mask_bits(sh, bits, Qt, Kt, idx, pws, ws_bytes - (idx_out ? 0 : mask_bytes), stream))
        return s;
    return from_hip(dsa::launch_attention(dsa::kFused, *sh, Q, K, V, idx, nullptr, nullptr, O, (hipStream_t)stream));
}

size_t dsa_threshold_workspace_bytes(const dsa_shape *sh)
{
    if (check_predict(sh) != DSA_OK || !dsa::threshold_supported(*sh)) return 0;
    return round_up_256(dsa::threshold_workspace_bytes(*sh));
}

dsa_status dsa_predict_mask_threshold(const dsa_shape *sh, const int8_t *Qt, const int8_t *Kt, int32_t theta,
                                      int32_t *row_ptr, int32_t *col, int64_t col_capacity, void *ws,
                                      size_t ws_bytes, void *stream)
{
    if (!sh || !Qt || !Kt || !row_ptr || !col || !ws) return DSA_ERR_NULL;
    if (dsa_status s = check_predict(sh)) return s;
    if (!dsa::threshold_supported(*sh)) return DSA_ERR_UNSUPPORTED;
    // row_ptr is 32-bit: the largest possible mask (every key of every unit) has to fit
    if ((int64_t)sh->B * sh->H * sh->L * sh->L > INT32_MAX) return DSA_ERR_UNSUPPORTED;
    if (col_capacity < 0 || col_capacity > INT32_MAX) return DSA_ERR_SHAPE;
    if (!aligned16(Qt) || !aligned16(Kt) || !aligned16(row_ptr) || !aligned16(col) || !aligned16(ws))
        return DSA_ERR_ALIGN;
    if (ws_bytes < dsa_threshold_workspace_bytes(sh)) return DSA_ERR_WORKSPACE;
    return from_hip(dsa::launch_predict_threshold(*sh, Qt, Kt, theta, row_ptr, col, col_capacity, ws,
                                                  (hipStream_t)stream));
}

dsa_status dsa_masked_attention_csr(const dsa_shape *sh, const void *Q, const void *K, const void *V,
                                    const int32_t *row_ptr, const int32_t *col, float *O, void *stream)
{
    if (!sh || !Q || !K || !V || !row_ptr || !col || !O) return DSA_ERR_NULL;
    if (dsa_status s = check_attention(sh)) return s;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(row_ptr) || !aligned16(col) || !aligned16(O))
        return DSA_ERR_ALIGN;
    return from_hip(dsa::launch_attention_csr(*sh, Q, K, V, row_ptr, col, O, (hipStream_t)stream));
}

dsa_status dsa_gather_roof(const dsa_shape *sh, const void *K, const void *V, const int32_t *idx, uint32_t *sink,
                           void *stream)
{
    if (!sh || !K || !V || !idx || !sink) return DSA_ERR_NULL;
    if (dsa_status s = check_attention(sh)) return s;
    if (!aligned16(K) || !aligned16(V) || !aligned16(idx) || !aligned16(sink)) return DSA_ERR_ALIGN;
    return from_hip(dsa::launch_gather_probe(*sh, K, V, idx, sink, (hipStream_t)stream));
}

dsa_status dsa_mfma_i8_sustained(int32_t blocks, int32_t iters, int32_t *sink, void *stream)
{
    if (!sink) return DSA_ERR_NULL;
    if (blocks < 1 || blocks > (1 << 20) || iters < 1) return DSA_ERR_SHAPE;
    if (!aligned16(sink)) return DSA_ERR_ALIGN;
    return from_hip(dsa::launch_mfma_i8_stream(blocks, iters, sink, (hipStream_t)stream));
}

const char *dsa_status_string(dsa_status s)
{
    switch (s) {
    case DSA_OK: return "ok";
    case DSA_ERR_NULL: return "null pointer";
    case DSA_ERR_SHAPE: return "dimension out of range";
    case DSA_ERR_UNSUPPORTED: return "unsupported configuration";
    case DSA_ERR_ALIGN: return "pointer not 16-byte aligned";
    case DSA_ERR_WORKSPACE: return "workspace missing or too small";
    case DSA_ERR_HIP: return "HIP launch failed";
    }
    return "unknown status";
}

const char *dsa_version(void) { return "0.1"; }

}  // extern "C"
