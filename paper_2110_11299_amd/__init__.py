"""MI355X-native Dynamic Sparse Attention forward path (arXiv 2110.11299).

`binding` is the Python face of the C-ABI library built from `csrc/`; `build` compiles it.
"""
from . import binding  # noqa: F401
from .binding import (DSA_BF16, DSA_F32, DsaError, DsaShape, dsa_approx_rowmax, dsa_attention_fwd, dsa_attention_fwd_bits,  # noqa: F401
                      dsa_attention_fwd_noalloc, dsa_masked_attention_csr, dsa_predict_mask_threshold,
                      dsa_masked_attention, dsa_mfma_i8_sustained, dsa_predict_mask, dsa_predict_mask_bits,
                      dsa_project_quantize, dsa_project_quantize_bits, dsa_project_quantize_ternary, dsa_sddmm, dsa_sparse_softmax, dsa_spmm,
                      keep_from_ratio, make_shape, workspace_bytes)
