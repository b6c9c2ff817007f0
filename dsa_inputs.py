"""Seeded synthetic inputs for the Dynamic Sparse Attention (DSA) forward path.

This module only *produces data*: Q, K, V tensors of shape [B, H, L, d] and the
int8 reduced-dimension projections Q~, K~ of shape [B, H, L, k] that the DSA
prediction path (paper section 3.1, "Design of Prediction Path") consumes.  It
holds none of the attention path's arithmetic (no scores, no top-k, no softmax)
and is shared by the CPU oracle's tests and the HIP library's tests, which
otherwise share no code.

The paper's own workloads (Long-Range Arena text / retrieval / image, section 4.1
and appendix A) are not available offline, so these tensors stand in for them:

* shapes follow the paper's profiling shape h=8, l=4096, d=64 (section 5.1,
  "Sparse Softmax Computation") and its DSA-90/95/99 keep ratios (section 4.2);
* values are "low-rank signal + noise": X = U W + E with U ~ N(0,1) [L, r],
  W ~ N(0, var=1/r) [r, d], E ~ N(0, sigma=0.1) [L, d], drawn independently for
  each of Q, K, V and each (b, h), so the exact score matrix has a few dominant
  directions, like the focused attention maps in the paper's figure 1;
* optional "global keys": n_global key positions per (b, h), sampled without
  replacement, whose K rows are multiplied by 4 -- the input-dependent global
  tokens the paper observes (section 1, section 5.1) and the source of the
  column locality its figure 11 exploits.  V is untouched.
* bf16 configs round Q, K, V to bfloat16 (round-to-nearest-even) once; the
  values returned are those rounded values held in float32, plus their raw
  16-bit patterns for upload.
* the projection R ~ N(0, var=1/k) [d, k] is one matrix shared by Q and K and by
  all (b, h) (the analogue of the shared random projection P of equation 5;
  same variance 1/k as sqrt(3/k){-1,0,1} with the usual 1/6, 2/3, 1/6 weights).
  Q~ = quant(Q R), K~ = quant(K R) with symmetric per-tensor int8 quantisation:
  s = max|x| / 127, q = clip(rint(x / s), -127, 127), computed in float64
  (rint = round half to even); all zeros if max|x| = 0.  The scale s never
  reaches the attention path: multiplying every approximate score by one
  positive constant cannot change a top-k.

Random numbers come from numpy's Philox generator with a fixed draw order:
R first, then for n in range(B*H): Uq, Wq, Eq, Uk, Wk, Ek, Uv, Wv, Ev, global
positions.
"""
from __future__ import annotations

from dataclasses import dataclass, field
import numpy as np


@dataclass(frozen=True)
class DsaConfig:
    """One DSA workload.  `keep` is the count the workload description prints
    for `ratio`; the libraries' own keep-from-ratio rules are tested against it."""
    name: str
    B: int
    H: int
    L: int
    d: int
    dtype: str          # "f32" or "bf16": storage type of Q, K, V
    rank: int           # r of the low-rank signal
    k: int              # projection dim of the prediction path
    vec: int            # mask granularity in query rows: 1 (fine-grained) or 8 (vector-wise)
    ratio: float        # keep ratio
    keep: int           # kept keys per row / group
    n_global: int = 0   # high-norm key positions per (b, h)
    seed: int = 0

    @property
    def N(self) -> int:
        return self.B * self.H

    @property
    def units(self) -> int:
        """Selection units (rows or 8-row groups) over the whole tensor."""
        return self.N * (self.L // self.vec)

    @property
    def scale(self) -> np.float32:
        return np.float32(1.0 / np.sqrt(np.float64(self.d)))


CONFIGS = {
    # Tiny fine-grained case the oracle finishes instantly.
    "C1": DsaConfig("C1", B=1, H=2, L=256, d=64, dtype="f32", rank=8, k=16, vec=1,
                    ratio=0.10, keep=26, seed=1101),
    # BERT-base-shaped layer.
    "C2": DsaConfig("C2", B=8, H=12, L=512, d=64, dtype="f32", rank=16, k=32, vec=1,
                    ratio=0.10, keep=51, seed=1102),
    # Vector-wise (8 query rows x 1 key column).
    "C3": DsaConfig("C3", B=4, H=16, L=2048, d=64, dtype="bf16", rank=32, k=32, vec=8,
                    ratio=0.05, keep=102, seed=1103),
    # Long sequence, fine-grained and vector-wise on the same tensors.
    "C4f": DsaConfig("C4f", B=2, H=8, L=4096, d=64, dtype="bf16", rank=32, k=32, vec=1,
                     ratio=0.05, keep=205, n_global=16, seed=1104),
    "C4v": DsaConfig("C4v", B=2, H=8, L=4096, d=64, dtype="bf16", rank=32, k=32, vec=8,
                     ratio=0.05, keep=205, n_global=16, seed=1104),
    # Stress.
    "C5": DsaConfig("C5", B=1, H=16, L=8192, d=128, dtype="bf16", rank=64, k=64, vec=8,
                    ratio=0.01, keep=82, n_global=32, seed=1105),
}


def custom_config(name="custom", *, B=1, H=1, L=64, d=64, dtype="f32", rank=4, k=16, vec=1,
                  keep=8, n_global=0, seed=7) -> DsaConfig:
    """A config of arbitrary shape for edge-case tests."""
    return DsaConfig(name, B=B, H=H, L=L, d=d, dtype=dtype, rank=rank, k=k, vec=vec,
                     ratio=keep / L, keep=keep, n_global=n_global, seed=seed)


def round_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even.  Finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> the same values as float32 (exact)."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize_int8(x: np.ndarray) -> np.ndarray:
    """Symmetric per-tensor int8 quantisation in float64 (see module docstring)."""
    x = np.asarray(x, dtype=np.float64)
    amax = float(np.max(np.abs(x))) if x.size else 0.0
    if amax == 0.0:
        return np.zeros(x.shape, dtype=np.int8)
    s = amax / 127.0
    return np.clip(np.rint(x / s), -127, 127).astype(np.int8)


@dataclass
class DsaInputs:
    cfg: DsaConfig
    Q: np.ndarray            # float32 [B,H,L,d]; bf16 configs: bf16-representable values
    K: np.ndarray
    V: np.ndarray
    Qt: np.ndarray           # int8 [B,H,L,k]
    Kt: np.ndarray
    R: np.ndarray            # float64 [d,k]
    global_pos: np.ndarray   # int64 [B*H, n_global]
    _bits: dict = field(default_factory=dict)

    def storage(self, which: str) -> np.ndarray:
        """The tensor as it is stored for the device: float32 array for "f32" configs,
        uint16 bfloat16 bit patterns for "bf16" configs."""
        x = getattr(self, which)
        if self.cfg.dtype == "f32":
            return x
        if which not in self._bits:
            self._bits[which] = round_to_bf16_bits(x)  # exact: x is already bf16-representable
        return self._bits[which]


def make_inputs(cfg: DsaConfig) -> DsaInputs:
    rng = np.random.Generator(np.random.Philox(cfg.seed))
    B, H, L, d, r, k = cfg.B, cfg.H, cfg.L, cfg.d, cfg.rank, cfg.k
    N = B * H
    R = rng.standard_normal((d, k)) * np.sqrt(1.0 / k)
    Q = np.empty((N, L, d), dtype=np.float32)
    K = np.empty((N, L, d), dtype=np.float32)
    V = np.empty((N, L, d), dtype=np.float32)
    gpos = np.zeros((N, cfg.n_global), dtype=np.int64)

    def low_rank_plus_noise():
        U = rng.standard_normal((L, r))
        W = rng.standard_normal((r, d)) * np.sqrt(1.0 / r)
        E = rng.standard_normal((L, d)) * 0.1
        return U @ W + E

    for n in range(N):
        q = low_rank_plus_noise()
        kk = low_rank_plus_noise()
        v = low_rank_plus_noise()
        if cfg.n_global:
            pos = rng.choice(L, size=cfg.n_global, replace=False)
            gpos[n] = np.sort(pos)
            kk[pos] *= 4.0
        Q[n], K[n], V[n] = q, kk, v

    if cfg.dtype == "bf16":
        Q = bf16_bits_to_f32(round_to_bf16_bits(Q))
        K = bf16_bits_to_f32(round_to_bf16_bits(K))
        V = bf16_bits_to_f32(round_to_bf16_bits(V))
    elif cfg.dtype != "f32":
        raise ValueError(f"unknown dtype {cfg.dtype!r}")

    Qt = quantize_int8(Q.astype(np.float64) @ R)
    Kt = quantize_int8(K.astype(np.float64) @ R)
    shp = (B, H, L)
    return DsaInputs(cfg, Q.reshape(shp + (d,)), K.reshape(shp + (d,)), V.reshape(shp + (d,)),
                     Qt.reshape(shp + (k,)), Kt.reshape(shp + (k,)), R, gpos)


def random_int8_case(seed: int, B: int, H: int, L: int, k: int, *, lo=-127, hi=127):
    """Uniform random int8 Q~, K~ in [lo, hi] -- a narrow range gives heavy score ties."""
    rng = np.random.Generator(np.random.Philox(seed))
    Qt = rng.integers(lo, hi + 1, size=(B, H, L, k), dtype=np.int64).astype(np.int8)
    Kt = rng.integers(lo, hi + 1, size=(B, H, L, k), dtype=np.int64).astype(np.int8)
    return Qt, Kt
