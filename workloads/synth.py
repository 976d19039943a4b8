"""Synthetic workloads shaped like the paper's models (Sec. 6.1 names Phi-3-Mini,
Phi-3-Medium, Llama-3-8B, Mistral-7B; only their MLP shapes are used here).

The paper evaluates on public text corpora with trained weights; neither is
available, so every input is drawn from ``numpy.random.default_rng(seed)``:

* weights ~ N(0, 0.02^2) generated in fp32, then stored as fp32, as bf16
  (round-to-nearest-even, done once here) or as int4 with one fp16 scale per
  group of 128 consecutive elements of a feature-major row;
* activations: iid N(0,1); iid Student-t(df=3) (heavy tails: a few channels
  dominate, as the paper's Sec. 5.2 / Fig. 7 describe for real activations);
  or a per-feature AR(1) process x_t = rho x_{t-1} + sqrt(1-rho^2) eps_t with
  unit-variance Laplace noise (temporally correlated, so a residency cache has
  something to exploit).

Layout convention (feature-major): a weight matrix that the paper writes as
W in R^{n_out x n_in} is stored as an array of shape [n_in][n_out]; stored row
i is the paper's column W[:, i], i.e. everything input feature i multiplies.
The up and gate matrices of one MLP are bundled per feature: stored row i is
[W^u[:, i] ; W^g[:, i]] (2*d_ff elements).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np


# --------------------------------------------------------------------------
# storage-format encoders (no method arithmetic)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (round-to-nearest-even) and return the 16-bit patterns.

    Inputs must be finite.  bf16 is the upper half of the fp32 pattern, so
    RNE is: add 0x7FFF plus the lsb of the kept half, then truncate.
    """
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def pack_int4_g128(w_fm: np.ndarray, group: int = 128) -> Tuple[np.ndarray, np.ndarray]:
    """Encode a feature-major fp32 matrix [n_in][n_out] as signed 4-bit codes.

    Per stored row, every ``group`` consecutive elements share one fp16 scale
    ``scale = fp16_rne(max|w| / 7)`` (a zero group gets scale 0 and codes 0);
    codes are ``q = clip(rint(w / scale), -8, 7)`` stored two per byte, the
    even element in the low nibble, as two's-complement nibbles.

    Returns (packed uint8 [n_in][n_out//2], scales float16 [n_in][n_out//group]).
    """
    w = np.ascontiguousarray(w_fm, dtype=np.float32)
    n_in, n_out = w.shape
    if n_out % group or group % 2:
        raise ValueError("n_out must be a multiple of the group size")
    g = w.reshape(n_in, n_out // group, group)
    amax = np.abs(g).max(axis=2)
    scales = (amax / np.float32(7.0)).astype(np.float16)
    s32 = scales.astype(np.float32)
    safe = np.where(s32 > 0, s32, np.float32(1.0))
    q = np.rint(g / safe[:, :, None])
    q = np.where(s32[:, :, None] > 0, q, 0.0)
    q = np.clip(q, -8, 7).astype(np.int8).reshape(n_in, n_out)
    nib = (q & 0xF).astype(np.uint8)
    packed = (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)
    return np.ascontiguousarray(packed), np.ascontiguousarray(scales)


def k_from_ratio(ratio: float, n: int) -> int:
    """Keep ratio -> integer k: nearest integer to ratio*n, clamped to [1, n]."""
    k = int(np.floor(float(ratio) * n + 0.5))
    return max(1, min(n, k))


# --------------------------------------------------------------------------
# weights
# --------------------------------------------------------------------------
def layer_weights(d_model: int, d_ff: int, seed: int, layer: int = 0,
                  dtype: str = "f32", std: float = 0.02):
    """Weights of one SwiGLU MLP, feature-major, for ``seed*1000 + layer``.

    Returns a dict with
      'ug'  : bundled up/gate, shape [d_model][2*d_ff]  (up first, then gate)
      'd'   : down,            shape [d_ff][d_model]
    as fp32 arrays (dtype 'f32'), uint16 bf16 bit patterns ('bf16'), or
    (packed uint8, fp16 scales) tuples ('int4').
    """
    rng = np.random.default_rng(seed * 1000 + layer)
    ug = rng.standard_normal((d_model, 2 * d_ff), dtype=np.float32)
    ug *= np.float32(std)
    dn = rng.standard_normal((d_ff, d_model), dtype=np.float32)
    dn *= np.float32(std)
    if dtype == "f32":
        return {"ug": ug, "d": dn}
    if dtype == "bf16":
        return {"ug": f32_to_bf16_bits(ug), "d": f32_to_bf16_bits(dn)}
    if dtype == "int4":
        # groups must not straddle the up/gate boundary: d_ff % 128 == 0 in all configs
        return {"ug": pack_int4_g128(ug), "d": pack_int4_g128(dn)}
    raise ValueError(dtype)


def layer_weights_split(d_model: int, d_ff: int, seed: int, layer: int = 0,
                        dtype: str = "f32", std: float = 0.02):
    """The same three matrices as ``layer_weights``, stored apart for the schemes that
    multiply one of W^u / W^g densely and gather whole rows of the other.

    Returns a dict with
      'u', 'g'           : feature-major, shape [d_model][d_ff]   (stored row i = column i)
      'u_rows', 'g_rows' : neuron-major,  shape [d_ff][d_model]   (stored row j = row j)
      'd'                : feature-major, shape [d_ff][d_model]
    in the storage format of ``dtype`` (a 4-bit matrix is quantised per stored row, so its
    two layouts hold slightly different values).
    """
    rng = np.random.default_rng(seed * 1000 + layer)
    ug = rng.standard_normal((d_model, 2 * d_ff), dtype=np.float32)
    ug *= np.float32(std)
    dn = rng.standard_normal((d_ff, d_model), dtype=np.float32)
    dn *= np.float32(std)
    mats = {"u": np.ascontiguousarray(ug[:, :d_ff]), "g": np.ascontiguousarray(ug[:, d_ff:]),
            "u_rows": np.ascontiguousarray(ug[:, :d_ff].T), "g_rows": np.ascontiguousarray(ug[:, d_ff:].T),
            "d": dn}
    if dtype == "f32":
        return mats
    if dtype == "bf16":
        return {k: f32_to_bf16_bits(v) for k, v in mats.items()}
    if dtype == "int4":
        return {k: pack_int4_g128(v) for k, v in mats.items()}
    raise ValueError(dtype)


# --------------------------------------------------------------------------
# activations
# --------------------------------------------------------------------------
def gaussian_tokens(n_tokens: int, n: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.standard_normal((n_tokens, n), dtype=np.float32)


def studentt_tokens(n_tokens: int, n: int, seed: int, df: float = 3.0) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.standard_t(df, size=(n_tokens, n)).astype(np.float32)


def ar1_laplace_stream(n_tokens: int, n: int, seed: int, rho: float = 0.8) -> np.ndarray:
    """x_0 = eps_0, x_t = rho*x_{t-1} + sqrt(1-rho^2)*eps_t, eps ~ Laplace(0, 1/sqrt 2)."""
    rng = np.random.default_rng(seed)
    eps = rng.laplace(0.0, 1.0 / np.sqrt(2.0), size=(n_tokens, n))
    out = np.empty((n_tokens, n), dtype=np.float64)
    out[0] = eps[0]
    c = np.sqrt(1.0 - rho * rho)
    for t in range(1, n_tokens):
        out[t] = rho * out[t - 1] + c * eps[t]
    return out.astype(np.float32)


def lru_warm_bits(n: int, capacity: int, seed: int) -> np.ndarray:
    """A random residency pattern with exactly ``capacity`` resident columns (bool[n])."""
    rng = np.random.default_rng(seed)
    bits = np.zeros(n, dtype=bool)
    bits[rng.choice(n, size=capacity, replace=False)] = True
    return bits


# --------------------------------------------------------------------------
# the five configurations
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    d_model: int
    d_ff: int
    n_layers: int
    dtype: str                 # 'f32' | 'bf16' | 'int4'
    n_tokens: int
    inputs: str                # 'gaussian' | 'studentt3' | 'ar1_laplace'
    keep_ratios: Tuple[float, ...]
    cache_fracs: Tuple[Optional[float], ...] = (None,)
    gamma: float = 0.2
    batch: Tuple[int, ...] = (1,)
    seed: int = 0
    note: str = ""

    def k_in(self, r: float) -> int:
        return k_from_ratio(r, self.d_model)

    def k_mid(self, r: float) -> int:
        return k_from_ratio(r, self.d_ff)

    def gathered_bytes(self, r: float) -> int:
        """Weight bytes one layer-token must read at batch 1 (int4: codes plus fp16 group scales)."""
        elems = 2 * self.k_in(r) * self.d_ff + self.k_mid(r) * self.d_model
        if self.dtype == "int4":
            return elems // 2 + (elems // 128) * 2
        return elems * {"f32": 4, "bf16": 2}[self.dtype]

    def tokens(self, layer: int = 0, n_tokens: Optional[int] = None, n: Optional[int] = None):
        """Input stream for one layer (layers get independent streams, not chained)."""
        nt = self.n_tokens if n_tokens is None else n_tokens
        n = self.d_model if n is None else n
        s = self.seed * 1000 + 500 + layer
        if self.inputs == "gaussian":
            return gaussian_tokens(nt, n, s)
        if self.inputs == "studentt3":
            return studentt_tokens(nt, n, s)
        if self.inputs == "ar1_laplace":
            return ar1_laplace_stream(nt, n, s)
        raise ValueError(self.inputs)


CONFIGS = {
    1: WorkloadConfig("tiny-f32", 512, 1536, 1, "f32", 16, "gaussian", (0.5,)),
    2: WorkloadConfig("phi3-mini-mlp-bf16", 3072, 8192, 1, "bf16", 256, "studentt3",
                      (0.25, 0.5, 0.75),
                      note="one layer shape; the benchmark rotates over distinct weight "
                           "copies so the 256 MB last-level cache cannot hold them"),
    3: WorkloadConfig("llama3-8b-mlp-stack-bf16", 4096, 14336, 32, "bf16", 512, "ar1_laplace",
                      (0.3,), cache_fracs=(0.5,)),
    4: WorkloadConfig("phi3-medium-mlp-stack-bf16", 5120, 17920, 40, "bf16", 1024, "ar1_laplace",
                      (0.2, 0.3, 0.4, 0.5), cache_fracs=(0.25, 0.5, 0.75)),
    5: WorkloadConfig("phi3-medium-mlp-stack-int4", 5120, 17920, 40, "int4", 1024, "ar1_laplace",
                      (0.3,), cache_fracs=(0.5,), batch=(1, 2, 4, 8)),
}
