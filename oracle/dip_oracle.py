"""CPU oracle for Dynamic Input Pruning (DIP) and its cache-aware variant (DIP-CA).

TEST INFRASTRUCTURE ONLY.  This file is the slow, literal reference that the
HIP library is checked against.  It may be imported by tests/, by
__graft_entry__.smoke() and by bench.py's cpu_baseline leg, and by nothing
else; the product path never routes through it.  It shares no code with the
HIP path and imports nothing from the package that binds it.

DIP is an approximation defined by a procedure, so the oracle is that
procedure taken step by step in the paper's order:

  Sec. 3, Eq. 1-2   MLP(x) = W^d GLU(x),  GLU(x) = W^u x (.) sigma(W^g x),
                    sigma = SiLU
  Sec. 3, Eq. 3     the sparse MLP uses column-masked W~^u, W~^g, W~^d
  Sec. 4 (DIP)      mask 1 = topK(|x|) removes columns of W^u and W^g;
                    mask 2 = topK(|GLU~(x)|) removes columns of W^d
  Sec. 5.2, Eq. 10   s = |x| (c + gamma (1 - c)) / ||x||_inf
  Sec. 5.2, Alg. 1  s -> m = topK(s, k) -> c' = cache_update(c, m) -> W~ = W (.) m

Arithmetic.  Scores are fp32, in exactly this operation order, round to
nearest even, no fused operations, denormals kept:  a = |x_i| ;
p = a if c_i else fl32(a * gamma) ;  s_i = fl32(p / M),  M = max_i |x_i|.
Matrix-vector sums are fp64 over the selected features in ascending index
order (a library matmul serves as that step); h~ and y are rounded to fp32
once, at the end.  Weights arrive in their storage format (fp32, bf16 bit
patterns, or int4 codes + fp16 scales) and are widened exactly to fp64.

Readings where the paper is silent (each is listed in the design notes):
ties in top-K go to the lowest index; zero-valued features are ordinary keys;
||x||_inf = 0 gives all-zero scores; the residency used for scoring is the
state before this token's update; LRU is set-valued with the rules in
``lru_update``.

Parity pins (tests/test_oracle_*.py): dense anchor against an independent
dense MLP; top-K against exhaustive enumeration; score identities; gathered
GEMV against unit vectors and masked dense products; LRU/LFU against textbook
list-based caches on tiny inputs.  The density-allocation rule of App. B and
Belady's policy are not implemented here ("parity unpinned": figures only).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np

F32 = np.float32
F64 = np.float64


# ---------------------------------------------------------------------------
# storage formats -> exact fp64 values
# ---------------------------------------------------------------------------
def widen_rows(w, rows: np.ndarray) -> np.ndarray:
    """Return the selected feature-major rows of a stored matrix as fp64.

    ``w`` is an fp32 array, a uint16 array of bf16 bit patterns, or a tuple
    (packed uint8 [n_in][n_out/2], fp16 scales [n_in][n_out/128]) of signed
    4-bit codes with w = scale * q (low nibble = even element).
    """
    if isinstance(w, tuple):
        packed, scales = w
        p = packed[rows]
        lo = (p & 0xF).astype(np.int16)
        hi = (p >> 4).astype(np.int16)
        lo = np.where(lo >= 8, lo - 16, lo)
        hi = np.where(hi >= 8, hi - 16, hi)
        q = np.empty((p.shape[0], p.shape[1] * 2), dtype=F64)
        q[:, 0::2] = lo
        q[:, 1::2] = hi
        group = q.shape[1] // scales.shape[1]
        s = scales[rows].astype(F64)
        return q * np.repeat(s, group, axis=1)
    if w.dtype == np.uint16:
        bits = w[rows].astype(np.uint32) << np.uint32(16)
        return bits.view(np.float32).astype(F64)
    if w.dtype == np.float32:
        return w[rows].astype(F64)
    raise TypeError("unsupported weight storage")


def n_rows(w) -> int:
    return (w[0] if isinstance(w, tuple) else w).shape[0]


def n_cols(w) -> int:
    return w[0].shape[1] * 2 if isinstance(w, tuple) else w.shape[1]


# ---------------------------------------------------------------------------
# Sec. 5.2 Eq. 10 / Alg. 1 step 1: scores
# ---------------------------------------------------------------------------
def score(v: np.ndarray, cache_bits: Optional[np.ndarray], gamma: float) -> np.ndarray:
    """Selection key for every feature.

    cache_bits None  ->  plain DIP key |v| (Sec. 4).
    otherwise        ->  Eq. 10 with c = cache_bits (bool[n]), all in fp32.
    """
    v = np.asarray(v, dtype=F32)
    a = np.abs(v)
    if cache_bits is None:
        return a
    c = np.asarray(cache_bits, dtype=bool)
    M = a.max() if a.size else F32(0)
    if M == 0:
        return np.zeros_like(a)
    g = F32(gamma)
    pen = (a * g).astype(F32)            # fl32(|x| * gamma)
    p = np.where(c, a, pen).astype(F32)  # c + gamma (1 - c) is 1 or gamma
    with np.errstate(under="ignore"):
        return (p / F32(M)).astype(F32)


# ---------------------------------------------------------------------------
# Alg. 1 step 2: m = topK(s, k)
# ---------------------------------------------------------------------------
def topk(s: np.ndarray, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """Exactly k features with the largest keys; among equal keys the lowest index wins.

    Full stable sort by descending key.  Returns (mask bool[n], idx ascending int64[k]).
    """
    s = np.asarray(s, dtype=F32)
    n = s.shape[0]
    if not (1 <= k <= n):
        raise ValueError("k out of range")
    order = np.argsort(-s.astype(F64), kind="stable")
    chosen = np.sort(order[:k])
    mask = np.zeros(n, dtype=bool)
    mask[chosen] = True
    return mask, chosen.astype(np.int64)


# ---------------------------------------------------------------------------
# Alg. 1 step 3: c' = cache_update(c, m)
# ---------------------------------------------------------------------------
@dataclass
class CacheState:
    """Residency of one linear layer's columns (Sec. 5.1).

    resident[i]  column i is in the cache (the paper's c)
    stamp[i]     LRU: step of last use;  LFU: number of uses so far
    step         1-based counter of updates applied + 1
    """
    n: int
    capacity: int
    policy: str = "lru"                       # 'lru' | 'lfu'
    resident: np.ndarray = field(default=None)
    stamp: np.ndarray = field(default=None)
    step: int = 1
    hits: int = 0
    lookups: int = 0

    def __post_init__(self):
        if self.resident is None:
            self.resident = np.zeros(self.n, dtype=bool)
        else:
            self.resident = np.array(self.resident, dtype=bool)
        if self.stamp is None:
            self.stamp = np.zeros(self.n, dtype=np.int64)
        else:
            self.stamp = np.array(self.stamp, dtype=np.int64)
        if not (0 <= self.capacity <= self.n):
            raise ValueError("capacity out of range")
        if int(self.resident.sum()) > self.capacity:
            raise ValueError("more resident columns than capacity")

    def copy(self) -> "CacheState":
        return CacheState(self.n, self.capacity, self.policy, self.resident.copy(),
                          self.stamp.copy(), self.step, self.hits, self.lookups)


def cache_update(st: CacheState, mask: np.ndarray) -> dict:
    """Apply one token's mask to the cache (in place) and return the event counts.

    Sec. 5.1: LRU evicts the resident whose last use lies farthest back; LFU
    keeps a use counter and evicts the rarest.  The mask arrives as a set, so:

      hits    H  = m & c            -> their priority is refreshed
      misses  Mi = m & ~c, ascending index
      free       = capacity - |c|
      victims V  = c & ~m           (a column used by this token is never evicted)
      n_ins      = min(|Mi|, free + |V|)
      evict the (n_ins - free)+ members of V with the smallest (priority, index)
      insert the first n_ins members of Mi; the rest bypass the cache
      (Sec. 6.4: with too little room part of the active set goes straight
      to the processing unit).

    Priority: LRU -> stamp = step of last use.  LFU -> stamp = use count; it
    counts every selection of the column, resident or not, and is kept when
    the column is evicted ("for the current session").
    """
    m = np.asarray(mask, dtype=bool)
    c = st.resident
    hit = m & c
    miss = m & ~c
    n_hit = int(hit.sum())
    miss_idx = np.flatnonzero(miss)
    free = st.capacity - int(c.sum())
    victims = np.flatnonzero(c & ~m)
    n_ins = min(miss_idx.size, free + victims.size)
    n_evict = max(0, n_ins - free)

    if st.policy == "lru":
        st.stamp[hit] = st.step
    elif st.policy == "lfu":
        st.stamp[m] += 1
    else:
        raise ValueError(st.policy)

    if n_evict:
        # smallest (priority, index): stable sort on priority keeps index order
        order = np.argsort(st.stamp[victims], kind="stable")
        c[victims[order[:n_evict]]] = False
    ins = miss_idx[:n_ins]
    c[ins] = True
    if st.policy == "lru":
        st.stamp[ins] = st.step
    st.step += 1
    st.hits += n_hit
    st.lookups += int(m.sum())
    return {"hits": n_hit, "misses": int(miss_idx.size), "inserted": int(n_ins),
            "evicted": int(n_evict), "bypassed": int(miss_idx.size - n_ins)}


# ---------------------------------------------------------------------------
# Alg. 1 step 4: W~ = W (.) m, applied as a product
# ---------------------------------------------------------------------------
def gathered_gemv(w, x: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """y[j] = sum over selected i (ascending) of W[j, i] x_i, in fp64.

    ``w`` is feature-major (stored row i = the paper's column i).  Masking the
    columns of W and multiplying by x is the same sum (Alg. 1 step 4).
    """
    idx = np.asarray(idx, dtype=np.int64)
    xs = np.asarray(x, dtype=F32)[idx].astype(F64)
    rows = widen_rows(w, idx)              # [k][n_out]
    return xs @ rows                       # fp64


def silu(z: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        return z / (1.0 + np.exp(-z))


def glu_from_preacts(ug: np.ndarray) -> np.ndarray:
    """Eq. 2: up (.) SiLU(gate) for a bundled pre-activation vector [up ; gate]; rounds to fp32."""
    f = ug.shape[0] // 2
    return (ug[:f] * silu(ug[f:])).astype(F32)


# ---------------------------------------------------------------------------
# Sec. 4 + Alg. 1 composed over one MLP, one token
# ---------------------------------------------------------------------------
def mlp_forward(w_ug, w_d, x, k_in: int, k_mid: int,
                cache_in: Optional[CacheState] = None,
                cache_mid: Optional[CacheState] = None,
                gamma: float = 0.2) -> dict:
    """One token through one DIP / DIP-CA SwiGLU MLP.

    w_ug: bundled up/gate, feature-major [d][2f];  w_d: feature-major [f][d].
    Caches (if given) are scored with their state before this token and then
    updated in place.  Returns every intermediate for stage-wise comparison.
    """
    x = np.asarray(x, dtype=F32)
    s1 = score(x, None if cache_in is None else cache_in.resident, gamma)
    m1, idx1 = topk(s1, k_in)
    ev1 = cache_update(cache_in, m1) if cache_in is not None else None
    h = glu_from_preacts(gathered_gemv(w_ug, x, idx1))
    s2 = score(h, None if cache_mid is None else cache_mid.resident, gamma)
    m2, idx2 = topk(s2, k_mid)
    ev2 = cache_update(cache_mid, m2) if cache_mid is not None else None
    y = gathered_gemv(w_d, h, idx2).astype(F32)
    return {"s_in": s1, "mask_in": m1, "idx_in": idx1, "h": h, "s_mid": s2,
            "mask_mid": m2, "idx_mid": idx2, "y": y, "ev_in": ev1, "ev_mid": ev2}


def mlp_forward_batched(w_ug, w_d, X, k_in: int, k_mid: int,
                        cache_in: Optional[CacheState] = None,
                        cache_mid: Optional[CacheState] = None,
                        gamma: float = 0.2) -> dict:
    """B rows through one layer: B independent batch-1 results (the paper is batch 1).

    All rows are scored against the cache state before the step; the caches are
    then updated once with the union of the per-row masks.
    """
    X = np.asarray(X, dtype=F32)
    B = X.shape[0]
    c_in = None if cache_in is None else cache_in.resident.copy()
    c_mid = None if cache_mid is None else cache_mid.resident.copy()
    M1, H, M2, Y = [], [], [], []
    for b in range(B):
        m1, idx1 = topk(score(X[b], c_in, gamma), k_in)
        h = glu_from_preacts(gathered_gemv(w_ug, X[b], idx1))
        m2, idx2 = topk(score(h, c_mid, gamma), k_mid)
        y = gathered_gemv(w_d, h, idx2).astype(F32)
        M1.append(m1); H.append(h); M2.append(m2); Y.append(y)
    M1 = np.stack(M1); M2 = np.stack(M2)
    ev1 = cache_update(cache_in, M1.any(axis=0)) if cache_in is not None else None
    ev2 = cache_update(cache_mid, M2.any(axis=0)) if cache_mid is not None else None
    return {"mask_in": M1, "h": np.stack(H), "mask_mid": M2, "y": np.stack(Y),
            "ev_in": ev1, "ev_mid": ev2}


def gathered_weight_elements(k_in: int, k_mid: int, d_model: int, d_ff: int) -> int:
    """Weight elements one token must read: two matrices at point 1, one at point 2 (Sec. 4)."""
    return 2 * k_in * d_ff + k_mid * d_model


# ---------------------------------------------------------------------------
# Sec. 3.2: the sibling schemes that prune on (partial) GLU activations
# ---------------------------------------------------------------------------
GLU_PRUNING, GATE_PRUNING, UP_PRUNING = "glu", "gate", "up"


def gathered_rowdot(w_rows, x: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """(W x)_j for the selected output neurons j, in fp64.

    ``w_rows`` is neuron-major (stored row j = the paper's row j), so removing the
    rows of W that a mask drops leaves exactly these dot products.
    """
    idx = np.asarray(idx, dtype=np.int64)
    return widen_rows(w_rows, idx) @ np.asarray(x, dtype=F32).astype(F64)


def glu_pruning_forward(w_ug, w_d, x, k: int) -> dict:
    """GLU pruning (Sec. 3.2): W^u x and W^g x are dense; topK(|GLU(x)|) removes columns of W^d."""
    x = np.asarray(x, dtype=F32)
    d = n_rows(w_ug)
    h = glu_from_preacts(gathered_gemv(w_ug, x, np.arange(d)))
    m, idx = topk(np.abs(h), k)
    y = gathered_gemv(w_d, h, idx).astype(F32)
    return {"a": h, "mask": m, "idx": idx, "h_sel": h[idx], "y": y}


def partial_pruning_forward(scheme: str, w_dense, w_rows, w_d, x, k: int) -> dict:
    """Gate pruning and Up pruning (Sec. 3.2).

    gate:  a = sigma(W^g x) dense,  m = topK(|a|),  W^u loses the rows and W^d the columns
           outside m:  h_j = (W^u x)_j a_j  for j in m.
    up:    a = W^u x dense,         m = topK(|a|),  W^g and W^d are pruned:
           h_j = a_j sigma((W^g x)_j)  for j in m.
    ``w_dense`` is the densely multiplied matrix, feature-major [d][f]; ``w_rows`` the
    other one, neuron-major [f][d]; ``w_d`` feature-major [f][d].  The partial
    activation a is rounded to fp32 once; that array is both the selection key and
    the factor of h.  h is returned compact (one value per selected neuron, ascending).
    """
    x = np.asarray(x, dtype=F32)
    d = n_rows(w_dense)
    pre = gathered_gemv(w_dense, x, np.arange(d))            # fp64, all f neurons
    if scheme == GATE_PRUNING:
        a = silu(pre).astype(F32)
    elif scheme == UP_PRUNING:
        a = pre.astype(F32)
    else:
        raise ValueError(scheme)
    m, idx = topk(np.abs(a), k)
    other = gathered_rowdot(w_rows, x, idx)                  # fp64, k neurons
    if scheme == GATE_PRUNING:
        h_sel = (other * a[idx].astype(F64)).astype(F32)
    else:
        h_sel = (a[idx].astype(F64) * silu(other)).astype(F32)
    h = np.zeros(a.shape[0], dtype=F32)
    h[idx] = h_sel
    y = gathered_gemv(w_d, h, idx).astype(F32)
    return {"a": a, "mask": m, "idx": idx, "h_sel": h_sel, "y": y}


def sibling_weight_elements(scheme: str, k: int, d_model: int, d_ff: int) -> int:
    """Weight elements one token reads under a Sec. 3.2 scheme with k kept GLU units."""
    if scheme == GLU_PRUNING:
        return 2 * d_model * d_ff + k * d_model
    if scheme in (GATE_PRUNING, UP_PRUNING):
        return d_model * d_ff + 2 * k * d_model
    raise ValueError(scheme)
