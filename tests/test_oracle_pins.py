"""Pins for the CPU oracle: each test checks oracle/dip_oracle.py against something
that is not the oracle -- a closed form, an identity the paper states, a textbook
routine, an independent library computation, or brute force on tiny inputs.
CPU only.
"""
import itertools
import json
import os
from collections import OrderedDict

import numpy as np
import pytest
import torch

from oracle import dip_oracle as O
from workloads import (f32_to_bf16_bits, k_from_ratio, layer_weights, pack_int4_g128,
                       studentt_tokens)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# --------------------------------------------------------------------------
# independent helpers (written without looking at the oracle's code paths)
# --------------------------------------------------------------------------
def greedy_topk(vals, k):
    """Definition by repeated extraction: k times take the largest remaining key,
    the lowest index among equals."""
    left = list(range(len(vals)))
    out = []
    for _ in range(k):
        best = left[0]
        for i in left[1:]:
            if vals[i] > vals[best]:
                best = i
        out.append(best)
        left.remove(best)
    return sorted(out)


def torch_dense_mlp(w_ug_fm, w_d_fm, x):
    """Eq. 1-2 with library routines only: W^d (W^u x * silu(W^g x)), fp64."""
    f = w_ug_fm.shape[1] // 2
    Wu = torch.from_numpy(w_ug_fm[:, :f].astype(np.float64)).T   # [f][d], paper orientation
    Wg = torch.from_numpy(w_ug_fm[:, f:].astype(np.float64)).T
    Wd = torch.from_numpy(w_d_fm.astype(np.float64)).T           # [d][f]
    xt = torch.from_numpy(x.astype(np.float64))
    glu = (Wu @ xt) * torch.nn.functional.silu(Wg @ xt)
    return glu.numpy(), (Wd @ glu).numpy()


def bf16_bits_to_f64_via_torch(bits):
    t = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16)
    return t.to(torch.float64).numpy()


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


# --------------------------------------------------------------------------
# golden: Eq. 10 worked by hand
# --------------------------------------------------------------------------
def test_eq10_hand_worked_cases():
    with open(os.path.join(GOLDEN, "eq10_hand_worked.json")) as fh:
        cases = json.load(fh)["cases"]
    for c in cases:
        x = np.array(c["x"], dtype=np.float32)
        cb = np.array(c["c"], dtype=bool)
        s = O.score(x, cb, c["gamma"])
        assert s.dtype == np.float32
        assert s.tolist() == c["s"], c["_why"]
        m, idx = O.topk(s, c["k"])
        assert m.astype(int).tolist() == c["mask"], c["_why"]


# --------------------------------------------------------------------------
# top-K
# --------------------------------------------------------------------------
def test_topk_exhaustive_small_alphabet():
    alphabet = [0.0, 0.5, 1.0, 2.0]
    for n in range(1, 7):
        for vals in itertools.product(alphabet, repeat=n):
            s = np.array(vals, dtype=np.float32)
            for k in range(1, n + 1):
                m, idx = O.topk(s, k)
                assert idx.tolist() == greedy_topk(vals, k)
                assert int(m.sum()) == k


@pytest.mark.parametrize("seed", range(4))
def test_topk_properties_with_heavy_ties(seed):
    rng = np.random.default_rng(seed)
    n = 1000 + 37 * seed
    s = rng.integers(0, 12, size=n).astype(np.float32) / 4    # many duplicates
    for k in (1, 7, n // 3, n - 1, n):
        m, idx = O.topk(s, k)
        assert int(m.sum()) == k and idx.size == k
        assert np.all(np.diff(idx) > 0)
        if k < n:
            T = s[m].min()
            assert T >= s[~m].max()
            # among keys equal to the threshold the selected ones are the lowest indices
            eq = np.flatnonzero(s == T)
            sel_eq = eq[m[eq]]
            assert np.array_equal(sel_eq, eq[:sel_eq.size])
            assert np.all(m[s > T])


def test_topk_negative_zero_and_zero_keys():
    s = np.abs(np.array([-0.0, 0.0, -0.0, 1.0], dtype=np.float32))
    m, idx = O.topk(s, 3)
    assert idx.tolist() == [0, 1, 3]          # zeros are ordinary keys, lowest index first


def test_topk_rejects_bad_k():
    s = np.ones(4, dtype=np.float32)
    for k in (0, 5, -1):
        with pytest.raises(ValueError):
            O.topk(s, k)


# --------------------------------------------------------------------------
# Eq. 10 identities
# --------------------------------------------------------------------------
def test_score_plain_dip_key_is_magnitude():
    x = studentt_tokens(1, 257, 3)[0]
    assert np.array_equal(O.score(x, None, 0.2), np.abs(x))


@pytest.mark.parametrize("seed", range(3))
def test_score_max_is_one_or_gamma(seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(300).astype(np.float32)
    c = rng.random(300) < 0.5
    j = int(np.argmax(np.abs(x)))
    g = np.float32(0.2)
    c[j] = True
    assert O.score(x, c, g).max() == np.float32(1.0)
    c[j] = False
    c[:] = False                                  # nothing cached: max is exactly gamma*M/M
    s = O.score(x, c, g)
    M = np.abs(x).max()
    assert s.max() == np.float32(np.float32(M * g) / M)


def test_score_scale_invariance_power_of_two():
    """The denominator makes the score insensitive to the activations' dynamic range
    (Sec. 5.2); for a power-of-two factor the invariance is bit-exact."""
    rng = np.random.default_rng(5)
    x = rng.standard_normal(512).astype(np.float32)
    c = rng.random(512) < 0.4
    s = O.score(x, c, 0.2)
    for a in (2.0, 0.25, 1024.0):
        assert np.array_equal(O.score((x * np.float32(a)).astype(np.float32), c, 0.2), s)


def test_gamma_one_is_plain_dip():
    """gamma = 1 is the DIP instance (Sec. 6.4): no re-weighting.  With ||x||_inf a power
    of two the division is exact, so the masks are identical bit for bit."""
    rng = np.random.default_rng(7)
    x = rng.standard_normal(400).astype(np.float32)
    x[17] = 4.0                                   # M = 4
    x = np.clip(x, -4, 4)
    c = rng.random(400) < 0.5
    for k in (1, 50, 200, 399):
        m_ca, _ = O.topk(O.score(x, c, 1.0), k)
        m_dip, _ = O.topk(O.score(x, None, 1.0), k)
        assert np.array_equal(m_ca, m_dip)


@pytest.mark.parametrize("fill", [False, True])
def test_uniform_cache_gives_dip_mask(fill):
    """c == 0 or c == 1 re-weights every feature alike, so the ranking is DIP's.
    M is a power of two and gamma = 0.25 so no new ties can appear through rounding."""
    rng = np.random.default_rng(11)
    x = rng.standard_normal(333).astype(np.float32)
    x = np.clip(x, -2, 2)
    x[5] = -2.0
    c = np.full(333, fill)
    for k in (1, 100, 332):
        m_ca, _ = O.topk(O.score(x, c, 0.25), k)
        m_dip, _ = O.topk(np.abs(x), k)
        assert np.array_equal(m_ca, m_dip)


def test_cached_dominates_equal_magnitude_uncached():
    """Sec. 5.2: the penalty biases selection towards cached columns.  Pairs of equal
    magnitude, one cached (at the HIGHER index so the tie rule cannot help it)."""
    rng = np.random.default_rng(13)
    mags = (rng.random(50).astype(np.float32) + np.float32(0.01))
    x = np.empty(100, dtype=np.float32)
    x[0::2] = mags
    x[1::2] = -mags
    c = np.zeros(100, dtype=bool)
    c[1::2] = True
    s = O.score(x, c, 0.2)
    assert np.all(s[1::2] > s[0::2])
    m, _ = O.topk(s, 50)
    # gamma = 0.2 and magnitudes within a factor 100 > 5 do not guarantee all cached win;
    # what is guaranteed is pairwise dominance:
    assert not np.any(m[0::2] & ~m[1::2])


def test_score_zero_vector():
    s = O.score(np.zeros(9, dtype=np.float32), np.ones(9, dtype=bool), 0.2)
    assert np.array_equal(s, np.zeros(9, dtype=np.float32))


def test_score_op_order_is_mul_then_div():
    """fl(fl(a*gamma)/M) differs from fl(a*fl(gamma/M)) and from fp64 evaluation for some
    inputs; the oracle must be the former.  Checked against Python floats rounded by hand."""
    import struct

    def f32(v):
        return struct.unpack("f", struct.pack("f", v))[0]

    rng = np.random.default_rng(17)
    x = (rng.random(2000).astype(np.float32) + np.float32(0.5))
    c = np.zeros(2000, dtype=bool)
    g = f32(0.2)
    s = O.score(x, c, g)
    M = float(np.abs(x).max())
    ref = [f32(f32(float(a) * g) / M) for a in x]        # double mul/div of fp32 values then
    # one rounding each: a*g is exact in double (24+24 bits), so f32() of it is the correctly
    # rounded fp32 product; p/M in double then rounded to fp32 is the correctly rounded
    # quotient except for double-rounding cases, which need > 53-24 = 29 equal bits: none here.
    assert s.tolist() == ref
    other = [f32(float(a) * f32(g / M)) for a in x]
    assert other != ref                                    # the test can tell the orders apart


# --------------------------------------------------------------------------
# storage formats and gathered GEMV
# --------------------------------------------------------------------------
def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(19)
    a = (rng.standard_normal(100000) * 0.02).astype(np.float32)
    ours = f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)


def test_widen_bf16_matches_torch_decode():
    rng = np.random.default_rng(23)
    bits = f32_to_bf16_bits((rng.standard_normal((16, 64)) * 0.02).astype(np.float32))
    got = O.widen_rows(bits, np.arange(16))
    assert np.array_equal(got, bf16_bits_to_f64_via_torch(bits))


def test_widen_int4_by_hand():
    rng = np.random.default_rng(29)
    w = (rng.standard_normal((3, 256)) * 0.02).astype(np.float32)
    packed, scales = pack_int4_g128(w)
    got = O.widen_rows((packed, scales), np.array([2, 0]))
    for out_r, r in enumerate((2, 0)):
        for j in (0, 1, 2, 127, 128, 255):
            byte = int(packed[r, j // 2])
            nib = (byte >> 4) if (j & 1) else (byte & 0xF)
            q = nib - 16 if nib >= 8 else nib
            want = float(scales[r, j // 128]) * q
            assert got[out_r, j] == want
    # quantisation sanity: error at most half a step
    full = O.widen_rows((packed, scales), np.arange(3))
    step = np.repeat(scales.astype(np.float64), 128, axis=1)
    assert np.all(np.abs(full - w) <= 0.5 * step + 1e-12)


@pytest.mark.parametrize("fmt", ["f32", "bf16", "int4"])
def test_gathered_gemv_unit_vector_returns_stored_row(fmt):
    w = layer_weights(128, 128, seed=1, layer=0, dtype=fmt)["ug"]
    n_in = O.n_rows(w)
    for i in (0, 17, n_in - 1):
        x = np.zeros(n_in, dtype=np.float32)
        x[i] = 1.0
        y = O.gathered_gemv(w, x, np.array([i]))
        assert y.shape == (O.n_cols(w),)
        assert np.array_equal(y, O.widen_rows(w, np.array([i]))[0])
        # a transposed layout would return a strided slice instead:
        if fmt == "f32":
            assert np.array_equal(y, w[i].astype(np.float64))


def test_gathered_gemv_equals_dense_product_on_masked_input():
    """W~ = W (.) m (Alg. 1 step 4): multiplying the column-masked matrix by x equals the
    dense product with the masked-out entries of x set to zero (library matmul)."""
    rng = np.random.default_rng(31)
    w = (rng.standard_normal((200, 96)) * 0.02).astype(np.float32)
    x = rng.standard_normal(200).astype(np.float32)
    m, idx = O.topk(np.abs(x), 70)
    y = O.gathered_gemv(w, x, idx)
    xm = np.where(m, x, 0).astype(np.float64)
    ref = (torch.from_numpy(w.astype(np.float64)).T @ torch.from_numpy(xm)).numpy()
    assert rel_l2(y, ref) < 1e-14
    # linearity in x
    y2 = O.gathered_gemv(w, (2 * x).astype(np.float32), idx)
    assert rel_l2(y2, 2 * y) < 1e-15


# --------------------------------------------------------------------------
# dense anchor: keep ratio 1.0 is the dense MLP (Eq. 1-3)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("fmt", ["f32", "bf16"])
def test_keep_ratio_one_equals_dense_mlp(fmt):
    d, f = 96, 224
    w = layer_weights(d, f, seed=2, layer=0, dtype=fmt)
    if fmt == "bf16":
        ug = bf16_bits_to_f64_via_torch(w["ug"])
        dn = bf16_bits_to_f64_via_torch(w["d"])
    else:
        ug, dn = w["ug"], w["d"]
    x = studentt_tokens(1, d, 4)[0]
    out = O.mlp_forward(w["ug"], w["d"], x, d, f)
    glu_ref, y_ref = torch_dense_mlp(np.asarray(ug), np.asarray(dn), x)
    assert rel_l2(out["h"], glu_ref) < 2e-7        # one fp32 rounding of h
    assert rel_l2(out["y"], y_ref) < 3e-7
    assert out["mask_in"].all() and out["mask_mid"].all()


def test_swapping_up_and_gate_is_detected():
    """The anchor must be able to fail: SiLU sits on the gate half only (Eq. 2)."""
    d, f = 64, 128
    w = layer_weights(d, f, seed=3, layer=0, dtype="f32")
    x = studentt_tokens(1, d, 5)[0]
    swapped = np.concatenate([w["ug"][:, f:], w["ug"][:, :f]], axis=1)
    good = O.mlp_forward(w["ug"], w["d"], x, d, f)["y"]
    bad = O.mlp_forward(swapped, w["d"], x, d, f)["y"]
    _, y_ref = torch_dense_mlp(w["ug"], w["d"], x)
    assert rel_l2(good, y_ref) < 3e-7
    assert rel_l2(bad, y_ref) > 1e-2


def test_sparse_forward_matches_masked_dense_chain():
    """Sec. 4: DIP equals the dense formulas applied to column-masked matrices."""
    d, f = 128, 320
    w = layer_weights(d, f, seed=4, layer=0, dtype="f32")
    x = studentt_tokens(1, d, 6)[0]
    k_in, k_mid = 40, 100
    out = O.mlp_forward(w["ug"], w["d"], x, k_in, k_mid)
    assert int(out["mask_in"].sum()) == k_in and int(out["mask_mid"].sum()) == k_mid
    m1 = np.asarray(greedy_topk(np.abs(x).tolist(), k_in))
    ug_masked = np.zeros_like(w["ug"])
    ug_masked[m1] = w["ug"][m1]
    glu_ref, _ = torch_dense_mlp(ug_masked, w["d"], x)
    assert rel_l2(out["h"], glu_ref) < 2e-7
    m2 = np.asarray(greedy_topk(np.abs(out["h"]).tolist(), k_mid))
    assert np.array_equal(np.flatnonzero(out["mask_mid"]), m2)
    d_masked = np.zeros_like(w["d"])
    d_masked[m2] = w["d"][m2]
    y_ref = (torch.from_numpy(d_masked.astype(np.float64)).T
             @ torch.from_numpy(out["h"].astype(np.float64))).numpy()
    assert rel_l2(out["y"], y_ref) < 3e-7


# --------------------------------------------------------------------------
# counting closed forms (Sec. 3.2, Sec. 4)
# --------------------------------------------------------------------------
def test_gathered_element_counts():
    for (d, f) in ((512, 1536), (3072, 8192), (5120, 17920)):
        for r in (0.25, 0.5, 0.75, 1.0):
            k_in, k_mid = k_from_ratio(r, d), k_from_ratio(r, f)
            got = O.gathered_weight_elements(k_in, k_mid, d, f)
            assert got == int(r * 3 * d * f)          # one ratio at both points touches r of the MLP
        # GLU pruning (only the down matrix is sparse) can remove at most 1/3 of the MLP,
        # gate/up pruning (one matrix dense) at most 2/3:
        dense = 3 * d * f
        glu_only = O.gathered_weight_elements(d, 1, d, f)
        assert 1 - glu_only / dense <= 1 / 3 + 1e-9
        assert (dense - d * f) / dense == pytest.approx(2 / 3)
    c3 = (k_from_ratio(0.3, 4096), k_from_ratio(0.3, 14336))
    assert c3 == (1229, 4301)


# --------------------------------------------------------------------------
# cache_update: LRU / LFU (Sec. 5.1)
# --------------------------------------------------------------------------
def classic_lru_faults(trace, frames):
    od = OrderedDict()
    faults = 0
    for p in trace:
        if p in od:
            od.move_to_end(p)
        else:
            faults += 1
            if len(od) >= frames:
                od.popitem(last=False)
            od[p] = True
    return faults, set(od)


def test_lru_textbook_reference_string():
    """The classic 20-reference page string with 3 frames gives 12 faults under LRU
    (operating-systems textbooks' standard example); single-item masks reduce the
    set-valued update to classical LRU."""
    trace = [7, 0, 1, 2, 0, 3, 0, 4, 2, 3, 0, 3, 2, 1, 2, 0, 1, 7, 0, 1]
    st = O.CacheState(n=8, capacity=3)
    faults = 0
    for p in trace:
        m = np.zeros(8, dtype=bool)
        m[p] = True
        ev = O.cache_update(st, m)
        faults += ev["misses"]
    assert faults == 12
    assert classic_lru_faults(trace, 3)[0] == 12
    assert set(np.flatnonzero(st.resident)) == classic_lru_faults(trace, 3)[1]


@pytest.mark.parametrize("seed", range(5))
def test_lru_single_item_traces_match_ordereddict(seed):
    rng = np.random.default_rng(seed)
    n, C = 12, int(rng.integers(1, 8))
    trace = rng.integers(0, n, size=200).tolist()
    st = O.CacheState(n=n, capacity=C)
    od = OrderedDict()
    for p in trace:
        m = np.zeros(n, dtype=bool)
        m[p] = True
        O.cache_update(st, m)
        if p in od:
            od.move_to_end(p)
        else:
            if len(od) >= C:
                od.popitem(last=False)
            od[p] = True
        assert set(np.flatnonzero(st.resident)) == set(od)


def naive_list_lru_step(lst, cap, mset):
    """Recency list, least recent first; items used in one step sit in index order.
    A resident used by this token is never the victim; if no victim exists the miss bypasses."""
    used = []
    for i in sorted(mset):
        if i in lst:
            used.append(i)
    for i in sorted(mset):
        if i in lst:
            continue
        if len(lst) < cap:
            lst.append(i)
            used.append(i)
            continue
        victim = next((j for j in lst if j not in mset), None)
        if victim is None:
            continue
        lst.remove(victim)
        lst.append(i)
        used.append(i)
    for i in sorted(used):
        lst.remove(i)
    lst.extend(sorted(used))
    return lst


def test_lru_set_valued_exhaustive_tiny():
    n = 4
    all_masks = [ms for r in range(1, n + 1) for ms in itertools.combinations(range(n), r)]
    for cap in range(0, n + 1):
        for seq in itertools.product(all_masks, repeat=3):
            st = O.CacheState(n=n, capacity=cap)
            lst = []
            for ms in seq:
                m = np.zeros(n, dtype=bool)
                m[list(ms)] = True
                before = st.resident.copy()
                O.cache_update(st, m)
                lst = naive_list_lru_step(lst, cap, set(ms))
                assert set(np.flatnonzero(st.resident)) == set(lst), (cap, seq)
                assert int(st.resident.sum()) <= cap
                assert np.all(st.resident[m & before])           # a hit is never evicted
                if len(ms) <= cap:
                    assert np.all(st.resident[m])                # everything selected fits
                elif before.sum() == cap:
                    assert int(st.resident.sum()) == cap
                    assert not np.any(st.resident & ~(before | m))


def test_lru_inclusion_property_hit_rate_monotone_in_capacity():
    rng = np.random.default_rng(41)
    n, k, T = 64, 8, 120
    x = np.cumsum(rng.standard_normal((T, n)), axis=0)           # slowly varying magnitudes
    masks = [O.topk(np.abs(x[t]).astype(np.float32), k)[0] for t in range(T)]
    prev_sets, prev_hits = None, -1
    for C in (8, 12, 16, 24, 32, 64):
        st = O.CacheState(n=n, capacity=C)
        sets = []
        for m in masks:
            O.cache_update(st, m)
            sets.append(set(np.flatnonzero(st.resident)))
        if prev_sets is not None:
            assert all(a <= b for a, b in zip(prev_sets, sets))  # smaller cache is a subset
            assert st.hits >= prev_hits
        prev_sets, prev_hits = sets, st.hits


def test_lru_bypass_when_active_set_exceeds_cache():
    """Sec. 6.4: below some sparsity the active set no longer fits; the cache then holds
    part of the current neurons and the rest is streamed without being cached."""
    st = O.CacheState(n=10, capacity=3)
    m = np.zeros(10, dtype=bool)
    m[[1, 2, 5, 7, 9]] = True
    ev = O.cache_update(st, m)
    assert ev == {"hits": 0, "misses": 5, "inserted": 3, "evicted": 0, "bypassed": 2}
    assert np.flatnonzero(st.resident).tolist() == [1, 2, 5]
    m2 = np.zeros(10, dtype=bool)
    m2[[2, 3, 4, 5, 6]] = True
    ev = O.cache_update(st, m2)
    # 2 and 5 hit and are protected; only column 1 can be evicted -> one insert, two bypass
    assert ev == {"hits": 2, "misses": 3, "inserted": 1, "evicted": 1, "bypassed": 2}
    assert np.flatnonzero(st.resident).tolist() == [2, 3, 5]


def test_lfu_single_item_trace_matches_counter_dict():
    rng = np.random.default_rng(43)
    n, C = 10, 4
    trace = rng.integers(0, n, size=300).tolist()
    st = O.CacheState(n=n, capacity=C, policy="lfu")
    counts = {i: 0 for i in range(n)}
    res = set()
    for p in trace:
        m = np.zeros(n, dtype=bool)
        m[p] = True
        O.cache_update(st, m)
        counts[p] += 1
        if p not in res:
            if len(res) >= C:
                victim = min(res, key=lambda j: (counts[j], j))
                res.remove(victim)
            res.add(p)
        assert set(np.flatnonzero(st.resident)) == res


def naive_counter_lfu_step(res, counts, cap, mset):
    """LFU by the book, one column after the other: every use is counted; a missed column takes
    a free place, else the place of the resident with the smallest (count, index) among those
    this token does not use; if there is none it is not cached."""
    for i in sorted(mset):
        counts[i] += 1
    for i in sorted(mset):
        if i in res:
            continue
        if len(res) < cap:
            res.add(i)
            continue
        cands = [j for j in res if j not in mset]
        if not cands:
            continue
        res.remove(min(cands, key=lambda j: (counts[j], j)))
        res.add(i)
    return res


@pytest.mark.parametrize("n,steps", [(4, 3), (3, 5)])
def test_lfu_set_valued_exhaustive_tiny(n, steps):
    """Every sequence of masks over n columns, every capacity: several misses and several
    evictions in one step, with equal use counts among the candidates (index decides)."""
    all_masks = [ms for r in range(1, n + 1) for ms in itertools.combinations(range(n), r)]
    for cap in range(0, n + 1):
        for seq in itertools.product(all_masks, repeat=steps):
            st = O.CacheState(n=n, capacity=cap, policy="lfu")
            res, counts = set(), [0] * n
            for ms in seq:
                m = np.zeros(n, dtype=bool)
                m[list(ms)] = True
                before = st.resident.copy()
                O.cache_update(st, m)
                res = naive_counter_lfu_step(res, counts, cap, set(ms))
                assert set(np.flatnonzero(st.resident)) == res, (cap, seq)
                assert st.stamp.tolist() == counts, (cap, seq)
                assert int(st.resident.sum()) <= cap
                assert np.all(st.resident[m & before])           # a hit is never evicted


# --------------------------------------------------------------------------
# DIP-CA composition (Alg. 1 inside the MLP)
# --------------------------------------------------------------------------
def test_cold_cache_first_token_equals_dip_and_uses_old_state():
    d, f = 128, 256
    w = layer_weights(d, f, seed=6, layer=0, dtype="f32")
    x = studentt_tokens(2, d, 8)
    x[:, 3] = 8.0
    x = np.clip(x, -8, 8)                     # M = 8: exact division
    ci = O.CacheState(n=d, capacity=64)
    cm = O.CacheState(n=f, capacity=128)
    ca = O.mlp_forward(w["ug"], w["d"], x[0], 32, 64, ci, cm, gamma=0.25)
    dip = O.mlp_forward(w["ug"], w["d"], x[0], 32, 64)
    assert np.array_equal(ca["mask_in"], dip["mask_in"])
    # the state after the update holds exactly this token's selection (it fits)
    assert np.array_equal(ci.resident, ca["mask_in"])
    assert ci.step == 2 and cm.step == 2
    # second token is scored with the state left by the first
    snap = ci.resident.copy()
    ca2 = O.mlp_forward(w["ug"], w["d"], x[1], 32, 64, ci, cm, gamma=0.25)
    assert np.array_equal(ca2["s_in"], O.score(x[1], snap, 0.25))


def test_cache_aware_masking_raises_hit_rate_on_correlated_stream():
    """Sec. 5.2's claim, statistically: biasing towards resident columns raises the hit rate."""
    from workloads import ar1_laplace_stream
    n, k, C, T = 512, 128, 256, 200
    xs = ar1_laplace_stream(T, n, seed=3)
    rates = {}
    for gamma in (1.0, 0.2):
        st = O.CacheState(n=n, capacity=C)
        for t in range(T):
            m, _ = O.topk(O.score(xs[t], st.resident, gamma), k)
            O.cache_update(st, m)
        rates[gamma] = st.hits / st.lookups
    assert rates[0.2] > rates[1.0]


def test_batched_rows_are_independent_and_cache_sees_union():
    d, f = 64, 128
    w = layer_weights(d, f, seed=7, layer=0, dtype="f32")
    X = studentt_tokens(3, d, 9)
    ci = O.CacheState(n=d, capacity=48)
    cm = O.CacheState(n=f, capacity=96)
    ci0, cm0 = ci.copy(), cm.copy()
    out = O.mlp_forward_batched(w["ug"], w["d"], X, 16, 32, ci, cm, gamma=0.2)
    for b in range(3):
        one = O.mlp_forward(w["ug"], w["d"], X[b], 16, 32, ci0.copy(), cm0.copy(), gamma=0.2)
        assert np.array_equal(out["mask_in"][b], one["mask_in"])
        assert np.array_equal(out["y"][b], one["y"])
    ref = ci0.copy()
    O.cache_update(ref, out["mask_in"].any(axis=0))
    assert np.array_equal(ref.resident, ci.resident)
