"""GPU tests of the two-tier residency path (columns cached in HBM slots, the full matrix in
pinned host memory): the result must be the bits of the single-tier forward on the same inputs
and cache states (same kernels, same summation order) and within tolerance of the oracle; the
slot map is not unique, so it is checked for validity: resident <=> has a slot, slots distinct
and below the capacity, and every slot holds a bit-exact copy of its column.
"""
import numpy as np
import pytest
import torch

from oracle import dip_oracle as O
from workloads import ar1_laplace_stream, layer_weights, lru_warm_bits
from gpu_util import (assert_product_close, bits_from_bool, bool_from_bits, dev_f32, dev_u32, glu_scale, host_u32,
                      make_weight, rel_l2, workspace)

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-3}


@pytest.fixture(scope="module")
def D():
    import paper_2412_01380_amd as D
    return D


def pinned(w):
    t = torch.from_numpy(w.view(np.int16) if w.dtype == np.uint16 else w)
    p = torch.empty(t.shape, dtype=t.dtype, pin_memory=True)
    p.copy_(t)
    return p


def check_slot_map(tw, cache_bits, n):
    slot_of = tw.slot_of.cpu().numpy()
    resident = bool_from_bits(host_u32(cache_bits), n)
    assert np.array_equal(slot_of >= 0, resident)
    used = slot_of[resident]
    assert used.size == np.unique(used).size and (used < tw.capacity).all()
    slots = tw.slots.cpu()
    host = tw.host
    cols = np.flatnonzero(resident)
    got = slots[torch.from_numpy(used.astype(np.int64))]
    want = host[torch.from_numpy(cols)]
    assert torch.equal(got.view(torch.uint8), want.contiguous().view(torch.uint8))


@pytest.mark.parametrize("fmt,d,f,r,frac,warm", [
    ("f32", 512, 1536, 0.5, 0.6, False), ("f32", 512, 1536, 0.5, 0.25, False),
    ("bf16", 512, 1536, 0.3, 0.5, True), ("bf16", 3072, 8192, 0.5, 0.5, False),
    ("bf16", 5120, 17920, 0.3, 0.25, False), ("f32", 200, 456, 0.4, 1.0, False),
    ("f32", 200, 456, 0.4, 0.0, False),
])
def test_tiered_forward_equals_single_tier(D, fmt, d, f, r, frac, warm):
    w = layer_weights(d, f, seed=51, layer=0, dtype=fmt)
    k_in, k_mid = max(1, int(r * d)), max(1, int(r * f))
    C_in, C_mid = int(frac * d), int(frac * f)
    mlp = D.Mlp(make_weight(D, w["ug"]), make_weight(D, w["d"]))
    tw_ug, tw_d = D.TieredWeight(pinned(w["ug"]), C_in), D.TieredWeight(pinned(w["d"]), C_mid)
    tmlp = D.TieredMlp(tw_ug, tw_d)
    caches = [[D.Cache(d, C_in), D.Cache(f, C_mid)] for _ in range(2)]   # [single tier, tiered]
    oc = [O.CacheState(n=d, capacity=C_in), O.CacheState(n=f, capacity=C_mid)]
    init = [None, None]
    if warm:
        wb = [lru_warm_bits(d, C_in, 1), lru_warm_bits(f, C_mid, 2)]
        init = [dev_u32(bits_from_bool(b)) for b in wb]
        oc = [O.CacheState(n=d, capacity=C_in, resident=wb[0]), O.CacheState(n=f, capacity=C_mid, resident=wb[1])]
    for pair in caches:
        for c, ib in zip(pair, init):
            D.dip_cache_init(c, ib)
    for tw, c in ((tw_ug, caches[1][0]), (tw_d, caches[1][1])):
        D.dip_tier_init(tw, c, workspace(D.dip_tier_init_workspace_bytes(tw)))
    torch.cuda.synchronize()
    check_slot_map(tw_ug, caches[1][0].bits, d)
    check_slot_map(tw_d, caches[1][1].bits, f)

    xs = ar1_laplace_stream(6, d, seed=52)
    ws1 = workspace(D.dip_swiglu_mlp_forward_workspace_bytes(mlp, k_in, k_mid))
    ws2 = workspace(D.dip_tiered_mlp_forward_workspace_bytes(tmlp, k_in, k_mid))
    y1 = torch.empty(d, dtype=torch.float32, device="cuda")
    y2 = torch.empty(d, dtype=torch.float32, device="cuda")
    dbg = D.Debug(d, f, k_in, k_mid)
    for t in range(xs.shape[0]):
        x = dev_f32(xs[t])
        D.dip_swiglu_mlp_forward(mlp, x, k_in, k_mid, caches[0][0], caches[0][1], 0.2, y1, None, ws1)
        D.dip_tiered_mlp_forward(tmlp, x, k_in, k_mid, caches[1][0], caches[1][1], 0.2, y2, dbg, ws2)
        torch.cuda.synchronize()
        assert torch.equal(y1, y2), t
        for a, b in zip(caches[0], caches[1]):
            assert torch.equal(a.bits, b.bits) and torch.equal(a.stamp, b.stamp) and torch.equal(a.meta, b.meta)
        check_slot_map(tw_ug, caches[1][0].bits, d)
        check_slot_map(tw_d, caches[1][1].bits, f)
        # against the oracle: stage replay on the GPU's own h~ (mask 2 depends on its bits)
        m1, idx1 = O.topk(O.score(xs[t], oc[0].resident, 0.2), k_in)
        assert np.array_equal(bool_from_bits(host_u32(dbg.mask_in), d), m1)
        O.cache_update(oc[0], m1)
        hg = dbg.h.cpu().numpy()
        pre = O.gathered_gemv(w["ug"], xs[t], idx1)
        assert_product_close(hg, O.glu_from_preacts(pre), fmt, k_in, "h", scale=glu_scale(pre), factor=3.0)
        m2, idx2 = O.topk(O.score(hg, oc[1].resident, 0.2), k_mid)
        assert np.array_equal(bool_from_bits(host_u32(dbg.mask_mid), f), m2)
        O.cache_update(oc[1], m2)
        assert_product_close(y2.cpu().numpy(), O.gathered_gemv(w["d"], hg, idx2), fmt, k_mid, "y")
        assert np.array_equal(bool_from_bits(host_u32(caches[1][1].bits), f), oc[1].resident)


def test_tiered_forward_rejects_mismatched_cache(D):
    d, f = 128, 256
    w = layer_weights(d, f, seed=53, layer=0, dtype="f32")
    tmlp = D.TieredMlp(D.TieredWeight(pinned(w["ug"]), 64), D.TieredWeight(pinned(w["d"]), 128))
    c_in, c_mid = D.Cache(d, 64), D.Cache(f, 100)       # c_mid capacity differs from its tier
    ws = workspace(D.dip_tiered_mlp_forward_workspace_bytes(tmlp, 32, 64))
    x, y = dev_f32(np.ones(d)), torch.empty(d, dtype=torch.float32, device="cuda")
    with pytest.raises(D.DipError):
        D.dip_tiered_mlp_forward(tmlp, x, 32, 64, c_in, c_mid, 0.2, y, None, ws)
