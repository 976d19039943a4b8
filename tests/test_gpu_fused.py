"""The one-launch form of a pruning point (the gathered product runs scores and top-K at its
own head) against the oracle and against the two-launch form.

Stage replay against the oracle on inputs built to hit every branch of the head: ties that
are split at the threshold, all-zero vectors, gamma 0 and 1, denormal scores (where many
distinct |x| share one rounded score, so the tie set of the rounded scores is wider than the
tie set of the magnitudes), k = 1 and k = n, vector lengths off every tile boundary.  Masks,
index lists and score bit patterns must be identical; h~ and y within the float tolerance.

Against the two-launch form with both forced to one launch shape: every output bit-equal.
"""
import numpy as np
import pytest
import torch

from oracle import dip_oracle as O
from workloads import ar1_laplace_stream, layer_weights, studentt_tokens
from gpu_util import (assert_product_close, glu_scale, bits_from_bool, bool_from_bits, dev_f32, host_u32, make_weight, rel_l2, workspace)

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-3, "int4": 2e-3}


@pytest.fixture()
def D():
    import paper_2412_01380_amd as D
    D.dip_set_fusion(True)
    D.dip_tune_gemv()
    yield D
    D.dip_set_fusion(True)
    D.dip_tune_gemv()


def _layer(D, d, f, fmt, seed, k_in, k_mid, w=None):
    w = w if w is not None else layer_weights(d, f, seed=seed, layer=0, dtype=fmt)
    mlp = D.Mlp(make_weight(D, w["ug"]), make_weight(D, w["d"]))
    return {"ug": w["ug"], "d": w["d"], "mlp": mlp, "fmt": fmt,
            "ws": workspace(D.dip_swiglu_mlp_forward_workspace_bytes(mlp, k_in, k_mid)),
            "dbg": D.Debug(d, f, k_in, k_mid), "y": torch.empty(d, dtype=torch.float32, device="cuda")}


def _replay(D, L, x, k_in, k_mid, gamma=0.2, caches=None, ocaches=None):
    """One forward call, every stage against the oracle on identical inputs."""
    mlp, dbg, y = L["mlp"], L["dbg"], L["y"]
    d, f = mlp.d_model, mlp.d_ff
    cin, cmid = caches if caches else (None, None)
    ocin, ocmid = ocaches if ocaches else (None, None)
    D.dip_swiglu_mlp_forward(mlp, dev_f32(x), k_in, k_mid, cin, cmid, gamma, y, dbg, L["ws"])
    torch.cuda.synchronize()
    s1 = O.score(x, None if ocin is None else ocin.resident, gamma)
    assert np.array_equal(dbg.s_in.cpu().numpy().view(np.uint32), s1.view(np.uint32)), "scores 1"
    m1, idx1 = O.topk(s1, k_in)
    assert np.array_equal(host_u32(dbg.mask_in), bits_from_bool(m1)), "mask 1"
    assert np.array_equal(dbg.idx_in.cpu().numpy(), idx1), "index list 1"
    h_gpu = dbg.h.cpu().numpy()
    pre = O.gathered_gemv(L["ug"], x, idx1)
    assert_product_close(h_gpu, O.glu_from_preacts(pre), L["fmt"], k_in, "h", scale=glu_scale(pre), factor=3.0)
    s2 = O.score(h_gpu, None if ocmid is None else ocmid.resident, gamma)
    assert np.array_equal(dbg.s_mid.cpu().numpy().view(np.uint32), s2.view(np.uint32)), "scores 2"
    m2, idx2 = O.topk(s2, k_mid)
    assert np.array_equal(host_u32(dbg.mask_mid), bits_from_bool(m2)), "mask 2"
    assert np.array_equal(dbg.idx_mid.cpu().numpy(), idx2), "index list 2"
    y_ref = O.gathered_gemv(L["d"], h_gpu, idx2).astype(np.float32)
    assert_product_close(y.cpu().numpy(), y_ref, L["fmt"], k_mid, "y")
    if ocin is not None:
        O.cache_update(ocin, m1)
        assert np.array_equal(bool_from_bits(host_u32(cin.bits), d), ocin.resident)
        assert np.array_equal(host_u32(cin.stamp).astype(np.int64), ocin.stamp)
    if ocmid is not None:
        O.cache_update(ocmid, m2)
        assert np.array_equal(bool_from_bits(host_u32(cmid.bits), f), ocmid.resident)
        assert np.array_equal(host_u32(cmid.stamp).astype(np.int64), ocmid.stamp)


def _caches(D, d, f, c_in, c_mid, seed=None):
    cin, cmid = D.Cache(d, c_in), D.Cache(f, c_mid)
    ocin, ocmid = O.CacheState(n=d, capacity=c_in), O.CacheState(n=f, capacity=c_mid)
    init = [None, None]
    if seed is not None:
        rng = np.random.default_rng(seed)
        for i, (n, c, oc) in enumerate(((d, c_in, ocin), (f, c_mid, ocmid))):
            bits = np.zeros(n, dtype=bool)
            bits[rng.choice(n, size=c, replace=False)] = True
            oc.resident[:] = bits
            init[i] = torch.from_numpy(bits_from_bool(bits).view(np.int32)).cuda()
    D.dip_cache_init(cin, init[0])
    D.dip_cache_init(cmid, init[1])
    return (cin, cmid), (ocin, ocmid)


@pytest.mark.parametrize("d,f,fmt", [(512, 1536, "f32"), (1000, 2056, "f32"), (1032, 1160, "bf16"),
                                     (2048, 5120, "int4"), (3072, 8192, "bf16")])
def test_forward_uses_the_one_launch_form(D, d, f, fmt):
    k_in, k_mid = d // 3, f // 3
    L = _layer(D, d, f, fmt, 1, k_in, k_mid)
    assert D.dip_fused_launch_shape(L["mlp"].w_ug, k_in, bundled=True) is not None
    assert D.dip_fused_launch_shape(L["mlp"].w_d, k_mid, bundled=False) is not None


@pytest.mark.parametrize("d,f,fmt,r", [(512, 1536, "f32", 0.5), (1000, 2056, "f32", 0.3),
                                       (1032, 1160, "bf16", 0.7), (2048, 5120, "int4", 0.3),
                                       (3072, 8192, "bf16", 0.25),
                                       # the widest instantiations: 32 keys per lane at point 2, 8 at point 1
                                       (256, 32768, "f32", 0.3), (8192, 1024, "bf16", 0.2)])
def test_stage_replay_random_tokens_dip_and_dipca(D, d, f, fmt, r):
    k_in, k_mid = max(1, round(r * d)), max(1, round(r * f))
    L = _layer(D, d, f, fmt, 2, k_in, k_mid)
    assert D.dip_fused_launch_shape(L["mlp"].w_ug, k_in, bundled=True) is not None
    assert D.dip_fused_launch_shape(L["mlp"].w_d, k_mid, bundled=False) is not None
    xs = studentt_tokens(3, d, seed=d)
    for t in range(3):
        _replay(D, L, xs[t], k_in, k_mid)
    caches, ocaches = _caches(D, d, f, d // 2, f // 2, seed=5)
    xs = ar1_laplace_stream(6, d, seed=f)
    for t in range(6):
        _replay(D, L, xs[t], k_in, k_mid, 0.2, caches, ocaches)


def _adversarial_inputs(d, rng):
    """Vectors that stress the selection: split ties, zeros, huge dynamic range, denormals."""
    out = {}
    x = rng.integers(-3, 4, size=d).astype(np.float32)            # seven distinct magnitudes
    out["heavy ties"] = x
    out["all zero"] = np.zeros(d, dtype=np.float32)
    x = np.zeros(d, dtype=np.float32)
    x[rng.choice(d, size=d // 10, replace=False)] = 1.5
    out["fewer non-zeros than k"] = x
    x = studentt_tokens(1, d, seed=3)[0]
    x[::7] = x[1]                                                   # one value many times
    out["one value repeated"] = x
    x = (rng.random(d).astype(np.float32) + 0.5) * np.float32(1e-22)
    x[5] = np.float32(1e18)                                         # scores of the rest are denormal
    out["denormal scores"] = x
    x = (rng.random(d).astype(np.float32) + 0.5) * np.float32(3e-39)
    out["denormal inputs"] = x
    x = (rng.random(d).astype(np.float32) + 0.5) * np.float32(1e-29)
    x[9] = np.float32(1e18)                                         # scores underflow to zero
    out["scores underflow"] = x
    x = np.full(d, 2.0, dtype=np.float32)
    x[::2] = np.nextafter(np.float32(2.0), np.float32(3.0))          # two neighbouring floats
    x[3] = 7.0
    out["neighbouring floats"] = x
    # The one-pass selection ranks the keys of the threshold bin (2^14 consecutive bit patterns,
    # counted down from the maximum) in registers when there are at most 64 of them and runs
    # the generic digits otherwise: m distinct keys in one such bin around the (d // 3)-th
    # largest, for m on both sides of 64 and with a pair of equal keys among them.
    top = np.float32(2.0).view(np.uint32)
    for m in (1, 63, 64, 65, 90):
        bits = np.empty(d, dtype=np.uint32)
        n_above = d // 3 - m // 2
        bits[:n_above] = top - rng.integers(1 << 14, 40 << 14, size=n_above).astype(np.uint32)
        bits[n_above:n_above + m] = top - np.uint32(50 << 14) - 1 - rng.permutation(m).astype(np.uint32)
        if m > 2:
            bits[n_above + 1] = bits[n_above]                    # a tie inside the bin
        rest = d - n_above - m
        bits[n_above + m:] = (rng.random(rest).astype(np.float32) * np.float32(1e-6)).view(np.uint32)
        bits[0] = top
        x = bits.view(np.float32).copy()
        x *= rng.choice(np.array([-1.0, 1.0], dtype=np.float32), size=d)
        out[f"threshold bin of {m}"] = x[rng.permutation(d)]
    return out


@pytest.mark.parametrize("d,f", [(520, 1544), (2052, 3080)])
@pytest.mark.parametrize("gamma", [0.2, 0.0, 1.0])
def test_stage_replay_adversarial_vectors_at_point_1(D, d, f, gamma):
    rng = np.random.default_rng(d)
    for k_in in (1, d // 3, d - 1, d):
        k_mid = f // 4
        L = _layer(D, d, f, "f32", 3, k_in, k_mid)
        for name, x in _adversarial_inputs(d, rng).items():
            for warm in (None, 11):
                caches, ocaches = _caches(D, d, f, d // 2, f // 2, seed=warm)
                try:
                    _replay(D, L, x, k_in, k_mid, gamma, caches, ocaches)
                except AssertionError as e:
                    raise AssertionError(f"{name}, k_in={k_in}, gamma={gamma}, warm={warm}: {e}") from e
            _replay(D, L, x, k_in, k_mid)          # plain DIP keys


def test_stage_replay_adversarial_vectors_at_point_2(D):
    """h~ with structure: identical weight rows make blocks of equal GLU outputs (split ties at
    the threshold of point 2), zero weights make h~ vanish (all scores zero)."""
    d, f, k_in = 512, 2056, 200
    rng = np.random.default_rng(0)
    w = layer_weights(d, f, seed=4, layer=0, dtype="f32")
    ug = w["ug"].copy()
    # 8 distinct GLU units repeated over and over: columns j and j + 8 of W^u, W^g coincide
    ug[:, :f] = np.tile(ug[:, :8], (1, f // 8))
    ug[:, f:] = np.tile(ug[:, f:f + 8], (1, f // 8))
    for name, ug_m in (("tied units", ug), ("zero up/gate", np.zeros_like(ug))):
        for k_mid in (1, 300, f // 2, f):
            L = _layer(D, d, f, "f32", 4, k_in, k_mid, w={"ug": ug_m, "d": w["d"]})
            x = studentt_tokens(1, d, seed=k_mid)[0]
            for warm in (None, 3):
                caches, ocaches = _caches(D, d, f, d // 2, f // 3, seed=warm)
                try:
                    _replay(D, L, x, k_in, k_mid, 0.2, caches, ocaches)
                except AssertionError as e:
                    raise AssertionError(f"{name}, k_mid={k_mid}, warm={warm}: {e}") from e
            _replay(D, L, x, k_in, k_mid)


def _run_tokens(D, L, xs, k_in, k_mid, d, f):
    (cin, cmid), _ = _caches(D, d, f, d // 2, f // 2, seed=8)
    out = []
    for x in xs:
        D.dip_swiglu_mlp_forward(L["mlp"], dev_f32(x), k_in, k_mid, cin, cmid, 0.2, L["y"], L["dbg"], L["ws"])
        torch.cuda.synchronize()
        dbg = L["dbg"]
        out.append([a.cpu().numpy().view(np.uint32).copy() for a in
                    (dbg.s_in, dbg.mask_in, dbg.idx_in, dbg.h, dbg.s_mid, dbg.mask_mid, dbg.idx_mid, L["y"],
                     cin.bits, cin.stamp, cin.meta, cmid.bits, cmid.stamp, cmid.meta)])
    return out


@pytest.mark.parametrize("d,f,fmt,lpr,ks", [(1024, 2048, "f32", 32, 3), (3072, 8192, "bf16", 32, 8),
                                            (2048, 5120, "int4", 16, 4), (1032, 1160, "bf16", 64, 2),
                                            (5120, 17920, "bf16", 32, 3)])
def test_one_launch_form_equals_two_launch_form_bit_for_bit(D, d, f, fmt, lpr, ks):
    k_in, k_mid = d // 2, f // 3
    D.dip_tune_gemv(lpr, 16, ks, 4)          # both forms, both products: one launch shape
    L = _layer(D, d, f, fmt, 6, k_in, k_mid)
    assert D.dip_fused_launch_shape(L["mlp"].w_ug, k_in, bundled=True) == (lpr, 16, ks, 4)
    xs = ar1_laplace_stream(4, d, seed=2)
    a = _run_tokens(D, L, xs, k_in, k_mid, d, f)
    D.dip_set_fusion(False)
    L2 = _layer(D, d, f, fmt, 6, k_in, k_mid)
    assert D.dip_fused_launch_shape(L2["mlp"].w_ug, k_in, bundled=True) is None
    b = _run_tokens(D, L2, xs, k_in, k_mid, d, f)
    names = ["s_in", "mask_in", "idx_in", "h", "s_mid", "mask_mid", "idx_mid", "y", "c_in.bits", "c_in.stamp",
             "c_in.meta", "c_mid.bits", "c_mid.stamp", "c_mid.meta"]
    for t, (u, v) in enumerate(zip(a, b)):
        for name, p, q in zip(names, u, v):
            assert np.array_equal(p, q), f"{name} differs at token {t}"
