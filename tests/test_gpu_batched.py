"""GPU parity of the small-batch forward (B = 1..8 rows, unioned column reads) against the
oracle, stage by stage on identical inputs as in test_gpu_parity.py: per-row masks are
bit-exact, h~ and y within tolerance, caches identical to the oracle's update with the union
of the row masks."""
import numpy as np
import pytest
import torch

from oracle import dip_oracle as O
from workloads import CONFIGS, ar1_laplace_stream, layer_weights
from gpu_util import (assert_product_close, bits_from_bool, bool_from_bits, dev_f32, glu_scale, host_u32, make_weight,
                      rel_l2, workspace)

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-5, "bf16": 2e-3, "int4": 2e-3}


@pytest.fixture(scope="module")
def D():
    import paper_2412_01380_amd as D
    return D


def run_steps(D, d, f, fmt, B, k_in, k_mid, steps, use_cache, seed, layer=0, cap_frac=0.5):
    w = layer_weights(d, f, seed=seed, layer=layer, dtype=fmt)
    mlp = D.Mlp(make_weight(D, w["ug"]), make_weight(D, w["d"]))
    vector = not (fmt == "int4" and B >= 3)       # that case runs on the matrix cores (own bar)
    ws = workspace(D.dip_swiglu_mlp_forward_batched_workspace_bytes(mlp, B, k_in, k_mid))
    wd, wf = (d + 31) // 32, (f + 31) // 32
    m1 = torch.empty(B, wd, dtype=torch.int32, device="cuda")
    m2 = torch.empty(B, wf, dtype=torch.int32, device="cuda")
    H = torch.empty(B, f, dtype=torch.float32, device="cuda")
    Y = torch.empty(B, d, dtype=torch.float32, device="cuda")
    cin = cmid = ocin = ocmid = None
    if use_cache:
        C_in, C_mid = int(cap_frac * d), int(cap_frac * f)
        cin, cmid = D.Cache(d, C_in), D.Cache(f, C_mid)
        D.dip_cache_init(cin)
        D.dip_cache_init(cmid)
        ocin, ocmid = O.CacheState(n=d, capacity=C_in), O.CacheState(n=f, capacity=C_mid)
    # every row is its own AR(1) stream
    streams = np.stack([ar1_laplace_stream(steps, d, seed=seed * 100 + b) for b in range(B)], axis=1)
    for t in range(steps):
        X = streams[t]
        D.dip_swiglu_mlp_forward_batched(mlp, dev_f32(X), B, k_in, k_mid, cin, cmid, 0.2, Y, m1, H, m2, ws)
        torch.cuda.synchronize()
        Hg, Yg = H.cpu().numpy(), Y.cpu().numpy()
        c_in = None if ocin is None else ocin.resident.copy()
        c_mid = None if ocmid is None else ocmid.resident.copy()
        M1, M2 = [], []
        for b in range(B):
            mb1, idx1 = O.topk(O.score(X[b], c_in, 0.2), k_in)
            assert np.array_equal(host_u32(m1[b]), bits_from_bool(mb1)), (t, b, "mask 1")
            pre = O.gathered_gemv(w["ug"], X[b], idx1)
            h_ref = O.glu_from_preacts(pre)
            assert rel_l2(Hg[b], h_ref) <= TOL[fmt], (t, b, "h")
            if vector:
                assert_product_close(Hg[b], h_ref, fmt, k_in, (t, b, "h"), scale=glu_scale(pre), factor=3.0)
            mb2, idx2 = O.topk(O.score(Hg[b], c_mid, 0.2), k_mid)
            assert np.array_equal(host_u32(m2[b]), bits_from_bool(mb2)), (t, b, "mask 2")
            y_ref = O.gathered_gemv(w["d"], Hg[b], idx2)
            assert rel_l2(Yg[b], y_ref) <= TOL[fmt], (t, b, "y")
            if vector:
                assert_product_close(Yg[b], y_ref, fmt, k_mid, (t, b, "y"))
            M1.append(mb1)
            M2.append(mb2)
        if use_cache:
            O.cache_update(ocin, np.any(M1, axis=0))
            O.cache_update(ocmid, np.any(M2, axis=0))
            assert np.array_equal(bool_from_bits(host_u32(cin.bits), d), ocin.resident)
            assert np.array_equal(host_u32(cin.stamp).astype(np.int64), ocin.stamp)
            assert np.array_equal(bool_from_bits(host_u32(cmid.bits), f), ocmid.resident)
            assert np.array_equal(host_u32(cmid.stamp).astype(np.int64), ocmid.stamp)
            assert cmid.meta_host()["cum_lookups"] == ocmid.lookups
    return Yg


@pytest.mark.parametrize("fmt", ["f32", "bf16", "int4"])
@pytest.mark.parametrize("B", [1, 2, 3, 8])
def test_batched_small_layer(D, fmt, B):
    run_steps(D, 512, 1536, fmt, B, 154, 461, steps=3, use_cache=True, seed=31)


def test_batched_ragged_shapes_no_cache(D):
    run_steps(D, 1000, 1144, "bf16", 5, 333, 401, steps=2, use_cache=False, seed=32)


def test_batch_one_equals_single_row_forward(D):
    """B = 1 through the batched entry point selects the same masks as the batch-1 call."""
    d, f, k_in, k_mid = 512, 1536, 200, 500
    w = layer_weights(d, f, seed=33, layer=0, dtype="bf16")
    mlp = D.Mlp(make_weight(D, w["ug"]), make_weight(D, w["d"]))
    x = ar1_laplace_stream(1, d, seed=5)
    ws1 = workspace(D.dip_swiglu_mlp_forward_workspace_bytes(mlp, k_in, k_mid))
    dbg = D.Debug(d, f, k_in, k_mid)
    y1 = torch.empty(d, dtype=torch.float32, device="cuda")
    D.dip_swiglu_mlp_forward(mlp, dev_f32(x[0]), k_in, k_mid, None, None, 0.2, y1, dbg, ws1)
    wsb = workspace(D.dip_swiglu_mlp_forward_batched_workspace_bytes(mlp, 1, k_in, k_mid))
    m1 = torch.empty(1, (d + 31) // 32, dtype=torch.int32, device="cuda")
    Y = torch.empty(1, d, dtype=torch.float32, device="cuda")
    D.dip_swiglu_mlp_forward_batched(mlp, dev_f32(x), 1, k_in, k_mid, None, None, 0.2, Y, m1, None, None, wsb)
    assert np.array_equal(host_u32(m1[0]), host_u32(dbg.mask_in))
    assert rel_l2(Y[0].cpu().numpy(), y1.cpu().numpy()) <= 1e-5


@pytest.mark.parametrize("B", [2, 8])
def test_config5_phi3_medium_int4_batched(D, B):
    cfg = CONFIGS[5]
    run_steps(D, cfg.d_model, cfg.d_ff, "int4", B, cfg.k_in(0.3), cfg.k_mid(0.3), steps=2,
              use_cache=True, seed=cfg.seed, layer=1)


@pytest.mark.parametrize("B", [3, 5, 8])
def test_batched_int4_matrix_core_edges(D, B):
    """int4 with three or more rows runs on the matrix cores: an odd number of 128-column
    scale groups (the last 256-column strip is half empty), shares shorter than one set of
    16 listed columns, and every keep count down to 1."""
    run_steps(D, 640, 1408, "int4", B, 211, 433, steps=2, use_cache=True, seed=34)
    run_steps(D, 640, 1408, "int4", B, 17, 33, steps=2, use_cache=False, seed=35)
    run_steps(D, 128, 128, "int4", B, 1, 1, steps=2, use_cache=True, seed=36)
    run_steps(D, 384, 1152, "int4", B, 384, 1152, steps=1, use_cache=False, seed=37)


@pytest.mark.parametrize("scale_log2", [0, -12, 12, -40, 30])
@pytest.mark.parametrize("B", [3, 8])
def test_batched_int4_matrix_core_accuracy_at_any_activation_scale(D, B, scale_log2):
    """The product on the matrix cores scales every row's activations by a power of two into a
    fixed range before they become fp16 operands and undoes it exactly: the error against the
    oracle must not depend on the magnitude of the activations (Sec. 5.2 normalises by
    ||x||_inf for the same reason), and rows of very different magnitudes may share a batch."""
    d, f, k_in, k_mid = 1024, 2816, 307, 845
    w = layer_weights(d, f, seed=38, layer=0, dtype="int4")
    mlp = D.Mlp(make_weight(D, w["ug"]), make_weight(D, w["d"]))
    ws = workspace(D.dip_swiglu_mlp_forward_batched_workspace_bytes(mlp, B, k_in, k_mid))
    H = torch.empty(B, f, dtype=torch.float32, device="cuda")
    Y = torch.empty(B, d, dtype=torch.float32, device="cuda")
    X = np.stack([ar1_laplace_stream(1, d, seed=380 + b)[0] for b in range(B)])
    X = (X * np.float32(2.0) ** scale_log2).astype(np.float32)
    X[1] *= np.float32(2.0 ** -9)             # one row far below the others
    D.dip_swiglu_mlp_forward_batched(mlp, dev_f32(X), B, k_in, k_mid, None, None, 0.2, Y, None, H, None, ws)
    torch.cuda.synchronize()
    Hg, Yg = H.cpu().numpy(), Y.cpu().numpy()
    assert np.all(np.isfinite(Hg)) and np.all(np.isfinite(Yg))
    for b in range(B):
        _, idx1 = O.topk(O.score(X[b], None, 0.2), k_in)
        pre = O.gathered_gemv(w["ug"], X[b], idx1)
        # the pre-activations carry the product's error; h~ = u * SiLU(g) is compared where it
        # is well conditioned (|g| not tiny relative to its scale is not needed: rel-L2 over all)
        assert rel_l2(Hg[b], O.glu_from_preacts(pre)) <= 2e-4, (b, "h")
        _, idx2 = O.topk(O.score(Hg[b], None, 0.2), k_mid)
        assert rel_l2(Yg[b], O.gathered_gemv(w["d"], Hg[b], idx2)) <= 2e-4, (b, "y")


def test_batched_config5_shape_batch_4(D):
    """B = 4 at the Phi-3-Medium int4 shape (the batch sizes 1, 2 and 8 are covered above)."""
    cfg = CONFIGS[5]
    run_steps(D, cfg.d_model, cfg.d_ff, "int4", 4, cfg.k_in(0.3), cfg.k_mid(0.3), steps=2, use_cache=True, seed=39)


@pytest.mark.parametrize("fmt,B", [("bf16", 2), ("int4", 4)])
def test_batched_stack_call_equals_per_layer_calls(D, fmt, B):
    """The batched forward over a stack in one call (cache updates of all layers in one launch
    at the end) against one batched call per layer: outputs and cache states bit-equal."""
    d, L = 512, 3
    ffs, k_in, k_mids = [1536, 2304, 1024], 150, [400, 700, 256]
    mlps, ws_one = [], []
    for l in range(L):
        w = layer_weights(d, ffs[l], seed=61, layer=l, dtype=fmt)
        mlps.append(D.Mlp(make_weight(D, w["ug"]), make_weight(D, w["d"])))
        ws_one.append(workspace(D.dip_swiglu_mlp_forward_batched_workspace_bytes(mlps[l], B, k_in, k_mids[l])))
    caches = [[D.Cache(d, 200) for _ in range(L)], [D.Cache(ffs[l], ffs[l] // 2) for l in range(L)],
              [D.Cache(d, 200) for _ in range(L)], [D.Cache(ffs[l], ffs[l] // 2) for l in range(L)]]
    for cs in caches:
        for c in cs:
            D.dip_cache_init(c)
    stack = D.MlpStack(mlps, caches[0], caches[1])
    ws = workspace(D.dip_swiglu_mlp_forward_batched_stack_workspace_bytes(stack, B, k_in, k_mids))
    Y = torch.empty(L, B, d, dtype=torch.float32, device="cuda")
    Y1 = torch.empty(B, d, dtype=torch.float32, device="cuda")
    for t in range(3):
        X = dev_f32(np.stack([ar1_laplace_stream(t + 1, d, seed=600 + l * 8 + b)[t] for l in range(L) for b in range(B)])
                    .reshape(L, B, d))
        D.dip_swiglu_mlp_forward_batched_stack(stack, X, B * d, B, k_in, k_mids, 0.2, Y, B * d, ws)
        for l in range(L):
            D.dip_swiglu_mlp_forward_batched(mlps[l], X[l], B, k_in, k_mids[l], caches[2][l], caches[3][l], 0.2, Y1,
                                             None, None, None, ws_one[l])
            torch.cuda.synchronize()
            assert torch.equal(Y[l].view(torch.int32), Y1.view(torch.int32)), (t, l, "y")
            for a, b in ((caches[0][l], caches[2][l]), (caches[1][l], caches[3][l])):
                assert torch.equal(a.bits, b.bits) and torch.equal(a.stamp, b.stamp) and torch.equal(a.meta, b.meta), (t, l)
