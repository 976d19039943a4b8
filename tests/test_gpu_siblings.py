"""GPU parity for the sibling schemes of Sec. 3.2 (GLU, Gate and Up pruning) through the C ABI.

Stage replay, as for DIP: the partial activation a comes out of the GPU's fp32 sums, so the
mask is compared with the oracle's selection applied to the GPU's own a, h with the oracle's
combination of that a with fp64 row products, and y with the oracle's down projection of the
GPU's own h.  a itself and the free-running y are compared in rel-L2.
"""
import numpy as np
import pytest
import torch

from oracle import dip_oracle as O
from workloads import layer_weights, layer_weights_split, studentt_tokens
from gpu_util import bool_from_bits, dev_f32, host_u32, make_weight, rel_l2, workspace

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-3, "int4": 2e-3}


@pytest.fixture(scope="module")
def D():
    import paper_2412_01380_amd as D
    return D


# ------------------------------------------------------------------ row-gathered dot products
@pytest.mark.parametrize("fmt,n_rows,n_cols,k", [
    ("f32", 96, 64, 96), ("f32", 300, 1000, 123), ("f32", 1536, 512, 768),
    ("bf16", 200, 72, 57), ("bf16", 8192, 3072, 4096), ("bf16", 1000, 5120, 1), ("bf16", 777, 8200, 300),
    ("int4", 256, 128, 100), ("int4", 1984, 5120, 900), ("int4", 640, 3072, 640),
    # rows longer than 16384 floats of x: more than 64 KB of LDS, several chunks per row
    ("f32", 64, 20480, 64), ("bf16", 128, 32768, 77),
])
def test_rowdot_matches_oracle(D, fmt, n_rows, n_cols, k):
    # a neuron-major matrix [n_rows][n_cols] is what layer_weights calls 'd' with d_ff = n_rows
    w = layer_weights(n_cols, n_rows, seed=21, layer=0, dtype=fmt)["d"]
    x = studentt_tokens(1, n_cols, seed=22)[0]
    rng = np.random.default_rng(23)
    idx = np.sort(rng.choice(n_rows, size=k, replace=False)).astype(np.int32)
    W = make_weight(D, w)
    out = torch.full((k,), float("nan"), dtype=torch.float32, device="cuda")
    D.dip_gathered_rowdot(W, dev_f32(x), torch.from_numpy(idx).cuda(), k, out)
    want = O.gathered_rowdot(w, x, idx)
    assert rel_l2(out.cpu().numpy(), want) <= TOL[fmt]
    # bit-repeatable
    out2 = torch.empty_like(out)
    D.dip_gathered_rowdot(W, dev_f32(x), torch.from_numpy(idx).cuda(), k, out2)
    assert torch.equal(out, out2)


def test_rowdot_unit_vector_returns_a_column(D):
    n_rows, n_cols = 130, 256
    w = layer_weights(n_cols, n_rows, seed=24, layer=0, dtype="f32")["d"]
    W = make_weight(D, w)
    idx = torch.arange(n_rows, dtype=torch.int32, device="cuda")
    out = torch.empty(n_rows, dtype=torch.float32, device="cuda")
    for c in (0, 63, 64, 255):
        e = np.zeros(n_cols, dtype=np.float32)
        e[c] = 1.0
        D.dip_gathered_rowdot(W, dev_f32(e), idx, n_rows, out)
        assert np.array_equal(out.cpu().numpy(), w[:, c])


# ------------------------------------------------------------------ gate / up pruning
def split_mlp(D, w, scheme):
    if scheme == "gate":
        return D.MlpSplit(make_weight(D, w["g"]), make_weight(D, w["u_rows"]), make_weight(D, w["d"])), w["g"], w["u_rows"]
    return D.MlpSplit(make_weight(D, w["u"]), make_weight(D, w["g_rows"]), make_weight(D, w["d"])), w["u"], w["g_rows"]


@pytest.mark.parametrize("scheme", ["gate", "up"])
@pytest.mark.parametrize("fmt,d,f,k", [
    ("f32", 512, 1536, 768), ("f32", 96, 200, 200), ("f32", 136, 328, 1),
    ("bf16", 512, 1536, 768), ("bf16", 3072, 8192, 4096), ("bf16", 3072, 8192, 2048),
    ("bf16", 5120, 17920, 5376), ("int4", 512, 1536, 500), ("int4", 5120, 17920, 5376),
])
def test_partial_pruning_stage_replay(D, scheme, fmt, d, f, k):
    w = layer_weights_split(d, f, seed=31, layer=0, dtype=fmt)
    mlp, w_dense, w_rows = split_mlp(D, w, scheme)
    code = D.DIP_GATE_PRUNING if scheme == "gate" else D.DIP_UP_PRUNING
    x = studentt_tokens(2, d, seed=32)
    dbg = D.PartialDebug(f, k)
    ws = workspace(D.dip_partial_pruning_forward_workspace_bytes(mlp, k))
    y = torch.empty(d, dtype=torch.float32, device="cuda")
    for t in range(2):
        D.dip_partial_pruning_forward(mlp, code, dev_f32(x[t]), k, y, dbg, ws)
        torch.cuda.synchronize()
        ref = O.partial_pruning_forward(scheme, w_dense, w_rows, w["d"], x[t], k)
        a = dbg.a.cpu().numpy()
        assert rel_l2(a, ref["a"]) <= TOL[fmt]
        # the oracle's selection on the GPU's own partial activation: exact
        m_want, idx_want = O.topk(np.abs(a), k)
        assert np.array_equal(bool_from_bits(host_u32(dbg.mask), f), m_want)
        assert np.array_equal(dbg.idx.cpu().numpy(), idx_want)
        # h from the GPU's a and fp64 row products
        other = O.gathered_rowdot(w_rows, x[t], idx_want)
        if scheme == "gate":
            h_want = other * a[idx_want].astype(np.float64)
        else:
            h_want = a[idx_want].astype(np.float64) * O.silu(other)
        h_sel = dbg.h_sel.cpu().numpy()
        assert rel_l2(h_sel, h_want) <= TOL[fmt]
        # y from the GPU's own h
        h_full = np.zeros(f, dtype=np.float32)
        h_full[idx_want] = h_sel
        y_want = O.gathered_gemv(w["d"], h_full, idx_want)
        assert rel_l2(y.cpu().numpy(), y_want) <= TOL[fmt]
        # free-running comparison when the masks agree
        if np.array_equal(ref["mask"], m_want):
            assert rel_l2(y.cpu().numpy(), ref["y"]) <= TOL[fmt]
    # without debug outputs the result is the same bits
    y2 = torch.empty_like(y)
    D.dip_partial_pruning_forward(mlp, code, dev_f32(x[1]), k, y2, None, ws)
    assert torch.equal(y, y2)


def test_partial_pruning_rejects_bad_arguments(D):
    d, f = 128, 256
    w = layer_weights_split(d, f, seed=33, layer=0, dtype="f32")
    mlp, _, _ = split_mlp(D, w, "gate")
    ws = workspace(D.dip_partial_pruning_forward_workspace_bytes(mlp, 10))
    x = dev_f32(np.ones(d))
    y = torch.empty(d, dtype=torch.float32, device="cuda")
    with pytest.raises(D.DipError):
        D.dip_partial_pruning_forward(mlp, 7, x, 10, y, None, ws)
    with pytest.raises(D.DipError):
        D.dip_partial_pruning_forward(mlp, D.DIP_GATE_PRUNING, x, f + 1, y, None, ws)
    bad = D.MlpSplit(make_weight(D, w["g"]), make_weight(D, w["u"]), make_weight(D, w["d"]))
    with pytest.raises(D.DipError):
        D.dip_partial_pruning_forward(bad, D.DIP_GATE_PRUNING, x, 10, y, None, ws)


# ------------------------------------------------------------------ GLU pruning
@pytest.mark.parametrize("fmt,d,f,k", [
    ("f32", 512, 1536, 768), ("f32", 100, 232, 17), ("bf16", 3072, 8192, 4096),
    ("bf16", 4096, 14336, 4301), ("int4", 5120, 17920, 5376),
])
def test_glu_pruning_stage_replay(D, fmt, d, f, k):
    w = layer_weights(d, f, seed=41, layer=0, dtype=fmt)
    mlp = D.Mlp(make_weight(D, w["ug"]), make_weight(D, w["d"]))
    x = studentt_tokens(1, d, seed=42)[0]
    h = torch.empty(f, dtype=torch.float32, device="cuda")
    mask = torch.empty((f + 31) // 32, dtype=torch.int32, device="cuda")
    idx = torch.empty(k, dtype=torch.int32, device="cuda")
    dbg = D.glu_debug(h=h, mask_mid=mask, idx_mid=idx)
    ws = workspace(D.dip_glu_pruning_forward_workspace_bytes(mlp, k))
    y = torch.empty(d, dtype=torch.float32, device="cuda")
    D.dip_glu_pruning_forward(mlp, dev_f32(x), k, y, dbg, ws)
    torch.cuda.synchronize()
    ref = O.glu_pruning_forward(w["ug"], w["d"], x, k)
    hg = h.cpu().numpy()
    assert rel_l2(hg, ref["a"]) <= TOL[fmt]
    m_want, idx_want = O.topk(np.abs(hg), k)
    assert np.array_equal(bool_from_bits(host_u32(mask), f), m_want)
    assert np.array_equal(idx.cpu().numpy(), idx_want)
    assert rel_l2(y.cpu().numpy(), O.gathered_gemv(w["d"], hg, idx_want)) <= TOL[fmt]
    if np.array_equal(ref["mask"], m_want):
        assert rel_l2(y.cpu().numpy(), ref["y"]) <= TOL[fmt]
    # the same result as DIP with nothing pruned at point 1
    y2 = torch.empty_like(y)
    ws2 = workspace(D.dip_swiglu_mlp_forward_workspace_bytes(mlp, d, k))
    D.dip_swiglu_mlp_forward(mlp, dev_f32(x), d, k, None, None, 0.2, y2, None, ws2)
    assert torch.equal(y, y2)
