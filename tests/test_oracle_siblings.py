"""Pins for the oracle's sibling schemes (Sec. 3.2: GLU, Gate and Up pruning).

Nothing here calls the HIP library.  The schemes are pinned to a case worked by hand with
scalar arithmetic, to the dense MLP when nothing is pruned, to the dense formulas applied
to explicitly masked matrices (library matmul, library SiLU, library top-k), and to the
sparsity limits the section states (one third for GLU pruning, two thirds for Gate / Up).
"""
import math

import numpy as np
import pytest
import torch

from oracle import dip_oracle as O
from workloads import layer_weights, layer_weights_split, studentt_tokens


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def sig(z):
    return z / (1.0 + math.exp(-z))


# the paper's orientation: W^g, W^u in R^{f x d}, W^d in R^{d x f}; d = 2, f = 3
WG = np.array([[1, 0], [0, 1], [-1, 0]], dtype=np.float32)
WU = np.array([[2, 0], [0, 0.5], [3, 3]], dtype=np.float32)
WD = np.array([[1, 1, 1], [1, -1, 0]], dtype=np.float32)
X = np.array([1, 2], dtype=np.float32)
# by hand: W^g x = (1, 2, -1), W^u x = (2, 1, 9)


def test_gate_pruning_hand_worked():
    # |sigma(W^g x)| = (0.731, 1.762, 0.269): the two largest are neurons 0 and 1
    out = O.partial_pruning_forward("gate", WG.T.copy(), WU, WD.T.copy(), X, 2)
    assert out["idx"].tolist() == [0, 1]
    h0, h1 = 2 * sig(1.0), 1 * sig(2.0)
    assert out["h_sel"] == pytest.approx([h0, h1], rel=1e-6)
    assert out["y"] == pytest.approx([h0 + h1, h0 - h1], rel=1e-6)


def test_up_pruning_hand_worked():
    # |W^u x| = (2, 1, 9): the two largest are neurons 0 and 2
    out = O.partial_pruning_forward("up", WU.T.copy(), WG, WD.T.copy(), X, 2)
    assert out["idx"].tolist() == [0, 2]
    h0, h2 = 2 * sig(1.0), 9 * sig(-1.0)
    assert out["h_sel"] == pytest.approx([h0, h2], rel=1e-6)
    assert out["y"] == pytest.approx([h0 + h2, h0], rel=1e-6)


def test_glu_pruning_hand_worked():
    # GLU(x) = (2 sig(1), 1 sig(2), 9 sig(-1)) = (1.462, 1.762, -2.420): keep neurons 1 and 2
    ug = np.concatenate([WU.T, WG.T], axis=1).copy()
    out = O.glu_pruning_forward(ug, WD.T.copy(), X, 2)
    assert out["idx"].tolist() == [1, 2]
    h1, h2 = sig(2.0), 9 * sig(-1.0)
    assert out["y"] == pytest.approx([h1 + h2, -h1], rel=1e-6)


def torch_masked_mlp(wu, wg, wd, x, key_fn, k):
    """Eq. 1-2 with the mask of Sec. 3.2 applied to dense intermediates; library routines only.
    wu, wg: [f][d]; wd: [d][f] (the paper's orientation), fp64 tensors."""
    u, g = wu @ x, wg @ x
    a = torch.nn.functional.silu(g)
    key = key_fn(u, a).abs().float()
    keep = torch.topk(key, k).indices
    m = torch.zeros_like(u)
    m[keep] = 1.0
    return np.sort(keep.numpy()), (wd @ (m * u * a)).numpy()


@pytest.mark.parametrize("scheme", ["glu", "gate", "up"])
@pytest.mark.parametrize("fmt", ["f32", "bf16"])
def test_schemes_equal_masked_dense_formulas(scheme, fmt):
    d, f, k = 96, 256, 77
    w32 = layer_weights_split(d, f, seed=11, layer=0, dtype="f32")
    w = layer_weights_split(d, f, seed=11, layer=0, dtype=fmt)
    wb = layer_weights(d, f, seed=11, layer=0, dtype=fmt)
    if fmt == "bf16":
        # what the storage holds, decoded by torch
        dec = lambda b: torch.from_numpy(b.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64)
    else:
        dec = lambda a: torch.from_numpy(a.astype(np.float64))
    wu, wg, wd = dec(w["u_rows"]), dec(w["g_rows"]), dec(w["d"]).T
    assert w32["u"].shape == (d, f) and w32["g_rows"].shape == (f, d)
    x = studentt_tokens(1, d, 12)[0]
    xt = torch.from_numpy(x.astype(np.float64))
    if scheme == "glu":
        out = O.glu_pruning_forward(wb["ug"], wb["d"], x, k)
        keep, y_ref = torch_masked_mlp(wu, wg, wd, xt, lambda u, a: u * a, k)
    elif scheme == "gate":
        out = O.partial_pruning_forward("gate", w["g"], w["u_rows"], w["d"], x, k)
        keep, y_ref = torch_masked_mlp(wu, wg, wd, xt, lambda u, a: a, k)
    else:
        out = O.partial_pruning_forward("up", w["u"], w["g_rows"], w["d"], x, k)
        keep, y_ref = torch_masked_mlp(wu, wg, wd, xt, lambda u, a: u, k)
    assert np.array_equal(out["idx"], keep)
    assert int(out["mask"].sum()) == k
    assert rel_l2(out["y"], y_ref) < 5e-7


@pytest.mark.parametrize("scheme", ["glu", "gate", "up"])
def test_keeping_everything_is_the_dense_mlp(scheme):
    d, f = 64, 128
    w = layer_weights_split(d, f, seed=13, layer=0, dtype="f32")
    wb = layer_weights(d, f, seed=13, layer=0, dtype="f32")
    x = studentt_tokens(1, d, 14)[0]
    xt = torch.from_numpy(x.astype(np.float64))
    wu = torch.from_numpy(w["u_rows"].astype(np.float64))
    wg = torch.from_numpy(w["g_rows"].astype(np.float64))
    wd = torch.from_numpy(w["d"].astype(np.float64)).T
    y_ref = (wd @ ((wu @ xt) * torch.nn.functional.silu(wg @ xt))).numpy()
    if scheme == "glu":
        y = O.glu_pruning_forward(wb["ug"], wb["d"], x, f)["y"]
    elif scheme == "gate":
        y = O.partial_pruning_forward("gate", w["g"], w["u_rows"], w["d"], x, f)["y"]
    else:
        y = O.partial_pruning_forward("up", w["u"], w["g_rows"], w["d"], x, f)["y"]
    assert rel_l2(y, y_ref) < 5e-7


def test_gate_and_up_pruning_differ_and_are_not_interchangeable():
    """Feeding the gate scheme the up matrix as its dense operand must change the result."""
    d, f, k = 64, 160, 40
    w = layer_weights_split(d, f, seed=15, layer=0, dtype="f32")
    x = studentt_tokens(1, d, 16)[0]
    gate = O.partial_pruning_forward("gate", w["g"], w["u_rows"], w["d"], x, k)
    wrong = O.partial_pruning_forward("gate", w["u"], w["g_rows"], w["d"], x, k)
    up = O.partial_pruning_forward("up", w["u"], w["g_rows"], w["d"], x, k)
    assert rel_l2(wrong["y"], gate["y"]) > 1e-2
    assert not np.array_equal(gate["mask"], up["mask"])


def test_sparsity_limits_of_the_schemes():
    """Sec. 3.2: GLU pruning removes at most one third of the MLP weights, Gate / Up pruning
    at most two thirds; DIP at equal ratios removes 1 - r."""
    for d, f in ((3072, 8192), (5120, 17920)):
        dense = 3 * d * f
        assert 1 - O.sibling_weight_elements("glu", 1, d, f) / dense < 1 / 3
        assert 1 - O.sibling_weight_elements("glu", 1, d, f) / dense > 1 / 3 - 1e-3
        for s in ("gate", "up"):
            assert 1 - O.sibling_weight_elements(s, 1, d, f) / dense < 2 / 3
            assert 1 - O.sibling_weight_elements(s, 1, d, f) / dense > 2 / 3 - 1e-3
            assert O.sibling_weight_elements(s, f, d, f) == dense
        assert O.sibling_weight_elements("glu", f, d, f) == dense
        # half of the GLU units kept: one sixth / one third of the MLP removed
        assert O.sibling_weight_elements("glu", f // 2, d, f) * 6 == 5 * dense
        assert O.sibling_weight_elements("gate", f // 2, d, f) * 3 == 2 * dense
