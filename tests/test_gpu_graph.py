"""The forward calls only launch kernels on the caller's stream (no allocation, no memset,
no host synchronisation), so a caller may capture them into a HIP graph and replay it.

A replay must give what the same calls give when issued one by one.  Each test replays its
graph several times, with new inputs copied into the captured buffers, eager library calls
and synchronisations between the replays, and compares every replay bit for bit with the
eager result on a second, identically initialised set of caches.
"""
import numpy as np
import pytest
import torch

from workloads import ar1_laplace_stream, layer_weights
from gpu_util import dev_f32, host_u32, make_weight, workspace

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def D():
    import paper_2412_01380_amd as D
    return D


def _bits(t):
    return t.cpu().numpy().view(np.uint32)


def _caches(D, L, d, f, c_in, c_mid):
    cins = [D.Cache(d, c_in) for _ in range(L)]
    cmids = [D.Cache(f, c_mid) for _ in range(L)]
    for c in cins + cmids:
        D.dip_cache_init(c)
    return cins, cmids


@pytest.mark.parametrize("fmt,use_cache", [("bf16", True), ("f32", False), ("int4", True)])
def test_stack_forward_replays_from_a_graph(D, fmt, use_cache):
    d, f, L = 512, 1536, 3
    k_in, k_mid = 150, 500
    mlps = []
    for l in range(L):
        w = layer_weights(d, f, seed=21, layer=l, dtype=fmt)
        mlps.append(D.Mlp(make_weight(D, w["ug"]), make_weight(D, w["d"])))
    ce, cg = (_caches(D, L, d, f, 200, 700), _caches(D, L, d, f, 200, 700)) if use_cache else ((None, None),) * 2
    stack_e = D.MlpStack(mlps, ce[0], ce[1])
    stack_g = D.MlpStack(mlps, cg[0], cg[1])
    nbytes = D.dip_swiglu_mlp_forward_stack_workspace_bytes(stack_e, k_in, k_mid)
    ws_e, ws_g = workspace(nbytes), workspace(nbytes)
    T = 6
    X = dev_f32(ar1_laplace_stream(L * T, d, seed=8).reshape(T, L, d))
    x_buf = torch.zeros(L, d, dtype=torch.float32, device="cuda")
    y_e = torch.empty(L, d, dtype=torch.float32, device="cuda")
    y_g = torch.zeros(L, d, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        D.dip_swiglu_mlp_forward_stack(stack_g, x_buf, d, k_in, k_mid, 0.2, y_g, d, ws_g)
    # capturing runs nothing: the graph's caches are still in their initial state
    for t in range(T):
        D.dip_swiglu_mlp_forward_stack(stack_e, X[t], d, k_in, k_mid, 0.2, y_e, d, ws_e)
        x_buf.copy_(X[t])
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(_bits(y_g), _bits(y_e)), (t, "y")
        if use_cache:
            for l in range(L):
                for a, b in ((ce[0][l], cg[0][l]), (ce[1][l], cg[1][l])):
                    assert np.array_equal(host_u32(a.bits), host_u32(b.bits)), (t, l, "residency")
                    assert np.array_equal(host_u32(a.stamp), host_u32(b.stamp)), (t, l, "stamps")
                    assert a.meta_host() == b.meta_host(), (t, l, "counters")


def test_batched_forward_replays_from_a_graph(D):
    d, f, B = 512, 1536, 4
    k_in, k_mid = 150, 500
    w = layer_weights(d, f, seed=22, layer=0, dtype="int4")
    mlp = D.Mlp(make_weight(D, w["ug"]), make_weight(D, w["d"]))
    (ce_in, ce_mid), (cg_in, cg_mid) = _caches(D, 1, d, f, 256, 768), _caches(D, 1, d, f, 256, 768)
    nbytes = D.dip_swiglu_mlp_forward_batched_workspace_bytes(mlp, B, k_in, k_mid)
    ws_e, ws_g = workspace(nbytes), workspace(nbytes)
    T = 5
    X = dev_f32(np.stack([ar1_laplace_stream(T, d, seed=30 + b) for b in range(B)], axis=1))
    x_buf = torch.zeros(B, d, dtype=torch.float32, device="cuda")
    y_e = torch.empty(B, d, dtype=torch.float32, device="cuda")
    y_g = torch.zeros(B, d, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        D.dip_swiglu_mlp_forward_batched(mlp, x_buf, B, k_in, k_mid, cg_in[0], cg_mid[0], 0.2, y_g,
                                         None, None, None, ws_g)
    for t in range(T):
        D.dip_swiglu_mlp_forward_batched(mlp, X[t], B, k_in, k_mid, ce_in[0], ce_mid[0], 0.2, y_e,
                                         None, None, None, ws_e)
        x_buf.copy_(X[t])
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(_bits(y_g), _bits(y_e)), (t, "y")
        for a, b in ((ce_in[0], cg_in[0]), (ce_mid[0], cg_mid[0])):
            assert np.array_equal(host_u32(a.bits), host_u32(b.bits)), (t, "residency")
            assert np.array_equal(host_u32(a.stamp), host_u32(b.stamp)), (t, "stamps")
