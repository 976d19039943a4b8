"""Guards of the cross-workgroup reduction of the gathered products (partial sums published
with write-through stores, a ticket per output strip, the last ticket holder adds them in
workgroup order).

1. Exact bits: a product split over G workgroups per strip must equal the G shares computed
   one by one (one workgroup per strip each, so no ticket is involved) and added on the host
   in fp32 in share order -- a stale or missing partial sum changes bits.
2. A bounded soak: about 2000 launches over mixed shapes, formats and both forms of the
   forward; every result must be bit-equal to the first one of its case.  Stops at the first
   mismatch."""
import numpy as np
import pytest
import torch

from oracle import dip_oracle as O
from workloads import ar1_laplace_stream, layer_weights, studentt_tokens
from gpu_util import dev_f32, dev_weight, make_weight, workspace

pytestmark = pytest.mark.gpu


@pytest.fixture()
def D():
    import paper_2412_01380_amd as D
    D.dip_set_fusion(True)
    D.dip_tune_gemv()
    yield D
    D.dip_set_fusion(True)
    D.dip_tune_gemv()


@pytest.mark.parametrize("fmt", ["f32", "bf16", "int4"])
@pytest.mark.parametrize("lpr,waves,ks,unroll", [(16, 8, 5, 4), (32, 16, 7, 4), (64, 16, 3, 4), (8, 4, 12, 2)])
def test_split_product_equals_host_sum_of_its_shares(D, fmt, lpr, waves, ks, unroll):
    n_in, n_out, k = 1536, 1536, 1111
    if fmt == "int4" and lpr == 64 and waves < 16:
        pytest.skip("strip wider than the workgroup")
    w = layer_weights(n_in, n_out // 2, seed=3, layer=0, dtype=fmt)["ug"]      # [n_in][n_out]
    W = make_weight(D, w)
    x = studentt_tokens(1, n_in, seed=4)[0]
    _, idx = O.topk(np.abs(x), k)
    idx_d = torch.from_numpy(idx.astype(np.int32)).cuda()
    xd = dev_f32(x)
    y = torch.empty(n_out, dtype=torch.float32, device="cuda")
    D.dip_tune_gemv(lpr, waves, ks, unroll)
    D.dip_gathered_gemv(W, xd, idx_d, k, y, workspace(D.dip_gathered_gemv_workspace_bytes(W, k)))
    whole = y.cpu().numpy().copy()
    # the shares the kernel cuts: ceil(k / ks) rounded up to a multiple of 8 rows each
    share = ((k + ks - 1) // ks + 7) // 8 * 8
    D.dip_tune_gemv(lpr, waves, 1, unroll)
    total = np.zeros(n_out, dtype=np.float32)
    for g in range(ks):
        kb, ke = min(k, g * share), min(k, (g + 1) * share)
        part = np.zeros(n_out, dtype=np.float32)
        if ke > kb:
            sub = idx_d[kb:ke].contiguous()
            D.dip_gathered_gemv(W, xd, sub, ke - kb, y, workspace(D.dip_gathered_gemv_workspace_bytes(W, ke - kb)))
            part = y.cpu().numpy().copy()
        total = (total + part).astype(np.float32)
    assert np.array_equal(whole.view(np.uint32), total.view(np.uint32))


def test_soak_two_thousand_launches_bit_equal(D):
    cases = []
    # the stand-alone product in several launch shapes
    for (fmt, n_in, n_out, k, shape) in [("bf16", 3072, 2048, 1536, (16, 8, 6, 4)), ("f32", 1500, 1536, 700, (32, 16, 9, 4)),
                                         ("int4", 2048, 2560, 900, (16, 8, 11, 4)), ("bf16", 4096, 1024, 2000, (64, 16, 13, 4))]:
        w = layer_weights(n_in, n_out // 2, seed=5, layer=0, dtype=fmt)["ug"]
        W = make_weight(D, w)
        x = studentt_tokens(1, n_in, seed=n_out)[0]
        _, idx = O.topk(np.abs(x), k)
        cases.append(("gemv", W, dev_f32(x), torch.from_numpy(idx.astype(np.int32)).cuda(), k,
                      torch.empty(n_out, dtype=torch.float32, device="cuda"), shape))
    # the forward in both forms (the one-launch form draws a ticket per strip in both products)
    for (fmt, d, f, fused) in [("bf16", 3072, 8192, True), ("bf16", 3072, 8192, False), ("int4", 2048, 5120, True),
                               ("f32", 1000, 2056, True)]:
        wts = layer_weights(d, f, seed=6, layer=0, dtype=fmt)
        mlp = D.Mlp(make_weight(D, wts["ug"]), make_weight(D, wts["d"]))
        k_in, k_mid = d // 3, f // 3
        ws = workspace(D.dip_swiglu_mlp_forward_workspace_bytes(mlp, k_in, k_mid))
        x = dev_f32(ar1_laplace_stream(1, d, seed=f)[0])
        cases.append(("mlp", mlp, x, k_in, k_mid, torch.empty(d, dtype=torch.float32, device="cuda"), ws, fused))
    first = [None] * len(cases)
    rounds = 250                                   # 8 cases x 250 = 2000 calls
    for it in range(rounds):
        for ci, c in enumerate(cases):
            if c[0] == "gemv":
                _, W, xd, idx_d, k, y, shape = c
                D.dip_tune_gemv(*shape)
                D.dip_gathered_gemv(W, xd, idx_d, k, y, workspace(D.dip_gathered_gemv_workspace_bytes(W, k)))
            else:
                _, mlp, xd, k_in, k_mid, y, ws, fused = c
                D.dip_tune_gemv()
                D.dip_set_fusion(fused)
                D.dip_swiglu_mlp_forward(mlp, xd, k_in, k_mid, None, None, 0.2, y, None, ws)
            if first[ci] is None:
                first[ci] = y.clone()
            else:
                assert torch.equal(y.view(torch.int32), first[ci].view(torch.int32)), (it, ci, c[0])
