"""The entry point that allocates nothing (dip_swiglu_mlp_forward_noalloc) against the
entry point it is a variant of (dip_swiglu_mlp_forward with a caller workspace): same
inputs, two calls in a row through the C ABI, the second on a smaller layer, so the built-in
scratch still holds the first call's contents when the second starts.  Masks, caches and
index lists must be bit-equal; h~ and y too, because both run the same kernels in the same
launch shape."""
import numpy as np
import pytest
import torch

from gpu_util import dev_f32, host_u32, make_weight, workspace
from workloads import ar1_laplace_stream, layer_weights

pytestmark = pytest.mark.gpu


def _run(D, d, f, r, dtype, seed, use_noalloc, n_tokens=3):
    k_in, k_mid = max(1, round(r * d)), max(1, round(r * f))
    w = layer_weights(d, f, seed=seed, layer=0, dtype=dtype)
    mlp = D.Mlp(make_weight(D, w["ug"]), make_weight(D, w["d"]))
    cin, cmid = D.Cache(d, d // 2), D.Cache(f, f // 2)
    D.dip_cache_init(cin)
    D.dip_cache_init(cmid)
    dbg = D.Debug(d, f, k_in, k_mid)
    y = torch.empty(d, dtype=torch.float32, device="cuda")
    ws = None if use_noalloc else workspace(D.dip_swiglu_mlp_forward_workspace_bytes(mlp, k_in, k_mid))
    xs = ar1_laplace_stream(n_tokens, d, seed=seed + 7)
    out = []
    for t in range(n_tokens):
        x = dev_f32(xs[t])
        if use_noalloc:
            D.dip_swiglu_mlp_forward_noalloc(mlp, x, k_in, k_mid, cin, cmid, 0.2, y, dbg)
        else:
            D.dip_swiglu_mlp_forward(mlp, x, k_in, k_mid, cin, cmid, 0.2, y, dbg, ws)
        torch.cuda.synchronize()
        out.append((host_u32(dbg.mask_in).copy(), dbg.idx_in.cpu().numpy().copy(),
                    dbg.h.cpu().numpy().view(np.uint32).copy(), host_u32(dbg.mask_mid).copy(),
                    dbg.idx_mid.cpu().numpy().copy(), y.cpu().numpy().view(np.uint32).copy(),
                    host_u32(cin.bits).copy(), host_u32(cin.stamp).copy(), host_u32(cin.meta).copy(),
                    host_u32(cmid.bits).copy(), host_u32(cmid.stamp).copy(), host_u32(cmid.meta).copy()))
    return out


NAMES = ["mask_in", "idx_in", "h", "mask_mid", "idx_mid", "y", "c_in.bits", "c_in.stamp", "c_in.meta",
         "c_mid.bits", "c_mid.stamp", "c_mid.meta"]


def test_noalloc_matches_workspace_entry_point_two_calls_second_smaller():
    import paper_2412_01380_amd as D
    # first a Phi-3-Mini-sized bf16 layer (split-K partials and tickets in the scratch), then a
    # smaller fp32 layer with a ragged last strip that reuses the same scratch bytes
    for (d, f, r, dtype, seed) in [(3072, 8192, 0.5, "bf16", 3), (520, 1544, 0.3, "f32", 4)]:
        ref = _run(D, d, f, r, dtype, seed, use_noalloc=False)
        got = _run(D, d, f, r, dtype, seed, use_noalloc=True)
        for t, (a, b) in enumerate(zip(ref, got)):
            for name, u, v in zip(NAMES, a, b):
                assert np.array_equal(u, v), f"{name} differs at token {t} of layer {d}x{f}"


def test_noalloc_rejects_layers_beyond_the_builtin_scratch():
    import paper_2412_01380_amd as D
    from paper_2412_01380_amd.libdip import _Mlp, _Weight
    import ctypes as C
    # validation happens on the host: fake pointers are never dereferenced
    d, f = 32768, 32768
    FAKE = 0x10000
    ug = _Weight(FAKE, None, D.DIP_F32, d, 2 * f, 0, 2 * f * 4)
    dn = _Weight(FAKE, None, D.DIP_F32, f, d, 0, d * 4)
    mlp = _Mlp(ug, dn)
    need = D.lib.dip_swiglu_mlp_forward_workspace_bytes(C.byref(mlp), d, f)
    assert need > D.DIP_STATIC_SCRATCH_BYTES
    st = D.lib.dip_swiglu_mlp_forward_noalloc(C.byref(mlp), FAKE, d, f, None, None, 0.2, FAKE, None, None)
    assert st == D.DIP_ERR_WORKSPACE
    assert "built-in" in D.dip_last_error()
