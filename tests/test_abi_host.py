"""Host-side checks that need no GPU: the shared library loads, exports every symbol the
header declares, and rejects bad arguments before touching the HIP runtime."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def D():
    import paper_2412_01380_amd as D
    return D


def header_functions():
    src = "".join(open(os.path.join(ROOT, "include", h)).read() for h in ("dip.h", "dip_devtools.h"))
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(dip_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol(D):
    names = header_functions()
    assert "dip_swiglu_mlp_forward" in names and "dip_prune_topk" in names
    for n in names:
        assert hasattr(D.lib, n), n
    assert sorted(D.EXPORTS) == names


def test_version(D):
    assert D.dip_version() == (0 << 16) | 1


FAKE = 0x10000  # a non-null, 256-aligned "device pointer"; validation never dereferences it


def test_topk_argument_validation(D):
    L = D.lib
    assert L.dip_prune_topk(None, 10, 3, FAKE, None, None) == D.DIP_ERR_INVALID_ARG
    assert L.dip_prune_topk(FAKE, 10, 3, None, None, None) == D.DIP_ERR_INVALID_ARG
    assert L.dip_prune_topk(FAKE, 10, 0, FAKE, None, None) == D.DIP_ERR_INVALID_ARG
    assert L.dip_prune_topk(FAKE, 10, 11, FAKE, None, None) == D.DIP_ERR_INVALID_ARG
    assert L.dip_prune_topk(FAKE, 0, 1, FAKE, None, None) == D.DIP_ERR_INVALID_ARG
    assert L.dip_prune_topk(FAKE, D.DIP_MAX_N + 1, 1, FAKE, None, None) == D.DIP_ERR_UNSUPPORTED
    assert "k must be" in D.dip_last_error() or "n must be" in D.dip_last_error()


def test_scores_argument_validation(D):
    L = D.lib
    assert L.dip_ca_scores(None, 8, None, 0.2, FAKE, None) == D.DIP_ERR_INVALID_ARG
    assert L.dip_ca_scores(FAKE, 8, FAKE, 1.5, FAKE, None) == D.DIP_ERR_INVALID_ARG
    assert L.dip_ca_scores(FAKE, 8, FAKE, -0.1, FAKE, None) == D.DIP_ERR_INVALID_ARG
    assert L.dip_ca_scores(FAKE, 8, FAKE, float("nan"), FAKE, None) == D.DIP_ERR_INVALID_ARG
    assert L.dip_ca_scores(FAKE, 0, None, 0.2, FAKE, None) == D.DIP_ERR_INVALID_ARG


def _weight(D, dtype=0, n_in=64, n_out=64, stride=None, data=FAKE):
    from paper_2412_01380_amd.libdip import _Weight
    eb = 4 if dtype == 0 else 2
    return _Weight(data, None, dtype, n_in, n_out, 0, stride if stride is not None else n_out * eb)


def test_gemv_argument_validation(D):
    L = D.lib
    w = _weight(D)
    ok_ws = L.dip_gathered_gemv_workspace_bytes(C.byref(w), 8)
    assert ok_ws >= 256
    call = lambda w, k=8, ws=FAKE, wsb=1 << 20, x=FAKE, idx=FAKE, y=FAKE: \
        L.dip_gathered_gemv(C.byref(w), x, idx, k, y, ws, wsb, None)
    assert call(w, k=0) == D.DIP_ERR_INVALID_ARG
    assert call(w, k=65) == D.DIP_ERR_INVALID_ARG
    assert call(w, x=None) == D.DIP_ERR_INVALID_ARG
    assert call(w, ws=None) == D.DIP_ERR_WORKSPACE
    assert call(w, wsb=8) == D.DIP_ERR_WORKSPACE
    assert call(w, ws=FAKE + 4) == D.DIP_ERR_WORKSPACE
    assert call(_weight(D, dtype=2, n_out=128)) == D.DIP_ERR_INVALID_ARG   # int4 without scales
    assert call(_weight(D, dtype=7)) == D.DIP_ERR_UNSUPPORTED
    assert call(_weight(D, n_out=66)) == D.DIP_ERR_UNSUPPORTED         # not a 16-byte multiple
    assert call(_weight(D, stride=100)) == D.DIP_ERR_INVALID_ARG       # stride < row
    assert call(_weight(D, data=FAKE + 2)) == D.DIP_ERR_UNSUPPORTED    # misaligned
    assert call(_weight(D, data=None)) == D.DIP_ERR_INVALID_ARG


def test_forward_argument_validation(D):
    from paper_2412_01380_amd.libdip import _Cache, _Mlp
    L = D.lib
    d, f = 64, 128
    mlp = _Mlp(_weight(D, 1, d, 2 * f), _weight(D, 1, f, d))
    need = L.dip_swiglu_mlp_forward_workspace_bytes(C.byref(mlp), 16, 32)
    assert need > 0

    def call(mlp=mlp, k_in=16, k_mid=32, cin=None, cmid=None, gamma=0.2, ws=FAKE, wsb=1 << 24, x=FAKE, y=FAKE):
        return L.dip_swiglu_mlp_forward(C.byref(mlp), x, k_in, k_mid, cin, cmid, gamma, y, None, ws, wsb, None)

    assert call(k_in=0) == D.DIP_ERR_INVALID_ARG
    assert call(k_in=d + 1) == D.DIP_ERR_INVALID_ARG
    assert call(k_mid=f + 1) == D.DIP_ERR_INVALID_ARG
    assert call(x=None) == D.DIP_ERR_INVALID_ARG
    assert call(wsb=need - 1) == D.DIP_ERR_WORKSPACE
    bad = _Mlp(_weight(D, 1, d, 2 * f), _weight(D, 1, f + 8, d))
    assert call(mlp=bad) == D.DIP_ERR_INVALID_ARG                      # shapes do not chain
    c_ok = _Cache(FAKE, FAKE, FAKE, d, 32, 0, 0)
    c_badn = _Cache(FAKE, FAKE, FAKE, d + 1, 32, 0, 0)
    c_badcap = _Cache(FAKE, FAKE, FAKE, d, d + 1, 0, 0)
    c_null = _Cache(None, FAKE, FAKE, d, 32, 0, 0)
    assert call(cin=C.byref(c_badn)) == D.DIP_ERR_INVALID_ARG
    assert call(cin=C.byref(c_badcap)) == D.DIP_ERR_INVALID_ARG
    assert call(cin=C.byref(c_null)) == D.DIP_ERR_INVALID_ARG
    assert call(cin=C.byref(c_ok), gamma=2.0) == D.DIP_ERR_INVALID_ARG
    assert L.dip_swiglu_mlp_forward_workspace_bytes(C.byref(bad), 16, 32) == 0


def test_cache_argument_validation(D):
    from paper_2412_01380_amd.libdip import _Cache
    L = D.lib
    assert L.dip_cache_update(None, FAKE, None) == D.DIP_ERR_INVALID_ARG
    c = _Cache(FAKE, FAKE, FAKE, 100, 50, 0, 0)
    assert L.dip_cache_update(C.byref(c), None, None) == D.DIP_ERR_INVALID_ARG
    c2 = _Cache(FAKE, FAKE, FAKE, 100, 50, 5, 0)
    assert L.dip_cache_update(C.byref(c2), FAKE, None) == D.DIP_ERR_INVALID_ARG
    assert L.dip_cache_init(C.byref(c2), None, None) == D.DIP_ERR_INVALID_ARG
    c3 = _Cache(FAKE, FAKE, FAKE, D.DIP_MAX_N + 1, 50, 0, 0)
    assert L.dip_cache_init(C.byref(c3), None, None) == D.DIP_ERR_UNSUPPORTED


def test_cache_blob_sizes_and_validation(D):
    assert D.dip_cache_blob_bytes(0) == 0 and D.dip_cache_blob_bytes(D.DIP_MAX_N + 1) == 0
    assert D.dip_cache_blob_bytes(1000) == 256 + 4096 + 256      # 128 B of bits, 4000 B of stamps, 32 B of meta
    assert D.dip_cache_state_bytes(1000) == (128, 4000, 32)
    with pytest.raises(D.DipError):
        D.dip_cache_state_bytes(0)
    assert D.lib.dip_cache_export(None, None, 0, None) == D.DIP_ERR_INVALID_ARG
    assert D.lib.dip_cache_import(None, None, 0, None) == D.DIP_ERR_INVALID_ARG


def test_tune_validation(D):
    assert D.lib.dip_tune_gemv(7, 0, 0, 0) == D.DIP_ERR_INVALID_ARG
    assert D.lib.dip_tune_gemv(0, 3, 0, 0) == D.DIP_ERR_INVALID_ARG
    assert D.lib.dip_tune_gemv(0, 0, 0, 0) == D.DIP_OK


def test_one_cache_state_for_two_pruning_points_is_rejected(D):
    """A cache is scored in one launch and updated at the end of the call: two pruning points (or
    two layers) that share one state would read it while it changes.  Rejected on the host."""
    from paper_2412_01380_amd.libdip import _Cache, _Mlp
    L = D.lib
    d = f = 64                                  # equal widths, so one state fits both points
    mlp = _Mlp(_weight(D, 1, d, 2 * f), _weight(D, 1, f, d))
    c = _Cache(FAKE, FAKE, FAKE, d, 32, 0, 0)
    other = _Cache(FAKE + 4096, FAKE, FAKE, d, 32, 0, 0)
    args = (C.byref(mlp), FAKE, 16, 16)
    tail = (0.2, FAKE, None, FAKE, 1 << 24, None)
    assert L.dip_swiglu_mlp_forward(*args, C.byref(c), C.byref(c), *tail) == D.DIP_ERR_INVALID_ARG
    assert "share" in D.dip_last_error()
    # the batched call applies the same rule
    assert L.dip_swiglu_mlp_forward_batched(C.byref(mlp), FAKE, 2, 16, 16, C.byref(c), C.byref(c), 0.2, FAKE,
                                            None, None, None, FAKE, 1 << 26, None) == D.DIP_ERR_INVALID_ARG
    # two layers of a stack with the same state at point 1
    mlps = (_Mlp * 2)(mlp, mlp)
    cin = (_Cache * 2)(c, c)
    cmid = (_Cache * 2)(other, _Cache(FAKE + 8192, FAKE, FAKE, d, 32, 0, 0))
    k = (C.c_int32 * 2)(16, 16)
    assert L.dip_swiglu_mlp_forward_stack(mlps, 2, FAKE, d, k, k, cin, cmid, 0.2, FAKE, d, FAKE, 1 << 26,
                                          None) == D.DIP_ERR_INVALID_ARG


def test_stack_and_no_alloc_argument_validation(D):
    from paper_2412_01380_amd.libdip import _Mlp
    L = D.lib
    d, f = 64, 128
    mlp = _Mlp(_weight(D, 1, d, 2 * f), _weight(D, 1, f, d))
    mlps = (_Mlp * 2)(mlp, mlp)
    k_in, k_mid = (C.c_int32 * 2)(16, 16), (C.c_int32 * 2)(32, 200)
    # per-layer k: layer 1 asks for more than d_ff
    assert L.dip_swiglu_mlp_forward_stack_workspace_bytes(mlps, 2, k_in, k_mid) == 0
    assert L.dip_swiglu_mlp_forward_stack(mlps, 2, FAKE, d, k_in, k_mid, None, None, 0.2, FAKE, d, FAKE, 1 << 26,
                                          None) == D.DIP_ERR_INVALID_ARG
    k_mid = (C.c_int32 * 2)(32, 64)
    need = L.dip_swiglu_mlp_forward_stack_workspace_bytes(mlps, 2, k_in, k_mid)
    assert need > 0
    assert L.dip_swiglu_mlp_forward_stack(mlps, 2, FAKE, d, k_in, k_mid, None, None, 0.2, FAKE, d, FAKE, need - 1,
                                          None) == D.DIP_ERR_WORKSPACE
    assert L.dip_swiglu_mlp_forward_stack(mlps, 0, FAKE, d, k_in, k_mid, None, None, 0.2, FAKE, d, FAKE, need,
                                          None) == D.DIP_ERR_INVALID_ARG
    assert L.dip_swiglu_mlp_forward_stack(mlps, 2, FAKE, d, None, k_mid, None, None, 0.2, FAKE, d, FAKE, need,
                                          None) == D.DIP_ERR_INVALID_ARG
    assert L.dip_swiglu_mlp_forward_batched_stack_workspace_bytes(mlps, 2, 9, k_in, k_mid) == 0      # batch > 8
    assert L.dip_swiglu_mlp_forward_batched_stack(mlps, 2, FAKE, 8 * d, 9, k_in, k_mid, None, None, 0.2, FAKE,
                                                  8 * d, FAKE, 1 << 26, None) == D.DIP_ERR_INVALID_ARG
    # the entry point that allocates nothing: bad arguments and layers beyond its built-in buffer are
    # turned away before the runtime is touched
    assert L.dip_swiglu_mlp_forward_noalloc(C.byref(mlp), FAKE, 0, 32, None, None, 0.2, FAKE, None,
                                            None) == D.DIP_ERR_INVALID_ARG
    big = _Mlp(_weight(D, 0, 16384, 2 * 32768), _weight(D, 0, 32768, 16384))
    assert L.dip_swiglu_mlp_forward_workspace_bytes(C.byref(big), 8192, 16384) + 2 * 4096 > D.DIP_STATIC_SCRATCH_BYTES
    assert L.dip_swiglu_mlp_forward_noalloc(C.byref(big), FAKE, 8192, 16384, None, None, 0.2, FAKE, None,
                                            None) == D.DIP_ERR_WORKSPACE
    assert "built-in" in D.dip_last_error()
