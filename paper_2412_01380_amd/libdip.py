"""ctypes binding of libdip.so: same names as the C ABI (include/dip.h), torch tensors in.

PyTorch is used for device memory and streams only.  Tensors must live on the GPU, be
contiguous and have the dtype the C signature states; the binding passes their data
pointers through unchanged.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
# DIP_LIBRARY points the binding at another build of the same ABI (e.g. an instrumented one)
lib_path = os.environ.get("DIP_LIBRARY") or os.path.join(HERE, "lib", "libdip.so")

DIP_OK, DIP_ERR_INVALID_ARG, DIP_ERR_UNSUPPORTED, DIP_ERR_WORKSPACE, DIP_ERR_HIP = range(5)
DIP_F32, DIP_BF16, DIP_INT4_G128 = 0, 1, 2
DIP_LRU, DIP_LFU = 0, 1
DIP_GATE_PRUNING, DIP_UP_PRUNING = 1, 2
DIP_MAX_N = 32768
DIP_CACHE_META_WORDS = 8
META = {"step": 0, "resident": 1, "hits": 2, "inserted": 3, "evicted": 4, "bypassed": 5,
        "cum_hits": 6, "cum_lookups": 7}


class DipError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"libdip status {status}: {msg}")
        self.status = status


class _Weight(C.Structure):
    _fields_ = [("data", C.c_void_p), ("scales", C.c_void_p), ("dtype", C.c_int32),
                ("n_in", C.c_int32), ("n_out", C.c_int32), ("reserved", C.c_int32),
                ("row_stride_bytes", C.c_int64)]


class _Mlp(C.Structure):
    _fields_ = [("w_ug", _Weight), ("w_d", _Weight)]


class _Cache(C.Structure):
    _fields_ = [("bits", C.c_void_p), ("stamp", C.c_void_p), ("meta", C.c_void_p),
                ("n", C.c_int32), ("capacity", C.c_int32), ("policy", C.c_int32),
                ("reserved", C.c_int32)]


class _Debug(C.Structure):
    _fields_ = [("s_in", C.c_void_p), ("mask_in", C.c_void_p), ("idx_in", C.c_void_p),
                ("h", C.c_void_p), ("s_mid", C.c_void_p), ("mask_mid", C.c_void_p),
                ("idx_mid", C.c_void_p)]


class _MlpSplit(C.Structure):
    _fields_ = [("w_dense", _Weight), ("w_rows", _Weight), ("w_d", _Weight)]


class _PartialDebug(C.Structure):
    _fields_ = [("a", C.c_void_p), ("mask", C.c_void_p), ("idx", C.c_void_p), ("h_sel", C.c_void_p)]


class _TieredWeight(C.Structure):
    _fields_ = [("full", _Weight), ("slots", C.c_void_p), ("slot_of", C.c_void_p),
                ("capacity", C.c_int32), ("reserved", C.c_int32)]


class _TieredMlp(C.Structure):
    _fields_ = [("w_ug", _TieredWeight), ("w_d", _TieredWeight)]


def _load() -> C.CDLL:
    if not os.path.exists(lib_path):
        raise ImportError(
            f"{lib_path} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()' "
            "or python paper_2412_01380_amd/build.py). There is no fallback path.")
    L = C.CDLL(lib_path)
    vp, i32, i64, f32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_size_t
    L.dip_version.restype = i32
    L.dip_version.argtypes = []
    L.dip_last_error.restype = C.c_char_p
    L.dip_last_error.argtypes = []
    L.dip_ca_scores.restype = i32
    L.dip_ca_scores.argtypes = [vp, i32, vp, f32, vp, vp]
    L.dip_prune_topk.restype = i32
    L.dip_prune_topk.argtypes = [vp, i32, i32, vp, vp, vp]
    L.dip_cache_init.restype = i32
    L.dip_cache_init.argtypes = [C.POINTER(_Cache), vp, vp]
    L.dip_cache_update.restype = i32
    L.dip_cache_update.argtypes = [C.POINTER(_Cache), vp, vp]
    L.dip_cache_state_bytes.restype = i32
    L.dip_cache_state_bytes.argtypes = [i32, C.POINTER(sz), C.POINTER(sz), C.POINTER(sz)]
    L.dip_cache_blob_bytes.restype = sz
    L.dip_cache_blob_bytes.argtypes = [i32]
    L.dip_cache_export.restype = i32
    L.dip_cache_export.argtypes = [C.POINTER(_Cache), vp, sz, vp]
    L.dip_cache_import.restype = i32
    L.dip_cache_import.argtypes = [C.POINTER(_Cache), vp, sz, vp]
    L.dip_gathered_gemv_workspace_bytes.restype = sz
    L.dip_gathered_gemv_workspace_bytes.argtypes = [C.POINTER(_Weight), i32]
    L.dip_gathered_gemv.restype = i32
    L.dip_gathered_gemv.argtypes = [C.POINTER(_Weight), vp, vp, i32, vp, vp, sz, vp]
    L.dip_swiglu_mlp_forward_workspace_bytes.restype = sz
    L.dip_swiglu_mlp_forward_workspace_bytes.argtypes = [C.POINTER(_Mlp), i32, i32]
    L.dip_swiglu_mlp_forward.restype = i32
    L.dip_swiglu_mlp_forward.argtypes = [C.POINTER(_Mlp), vp, i32, i32, C.POINTER(_Cache),
                                         C.POINTER(_Cache), f32, vp, C.POINTER(_Debug), vp, sz, vp]
    L.dip_swiglu_mlp_forward_noalloc.restype = i32
    L.dip_swiglu_mlp_forward_noalloc.argtypes = [C.POINTER(_Mlp), vp, i32, i32, C.POINTER(_Cache),
                                                 C.POINTER(_Cache), f32, vp, C.POINTER(_Debug), vp]
    L.dip_swiglu_mlp_forward_stack.restype = i32
    L.dip_swiglu_mlp_forward_stack.argtypes = [C.POINTER(_Mlp), i32, vp, i64, C.POINTER(i32), C.POINTER(i32),
                                               C.POINTER(_Cache), C.POINTER(_Cache), f32, vp, i64,
                                               vp, sz, vp]
    L.dip_swiglu_mlp_forward_stack_workspace_bytes.restype = sz
    L.dip_swiglu_mlp_forward_stack_workspace_bytes.argtypes = [C.POINTER(_Mlp), i32, C.POINTER(i32), C.POINTER(i32)]
    L.dip_swiglu_mlp_forward_batched_workspace_bytes.restype = sz
    L.dip_swiglu_mlp_forward_batched_workspace_bytes.argtypes = [C.POINTER(_Mlp), i32, i32, i32]
    L.dip_swiglu_mlp_forward_batched.restype = i32
    L.dip_swiglu_mlp_forward_batched.argtypes = [C.POINTER(_Mlp), vp, i32, i32, i32, C.POINTER(_Cache),
                                                 C.POINTER(_Cache), f32, vp, vp, vp, vp, vp, sz, vp]
    L.dip_swiglu_mlp_forward_batched_stack_workspace_bytes.restype = sz
    L.dip_swiglu_mlp_forward_batched_stack_workspace_bytes.argtypes = [C.POINTER(_Mlp), i32, i32, C.POINTER(i32),
                                                                       C.POINTER(i32)]
    L.dip_swiglu_mlp_forward_batched_stack.restype = i32
    L.dip_swiglu_mlp_forward_batched_stack.argtypes = [C.POINTER(_Mlp), i32, vp, i64, i32, C.POINTER(i32),
                                                       C.POINTER(i32), C.POINTER(_Cache), C.POINTER(_Cache), f32,
                                                       vp, i64, vp, sz, vp]
    L.dip_glu_pruning_forward_workspace_bytes.restype = sz
    L.dip_glu_pruning_forward_workspace_bytes.argtypes = [C.POINTER(_Mlp), i32]
    L.dip_glu_pruning_forward.restype = i32
    L.dip_glu_pruning_forward.argtypes = [C.POINTER(_Mlp), vp, i32, vp, C.POINTER(_Debug), vp, sz, vp]
    L.dip_gathered_rowdot.restype = i32
    L.dip_gathered_rowdot.argtypes = [C.POINTER(_Weight), vp, vp, i32, vp, vp]
    L.dip_partial_pruning_forward_workspace_bytes.restype = sz
    L.dip_partial_pruning_forward_workspace_bytes.argtypes = [C.POINTER(_MlpSplit), i32]
    L.dip_partial_pruning_forward.restype = i32
    L.dip_partial_pruning_forward.argtypes = [C.POINTER(_MlpSplit), i32, vp, i32, vp,
                                              C.POINTER(_PartialDebug), vp, sz, vp]
    L.dip_tier_init_workspace_bytes.restype = sz
    L.dip_tier_init_workspace_bytes.argtypes = [C.POINTER(_TieredWeight)]
    L.dip_tier_init.restype = i32
    L.dip_tier_init.argtypes = [C.POINTER(_TieredWeight), C.POINTER(_Cache), vp, sz, vp]
    L.dip_tiered_mlp_forward_workspace_bytes.restype = sz
    L.dip_tiered_mlp_forward_workspace_bytes.argtypes = [C.POINTER(_TieredMlp), i32, i32]
    L.dip_tiered_mlp_forward.restype = i32
    L.dip_tiered_mlp_forward.argtypes = [C.POINTER(_TieredMlp), vp, i32, i32, C.POINTER(_Cache),
                                         C.POINTER(_Cache), f32, vp, C.POINTER(_Debug), vp, sz, vp]
    L.dip_tune_gemv.restype = i32
    L.dip_tune_gemv.argtypes = [i32, i32, i32, i32]
    L.dip_gemv_launch_shape.restype = i32
    L.dip_gemv_launch_shape.argtypes = [C.POINTER(_Weight), i32, i32, C.POINTER(i32)]
    L.dip_set_fusion.restype = i32
    L.dip_set_fusion.argtypes = [i32]
    L.dip_fused_launch_shape.restype = i32
    L.dip_fused_launch_shape.argtypes = [C.POINTER(_Weight), i32, i32, C.POINTER(i32)]
    L.dip_stream_read.restype = i32
    L.dip_stream_read.argtypes = [vp, sz, vp, vp]
    L.dip_profile_enable.restype = i32
    L.dip_profile_enable.argtypes = [i32]
    L.dip_profile_read.restype = i32
    L.dip_profile_read.argtypes = [i32, C.POINTER(C.c_double), C.POINTER(i32)]
    L.dip_profile_disable.restype = i32
    L.dip_profile_disable.argtypes = []
    return L


lib = _load()

EXPORTS = ["dip_version", "dip_last_error", "dip_ca_scores", "dip_prune_topk", "dip_cache_init",
           "dip_cache_update", "dip_cache_state_bytes", "dip_cache_blob_bytes", "dip_cache_export",
           "dip_cache_import", "dip_gathered_gemv_workspace_bytes", "dip_gathered_gemv",
           "dip_swiglu_mlp_forward_workspace_bytes", "dip_swiglu_mlp_forward",
           "dip_swiglu_mlp_forward_noalloc", "dip_swiglu_mlp_forward_stack",
           "dip_swiglu_mlp_forward_stack_workspace_bytes", "dip_swiglu_mlp_forward_batched_workspace_bytes",
           "dip_swiglu_mlp_forward_batched", "dip_swiglu_mlp_forward_batched_stack_workspace_bytes",
           "dip_swiglu_mlp_forward_batched_stack", "dip_glu_pruning_forward_workspace_bytes",
           "dip_glu_pruning_forward", "dip_gathered_rowdot",
           "dip_partial_pruning_forward_workspace_bytes", "dip_partial_pruning_forward", "dip_tier_init_workspace_bytes",
           "dip_tier_init", "dip_tiered_mlp_forward_workspace_bytes", "dip_tiered_mlp_forward", "dip_tune_gemv", "dip_gemv_launch_shape", "dip_set_fusion", "dip_fused_launch_shape", "dip_stream_read", "dip_profile_enable", "dip_profile_read",
           "dip_profile_disable"]


def dip_last_error() -> str:
    return lib.dip_last_error().decode()


def _check(st: int) -> None:
    if st != DIP_OK:
        raise DipError(st, dip_last_error())


def _ptr(t, dtype=None) -> Optional[int]:
    """Device pointer of a torch tensor (None -> NULL)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda:
        raise TypeError("libdip takes device tensors")
    if not t.is_contiguous():
        raise TypeError("libdip takes contiguous tensors")
    if dtype is not None and t.dtype not in (dtype if isinstance(dtype, tuple) else (dtype,)):
        raise TypeError(f"expected dtype {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    import torch
    if stream is None:
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


class Weight:
    """A feature-major weight matrix on the device: tensor [n_in][n_out], fp32 or bf16
    (bf16 may be given as torch.bfloat16, int16 or uint16 holding the bit patterns), or
    int4-g128: `data` uint8 [n_in][n_out/2] (low nibble = even element) with `scales`
    float16 [n_in][n_out/128]."""

    def __init__(self, data, scales=None):
        import torch
        if data.dim() != 2 or not data.is_cuda or data.stride(1) != 1:
            raise TypeError("weight must be a 2-D device tensor with unit inner stride")
        n_out = data.shape[1]
        sptr = None
        if scales is not None:
            if data.dtype != torch.uint8 or scales.dtype != torch.float16:
                raise TypeError("int4 weights are uint8 codes with float16 scales")
            n_out = data.shape[1] * 2
            if (not scales.is_cuda or not scales.is_contiguous()
                    or tuple(scales.shape) != (data.shape[0], n_out // 128)):
                raise TypeError("scales must be a contiguous device tensor [n_in][n_out/128]")
            dt = DIP_INT4_G128
            sptr = scales.data_ptr()
        elif data.dtype == torch.float32:
            dt = DIP_F32
        elif data.dtype in (torch.bfloat16, torch.int16, torch.uint16):
            dt = DIP_BF16
        else:
            raise TypeError(f"unsupported weight dtype {data.dtype}")
        self.tensor, self.scales = data, scales
        self.c = _Weight(data.data_ptr(), sptr, dt, data.shape[0], n_out, 0,
                         data.stride(0) * data.element_size())


class Mlp:
    """w_ug: bundled up/gate [d_model][2*d_ff]; w_d: down [d_ff][d_model] (feature-major)."""

    def __init__(self, w_ug: Weight, w_d: Weight):
        self.w_ug, self.w_d = w_ug, w_d
        self.c = _Mlp(w_ug.c, w_d.c)
        self.d_model = w_ug.c.n_in
        self.d_ff = w_d.c.n_in


class Cache:
    """Residency state of one layer's columns, held in caller-owned device tensors."""

    def __init__(self, n: int, capacity: int, policy: int = DIP_LRU, device="cuda"):
        import torch
        self.n, self.capacity, self.policy = n, capacity, policy
        self.bits = torch.zeros((n + 31) // 32, dtype=torch.int32, device=device)
        self.stamp = torch.zeros(n, dtype=torch.int32, device=device)
        self.meta = torch.zeros(DIP_CACHE_META_WORDS, dtype=torch.int32, device=device)
        self.c = _Cache(self.bits.data_ptr(), self.stamp.data_ptr(), self.meta.data_ptr(), n,
                        capacity, policy, 0)

    def meta_host(self) -> dict:
        m = self.meta.cpu().numpy().view("uint32")
        return {k: int(m[i]) for k, i in META.items()}


class Debug:
    """Stage outputs of one forward call (device tensors allocated by the caller)."""

    def __init__(self, d_model: int, d_ff: int, k_in: int, k_mid: int, device="cuda"):
        import torch
        self.s_in = torch.empty(d_model, dtype=torch.float32, device=device)
        self.mask_in = torch.empty((d_model + 31) // 32, dtype=torch.int32, device=device)
        self.idx_in = torch.empty(k_in, dtype=torch.int32, device=device)
        self.h = torch.empty(d_ff, dtype=torch.float32, device=device)
        self.s_mid = torch.empty(d_ff, dtype=torch.float32, device=device)
        self.mask_mid = torch.empty((d_ff + 31) // 32, dtype=torch.int32, device=device)
        self.idx_mid = torch.empty(k_mid, dtype=torch.int32, device=device)
        self.c = _Debug(self.s_in.data_ptr(), self.mask_in.data_ptr(), self.idx_in.data_ptr(),
                        self.h.data_ptr(), self.s_mid.data_ptr(), self.mask_mid.data_ptr(),
                        self.idx_mid.data_ptr())


class MlpSplit:
    """Matrices for gate / up pruning: w_dense feature-major [d_model][d_ff] (W^g for gate
    pruning, W^u for up pruning), w_rows neuron-major [d_ff][d_model] (the other one of the
    pair), w_d feature-major [d_ff][d_model]."""

    def __init__(self, w_dense: Weight, w_rows: Weight, w_d: Weight):
        self.w_dense, self.w_rows, self.w_d = w_dense, w_rows, w_d
        self.c = _MlpSplit(w_dense.c, w_rows.c, w_d.c)
        self.d_model = w_dense.c.n_in
        self.d_ff = w_dense.c.n_out


class PartialDebug:
    """Stage outputs of dip_partial_pruning_forward (device tensors allocated by the caller)."""

    def __init__(self, d_ff: int, k: int, device="cuda"):
        import torch
        self.a = torch.empty(d_ff, dtype=torch.float32, device=device)
        self.mask = torch.empty((d_ff + 31) // 32, dtype=torch.int32, device=device)
        self.idx = torch.empty(k, dtype=torch.int32, device=device)
        self.h_sel = torch.empty(k, dtype=torch.float32, device=device)
        self.c = _PartialDebug(self.a.data_ptr(), self.mask.data_ptr(), self.idx.data_ptr(),
                               self.h_sel.data_ptr())


class TieredWeight:
    """A matrix in two tiers: `host` is the whole feature-major matrix in pinned host memory
    (fp32, or bf16 given as bfloat16 / int16 / uint16 bit patterns), `capacity` rows of HBM
    are its cache.  The slot map lives on the device."""

    def __init__(self, host, capacity: int, device="cuda"):
        import torch
        if host.is_cuda or not host.is_pinned() or host.dim() != 2 or host.stride(1) != 1:
            raise TypeError("the slow tier must be a 2-D pinned host tensor with unit inner stride")
        if host.dtype == torch.float32:
            dt = DIP_F32
        elif host.dtype in (torch.bfloat16, torch.int16, torch.uint16):
            dt = DIP_BF16
        else:
            raise TypeError(f"unsupported tier dtype {host.dtype}")
        self.host, self.capacity = host, capacity
        self.slots = torch.zeros((max(capacity, 1), host.shape[1]), dtype=host.dtype, device=device)
        self.slot_of = torch.full((host.shape[0],), -1, dtype=torch.int32, device=device)
        stride = host.stride(0) * host.element_size()
        # pinned host memory is mapped into the device's address space at the same address
        full = _Weight(host.data_ptr(), None, dt, host.shape[0], host.shape[1], 0, stride)
        self.c = _TieredWeight(full, self.slots.data_ptr(), self.slot_of.data_ptr(), capacity, 0)


class TieredMlp:
    def __init__(self, w_ug: TieredWeight, w_d: TieredWeight):
        self.w_ug, self.w_d = w_ug, w_d
        self.c = _TieredMlp(w_ug.c, w_d.c)
        self.d_model = w_ug.c.full.n_in
        self.d_ff = w_d.c.full.n_in


def dip_version() -> int:
    return lib.dip_version()


def dip_ca_scores(x, n: int, cache_bits, gamma: float, s_out, stream=None) -> None:
    import torch
    _check(lib.dip_ca_scores(_ptr(x, torch.float32), n, _ptr(cache_bits, torch.int32), gamma,
                             _ptr(s_out, torch.float32), _stream(stream)))


def dip_prune_topk(s, n: int, k: int, mask_out, idx_out, stream=None) -> None:
    import torch
    _check(lib.dip_prune_topk(_ptr(s, torch.float32), n, k, _ptr(mask_out, torch.int32),
                              _ptr(idx_out, torch.int32), _stream(stream)))


def dip_cache_init(cache: Cache, initial_bits=None, stream=None) -> None:
    import torch
    _check(lib.dip_cache_init(C.byref(cache.c), _ptr(initial_bits, torch.int32), _stream(stream)))


def dip_cache_update(cache: Cache, mask_bits, stream=None) -> None:
    import torch
    _check(lib.dip_cache_update(C.byref(cache.c), _ptr(mask_bits, torch.int32), _stream(stream)))


def dip_cache_state_bytes(n: int):
    """(bits, stamp, meta) array sizes in bytes for a cache over n columns."""
    b, s_, m = C.c_size_t(0), C.c_size_t(0), C.c_size_t(0)
    _check(lib.dip_cache_state_bytes(n, C.byref(b), C.byref(s_), C.byref(m)))
    return b.value, s_.value, m.value


def dip_cache_blob_bytes(n: int) -> int:
    return lib.dip_cache_blob_bytes(n)


def _blob_ptr(blob):
    """Device tensor or (pinned) host tensor -> raw pointer; the C side copies with hipMemcpyDefault."""
    if not blob.is_contiguous():
        raise TypeError("blob must be contiguous")
    return blob.data_ptr()


def dip_cache_export(cache: Cache, blob, stream=None) -> None:
    _check(lib.dip_cache_export(C.byref(cache.c), _blob_ptr(blob), blob.numel() * blob.element_size(),
                                _stream(stream)))


def dip_cache_import(cache: Cache, blob, stream=None) -> None:
    _check(lib.dip_cache_import(C.byref(cache.c), _blob_ptr(blob), blob.numel() * blob.element_size(),
                                _stream(stream)))


def dip_gathered_gemv_workspace_bytes(w: Weight, k: int) -> int:
    return lib.dip_gathered_gemv_workspace_bytes(C.byref(w.c), k)


def dip_gathered_gemv(w: Weight, x, idx, k: int, y_out, ws, stream=None) -> None:
    import torch
    _check(lib.dip_gathered_gemv(C.byref(w.c), _ptr(x, torch.float32), _ptr(idx, torch.int32), k,
                                 _ptr(y_out, torch.float32), _ptr(ws), ws.numel() * ws.element_size(),
                                 _stream(stream)))


def dip_swiglu_mlp_forward_workspace_bytes(mlp: Mlp, k_in: int, k_mid: int) -> int:
    return lib.dip_swiglu_mlp_forward_workspace_bytes(C.byref(mlp.c), k_in, k_mid)


def dip_swiglu_mlp_forward(mlp: Mlp, x, k_in: int, k_mid: int, cache_in: Optional[Cache],
                           cache_mid: Optional[Cache], gamma: float, y_out, dbg: Optional[Debug],
                           ws, stream=None) -> None:
    import torch
    _check(lib.dip_swiglu_mlp_forward(
        C.byref(mlp.c), _ptr(x, torch.float32), k_in, k_mid,
        C.byref(cache_in.c) if cache_in is not None else None,
        C.byref(cache_mid.c) if cache_mid is not None else None,
        gamma, _ptr(y_out, torch.float32), C.byref(dbg.c) if dbg is not None else None,
        _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))


DIP_STATIC_SCRATCH_BYTES = 4 << 20


def dip_swiglu_mlp_forward_noalloc(mlp: Mlp, x, k_in: int, k_mid: int, cache_in: Optional[Cache],
                                   cache_mid: Optional[Cache], gamma: float, y_out,
                                   dbg: Optional[Debug], stream=None) -> None:
    import torch
    _check(lib.dip_swiglu_mlp_forward_noalloc(
        C.byref(mlp.c), _ptr(x, torch.float32), k_in, k_mid,
        C.byref(cache_in.c) if cache_in is not None else None,
        C.byref(cache_mid.c) if cache_mid is not None else None,
        gamma, _ptr(y_out, torch.float32), C.byref(dbg.c) if dbg is not None else None,
        _stream(stream)))


class MlpStack:
    """Host arrays of descriptors for dip_swiglu_mlp_forward_stack (built once, reused)."""

    def __init__(self, mlps: Sequence[Mlp], caches_in: Optional[Sequence[Cache]] = None,
                 caches_mid: Optional[Sequence[Cache]] = None):
        n = len(mlps)
        self.n = n
        self.mlps = (_Mlp * n)(*[m.c for m in mlps])
        self.cin = (_Cache * n)(*[c.c for c in caches_in]) if caches_in else None
        self.cmid = (_Cache * n)(*[c.c for c in caches_mid]) if caches_mid else None
        self._keep = (list(mlps), caches_in, caches_mid)


def _k_array(k, n: int):
    """One k for all layers, or a sequence of n_layers values -> a host int32 array."""
    vals = [int(k)] * n if isinstance(k, int) else [int(v) for v in k]
    if len(vals) != n:
        raise ValueError(f"expected {n} values of k, got {len(vals)}")
    return (C.c_int32 * n)(*vals)


def dip_swiglu_mlp_forward_stack_workspace_bytes(stack: MlpStack, k_in, k_mid) -> int:
    return lib.dip_swiglu_mlp_forward_stack_workspace_bytes(stack.mlps, stack.n, _k_array(k_in, stack.n),
                                                            _k_array(k_mid, stack.n))


def dip_swiglu_mlp_forward_stack(stack: MlpStack, x, x_stride: int, k_in, k_mid,
                                 gamma: float, y_out, y_stride: int, ws, stream=None) -> None:
    """k_in / k_mid: an int for all layers, a sequence of per-layer values, or a ctypes int32 array."""
    import torch
    ki = k_in if isinstance(k_in, C.Array) else _k_array(k_in, stack.n)
    km = k_mid if isinstance(k_mid, C.Array) else _k_array(k_mid, stack.n)
    _check(lib.dip_swiglu_mlp_forward_stack(
        stack.mlps, stack.n, _ptr(x, torch.float32), x_stride, ki, km, stack.cin, stack.cmid,
        gamma, _ptr(y_out, torch.float32), y_stride, _ptr(ws), ws.numel() * ws.element_size(),
        _stream(stream)))


def dip_swiglu_mlp_forward_batched_workspace_bytes(mlp: Mlp, batch: int, k_in: int, k_mid: int) -> int:
    return lib.dip_swiglu_mlp_forward_batched_workspace_bytes(C.byref(mlp.c), batch, k_in, k_mid)


def dip_swiglu_mlp_forward_batched(mlp: Mlp, X, batch: int, k_in: int, k_mid: int,
                                   cache_in: Optional[Cache], cache_mid: Optional[Cache], gamma: float,
                                   Y, mask_in_out, h_out, mask_mid_out, ws, stream=None) -> None:
    import torch
    _check(lib.dip_swiglu_mlp_forward_batched(
        C.byref(mlp.c), _ptr(X, torch.float32), batch, k_in, k_mid,
        C.byref(cache_in.c) if cache_in is not None else None,
        C.byref(cache_mid.c) if cache_mid is not None else None,
        gamma, _ptr(Y, torch.float32), _ptr(mask_in_out, torch.int32), _ptr(h_out, torch.float32),
        _ptr(mask_mid_out, torch.int32), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))


def dip_swiglu_mlp_forward_batched_stack_workspace_bytes(stack: MlpStack, batch: int, k_in, k_mid) -> int:
    return lib.dip_swiglu_mlp_forward_batched_stack_workspace_bytes(stack.mlps, stack.n, batch, _k_array(k_in, stack.n),
                                                                    _k_array(k_mid, stack.n))


def dip_swiglu_mlp_forward_batched_stack(stack: MlpStack, X, x_stride: int, batch: int, k_in, k_mid, gamma: float,
                                         Y, y_stride: int, ws, stream=None) -> None:
    """X: [n_layers][batch][d_model] (layer stride x_stride floats), Y likewise; k as in the stack call."""
    import torch
    ki = k_in if isinstance(k_in, C.Array) else _k_array(k_in, stack.n)
    km = k_mid if isinstance(k_mid, C.Array) else _k_array(k_mid, stack.n)
    _check(lib.dip_swiglu_mlp_forward_batched_stack(
        stack.mlps, stack.n, _ptr(X, torch.float32), x_stride, batch, ki, km, stack.cin, stack.cmid, gamma,
        _ptr(Y, torch.float32), y_stride, _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))


def dip_glu_pruning_forward_workspace_bytes(mlp: Mlp, k: int) -> int:
    return lib.dip_glu_pruning_forward_workspace_bytes(C.byref(mlp.c), k)


def dip_glu_pruning_forward(mlp: Mlp, x, k: int, y_out, dbg, ws, stream=None) -> None:
    """dbg: a ctypes _Debug whose point-1 members are NULL (see glu_debug), or None."""
    import torch
    _check(lib.dip_glu_pruning_forward(
        C.byref(mlp.c), _ptr(x, torch.float32), k, _ptr(y_out, torch.float32),
        C.byref(dbg) if dbg is not None else None, _ptr(ws), ws.numel() * ws.element_size(),
        _stream(stream)))


def glu_debug(h=None, s_mid=None, mask_mid=None, idx_mid=None) -> _Debug:
    """Debug descriptor for dip_glu_pruning_forward: only the point-2 members exist."""
    import torch
    return _Debug(None, None, None, _ptr(h, torch.float32), _ptr(s_mid, torch.float32),
                  _ptr(mask_mid, torch.int32), _ptr(idx_mid, torch.int32))


def dip_gathered_rowdot(w_rows: Weight, x, idx, k: int, out, stream=None) -> None:
    import torch
    _check(lib.dip_gathered_rowdot(C.byref(w_rows.c), _ptr(x, torch.float32), _ptr(idx, torch.int32),
                                   k, _ptr(out, torch.float32), _stream(stream)))


def dip_partial_pruning_forward_workspace_bytes(mlp: MlpSplit, k: int) -> int:
    return lib.dip_partial_pruning_forward_workspace_bytes(C.byref(mlp.c), k)


def dip_partial_pruning_forward(mlp: MlpSplit, scheme: int, x, k: int, y_out,
                                dbg: Optional[PartialDebug], ws, stream=None) -> None:
    import torch
    _check(lib.dip_partial_pruning_forward(
        C.byref(mlp.c), scheme, _ptr(x, torch.float32), k, _ptr(y_out, torch.float32),
        C.byref(dbg.c) if dbg is not None else None, _ptr(ws), ws.numel() * ws.element_size(),
        _stream(stream)))


def dip_tier_init_workspace_bytes(tw: TieredWeight) -> int:
    return lib.dip_tier_init_workspace_bytes(C.byref(tw.c))


def dip_tier_init(tw: TieredWeight, cache: Cache, ws, stream=None) -> None:
    _check(lib.dip_tier_init(C.byref(tw.c), C.byref(cache.c), _ptr(ws), ws.numel() * ws.element_size(),
                             _stream(stream)))


def dip_tiered_mlp_forward_workspace_bytes(mlp: TieredMlp, k_in: int, k_mid: int) -> int:
    return lib.dip_tiered_mlp_forward_workspace_bytes(C.byref(mlp.c), k_in, k_mid)


def dip_tiered_mlp_forward(mlp: TieredMlp, x, k_in: int, k_mid: int, cache_in: Cache, cache_mid: Cache,
                           gamma: float, y_out, dbg: Optional[Debug], ws, stream=None) -> None:
    import torch
    _check(lib.dip_tiered_mlp_forward(
        C.byref(mlp.c), _ptr(x, torch.float32), k_in, k_mid, C.byref(cache_in.c), C.byref(cache_mid.c),
        gamma, _ptr(y_out, torch.float32), C.byref(dbg.c) if dbg is not None else None,
        _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))


def dip_tune_gemv(lanes_per_row: int = 0, waves: int = 0, ksplit: int = 0, unroll: int = 0) -> None:
    _check(lib.dip_tune_gemv(lanes_per_row, waves, ksplit, unroll))


def dip_gemv_launch_shape(w: Weight, k: int, bundled: bool = False):
    """(lanes_per_row, waves, ksplit, unroll) the library would launch with."""
    out = (C.c_int32 * 4)()
    _check(lib.dip_gemv_launch_shape(C.byref(w.c), k, 1 if bundled else 0, out))
    return tuple(out)


def dip_set_fusion(on: bool) -> None:
    _check(lib.dip_set_fusion(1 if on else 0))


def dip_fused_launch_shape(w: Weight, k: int, bundled: bool = False):
    """(lanes_per_row, waves, ksplit, unroll) of the one-launch form, or None when the forward
    calls launch selection and product apart for this shape."""
    out = (C.c_int32 * 4)()
    st = lib.dip_fused_launch_shape(C.byref(w.c), k, 1 if bundled else 0, out)
    if st == DIP_ERR_UNSUPPORTED:
        return None
    _check(st)
    return tuple(out)


def dip_stream_read(src, sink, stream=None) -> None:
    """Plain streaming read of the whole tensor `src` (timed as profile kind 8)."""
    _check(lib.dip_stream_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream(stream)))


def dip_profile_enable(max_launches: int) -> None:
    _check(lib.dip_profile_enable(max_launches))


def dip_profile_read(kind: int):
    """(total milliseconds, launches) of one kernel kind since dip_profile_enable()."""
    ms, n = C.c_double(0.0), C.c_int32(0)
    _check(lib.dip_profile_read(kind, C.byref(ms), C.byref(n)))
    return ms.value, n.value


def dip_profile_disable() -> None:
    _check(lib.dip_profile_disable())
