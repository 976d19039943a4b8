"""Helpers shared by the GPU parity tests: host<->device marshalling and comparisons.
No method arithmetic lives here."""
import numpy as np
import torch


def bits_from_bool(m: np.ndarray) -> np.ndarray:
    """bool[n] -> uint32 words, feature i = bit (i & 31) of word (i >> 5)."""
    n = m.shape[0]
    pad = (-n) % 32
    b = np.concatenate([m.astype(np.uint8), np.zeros(pad, dtype=np.uint8)])
    return np.packbits(b, bitorder="little").view(np.uint32).copy()


def bool_from_bits(words: np.ndarray, n: int) -> np.ndarray:
    w = np.ascontiguousarray(words).view(np.uint8)
    return np.unpackbits(w, bitorder="little")[:n].astype(bool)


def dev_u32(words: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(words.view(np.int32).copy()).cuda()


def host_u32(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint32)


def dev_f32(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def dev_weight(w):
    """fp32 array, uint16 bf16 bit patterns, or an int4 (codes, scales) pair -> what
    paper_2412_01380_amd.Weight(...) accepts (a tensor, or a (codes, scales) tuple of tensors)."""
    if isinstance(w, tuple):
        return (torch.from_numpy(w[0]).cuda(), torch.from_numpy(w[1]).cuda())
    if w.dtype == np.uint16:
        return torch.from_numpy(w.view(np.int16).copy()).cuda()
    return torch.from_numpy(np.ascontiguousarray(w, dtype=np.float32)).cuda()


def rel_l2(a, b) -> float:
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def workspace(nbytes: int) -> torch.Tensor:
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")


def make_weight(D, w):
    """Device Weight descriptor for any stored format of workloads.layer_weights."""
    t = dev_weight(w)
    return D.Weight(*t) if isinstance(t, tuple) else D.Weight(t)
