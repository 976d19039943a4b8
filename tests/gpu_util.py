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


# ---- float comparisons of a product of k selected rows --------------------------------------
NORTH_STAR = {"f32": 1e-5, "bf16": 2e-3, "int4": 2e-3}   # the stated bars (rel-L2)
VECTOR_BAR = 1e-5   # fp32 FMAs over exactly widened weights land near 1e-7 in every format:
                    # a regression bar 100x above that, 200x below the bf16 / int4 bar


def elem_bound(k: int) -> float:
    """Per-element error of an fp32 running sum of k products, relative to the largest output:
    each of the k roundings is at most 2^-24 of a partial sum no larger (up to a small factor)
    than the largest output, and they add like a random walk: c = 4 sqrt(k) 2^-24 (+ a few ulp
    for the conversions and the epilogue).  One selected row dropped from one strip moves an
    element by about 1/(4 sqrt(k)) of the largest output -- thousands of times this bound."""
    return (4.0 * np.sqrt(float(k)) + 8.0) * 2.0 ** -24


def assert_product_close(got, ref, fmt: str, k: int, what="", vector=True, scale=None, factor=1.0):
    """rel-L2 within the stated bar (and within VECTOR_BAR on the vector-ALU paths), and every
    element within elem_bound(k) of the reference, in units of `scale` (default: max |ref|)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    top = float(np.max(np.abs(ref), initial=0.0)) if scale is None else float(scale)
    if top < 1e-30:      # down in the denormal range single roundings are as large as the values
        assert float(np.max(np.abs(got), initial=0.0)) < 1e-29, what
        return 0.0
    e = rel_l2(got, ref)
    assert e <= NORTH_STAR[fmt], (what, "rel-L2", e)
    if vector:
        assert e <= VECTOR_BAR, (what, "rel-L2 (vector path)", e)
    worst = float(np.max(np.abs(got - ref)))
    bound = factor * elem_bound(k) * top
    assert worst <= bound, (what, "max |diff|", worst, "bound", bound)
    return e


def glu_scale(preacts) -> float:
    """Scale for the element bound of h = u * SiLU(g) from the reference pre-activations
    [u ; g]: both factors carry a sum's error, so the unit is max|u| * max|SiLU(g)|."""
    p = np.asarray(preacts, dtype=np.float64)
    f = p.shape[0] // 2
    u, g = p[:f], p[f:]
    return float(np.max(np.abs(u), initial=0.0) * np.max(np.abs(g / (1.0 + np.exp(-g))), initial=0.0))
