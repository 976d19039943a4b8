"""Seeded random sweeps of the selection kernel against the oracle: vector lengths anywhere in
[1, 32768] (every instantiation of the kernel, ragged tails), keep counts anywhere in [1, n],
value distributions with and without ties, scores with and without a residency mask, and
cache updates with random capacities and both policies.  Everything here is bit-exact."""
import numpy as np
import pytest
import torch

from oracle import dip_oracle as O
from gpu_util import bits_from_bool, bool_from_bits, dev_f32, dev_u32, host_u32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def D():
    import paper_2412_01380_amd as D
    return D


def _random_scores(rng, n, kind):
    if kind == 0:
        return np.abs(rng.standard_normal(n)).astype(np.float32)
    if kind == 1:
        return np.abs(rng.standard_t(2, n)).astype(np.float32)                 # heavy tails
    if kind == 2:
        return (rng.integers(0, 7, n) / 3).astype(np.float32)                  # seven values
    if kind == 3:
        return np.where(rng.random(n) < 0.5, 0, rng.random(n)).astype(np.float32)   # half zeros
    if kind == 4:
        return (1 + rng.integers(0, 3, n) * 2.0 ** -23).astype(np.float32)     # differ in the last bits
    return (rng.random(n) * 2.0 ** rng.integers(-140, 100, n).astype(np.float64)).astype(np.float32)  # all binades


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_scores_and_topk_random_sweep(D, seed):
    rng = np.random.default_rng(1000 + seed)
    for case in range(120):
        n = int(rng.choice([rng.integers(1, 200), rng.integers(200, 5000), rng.integers(5000, 32769),
                            1024 * rng.integers(1, 33)]))
        k = int(rng.integers(1, n + 1))
        s = _random_scores(rng, n, case % 6)
        if case % 2:
            c = rng.random(n) < 0.5
            x = (s * rng.choice([-1, 1], n)).astype(np.float32)
            got = torch.empty(n, dtype=torch.float32, device="cuda")
            D.dip_ca_scores(dev_f32(x), n, dev_u32(bits_from_bool(c)), 0.2, got)
            s = O.score(x, c, 0.2)
            assert np.array_equal(got.cpu().numpy().view(np.uint32), s.view(np.uint32)), (case, n, "scores")
        m_ref, idx_ref = O.topk(s, k)
        mask = torch.empty((n + 31) // 32, dtype=torch.int32, device="cuda")
        idx = torch.empty(k, dtype=torch.int32, device="cuda")
        D.dip_prune_topk(dev_f32(s), n, k, mask, idx)
        assert np.array_equal(host_u32(mask), bits_from_bool(m_ref)), (case, n, k, "mask")
        assert np.array_equal(idx.cpu().numpy().astype(np.int64), idx_ref), (case, n, k, "index list")


@pytest.mark.parametrize("seed", [1, 2])
def test_cache_update_random_sweep(D, seed):
    rng = np.random.default_rng(2000 + seed)
    for case in range(24):
        n = int(rng.choice([rng.integers(1, 300), rng.integers(300, 6000), rng.integers(6000, 32769)]))
        cap = int(rng.integers(0, n + 1))
        policy = "lru" if case % 2 == 0 else "lfu"
        cache = D.Cache(n, cap, D.DIP_LRU if policy == "lru" else D.DIP_LFU)
        D.dip_cache_init(cache)
        st = O.CacheState(n=n, capacity=cap, policy=policy)
        base = rng.standard_normal(n)
        for t in range(int(rng.integers(4, 12))):
            k = int(rng.integers(1, n + 1)) if t % 3 == 0 else int(rng.integers(1, max(2, n // 3)))
            base = 0.8 * base + 0.6 * rng.standard_normal(n)
            m, _ = O.topk(np.abs(base).astype(np.float32), k)
            D.dip_cache_update(cache, dev_u32(bits_from_bool(m)))
            O.cache_update(st, m)
            assert np.array_equal(bool_from_bits(host_u32(cache.bits), n), st.resident), (case, n, cap, policy, t)
            assert np.array_equal(host_u32(cache.stamp).astype(np.int64), st.stamp), (case, n, cap, policy, t)
            meta = cache.meta_host()
            assert meta["cum_hits"] == st.hits and meta["cum_lookups"] == st.lookups
