"""Host-side two-tier byte / latency model (the paper's "HW simulator", Sec. 6.1 and App. A).

The paper estimates mobile throughput by counting the bytes that move Flash -> DRAM (cache
misses) and DRAM -> processing unit (everything a token touches) and dividing by the two
bandwidths; compute time is ignored.  Layers that are never pruned (attention, embeddings,
KV cache) are pinned in DRAM and the rest of the DRAM is the MLP column cache, split evenly
over the MLP layers (App. A).  This module is that arithmetic, fed by the hit / miss
counters that the GPU path keeps in its cache state (dip_cache.meta); it moves no data.

The paper does not say whether the two transfers overlap.  Its printed dense throughputs
(Table 2, Tables 6-7) are reproduced to the printed precision by
`1 / max(flash_time, dram_time)`, so `overlap=True` is the default; `overlap=False` adds them.
"""
from __future__ import annotations

from dataclasses import dataclass

GB = 1e9


@dataclass(frozen=True)
class Device:
    """Bandwidths of the simulated device; defaults are the paper's Apple-A18 setting."""
    dram_gbps: float = 60.0
    flash_gbps: float = 1.0


def token_seconds(flash_bytes: float, dram_bytes: float, dev: Device = Device(), overlap: bool = True) -> float:
    """Latency of one token that reads `flash_bytes` from Flash and `dram_bytes` through DRAM."""
    tf = flash_bytes / (dev.flash_gbps * GB)
    td = dram_bytes / (dev.dram_gbps * GB)
    return max(tf, td) if overlap else tf + td


def dense_tokens_per_second(model_bytes: float, dram_bytes: float, dev: Device = Device(),
                            overlap: bool = True) -> float:
    """Dense model streamed from Flash: every token needs every weight; what does not fit in
    DRAM is re-read from Flash for each token."""
    miss = max(0.0, model_bytes - dram_bytes)
    return 1.0 / token_seconds(miss, model_bytes, dev, overlap)


def sparse_tokens_per_second(static_bytes: float, layers: int, col_bytes_in: float, col_bytes_mid: float,
                             selected_in: float, selected_mid: float, hit_rate_in: float,
                             hit_rate_mid: float, dev: Device = Device(), overlap: bool = True) -> float:
    """DIP / DIP-CA decode: per layer and token `selected_*` columns are used (k_in of the
    bundled up/gate columns, k_mid of the down columns); a fraction `hit_rate_*` of them is
    resident in the DRAM cache, the rest comes from Flash.  `static_bytes` (attention,
    embeddings, KV cache) are read from DRAM for every token and never from Flash."""
    used = layers * (selected_in * col_bytes_in + selected_mid * col_bytes_mid)
    missed = layers * (selected_in * (1.0 - hit_rate_in) * col_bytes_in
                       + selected_mid * (1.0 - hit_rate_mid) * col_bytes_mid)
    return 1.0 / token_seconds(missed, static_bytes + used, dev, overlap)


def hit_rates_from_meta(meta_in: dict, meta_mid: dict) -> tuple:
    """Cumulative hit rates from two dip_cache meta dictionaries (Cache.meta_host())."""
    hi = meta_in["cum_hits"] / max(1, meta_in["cum_lookups"])
    hm = meta_mid["cum_hits"] / max(1, meta_mid["cum_lookups"])
    return hi, hm
