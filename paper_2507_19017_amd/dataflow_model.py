"""Closed-form volume and memory estimates the paper uses to motivate its two techniques.

Pure arithmetic, no GPU work: Eq. (1) and Eq. (2) (communication volume of the sample flow
through a centralized replay buffer), Eq. (4) (volume per warehouse with the distributed
transfer dock) and Eq. (3) (redundant memory of the resharding flow without the swap; the
same formula is exported by the C library as reshard_redundant_memory_bytes).  Symbols
follow the paper: G global batch, N responses per prompt, B bytes per element, PL / SL
maximum prompt / response length, n number of response-length items, M number of scalars,
C transfer-dock controllers, S warehouses.
"""

from __future__ import annotations

GIB = 1024 ** 3


def cv_gb(G: int, N: int, B: int, PL: int, n: int, SL: int, M: int) -> float:
    """Eq. (1): volume of one request of a batch from the replay buffer, in GB (2^30 bytes)."""
    return G * N * B * (PL + n * SL + M) / GIB


def tcv_gb(G: int, N: int, B: int, PL: int, n: int, SL: int, M: int) -> float:
    """Eq. (2): total volume of the last three steps of the replay-buffer flow, in GB."""
    return G * N * B * (2 * PL + 3 * n * SL + 8 * M) / GIB


def td_tcv_gb(G: int, N: int, B: int, PL: int, n: int, SL: int, M: int, C: int, S: int) -> float:
    """Eq. (4): total volume per transfer-dock warehouse (C controllers, S warehouses), in GB."""
    return G * N * B * (2 * PL + 3 * n * SL + 8 * (C + 1) * M) / S / GIB


def dispatch_seconds(volume_gb: float, link_mb_per_s: float) -> float:
    """Time to move `volume_gb` (2^30-byte GB) over a link of `link_mb_per_s` (2^20-byte MB/s);
    Table 1's 1 GB/s column is 1024 MB/s."""
    return volume_gb * 1024.0 / link_mb_per_s


def redundant_memory_gb(GDP: int, TW: float, UTP: int, EW: float, GEP: int) -> float:
    """Eq. (3): R = GDP * (TW / UTP + EW / GEP), in the unit of TW and EW."""
    return GDP * (TW / UTP + EW / GEP)
