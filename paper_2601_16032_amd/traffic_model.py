"""Analytic L2 traffic of the tiled attention forward (paper Sec. 3.2, Sec. 3.3), in sectors and bytes.

Host-side reporting helpers: these give the algorithmic byte counts that the benchmark and the
profile summaries quote beside the measured counters.  No GPU work.
"""
from __future__ import annotations


def l2_sectors_noncausal(S: int, T: int, D: int = 64, E: int = 2, C: int = 32) -> float:
    """Sec. 3.2: Q and O are touched once, K and V once per query tile:  M = 2(SDE/C + S^2 DE/(TC))."""
    return 2.0 * (S * D * E / C + S * S * D * E / (T * C))


def l2_sectors_causal(S: int, T: int, D: int = 64, E: int = 2, C: int = 32) -> float:
    """Sec. 3.2 with a causal mask, as printed: M = (2 SDE/C)(S/2T + 1/2), i.e. 8S(S/2T + 1/2) at
    D=64, E=2, C=32.  (The printed form halves the Q/O term along with the K/V term.)"""
    return (2.0 * S * D * E / C) * (S / (2.0 * T) + 0.5)


def cold_miss_sectors(S: int, D: int = 64, E: int = 2, C: int = 32) -> float:
    """Sec. 3.3: every sector of Q, K, V, O missed once: 4 SDE/C."""
    return 4.0 * S * D * E / C


def l2_read_bytes(B: int, H: int, N: int, d: int, tile_q: int, causal: bool, elem_bytes: int = 2) -> float:
    """Bytes requested from L2 by one forward: Q once plus K and V once per query tile (Sec. 3.2 in
    bytes, for a query tile of `tile_q` rows); causal: tile i of n = N/tile_q reads (i+1)/n of K/V."""
    n = -(-N // tile_q)
    q = N * d * elem_bytes
    kv_once = 2.0 * N * d * elem_bytes
    kv = kv_once * n if not causal else kv_once * (n + 1) / 2.0
    return float(B * H) * (q + kv)


def compulsory_bytes(B: int, H: int, N: int, d: int, elem_bytes: int = 2, out_bytes: int = 2) -> float:
    """Q, K, V read once and O written once."""
    return float(B * H) * N * d * (3 * elem_bytes + out_bytes)


def lru_kv_miss_bytes(N: int, d: int, tile_q: int, workgroups_per_domain: int, capacity_bytes: float,
                      sawtooth: bool, elem_bytes: int = 2) -> float:
    """K/V bytes one head misses in the L2 of one domain when `workgroups_per_domain` workgroups
    walk K/V in lockstep, round after round, and the cache keeps the most recent `capacity_bytes`
    (Sec. 3.3 threshold, Sec. 3.4 lockstep reuse, Sec. 4 reuse distance): every round after the
    first re-misses everything under the cyclic order, and everything but the cache's worth it
    starts from under the sawtooth order."""
    kv = 2.0 * N * d * elem_bytes
    rounds = -(-(-(-N // tile_q)) // workgroups_per_domain)
    if kv <= capacity_bytes:
        return kv
    if not sawtooth:
        return rounds * kv
    return kv + (rounds - 1) * (kv - capacity_bytes)
