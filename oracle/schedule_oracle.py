"""Oracle for the work decode and the K/V scan direction -- TEST INFRASTRUCTURE ONLY.

Written from the paper's description, in plain Python lists: persistent workgroups take query
tiles in a grid-stride loop (Sec. 2.2, Alg. 2) and flip the K/V scan direction on every other
local iteration (Sec. 4, Alg. 4).  The reuse the method relies on happens among workgroups that
share one L2 (Sec. 3.4); on MI355X that is one XCD, and hardware places workgroup w on XCD
w mod 8.  Reading used here (stated in the design notes): the grid-stride loop runs per cache
domain.

  * B*H heads, ceil(N/T_q) query tiles each.  A head is cut into `parts` interleaved subsets of
    its tiles (parts = 8 / gcd(B*H, 8)); chunk c = head*parts + part belongs to domain c mod 8 and
    the chunks of a domain are processed in increasing c.
  * The `slots` workgroups of a domain stride over a chunk's tile list with stride `slots`
    (Alg. 2 with G = slots); one pass of all slots is a round.  Odd rounds hand the tiles out in
    reverse slot order; causal chunks list their tiles from the longest to the shortest.
  * Scan direction (Alg. 4): forward on even rounds, backward on odd rounds, the round count
    restarting with every chunk (a new chunk brings new K/V, so there is nothing to re-use by
    walking backward into it); N_KV is the number of K/V tiles visible to the query tile.

Nothing here is shared with the GPU library.
"""
from __future__ import annotations

from math import gcd

T_Q, T_KV, DOMAINS, MAX_SLOTS = 128, 64, 8, 64


def ceil_div(a: int, b: int) -> int:
    return -(-a // b)


def launch_geometry(B: int, H: int, N: int):
    heads = B * H
    q_tiles = ceil_div(N, T_Q)
    parts = DOMAINS // gcd(heads, DOMAINS)
    largest_part = ceil_div(q_tiles, parts)
    slots = min(largest_part, MAX_SLOTS)
    rounds = ceil_div(largest_part, slots)
    return {"grid": DOMAINS * slots, "slots": slots, "parts": parts, "q_tiles": q_tiles,
            "rounds_per_chunk": rounds, "chunks_per_domain": heads * parts // DOMAINS}


def schedule(B: int, H: int, N: int, causal: bool, scan_order: str):
    """Return {workgroup: [(head, query tile, first K/V tile, last K/V tile), ...]} in the order
    each workgroup processes its tiles."""
    geo = launch_geometry(B, H, N)
    heads, parts, slots = B * H, geo["parts"], geo["slots"]
    kv_tiles = ceil_div(N, T_KV)
    out = {}
    for wg in range(geo["grid"]):
        domain, slot = wg % DOMAINS, wg // DOMAINS
        my_chunks = [c for c in range(heads * parts) if c % DOMAINS == domain]
        recs = []
        for c in my_chunks:
            head, part = divmod(c, parts)
            tiles = list(range(part, geo["q_tiles"], parts))
            if causal:
                tiles.reverse()                       # longest tile first
            for r in range(geo["rounds_per_chunk"]):
                hand_out = list(range(slots)) if r % 2 == 0 else list(range(slots - 1, -1, -1))
                pos = r * slots + hand_out.index(slot)
                if pos < len(tiles):
                    t = tiles[pos]
                    if causal:
                        last_row = min((t + 1) * T_Q, N)   # rows of the tile are t*T_Q .. last_row-1
                        n_kv = ceil_div(last_row, T_KV)
                    else:
                        n_kv = kv_tiles
                    backward = scan_order == "sawtooth" and r % 2 == 1
                    recs.append((head, t, n_kv - 1, 0) if backward else (head, t, 0, n_kv - 1))
        out[wg] = recs
    return out
