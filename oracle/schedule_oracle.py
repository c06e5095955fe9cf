"""Oracle for the work decode and the K/V scan direction -- TEST INFRASTRUCTURE ONLY.

Written from the paper's description, in plain Python lists: persistent workgroups take query
tiles in a grid-stride loop (Sec. 2.2, Alg. 2) and flip the K/V scan direction on every other
local iteration (Sec. 4, Alg. 4).  The reuse the method relies on happens among workgroups that
share one L2 (Sec. 3.4); on MI355X that is one XCD, and hardware places workgroup w on XCD
w mod 8.  Reading used here (stated in the design notes): the grid-stride loop runs per cache
domain.

  * B*H heads, ceil(N/tile_q) query tiles each.  A head is cut into `parts` interleaved subsets of
    its tiles (parts = 8 / gcd(B*H, 8)); chunk c = head*parts + part belongs to domain c mod 8 and
    the chunks of a domain are processed in increasing c.
  * The `slots` workgroups of a domain stride over a chunk's tile list with stride `slots`
    (Alg. 2 with G = slots); one pass of all slots is a round.  Rounds are numbered through all
    chunks of the domain and the odd ones hand the tiles out in reverse slot order; causal chunks
    list their tiles from the longest to the shortest.
  * Scan direction (Alg. 4): forward on even rounds, backward on odd rounds, the round count
    restarting with every chunk (a new chunk brings new K/V, so there is nothing to re-use by
    walking backward into it); N_KV is the number of K/V tiles visible to the query tile.

Variants kept for comparison (same records, other hand-out):
  * a smaller `resident`: fewer workgroups per domain (Sec. 3.4's sweep over active CTAs).
  * decode "linear": the printed Alg. 2 -- one list of all (head, tile) pairs, tile fastest;
    persistent workgroup k takes entries k, k+G, k+2G, ... and walks backward on its odd local
    iterations (Alg. 4 as printed).
  * launch "grid" (Alg. 3): one workgroup per `tiles_per_workgroup` consecutive entries of the
    list (linear decode) or of a chunk's tile list (domain decode, workgroups of a domain
    numbered chunk after chunk); with two tiles per workgroup the second is walked backward
    under the sawtooth order (Sec. 4.3, the variant that advances the loop by two).

The tile height `tile_q` (query rows per workgroup tile) and `resident` (how many workgroups of one domain run
at the same time, the G of Alg. 2 per domain) are inputs: they are properties of the kernel that runs the
schedule, not of the method, and the tests take them from the library's launch query or from hand-listed
cases.  Nothing here is shared with the GPU library.
"""
from __future__ import annotations

from math import gcd

T_KV, DOMAINS = 64, 8


def ceil_div(a: int, b: int) -> int:
    return -(-a // b)


def launch_geometry(B: int, H: int, N: int, *, tile_q: int, resident: int, launch: str = "persistent",
                    decode: str = "domain", tiles_per_workgroup: int = 2):
    heads = B * H
    q_tiles = ceil_div(N, tile_q)
    total = heads * q_tiles
    if decode == "linear":
        if launch == "persistent":
            slots = min(ceil_div(total, DOMAINS), resident)
            local = ceil_div(total, DOMAINS * slots)
        else:
            slots = ceil_div(ceil_div(total, tiles_per_workgroup), DOMAINS)
            local = tiles_per_workgroup
        return {"grid": DOMAINS * slots, "slots": slots, "parts": 1, "q_tiles": q_tiles, "max_local": local,
                "tile_q": tile_q}
    parts = DOMAINS // gcd(heads, DOMAINS)
    largest_part = ceil_div(q_tiles, parts)
    chunks_per_domain = heads * parts // DOMAINS
    if launch == "persistent":
        slots = min(largest_part, resident)
        rounds = ceil_div(largest_part, slots)
        return {"grid": DOMAINS * slots, "slots": slots, "parts": parts, "q_tiles": q_tiles,
                "rounds_per_chunk": rounds, "chunks_per_domain": chunks_per_domain,
                "max_local": chunks_per_domain * rounds, "tile_q": tile_q}
    units = ceil_div(largest_part, tiles_per_workgroup)
    slots = chunks_per_domain * units
    return {"grid": DOMAINS * slots, "slots": slots, "parts": parts, "q_tiles": q_tiles,
            "units_per_chunk": units, "chunks_per_domain": chunks_per_domain, "max_local": tiles_per_workgroup,
            "tile_q": tile_q}


def visible_kv(t: int, N: int, causal: bool, tile_q: int) -> int:
    """Number of K/V tiles query tile t (of tile_q rows) has to visit."""
    if not causal:
        return ceil_div(N, T_KV)
    last_row = min((t + 1) * tile_q, N)       # rows of the tile are t*tile_q .. last_row-1
    return ceil_div(last_row, T_KV)


def record(head: int, t: int, N: int, causal: bool, backward: bool, tile_q: int):
    n_kv = visible_kv(t, N, causal, tile_q)
    return (head, t, n_kv - 1, 0) if backward else (head, t, 0, n_kv - 1)


def schedule(B: int, H: int, N: int, causal: bool, scan_order: str, *, tile_q: int, resident: int,
             launch: str = "persistent", decode: str = "domain", tiles_per_workgroup: int = 2):
    """Return {workgroup: [(head, query tile, first K/V tile, last K/V tile), ...]} in the order
    each workgroup processes its tiles."""
    geo = launch_geometry(B, H, N, tile_q=tile_q, resident=resident, launch=launch, decode=decode,
                          tiles_per_workgroup=tiles_per_workgroup)
    heads, parts, slots, grid, tq = B * H, geo["parts"], geo["slots"], geo["grid"], geo["tile_q"]
    saw = scan_order == "sawtooth"
    out = {}
    if decode == "linear":
        work = [(head, t) for head in range(heads) for t in range(geo["q_tiles"])]
        for wg in range(grid):
            mine = work[wg::grid] if launch == "persistent" else \
                work[wg * tiles_per_workgroup:(wg + 1) * tiles_per_workgroup]
            out[wg] = [record(head, t, N, causal, saw and i % 2 == 1, tq) for i, (head, t) in enumerate(mine)]
        return out
    for domain in range(DOMAINS):
        my_chunks = [c for c in range(heads * parts) if c % DOMAINS == domain]
        chunk_tiles = []
        for c in my_chunks:
            head, part = divmod(c, parts)
            tiles = list(range(part, geo["q_tiles"], parts))
            if causal:
                tiles.reverse()                       # longest tile first
            chunk_tiles.append((head, tiles))
        if launch == "grid":
            m = 0                                     # workgroups of the domain, chunk after chunk
            for head, tiles in chunk_tiles:
                for unit in range(geo["units_per_chunk"]):
                    mine = tiles[unit * tiles_per_workgroup:(unit + 1) * tiles_per_workgroup]
                    out[m * DOMAINS + domain] = [record(head, t, N, causal, saw and i % 2 == 1, tq)
                                                 for i, t in enumerate(mine)]
                    m += 1
            continue
        for slot in range(slots):
            recs = []
            for n_chunk, (head, tiles) in enumerate(chunk_tiles):
                for r in range(geo["rounds_per_chunk"]):
                    nth_round = n_chunk * geo["rounds_per_chunk"] + r
                    hand_out = list(range(slots)) if nth_round % 2 == 0 else list(range(slots - 1, -1, -1))
                    pos = r * slots + hand_out.index(slot)
                    if pos < len(tiles):
                        recs.append(record(head, tiles[pos], N, causal, saw and r % 2 == 1, tq))
            out[slot * DOMAINS + domain] = recs
    return out
