"""The paper's cache studies as sweeps over the attention kernel (one GPU).

Each study is a list of points (shape, launch variant, scan order).  A point is run as
`--warmup` untimed plus `--launches` timed launches of the HIP kernel through the C ABI (after `--settle-ms`
of untimed launches where the times are what the run is for), timed with events on the launch stream, and printed as one JSON line together with what the traffic model
(Sec. 3.2-3.4, Sec. 4) predicts for it.  Run the same command under `rocprofv3 --pmc ...
--kernel-trace` to get the L2 counters of every launch: the attention dispatches appear in the
order of the points, `warmup + launches` per point, which the `dispatches` field of each line
restates.

Studies
  seqlen    Sec. 3.2 / 3.3: sequence length 2K...128K at B=1, H in {1, 8}, d in {64, 128}:
            L2 requests against 2NdE(1 + N/T_q) (T_q = 128, or 256 where the library picks its wide
            variant), and where non-compulsory misses set in.
  resident  Sec. 3.4: G = 8 w persistent workgroups, w = 1...64 (96 at d = 64) per XCD: hit rate against 1 - 1/w;
            the sawtooth points a second time with qo_streaming = 4 (Q and O tiles as ordinary cached traffic).
  decode    Sec. 2.2 Alg. 2 as printed (one linear stride over all XCDs) against the per-XCD decode.
  launch    Alg. 3 (direct launch, one or two query tiles per workgroup) against the persistent
            launch, both scan orders (Sec. 4.3's two program variants).
  batch     Sec. 4.2 / 4.3 shapes: d = 64, N = 128K (and 32K), B in {1, 2, 4, 8}, plain and causal.
  heads     Alg. 2 against Alg. 3 where heads are short and come several to an XCD (B*H = 16...128, N = 512...8K):
            the persistent launch, the direct launch with one tile per workgroup, and what attn_fwd picks by itself.

A point without a variant runs what attn_fwd runs (launch left open); a variant pins the persistent launch unless
it names the other.

Inputs are seeded N(0,1) values rounded to fp16 (`workloads.make_random`), scale 1/sqrt(d).
"""
from __future__ import annotations

import argparse
import json
import math
import sys
import time

from . import traffic_model as tm
from . import workloads

L2_BYTES_PER_XCD = 4 * 2 ** 20


def _pt(B, H, N, d, causal=False, order="sawtooth", **variant):
    return {"B": B, "H": H, "N": N, "d": d, "causal": causal, "order": order, "variant": variant}


def study_points(study: str):
    pts = []
    if study == "seqlen":
        for H in (1, 8):
            for d in (64, 128):
                for N in (2048, 4096, 8192, 16384, 32768, 65536, 131072):
                    if H == 8 and N > 65536:
                        continue
                    for order in ("cyclic", "sawtooth"):
                        pts.append(_pt(1, H, N, d, order=order))
    elif study == "resident":
        for (H, N, d) in ((8, 32768, 64), (32, 16384, 128)):
            for w in (1, 2, 4, 8, 16, 32, 64) + ((96,) if d == 64 else ()):
                for order in ("cyclic", "sawtooth"):
                    pts.append(_pt(1, H, N, d, order=order, slots_per_domain=w))
                # the same turn-around with Q and O tiles passing the L2 as ordinary cached traffic
                pts.append(_pt(1, H, N, d, order="sawtooth", slots_per_domain=w, qo_streaming=4))
    elif study == "decode":
        for (B, H, N, d, causal) in ((1, 32, 16384, 128, False), (1, 16, 32768, 128, True), (8, 1, 32768, 64, False)):
            for decode in ("domain", "linear"):
                for order in ("cyclic", "sawtooth"):
                    pts.append(_pt(B, H, N, d, causal, order, decode=decode))
    elif study == "launch":
        for (B, H, N, d, causal) in ((1, 32, 16384, 128, False), (1, 16, 32768, 128, True)):
            for var in ({}, {"launch": "grid", "tiles_per_workgroup": 1}, {"launch": "grid", "tiles_per_workgroup": 2},
                        {"launch": "grid", "decode": "linear", "tiles_per_workgroup": 2}):
                for order in ("cyclic", "sawtooth"):
                    if var.get("tiles_per_workgroup") == 1 and order == "sawtooth":
                        continue        # one tile per workgroup: nothing to alternate
                    pts.append(_pt(B, H, N, d, causal, order, **var))
    elif study == "batch":
        for N in (32768, 131072):
            for causal in (False, True):
                for B in (1, 2, 4, 8):
                    for order in ("cyclic", "sawtooth"):
                        pts.append(_pt(B, 1, N, 64, causal, order))
    elif study == "heads":
        for d in (64, 128):
            for (H, N) in ((128, 512), (64, 1024), (64, 2048), (16, 2048), (24, 2048), (16, 4096), (32, 4096), (32, 8192)):
                for causal in (False, True):
                    # (what attn_fwd picks comes last: the first point of a shape meets a cold clock)
                    for var in ({"launch": "persistent", "kv_halves": 1},
                                {"launch": "grid", "tiles_per_workgroup": 1, "kv_halves": 1}, {}):
                        pts.append(_pt(1, H, N, d, causal, "sawtooth", **var))
    else:
        raise SystemExit(f"unknown study {study!r}")
    return pts


def model(pt, info):
    """What Sec. 3.2-3.4 and Sec. 4 predict for a point, in bytes."""
    B, H, N, d, causal = pt["B"], pt["H"], pt["N"], pt["d"], pt["causal"]
    kv_head = 2 * N * d * 2
    out = {"l2_read_bytes": tm.l2_read_bytes(B, H, N, d, info["tile_q"], causal),
           "compulsory_bytes": tm.compulsory_bytes(B, H, N, d),
           "kv_bytes_per_head": kv_head,
           "kv_over_l2": kv_head / L2_BYTES_PER_XCD}
    if not causal and pt["variant"].get("decode", "domain") == "domain" and pt["variant"].get("launch", "persistent") == "persistent":
        # every domain that holds a part of a head walks that head's K/V once per round
        # (a domain that holds 1/parts of a head's query tiles sees them as tiles `parts` times as tall)
        per_domain_head = tm.lru_kv_miss_bytes(N, d, info["tile_q"] * info["parts_per_head"], info["slots"],
                                               L2_BYTES_PER_XCD, pt["order"] == "sawtooth")
        out["lru_kv_miss_bytes"] = per_domain_head * B * H * info["parts_per_head"]
        out["lockstep_hit_rate"] = 1.0 - 1.0 / info["slots"]
    return out


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--study", required=True, choices=["seqlen", "resident", "decode", "launch", "batch", "heads"])
    ap.add_argument("--points", default="", help="comma-separated point indices or a:b ranges (default: all)")
    ap.add_argument("--launches", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--settle-ms", type=float, default=0.0,
                    help="untimed launches of a point for this long before its warm-up, so that the clock has settled "
                         "(for runs that are timed; leave at 0 under the profiler)")
    ap.add_argument("--list", action="store_true", help="print the points and exit (needs no GPU)")
    args = ap.parse_args(argv)

    pts = study_points(args.study)
    chosen = list(range(len(pts)))
    if args.points:
        chosen = []
        for tok in args.points.split(","):
            if ":" in tok:
                a, b = tok.split(":")
                chosen += list(range(int(a), int(b)))
            else:
                chosen.append(int(tok))
    if args.list:
        for i in chosen:
            print(json.dumps({"point": i, **pts[i]}))
        return 0

    import torch
    from . import binding as sa
    if not torch.cuda.is_available():
        raise SystemExit("sweeps need a GPU (there is no CPU path)")
    sa.lib()
    stream = torch.cuda.current_stream()
    cache = {}
    dispatch = 0
    for i in chosen:
        pt = pts[i]
        key = (pt["B"], pt["H"], pt["N"], pt["d"])
        if key not in cache:
            cache.clear()
            torch.cuda.empty_cache()
            Q, K, V = workloads.make_random(*key, "f16", seed=1234 + pt["N"] % 977, device="cuda")
            cache[key] = (Q, K, V, torch.empty_like(Q))
        Q, K, V, O = cache[key]
        var = sa.variant(**pt["variant"]) if pt["variant"] else None      # None: what attn_fwd runs
        info = sa.attn_fwd_variant_launch_info(*key, pt["causal"], var, "f16")
        scale = 1.0 / math.sqrt(pt["d"])

        def launch():
            sa.attn_fwd_variant(Q, K, V, O, scale=scale, causal=pt["causal"], scan_order=pt["order"], variant=var)

        settle = 0
        if args.settle_ms > 0:
            t0 = time.perf_counter()
            while (time.perf_counter() - t0) * 1e3 < args.settle_ms:
                launch()
                settle += 1
                if settle % 8 == 0:
                    torch.cuda.synchronize()
        for _ in range(args.warmup):
            launch()
        # A timed sample is `reps` launches back to back: 1 under the profiler, in a timed run as many as fill about
        # 0.3 ms, so that the host's own time per launch does not show in short kernels.
        reps = 1
        if args.settle_ms > 0:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            launch()
            e1.record(stream)
            torch.cuda.synchronize()
            settle += 1
            reps = max(1, min(64, int(0.3 / max(e0.elapsed_time(e1), 1e-3)) + 1))
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.launches + 1)]
        ev[0].record(stream)
        for k in range(args.launches):
            for _ in range(reps):
                launch()
            ev[k + 1].record(stream)
        torch.cuda.synchronize()
        ms = sorted(ev[k].elapsed_time(ev[k + 1]) / reps for k in range(args.launches))
        flops = 4.0 * pt["B"] * pt["H"] * pt["N"] ** 2 * pt["d"] * (0.5 if pt["causal"] else 1.0)
        n = settle + args.warmup + args.launches * reps
        print(json.dumps({"study": args.study, "point": i, **pt, "grid": info["grid"], "slots": info["slots"],
                          "tile_q": info["tile_q"], "launch": ("persistent", "grid")[info["launch"]],
                          "parts_per_head": info["parts_per_head"], "ms_median": ms[len(ms) // 2], "ms_min": ms[0],
                          "tflops": flops / (ms[len(ms) // 2] * 1e-3) / 1e12, "model": model(pt, info),
                          "dispatches": [dispatch, dispatch + n]}), flush=True)
        dispatch += n
    return 0


if __name__ == "__main__":
    sys.exit(main())
