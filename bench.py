#!/usr/bin/env python3
"""Benchmark of the attention forward hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 4] [--scan-order sawtooth]

A "step" is one attn_fwd call (work decode, scan-direction choice, Q load, K/V streaming, both
contractions, online softmax, epilogue) over one batch of the seeded synthetic workload, inputs
resident in HBM.  Prints ONE JSON line: whole-job TFLOP/s of the sawtooth order (4*B*H*N^2*d flops,
halved under a causal mask), the MFMA roofline of the kernel measured live with events on the
launch stream, the cyclic order timed the same way, and the fp64 CPU oracle timed on a bounded
sample of the same workload (reported baseline only).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_PEAK_TFLOPS_16BIT = 2500.0   # MI355X dense fp16/bf16 matrix peak



def profiled_counters(workload_name: str, workspace: bool):
    """HBM-side bytes and TCC (L2) misses per launch and scan order, read from the committed rocprofv3 summary of
    this workload (profiles/attn_fwd_<workload>[_workspace].txt: `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` /
    `TCC_MISS_sum` runs of this script, the byte counters scaled by their reading for a plain 1 GiB copy in the same
    run).  They are profile figures, not measured in this run: the line names the file they come from.  Returns
    (traffic bytes by order, misses by order, path relative to the repository) or ({}, {}, None) without a summary."""
    rel = os.path.join("profiles", f"attn_fwd_{workload_name}" + ("_workspace" if workspace else "") + ".txt")
    path = os.path.join(ROOT, rel)
    traffic, misses = {}, {}
    if not os.path.exists(path):
        return traffic, misses, None
    for line in open(path):
        t = line.split()
        if len(t) >= 3 and t[0] == "TCC_MISS_sum" and t[1] in ("sawtooth", "cyclic"):
            misses[t[1]] = float(t[2])
        if len(t) >= 4 and t[0] in ("sawtooth", "cyclic") and "bytes per launch" in line and "total" in t:
            traffic[t[0]] = float(t[t.index("total") + 1])
    return traffic, misses, rel


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", type=int, default=4, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--scan-order", default="both", choices=["both", "sawtooth", "cyclic"],
                    help="'both' times sawtooth (the headline) and cyclic; a single order is for profiling")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-mfma-probe", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (reference reading for FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--ramp-ms", type=float, default=60.0,
                    help="untimed launches for this long before the warm-up steps, so that the clock has settled")
    ap.add_argument("--workspace", action="store_true",
                    help="bf16 workloads: call attn_fwd_workspace with a caller-allocated workspace (binary16 copies "
                         "of K and V feed the 64-rows-per-wavefront kernel where it applies) instead of attn_fwd")
    ap.add_argument("--rows-per-wavefront", type=int, default=0, choices=[0, 32, 64],
                    help="0: what attn_fwd picks by itself; 32 or 64: that kernel shape through attn_fwd_variant")
    ap.add_argument("--kv-halves", type=int, default=0, choices=[0, 1, 2],
                    help="0: what attn_fwd picks by itself; 1: every wavefront walks the whole K/V scan; 2: 64-row tiles, "
                         "two wavefronts per half of the scan (small unmasked fp16 problems), through attn_fwd_variant")
    ap.add_argument("--align-rounds", action="store_true",
                    help="the workgroups of an XCD wait for each other after every round, not only between heads "
                         "(attn_fwd_variant; a study of how much the scan order can save at best)")
    ap.add_argument("--qo-streaming", type=int, default=0, choices=[0, 1, 2, 3, 4],
                    help="0: what attn_fwd does (3 on these workloads but the first two, where it is 1); 3: Q tiles in and O tiles out through LDS, whole lines, non-temporal; "
                         "1: O only; 2: Q only; 4: neither (every lane loads and stores its own pieces, cached), "
                         "through attn_fwd_variant: a study of what the tiles touched once cost the K/V tail in the L2")
    ap.add_argument("--evict", action="store_true",
                    help="overwrite a 1 GiB scratch buffer before every step so each launch starts cache-cold")
    return ap.parse_args()


def time_order(launch, torch, order, steps, warmup, evict_buf=None):
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        if evict_buf is not None:
            evict_buf.zero_()
        launch(order, stream)
    torch.cuda.synchronize()
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    t0 = time.perf_counter()
    for i in range(steps):
        if evict_buf is not None:
            evict_buf.zero_()
        starts[i].record(stream)
        launch(order, stream)
        stops[i].record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    kernel_ms = sum(a.elapsed_time(b) for a, b in zip(starts, stops)) / steps
    return wall_ms, kernel_ms


def mfma_probe(sa, torch):
    """Matrix rate this chip sustains (context for roofline.frac, which uses the datasheet peak)."""
    res = {"unit": "TFLOP/s"}
    for mode, key in ((0, "zero_operands"), (1, "live_operands_in_registers"), (2, "live_operands_lds_fed")):
        for _ in range(10):                      # some tens of milliseconds: the clock settles
            sa.sawattn_mfma_probe(4000, mode)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        flops = sum(sa.sawattn_mfma_probe(4000, mode) for _ in range(10))
        e1.record()
        torch.cuda.synchronize()
        res[key] = flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
    return res


def cpu_baseline(w, Q, K, V, target_seconds):
    """Time the oracle, as it stands, on a bounded sample of the workload: evenly spaced query rows
    of as many (batch, head) pairs as fit in about `target_seconds` of CPU time."""
    from oracle import attn_oracle
    threads = attn_oracle.num_threads()

    def run(b, h, n_rows):
        rows = [int(i * w.N / n_rows) for i in range(n_rows)]
        q, k, v = Q[b:b + 1, h:h + 1], K[b:b + 1, h:h + 1], V[b:b + 1, h:h + 1]
        t0 = time.perf_counter()
        attn_oracle.attention(q, k, v, w.scale, causal=w.causal, rows=rows)
        dt = time.perf_counter() - t0
        # flops of exactly these rows (a causal row i has i+1 visible keys)
        fl = sum(4.0 * ((r + 1) if w.causal else w.N) * w.d for r in rows)
        return dt, fl

    run(0, 0, min(w.N, 16))                        # first call loads the library and starts the threads
    # Whole heads (all their query rows) one after another until the time is used up; the last head is cut to the
    # rows that still fit, judged by the rate seen so far (first head: by a 1024-row calibration run, not counted).
    dt0, fl0 = run(0, 0, min(w.N, 1024))
    rate = fl0 / max(dt0, 1e-6)                    # flop per second
    total_dt = total_fl = 0.0
    rows_done, heads_done = 0, 0
    head_fl = 4.0 * w.N * w.N * w.d * (0.5 if w.causal else 1.0)
    for idx in range(w.B * w.H):
        left = target_seconds - total_dt
        if left < 0.05 * target_seconds:
            break
        n = w.N if head_fl / rate <= left else max(64, int(w.N * left * rate / head_fl))
        n = min(n, w.N)
        dt, fl = run(idx // w.H, idx % w.H, n)
        total_dt += dt
        total_fl += fl
        rows_done += n
        heads_done += 1
        rate = total_fl / total_dt
        if n < w.N:
            break
    return {"value": total_fl / total_dt / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": f"{rows_done} evenly spaced query rows over the first {heads_done} (batch, head) pairs of "
                      f"{w.name}: {total_fl:.3e} flop in {total_dt:.1f} s, fp64, full score rows",
            "seconds": total_dt}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2601_16032_amd import binding as sa
    from paper_2601_16032_amd import workloads
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    sa.lib()   # raises if the HIP library is not built: there is no fallback
    torch.cuda.set_device(0)
    w = workloads.WORKLOADS[args.workload]
    Q, K, V = workloads.make_qkv(w)
    Qd, Kd, Vd = Q.cuda(), K.cuda(), V.cuda()
    # the output type the parity tests use for this workload: fp16 for fp16 inputs, fp32 for bf16 inputs
    o_dtype = torch.float16 if w.dtype == "f16" else torch.float32
    O = torch.empty(Qd.shape, dtype=o_dtype, device="cuda")
    evict_buf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda") if args.evict else None
    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    info = sa.attn_fwd_launch_info(w.B, w.H, w.N, w.d, w.causal, dtype=w.dtype)
    var = sa.variant(rows_per_wavefront=args.rows_per_wavefront, align_rounds=int(args.align_rounds),
                     kv_halves=args.kv_halves, qo_streaming=args.qo_streaming) \
        if (args.rows_per_wavefront or args.align_rounds or args.kv_halves or args.qo_streaming) else None
    if var is not None:
        info = sa.attn_fwd_variant_launch_info(w.B, w.H, w.N, w.d, w.causal, var, w.dtype)
    ws, ws_bytes = None, 0
    if args.workspace:
        ws_bytes, info = sa.attn_fwd_workspace_bytes(w.B, w.H, w.N, w.d, w.causal, var, w.dtype)
        ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")

    def launch(order, stream):
        if ws is not None:
            sa.attn_fwd_workspace(Qd, Kd, Vd, O, scale=w.scale, causal=w.causal, scan_order=order, stream=stream,
                                  workspace=ws, variant=var)
        elif var is not None:
            sa.attn_fwd_variant(Qd, Kd, Vd, O, scale=w.scale, causal=w.causal, scan_order=order, stream=stream,
                                variant=var)
        else:
            sa.attn_fwd(Qd, Kd, Vd, O, scale=w.scale, causal=w.causal, scan_order=order, stream=stream)

    orders = ["sawtooth", "cyclic"] if args.scan_order == "both" else [args.scan_order]
    # Bring the chip to the clock it sustains under this kernel before anything is timed: it leaves idle at a low
    # clock and settles, under matrix load, well below its peak clock within some tens of milliseconds.  Without
    # this the order timed first reads up to 10 % slower than the second on the sub-millisecond workloads.
    t_ramp = time.perf_counter()
    while time.perf_counter() - t_ramp < args.ramp_ms * 1e-3:
        for _ in range(4):
            launch(orders[0], torch.cuda.current_stream())
        torch.cuda.synchronize()
    res = {}
    for order in orders:
        wall_ms, kernel_ms = time_order(launch, torch, order, args.steps, args.warmup, evict_buf)
        res[order] = {"ms_per_step": wall_ms, "kernel_ms": kernel_ms,
                      "tflops": w.flops / (kernel_ms * 1e-3) / 1e12,
                      "tflops_wall": w.flops / (wall_ms * 1e-3) / 1e12}
    head = orders[0]
    r = res[head]
    traffic, misses, profile = profiled_counters(w.name, bool(ws_bytes)) if var is None else ({}, {}, None)
    kernel = f"attn_fwd_kernel<d={w.d}, {w.dtype if not ws_bytes else 'f16 copies'}, {'causal' if w.causal else 'full'}, " \
             + ("32 rows per wavefront, the two halves of the scan at once>" if info["tile_q"] == 64
                else f"{info['tile_q'] // 4} rows per wavefront>")
    out = {
        "metric": "attention fwd TFLOP/s (fp16, N=16k, d=128) + L2 miss count, sawtooth vs cyclic",
        "value": r["tflops_wall"],
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": r["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "H": w.H, "N": w.N, "d": w.d, "causal": w.causal,
                   "scan_order": head, "out_dtype": str(o_dtype).replace("torch.", ""), "flops_per_step": w.flops,
                   "launch": info, "kernel": kernel, "cache_cold_steps": bool(args.evict),
                   "entry_point": "attn_fwd_workspace" if ws is not None else
                                  ("attn_fwd_variant" if var is not None else "attn_fwd"),
                   "workspace_bytes": ws_bytes},
        "roofline": {"bound": "mfma", "achieved": r["tflops"], "peak": MFMA_PEAK_TFLOPS_16BIT,
                     "unit": "TFLOP/s", "frac": r["tflops"] / MFMA_PEAK_TFLOPS_16BIT,
                     "traffic": traffic.get(head), "traffic_source": profile,
                     "kernel_ms": r["kernel_ms"], "kernel": kernel},
        "scan_orders": {o: {"tflops": res[o]["tflops"], "kernel_ms": res[o]["kernel_ms"],
                            "tcc_miss_profiled": misses.get(o), "hbm_bytes_profiled": traffic.get(o)} for o in orders},
        "counters_from": profile,
    }
    if not args.no_mfma_probe:
        out["mfma_probe"] = mfma_probe(sa, torch)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, Q, K, V, args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
