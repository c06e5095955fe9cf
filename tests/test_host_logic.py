"""CPU-only tests of the host side: the C ABI surface, argument validation, the work decode /
scan-direction schedule against its oracle, and the traffic model against the paper's counters."""
import ctypes
import math
import os
import re

import numpy as np
import pytest
import torch

from oracle import schedule_oracle as so
from paper_2601_16032_amd import binding, traffic_model
from tests.util import oracle_inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def sa():
    binding.lib()
    return binding


# ------------------------------------------------------------------ C ABI surface
def test_library_exports_every_declared_symbol(sa):
    header = open(os.path.join(ROOT, "include", "sawattn.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = re.findall(r"\b(?:int|const char\*)\s+(\w+)\s*\(", header)
    # the four entry points a caller of the method needs, under their plain names, and the rest
    assert set(names) >= {"attn_fwd", "attn_fwd_launch_info", "attn_last_error", "attn_version"}
    assert set(names) >= {"attn_fwd_variant", "attn_fwd_variant_launch_info", "attn_fwd_plan", "attn_fwd_workspace",
                          "attn_fwd_workspace_bytes", "sawattn_last_error", "sawattn_version"}
    L = sa.lib()
    for n in names:
        assert hasattr(L, n), f"{n} is declared in sawattn.h but not exported"
    assert sa.attn_version() >= 200 and sa.sawattn_version() == sa.attn_version()
    assert L.attn_last_error() is not None and sa.sawattn_last_error() == sa.attn_last_error()
    # the benchmark's probe is a library of its own with a header of its own
    probe = open(os.path.join(ROOT, "include", "sawattn_probe.h")).read()
    probe = re.sub(r"/\*.*?\*/", "", probe, flags=re.S)
    P = sa.probe_lib()
    for n in re.findall(r"\b(?:int|const char\*)\s+(\w+)\s*\(", probe):
        assert hasattr(P, n), f"{n} is declared in sawattn_probe.h but not exported"
    assert not hasattr(L, "sawattn_mfma_probe")


def test_argument_validation_without_a_gpu(sa):
    """Every case below is rejected before anything is launched, so fake pointers are safe."""
    L = sa.lib()
    ok_ptr = 0x1000
    base = dict(Q=ok_ptr, K=ok_ptr, V=ok_ptr, O=0x100000, B=1, H=1, N=128, d=64, scale=0.125, causal=0,
                scan=1, idt=0, odt=0)

    def call(**kw):
        a = dict(base, **kw)
        return L.attn_fwd(a["Q"], a["K"], a["V"], a["O"], a["B"], a["H"], a["N"], a["d"], a["scale"],
                          a["causal"], a["scan"], a["idt"], a["odt"], None)

    assert call(Q=None) == binding.ERR_INVALID_ARG
    assert call(O=None) == binding.ERR_INVALID_ARG
    assert call(K=ok_ptr + 8) == binding.ERR_INVALID_ARG          # misaligned
    assert "aligned" in sa.attn_last_error()
    assert call(B=0) == binding.ERR_INVALID_ARG
    assert call(N=-5) == binding.ERR_INVALID_ARG
    assert call(d=96) == binding.ERR_UNSUPPORTED
    assert "64 or 128" in sa.attn_last_error()
    assert call(scale=float("nan")) == binding.ERR_INVALID_ARG
    assert call(scale=float("inf")) == binding.ERR_INVALID_ARG
    assert call(scan=2) == binding.ERR_INVALID_ARG
    assert call(idt=2) == binding.ERR_INVALID_ARG                 # fp32 inputs are not accepted
    assert call(odt=3) == binding.ERR_INVALID_ARG
    assert call(O=ok_ptr + 128 * 64 * 2 - 16) == binding.ERR_INVALID_ARG   # O starts inside Q
    assert "overlap" in sa.attn_last_error()
    assert call(Q=0x100000, K=0x200000, V=0x300000, O=0x300000 - 128 * 64 * 4 + 16, odt=2) == binding.ERR_INVALID_ARG
    assert call(B=1 << 20, H=1 << 10, N=1 << 20) == binding.ERR_INVALID_ARG   # size overflow
    with pytest.raises(binding.SawattnError):
        sa.attn_fwd_launch_info(1, 1, 128, 80)
    info = binding.LaunchInfo()
    assert L.attn_fwd_launch_info(1, 1, 128, 64, 0, 7, 0, ctypes.byref(info)) == binding.ERR_INVALID_ARG   # scan order
    assert L.attn_fwd_launch_info(1, 1, 128, 64, 0, 1, 2, ctypes.byref(info)) == binding.ERR_INVALID_ARG   # fp32 inputs
    assert L.attn_fwd_launch_info(1, 1, 128, 64, 0, 1, 0, None) == binding.ERR_INVALID_ARG
    # the entry point with the built-in scratch array: the same checks, and its size limit, before anything runs
    def static_call(**kw):
        a = dict(base, **kw)
        return L.attn_fwd_static(a["Q"], a["K"], a["V"], a["O"], a["B"], a["H"], a["N"], a["d"], a["scale"],
                                 a["causal"], a["scan"], a["idt"], a["odt"], None)
    assert static_call(Q=None) == binding.ERR_INVALID_ARG
    assert static_call(d=96) == binding.ERR_UNSUPPORTED
    big = dict(Q=1 << 40, K=2 << 40, V=3 << 40, O=4 << 40, B=1, H=8, N=32768, d=128, idt=1, odt=2)   # bf16, 128 MiB of copies
    assert static_call(**big) == binding.ERR_UNSUPPORTED
    assert "scratch" in sa.attn_last_error() and str(64 << 20) in sa.attn_last_error()


# ------------------------------------------------------------------ schedule oracle: what must hold
SHAPES = [(1, 1, 256), (1, 8, 2048), (1, 16, 8192), (1, 32, 16384), (4, 32, 32768), (2, 3, 333),
          (1, 12, 1000), (3, 7, 300), (1, 8, 128 * 70), (1, 2, 1), (5, 1, 129), (1, 64, 100)]


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("B,H,N", SHAPES)
@pytest.mark.parametrize("tile_q,resident", [(128, 64), (256, 32), (128, 96), (64, 5)])
def test_schedule_oracle_covers_every_tile_once_and_alternates(B, H, N, causal, tile_q, resident):
    sched = so.schedule(B, H, N, causal, "sawtooth", tile_q=tile_q, resident=resident)
    geo = so.launch_geometry(B, H, N, tile_q=tile_q, resident=resident)
    seen = {}
    for wg, recs in sched.items():
        for (head, t, first, last) in recs:
            assert (head, t) not in seen
            seen[(head, t)] = wg
            n_kv = -(-min((t + 1) * geo["tile_q"], N) // 64) if causal else -(-N // 64)
            assert {first, last} == {0, n_kv - 1}             # the whole visible range, one direction
    assert set(seen) == {(h, t) for h in range(B * H) for t in range(geo["q_tiles"])}
    # a head's tiles stay inside the domains it is assigned to, and workgroups of one domain that
    # work in the same round walk in the same direction
    for (head, t), wg in seen.items():
        part = t % geo["parts"]
        assert wg % 8 == (head * geo["parts"] + part) % 8
    cyc = so.schedule(B, H, N, causal, "cyclic", tile_q=tile_q, resident=resident)
    for wg in sched:
        assert [r[:2] for r in cyc[wg]] == [r[:2] for r in sched[wg]]   # same tiles, only direction differs
        assert all(r[2] == 0 for r in cyc[wg])


VARIANTS = [dict(decode="linear"), dict(launch="grid"), dict(launch="grid", tiles_per_workgroup=1),
            dict(launch="grid", decode="linear"), dict(launch="grid", decode="linear", tiles_per_workgroup=1),
            dict(slots_per_domain=1), dict(slots_per_domain=5), dict(decode="linear", slots_per_domain=7)]
WIDE_VARIANTS = [dict(rows_per_wavefront=64), dict(rows_per_wavefront=64, launch="grid"),
                 dict(rows_per_wavefront=64, decode="linear", slots_per_domain=3), dict(rows_per_wavefront=32)]


def oracle_kw(kw, tile_q=128, resident=96):
    """The schedule oracle's inputs for a variant description of the library (d = 64 kernel unless said otherwise)."""
    out = {k: v for k, v in kw.items() if k in ("launch", "decode", "tiles_per_workgroup")}
    out["tile_q"] = tile_q
    out["resident"] = kw.get("slots_per_domain") or resident
    return out


@pytest.mark.parametrize("kw", VARIANTS, ids=lambda kw: "-".join(f"{k}={v}" for k, v in kw.items()))
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("B,H,N", SHAPES)
def test_schedule_oracle_variants_cover_every_tile_once(B, H, N, causal, kw):
    sched = so.schedule(B, H, N, causal, "sawtooth", **oracle_kw(kw))
    geo = so.launch_geometry(B, H, N, **oracle_kw(kw))
    assert len(sched) == geo["grid"] and geo["grid"] % 8 == 0
    seen = set()
    for wg, recs in sched.items():
        assert len(recs) <= geo["max_local"]
        for i, (head, t, first, last) in enumerate(recs):
            assert (head, t) not in seen
            seen.add((head, t))
            n_kv = -(-min((t + 1) * geo["tile_q"], N) // 64) if causal else -(-N // 64)
            assert {first, last} == {0, n_kv - 1}
            if kw.get("launch") == "grid" or kw.get("decode") == "linear":
                assert (first > last) == (i % 2 == 1 and n_kv > 1)     # own iteration parity
            if kw.get("decode", "domain") == "domain":
                assert wg % 8 == (head * geo["parts"] + t % geo["parts"]) % 8
    assert seen == {(h, t) for h in range(B * H) for t in range(geo["q_tiles"])}
    if "slots_per_domain" in kw:
        assert geo["slots"] <= kw["slots_per_domain"]


def test_schedule_oracle_linear_stride_by_hand():
    """Printed Alg. 2 on 3 heads x 5 tiles (N = 640) with G = 8: workgroup 1 takes linear indices
    1 and 9, i.e. (head 0, tile 1) forward and (head 1, tile 4) backward; workgroup 7 takes 7 only."""
    s = so.schedule(1, 3, 640, False, "sawtooth", decode="linear", tile_q=128, resident=1)
    assert s[1] == [(0, 1, 0, 9), (1, 4, 9, 0)]
    assert s[7] == [(1, 2, 0, 9)]
    g = so.schedule(1, 3, 640, True, "sawtooth", launch="grid", decode="linear", tile_q=128, resident=64)
    assert g[2] == [(0, 4, 0, 9), (1, 0, 1, 0)]              # indices 4, 5: last tile of head 0, first of head 1


@pytest.mark.parametrize("B,H,N,causal", [(1, 8, 2048, False), (1, 16, 8192, True), (1, 32, 16384, False),
                                          (4, 32, 32768, True)])
def test_schedule_gives_every_workgroup_the_same_number_of_tile_steps(sa, B, H, N, causal):
    """On the benchmark shapes every workgroup walks the same number of K/V tiles in total: causal
    tiles (tile i costs i+1) are paired long with short inside a head when it has an even number
    of rounds, across two heads when it has one round (workload 3)."""
    trace, count = sa.attn_fwd_plan(B, H, N, 128, causal, "sawtooth", dtype="bf16" if causal else "f16")
    cost = [sum(abs(int(a) - int(b)) + 1 for (_, _, a, b) in trace[wg, : int(count[wg])].tolist())
            for wg in range(trace.shape[0])]
    assert max(cost) == min(cost)


def test_schedule_oracle_hand_example():
    """B*H = 8, N = 128*130: one head per domain, 64 slots, 3 rounds (64 + 64 + 2 tiles).
    Slot 5 of domain 3: round 0 -> tile 5 forward; round 1 (reverse hand-out) -> tile 64 + 58
    backward; round 2 (2 tiles, forward hand-out) -> nothing."""
    s = so.schedule(1, 8, 128 * 130, False, "sawtooth", tile_q=128, resident=64)
    n_kv = 128 * 130 // 64
    assert s[5 * 8 + 3] == [(3, 5, 0, n_kv - 1), (3, 64 + 58, n_kv - 1, 0)]
    assert s[1 * 8 + 3] == [(3, 1, 0, n_kv - 1), (3, 64 + 62, n_kv - 1, 0), (3, 129, 0, n_kv - 1)]


def test_schedule_oracle_hand_example_wide_tiles():
    """Same with 256-row tiles and 32 resident workgroups per domain: N = 256*70 gives 70 tiles, 3 rounds
    (32 + 32 + 6).  Slot 5 of domain 3: tile 5 forward, tile 32 + 26 backward, tile 64 + 5 forward; slot 7 has no
    third tile."""
    s = so.schedule(1, 8, 256 * 70, False, "sawtooth", tile_q=256, resident=32)
    n_kv = 256 * 70 // 64
    assert s[5 * 8 + 3] == [(3, 5, 0, n_kv - 1), (3, 58, n_kv - 1, 0), (3, 69, 0, n_kv - 1)]
    assert s[7 * 8 + 3] == [(3, 7, 0, n_kv - 1), (3, 56, n_kv - 1, 0)]


# ------------------------------------------------------------------ the library's choice of kernel shape, case by case
# (B, H, N, d, causal, dtype) -> (query rows per workgroup tile, workgroups per XCD, workgroups launched).
# Resident workgroups per XCD: 32 CUs x 2 at d = 128 (64 KiB LDS, 256 registers each), x 3 at d = 64, x 1 with
# 256-row tiles (128 KiB LDS, 512 registers).  256-row tiles where the measured break-even says so: d = 128,
# at least 32 such tiles of a head per XCD (64 under the causal mask).
KERNEL_CHOICE = [
    ((1, 1, 256, 64, False, "f16"), (64, 1, 8, "persistent")),            # workload 1: four 64-row tiles, one head over 8 XCDs
    ((1, 8, 2048, 64, False, "f16"), (64, 32, 256, "persistent")),        # workload 2: 32 tiles of 64 rows per head, one head per XCD
    ((1, 8, 2048, 64, True, "f16"), (64, 32, 256, "persistent")),         # ... also under the causal mask
    ((1, 8, 2048, 64, False, "bf16"), (64, 32, 256, "persistent")),       # ... and for bfloat16 inputs
    ((1, 8, 2000, 64, False, "f16"), (64, 32, 256, "persistent")),        # ... ragged lengths included (16 tiles of 128 rows)
    ((1, 8, 2048 + 64, 128, False, "f16"), (128, 17, 136, "persistent")),  # 17 tiles of 128 rows per head: 136 in all, too
                                                                            # many at d = 128
    ((1, 8, 4096, 64, False, "f16"), (64, 64, 512, "persistent")),        # ... d = 64: up to 256 tiles of 128 rows
    ((1, 8, 6144, 64, False, "f16"), (64, 64, 512, "persistent")),        # ... up to 384 (96 tiles of 64 rows per head)
    ((1, 8, 6144 + 64, 64, False, "f16"), (128, 49, 392, "persistent")),  # ... 392: too many
    ((1, 8, 8192, 64, True, "f16"), (64, 64, 512, "persistent")),         # ... under the causal mask up to 512
    ((1, 8, 8192 + 64, 64, True, "f16"), (128, 65, 520, "persistent")),
    ((1, 32, 1024, 64, False, "f16"), (128, 32, 256, "grid")),            # ... and only for N >= 2048: 256 tiles, short scans
    ((1, 16, 1024, 128, False, "f16"), (64, 32, 256, "grid")),  # 128 tiles of 128 rows: still at most half the CUs; two
                                                            # heads of 16 tiles (64 rows) per XCD: side by side
    ((1, 17, 1024, 128, False, "f16"), (128, 17, 136, "grid")),     # 136 tiles: no longer halved; 17 heads in 8 parts of
                                                                    # one tile each: 17 one-tile chunks per XCD, side by side
    ((1, 16, 8192, 128, True, "bf16"), (128, 64, 512, "persistent")),     # workload 3
    ((1, 32, 16384, 128, False, "f16"), (256, 32, 256, "persistent")),    # workload 4: 64 tiles of 256 rows per head
    ((4, 32, 32768, 128, True, "bf16"), (256, 32, 256, "persistent")),    # workload 5: 128 tiles of 256 rows per head
    ((1, 8, 256 * 31, 128, False, "f16"), (128, 62, 496, "persistent")),  # one tile short of the break-even
    ((1, 8, 256 * 32, 128, False, "f16"), (256, 32, 256, "persistent")),
    ((1, 8, 256 * 55, 128, True, "f16"), (128, 64, 512, "persistent")),   # under the mask the break-even is nearly twice as
    ((1, 8, 256 * 56, 128, True, "f16"), (256, 32, 256, "persistent")),   # far out
    ((1, 8, 256 * 64, 128, True, "f16"), (256, 32, 256, "persistent")),
    ((1, 8, 256 * 65, 128, True, "f16"), (128, 64, 512, "persistent")),   # 65 of 96: a third round with one tile
    ((1, 8, 256 * 36, 128, False, "f16"), (128, 64, 512, "persistent")),  # 36 of 64: a second round with four tiles
    ((1, 8, 256 * 56, 128, False, "f16"), (256, 32, 256, "persistent")),  # 56 of 64
    ((1, 8, 256 * 72, 128, False, "f16"), (128, 64, 512, "persistent")),  # 72 of 96
    ((1, 8, 256 * 70, 64, False, "f16"), (128, 96, 768, "persistent")),   # d = 64: three workgroups per CU
    ((1, 8, 256 * 88, 128, False, "bf16"), (256, 32, 256, "persistent")),  # the element type plays no part
    ((1, 1, 256 * 8 * 32, 128, False, "f16"), (256, 32, 256, "persistent")),   # one head over 8 XCDs: 32 tiles each
    ((1, 1, 256 * 8 * 31, 128, False, "f16"), (128, 62, 496, "persistent")),
    ((2, 3, 333, 128, False, "f16"), (64, 6, 48, "grid")),          # 6 heads of 6 tiles of 64 rows (18 of 128: a small
                                                                    # problem), 4 parts per head of at most 2 tiles; 3
                                                                    # chunks per XCD, side by side
    ((2, 3, 333, 128, False, "bf16"), (64, 6, 48, "grid")),         # ... whatever the input type
    # short heads, several per XCD: the direct launch, one tile per workgroup, all heads of an XCD side by side
    ((1, 128, 512, 64, False, "f16"), (128, 64, 512, "grid")),      # 16 heads of 4 tiles per XCD
    ((1, 64, 2048, 64, True, "f16"), (128, 128, 1024, "grid")),     # 8 heads of 16 tiles per XCD, causal
    ((1, 16, 4096, 64, False, "f16"), (128, 64, 512, "grid")),      # 2 heads of 32 tiles per XCD, no mask
    ((1, 16, 4096, 128, True, "f16"), (128, 32, 256, "persistent")),  # ... causal: a long and a short tile per workgroup
    ((1, 16, 2048, 128, True, "f16"), (128, 32, 256, "grid")),      # ... unless both heads' tiles (2 x 16) fit the 32 CUs
    ((1, 16, 2048, 64, True, "f16"), (64, 32, 256, "persistent")),  # (at d = 64 this is still a small problem: 64-row tiles,
                                                                    # 2 x 32 of them per XCD, a long and a short one each)
    ((1, 32, 8192, 64, True, "f16"), (128, 64, 512, "persistent")),  # 4 causal heads of 64 tiles: more than half of 96
    ((1, 32, 4096, 128, True, "bf16"), (128, 128, 1024, "grid")),   # 4 causal heads of 32 tiles per XCD
    ((1, 32, 8192, 128, True, "bf16"), (128, 64, 512, "persistent")),  # a head fills its XCD (64 tiles for 64 workgroups)
]


@pytest.mark.parametrize("shape,want", KERNEL_CHOICE)
def test_kernel_choice_by_hand_listed_cases(sa, shape, want):
    B, H, N, d, causal, dtype = shape
    info = sa.attn_fwd_launch_info(B, H, N, d, causal, dtype=dtype)
    assert (info["tile_q"], info["slots"], info["grid"], ["persistent", "grid"][info["launch"]]) == want
    assert info["tiles_per_workgroup"] == 1      # (two only when a variant asks for the grid launch without saying)
    assert info == sa.attn_fwd_launch_info(B, H, N, d, causal, "cyclic", dtype)     # the order plays no part
    assert info == sa.attn_fwd_variant_launch_info(B, H, N, d, causal, None, dtype)
    assert info["tile_kv"] == 64 and info["block_threads"] == 256 and info["domains"] == 8
    # 8 KiB per K/V tile at d = 64, 16 at d = 128: two K and two V buffers; four each with 256-row tiles; two sets of
    # two each with 64-row tiles (the two halves of the scan at once)
    assert info["lds_bytes"] == {(128, 128): 65536, (128, 64): 32768, (256, 128): 131072, (64, 64): 65536,
                                 (64, 128): 131072}[(info["tile_q"], d)]
    # a request for more workgroups per XCD than fit with 256-row tiles keeps 128-row tiles
    if want[0] == 256:
        assert sa.attn_fwd_variant_launch_info(B, H, N, d, causal, sa.variant(slots_per_domain=64), dtype)["tile_q"] == 128


# ------------------------------------------------------------------ host plan == oracle
@pytest.mark.parametrize("order", ["cyclic", "sawtooth"])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("B,H,N", SHAPES)
def test_host_plan_matches_schedule_oracle(sa, B, H, N, causal, order):
    # d = 64 runs up to 96 workgroups per domain, d = 128 up to 64, or 32 of twice the size for long fp16 inputs
    for d, dtype in ((128, "f16"), (128, "bf16"), (64, "f16")):
        info = sa.attn_fwd_launch_info(B, H, N, d, causal, dtype=dtype)
        okw = oracle_inputs(info, d)
        geo = so.launch_geometry(B, H, N, **okw)
        assert info["grid"] == geo["grid"] and info["slots"] == geo["slots"]
        assert info["parts_per_head"] == geo["parts"] and info["q_tiles_per_head"] == geo["q_tiles"]
        trace, count = sa.attn_fwd_plan(B, H, N, d, causal, order, dtype=dtype)
        want = so.schedule(B, H, N, causal, order, **okw)
        for wg in range(info["grid"]):
            got = [tuple(r) for r in trace[wg, : int(count[wg])].tolist()]
            assert got == want[wg], f"workgroup {wg} d={d} {dtype}"


@pytest.mark.parametrize("kw", VARIANTS, ids=lambda kw: "-".join(f"{k}={v}" for k, v in kw.items()))
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("B,H,N", SHAPES)
def test_host_plan_of_variants_matches_schedule_oracle(sa, B, H, N, causal, kw):
    var = sa.variant(kv_halves=1, **kw)      # 128-row tiles also where the default would halve the scan
    info = sa.attn_fwd_variant_launch_info(B, H, N, 64, causal, var)
    geo = so.launch_geometry(B, H, N, **oracle_kw(kw))
    assert info["grid"] == geo["grid"] and info["slots"] == geo["slots"]
    assert info["max_local_tiles"] == geo["max_local"]
    for order in ("cyclic", "sawtooth"):
        trace, count = sa.attn_fwd_plan(B, H, N, 64, causal, order, var)
        want = so.schedule(B, H, N, causal, order, **oracle_kw(kw))
        for wg in range(info["grid"]):
            got = [tuple(r) for r in trace[wg, : int(count[wg])].tolist()]
            assert got == want[wg], f"workgroup {wg} {order}"


@pytest.mark.parametrize("kw", [dict(), dict(launch="grid"), dict(decode="linear", slots_per_domain=3)],
                         ids=lambda kw: "-".join(f"{k}={v}" for k, v in kw.items()) or "default")
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("B,H,N", [(1, 1, 256), (1, 8, 2048), (2, 3, 384), (1, 32, 16384)])
def test_host_plan_with_halved_scan_matches_schedule_oracle(sa, B, H, N, d, kw):
    """kv_halves = 2: 64-row tiles, two workgroups per CU at d = 64 and one at d = 128 (hand-listed in util.py);
    the work decode is the same function of the tile height as everywhere else."""
    var = sa.variant(kv_halves=2, **kw)
    info = sa.attn_fwd_variant_launch_info(B, H, N, d, False, var)
    assert info["tile_q"] == 64 and info["lds_bytes"] == (65536 if d == 64 else 131072)
    okw = oracle_inputs(info, d, kw)
    assert okw["resident"] == kw.get("slots_per_domain", 64 if d == 64 else 32)
    geo = so.launch_geometry(B, H, N, **okw)
    assert info["grid"] == geo["grid"] and info["slots"] == geo["slots"] and info["max_local_tiles"] == geo["max_local"]
    for order in ("cyclic", "sawtooth"):
        trace, count = sa.attn_fwd_plan(B, H, N, d, False, order, var)
        want = so.schedule(B, H, N, False, order, **okw)
        for wg in range(info["grid"]):
            assert [tuple(r) for r in trace[wg, : int(count[wg])].tolist()] == want[wg], f"workgroup {wg} {order}"


def test_launch_left_open_in_a_variant_is_what_attn_fwd_runs(sa):
    """launch = "auto" in a variant gives the launch attn_fwd picks; with slots_per_domain or the linear decode
    given, that is the persistent one."""
    for shape in ((1, 128, 512, 64, False), (1, 64, 2048, 64, True), (1, 16, 4096, 64, True), (1, 32, 16384, 128, False)):
        assert sa.attn_fwd_variant_launch_info(*shape, sa.variant(launch="auto")) == sa.attn_fwd_launch_info(*shape)
    assert sa.attn_fwd_launch_info(1, 128, 512, 64, False)["launch"] == sa.LAUNCH_GRID
    assert sa.attn_fwd_variant_launch_info(1, 128, 512, 64, False, sa.variant(launch="auto", slots_per_domain=5))["launch"] \
        == sa.LAUNCH_PERSISTENT
    assert sa.attn_fwd_variant_launch_info(1, 128, 512, 64, False, sa.variant(launch="auto", decode="linear"))["launch"] \
        == sa.LAUNCH_PERSISTENT
    assert sa.attn_fwd_variant_launch_info(1, 128, 512, 64, False, sa.variant())["launch"] == sa.LAUNCH_PERSISTENT


def test_halved_scan_is_refused_where_it_does_not_apply(sa):
    for args, kw in (((1, 8, 2048, 128, False), dict(kv_halves=2, rows_per_wavefront=64)),):
        with pytest.raises(sa.SawattnError) as e:
            sa.attn_fwd_variant_launch_info(*args, sa.variant(**kw))
        assert e.value.code == sa.ERR_UNSUPPORTED
    assert sa.attn_fwd_variant_launch_info(1, 8, 2048, 64, False, sa.variant(kv_halves=2), "bf16")["tile_q"] == 64
    for bad in (-1, 3):
        with pytest.raises(sa.SawattnError) as e:
            sa.attn_fwd_variant_launch_info(1, 8, 2048, 64, False, sa.variant(kv_halves=bad))
        assert e.value.code == sa.ERR_INVALID_ARG
    # kv_halves = 1 keeps 128-row tiles where the default would halve
    assert sa.attn_fwd_variant_launch_info(1, 8, 2048, 64, False, sa.variant(kv_halves=1))["tile_q"] == 128
    assert sa.attn_fwd_launch_info(1, 8, 2048, 64, False)["tile_q"] == 64


@pytest.mark.parametrize("kw", WIDE_VARIANTS, ids=lambda kw: "-".join(f"{k}={v}" for k, v in kw.items()))
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("B,H,N", SHAPES)
def test_host_plan_with_rows_per_wavefront_matches_schedule_oracle(sa, B, H, N, causal, kw):
    var = sa.variant(kv_halves=1, **kw)      # (32 rows per wavefront is also what the halved scan runs, on 64-row tiles)
    info = sa.attn_fwd_variant_launch_info(B, H, N, 128, causal, var)
    rows = kw["rows_per_wavefront"]
    okw = oracle_kw(kw, tile_q=4 * rows, resident=32 if rows == 64 else 64)
    geo = so.launch_geometry(B, H, N, **okw)
    assert info["tile_q"] == 4 * rows
    assert info["grid"] == geo["grid"] and info["slots"] == geo["slots"] and info["q_tiles_per_head"] == geo["q_tiles"]
    trace, count = sa.attn_fwd_plan(B, H, N, 128, causal, "sawtooth", var)
    want = so.schedule(B, H, N, causal, "sawtooth", **okw)
    seen = set()
    for wg in range(info["grid"]):
        got = [tuple(r) for r in trace[wg, : int(count[wg])].tolist()]
        assert got == want[wg], f"workgroup {wg}"
        seen |= {(h, t) for (h, t, _, _) in got}
    assert seen == {(h, t) for h in range(B * H) for t in range(geo["q_tiles"])}


@pytest.mark.parametrize("N,d,want", [
    (256, 64, 1), (2048, 64, 1), (8191, 64, 1), (8192, 64, 3), (32768, 64, 3),      # K+V of a head: N * d * 4 bytes
    (512, 128, 1), (4095, 128, 1), (4096, 128, 3), (8192, 128, 3), (16384, 128, 3),
])
def test_q_tiles_are_streamed_only_past_half_an_l2(sa, N, d, want):
    """What attn_fwd does with the tiles touched once, cases listed by hand: O always through LDS as whole
    non-temporal lines (1), Q as well (3) from 2 MiB of K+V per head on; a variant's choice is reported as given."""
    for causal in (False, True):
        assert sa.attn_fwd_launch_info(1, 8, N, d, causal, "sawtooth", "f16")["qo_streaming"] == want
        assert sa.attn_fwd_variant_launch_info(2, 3, N, d, causal, sa.variant(), "bf16")["qo_streaming"] == want
        for mode in (1, 2, 3, 4):
            assert sa.attn_fwd_variant_launch_info(1, 8, N, d, causal, sa.variant(qo_streaming=mode))["qo_streaming"] == mode


def test_variant_fields_are_validated(sa):
    vli = sa.attn_fwd_variant_launch_info
    for bad in (dict(launch=3), dict(launch=-1), dict(decode=-1), dict(slots_per_domain=65), dict(slots_per_domain=-1),
                dict(tiles_per_workgroup=3), dict(align_rounds=2), dict(align_rounds=-1), dict(qo_streaming=5),
                dict(qo_streaming=-1)):
        with pytest.raises(binding.SawattnError) as e:
            vli(1, 8, 2048, 128, False, sa.variant(**bad))
        assert e.value.code == binding.ERR_INVALID_ARG and "variant." in str(e.value)
    with pytest.raises(binding.SawattnError) as e:
        vli(1, 8, 2048, 64, False, sa.variant(rows_per_wavefront=64))
    assert e.value.code == binding.ERR_UNSUPPORTED
    assert vli(1, 8, 2048, 128, False, sa.variant(rows_per_wavefront=64), dtype="bf16")["tile_q"] == 256
    with pytest.raises(binding.SawattnError):
        vli(1, 8, 2048, 128, False, sa.variant(rows_per_wavefront=64, slots_per_domain=33))
    with pytest.raises(binding.SawattnError):
        vli(1, 8, 2048, 128, False, sa.variant(rows_per_wavefront=48))
    assert vli(1, 8, 128 * 200, 64, False, sa.variant(slots_per_domain=96))["slots"] == 96
    with pytest.raises(binding.SawattnError):
        vli(1, 8, 128 * 200, 64, False, sa.variant(slots_per_domain=97))


def test_workspace_bytes_follow_the_choice_of_kernel(sa):
    """A workspace is asked for exactly where bfloat16 inputs, once converted, would run the 64-row kernel."""
    for (B, H, N, d, causal, dtype, kw, want_rows) in (
            (4, 32, 32768, 128, True, "bf16", {}, 64),            # workload 5
            (1, 16, 8192, 128, True, "bf16", {}, 32),             # workload 3: too short under the mask
            (1, 16, 8192, 128, False, "bf16", {}, 64),
            (1, 16, 8192, 128, True, "bf16", dict(rows_per_wavefront=64), 64),
            (1, 16, 32768, 128, False, "bf16", dict(rows_per_wavefront=32), 32),
            (1, 8, 32768, 64, False, "bf16", {}, 32),
            (1, 32, 16384, 128, False, "f16", {}, 64)):            # binary16 needs no copies
        var = sa.variant(**kw) if kw else None
        need, info = sa.attn_fwd_workspace_bytes(B, H, N, d, causal, var, dtype)
        assert info["tile_q"] == 4 * want_rows, (B, H, N, d, causal, dtype, kw)
        assert need == (4 * B * H * N * d if dtype == "bf16" and want_rows == 64 else 0)
        # the geometry is the binary16 one where copies are made, the plain one elsewhere
        as_if = "f16" if need else dtype
        assert info == sa.attn_fwd_variant_launch_info(B, H, N, d, causal, var, as_if)
    with pytest.raises(binding.SawattnError):
        sa.attn_fwd_workspace_bytes(1, 8, 2048, 80, False)


# ------------------------------------------------------------------ traffic model vs the paper's counters
def test_sector_model_matches_printed_counters():
    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "l2_sector_counters.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 4
    for table, S, total, from_tex in rows:
        model = traffic_model.l2_sectors_noncausal(int(S), T=80)
        assert abs(model - int(total)) / int(total) < 0.01        # Table 3: mean error 0.45 %
        assert abs(model - int(from_tex)) / int(from_tex) < 0.01
    # the closed forms the paper prints for D=64, fp16, 32-byte sectors
    S, T = 4096, 64
    assert traffic_model.l2_sectors_noncausal(S, T) == pytest.approx(8 * S * (1 + S / T))
    assert traffic_model.l2_sectors_causal(S, T) == pytest.approx(8 * S * (S / (2 * T) + 0.5))
    assert traffic_model.cold_miss_sectors(S) == 16 * S


def test_byte_model_and_lru_model():
    # workload 4: Q + 128 passes over K,V per head
    b = traffic_model.l2_read_bytes(1, 32, 16384, 128, 128, False)
    assert b == 32 * (16384 * 128 * 2) * (1 + 2 * 128)
    assert traffic_model.l2_read_bytes(1, 1, 1024, 64, 128, True) == 1024 * 64 * 2 * (1 + 2 * 9 / 2)
    assert traffic_model.compulsory_bytes(1, 32, 16384, 128) == 512 * 2 ** 20
    kv = 2 * 16384 * 128 * 2
    assert traffic_model.lru_kv_miss_bytes(16384, 128, 128, 64, 4 * 2 ** 20, False) == 2 * kv
    assert traffic_model.lru_kv_miss_bytes(16384, 128, 128, 64, 4 * 2 ** 20, True) == 2 * kv - 4 * 2 ** 20
    assert traffic_model.lru_kv_miss_bytes(2048, 64, 128, 16, 4 * 2 ** 20, False) == 2 * 2048 * 64 * 2
    # the paper's high-level-kernel experiment (Sec. 4.3): batch 8, S = 128K, D = 64, tile 64,
    # 48 lock-stepped workgroups on a 24 MiB L2: cyclic misses ~ all-access sectors / 48 ~ 3.6e8,
    # reported ~3.7e8; sawtooth reported ~1.2e8
    S = 131072
    all_access = 8 * traffic_model.l2_sectors_noncausal(S, 64)
    assert all_access / 48 == pytest.approx(3.7e8, rel=0.05)


# ------------------------------------------------------------------ the benchmark's profile figures come from profiles/
def test_bench_reads_its_counter_figures_from_the_committed_profiles():
    """bench.py reports HBM-side bytes and L2 misses per scan order as profile figures: they are parsed from the
    rocprofv3 summary of the workload, so they cannot drift from it; every workload has a summary."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    from paper_2601_16032_amd import workloads
    for k, w in workloads.WORKLOADS.items():
        for ws in ([False, True] if k == 5 else [False]):
            traffic, misses, rel = bench.profiled_counters(w.name, ws)
            assert rel is not None and os.path.exists(os.path.join(ROOT, rel)), (w.name, ws)
            text = open(os.path.join(ROOT, rel)).read()
            for order in ("sawtooth", "cyclic"):
                assert traffic[order] > 0 and misses[order] > 0
                assert f"total {traffic[order]:.4e} bytes per launch" in text
                # at least the bytes every launch has to move: Q, K, V read once
                assert traffic[order] >= 3 * w.B * w.H * w.N * w.d * 2 * 0.5
            assert set(traffic) == set(misses) == {"sawtooth", "cyclic"}
    assert bench.profiled_counters("no_such_workload", False) == ({}, {}, None)


def test_build_refuses_wide_kernels_that_spill():
    """The build reads the compiler's resource remarks and refuses a library whose 64-rows-per-wavefront kernels
    need scratch memory (their inline-assembly MFMAs are only sound without spills)."""
    from paper_2601_16032_amd import build as hip_build

    def remarks(scratch_of_one):
        lines = []
        for i, (bf, ca, nh) in enumerate([(0, 0, 2), (0, 1, 2), (1, 0, 2), (1, 1, 2), (0, 0, 1)]):
            name = f"_ZN7sawattn15attn_fwd_kernelILi128ELb{bf}ELb{ca}ELi{nh}ELb0EEEvNS_6ParamsE"
            scratch = scratch_of_one if i == 2 else (16 if nh == 1 else 0)
            lines += [f"x.hip:1:1: remark: Function Name: {name} [-Rpass-analysis=kernel-resource-usage]",
                      "x.hip:1:1: remark:     VGPRs: 233 [-Rpass-analysis=kernel-resource-usage]",
                      f"x.hip:1:1: remark:     ScratchSize [bytes/lane]: {scratch} [-Rpass-analysis=kernel-resource-usage]",
                      "x.hip:1:1: remark:     Occupancy [waves/SIMD]: 1 [-Rpass-analysis=kernel-resource-usage]"]
        return "\n".join(lines)

    res = hip_build.kernel_resources(remarks(0))
    assert len(res) == 5
    assert res["_ZN7sawattn15attn_fwd_kernelILi128ELb0ELb0ELi2ELb0EEEvNS_6ParamsE"] == {"VGPRs": 233, "ScratchSize": 0, "Occupancy": 1}
    hip_build.check_wide_kernels(res)                       # 32-row kernels may spill a little, wide ones not at all
    with pytest.raises(RuntimeError, match="must not use scratch"):
        hip_build.check_wide_kernels(hip_build.kernel_resources(remarks(188)))
    with pytest.raises(RuntimeError, match="expected the resource usage of 4"):
        hip_build.check_wide_kernels({})


def test_header_is_plain_c_and_the_binding_mirrors_its_structs(tmp_path):
    """include/sawattn.h compiles as C99 on its own, and the ctypes mirrors in binding.py have the header's field
    names, order, offsets and sizes (read back from a program gcc builds from the header)."""
    import ctypes
    import re
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    header = open(os.path.join(root, "include", "sawattn.h")).read()
    fields = {}
    for name in ("sawattn_variant", "sawattn_launch_info"):
        body = re.search(r"typedef struct %s \{(.*?)\} %s;" % (name, name), header, re.S).group(1)
        body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
        fields[name] = re.findall(r"\bint\s+(\w+)\s*;", body)
    prints = "".join('printf("%s.%s %%zu\\n", offsetof(%s, %s));\n' % (s, f, s, f) for s, fs in fields.items() for f in fs)
    prints += "".join('printf("%s %%zu\\n", sizeof(%s));\n' % (s, s) for s in fields)
    src = tmp_path / "abi.c"
    src.write_text('#include <stddef.h>\n#include <stdio.h>\n#include "sawattn.h"\nint main(void) {\n' + prints + "return 0; }\n")
    exe = tmp_path / "abi"
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(root, "include"), str(src), "-o", str(exe)],
                   check=True, capture_output=True)
    got = dict(line.split() for line in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines())
    for cname, mirror in (("sawattn_variant", binding.Variant), ("sawattn_launch_info", binding.LaunchInfo)):
        assert [n for n, _ in mirror._fields_] == fields[cname]
        assert int(got[cname]) == ctypes.sizeof(mirror)
        for n, _ in mirror._fields_:
            assert int(got[f"{cname}.{n}"]) == getattr(mirror, n).offset
