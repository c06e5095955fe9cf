"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on the same
seeded inputs.  Tolerance: max-abs 2e-3 and relative-L2 1e-3 (tests/util.py)."""
import math

import numpy as np
import pytest
import torch

from paper_2601_16032_amd import binding, workloads
from tests.util import assert_close, errors, oracle_inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sa():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2601_16032_amd import binding
    binding.lib()
    return binding


def run_gpu(sa, Q, K, V, scale, causal, order, o_dtype=None):
    O = sa.attn_fwd(Q.cuda(), K.cuda(), V.cuda(), scale=scale, causal=causal, scan_order=order,
                    o_dtype=o_dtype)
    torch.cuda.synchronize()
    return O.double().cpu().numpy()


ORDERS = ["cyclic", "sawtooth"]


# ------------------------------------------------------------------ small workloads, every element
@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("cfg", [1, 2])
def test_small_workloads_all_elements(sa, oracle, cfg, order):
    w = workloads.WORKLOADS[cfg]
    Q, K, V = workloads.make_qkv(w)
    want = oracle.attention(Q, K, V, w.scale, causal=w.causal)
    got = run_gpu(sa, Q, K, V, w.scale, w.causal, order)
    print(w.name, order, assert_close(got, want, f"{w.name} {order}"))
    got32 = run_gpu(sa, Q, K, V, w.scale, w.causal, order, o_dtype=torch.float32)
    print(w.name, order, "f32 out", assert_close(got32, want, f"{w.name} {order} f32"))


# ------------------------------------------------------------------ ragged and tiny shapes
RAGGED = [1, 2, 5, 31, 32, 33, 63, 64, 65, 127, 128, 129, 191, 200, 257, 333, 640, 1000]


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("d", [64, 128])
def test_ragged_lengths(sa, oracle, d, dtype, causal):
    for k, N in enumerate(RAGGED):
        B, H = (1, 1) if k % 3 == 0 else ((2, 3) if k % 3 == 1 else (1, 8))
        Q, K, V = workloads.make_random(B, H, N, d, dtype, seed=1000 + N)
        scale = 1.0 / math.sqrt(d)
        want = oracle.attention(Q, K, V, scale, causal=causal)
        for order in ORDERS:
            got = run_gpu(sa, Q, K, V, scale, causal, order, o_dtype=torch.float32)
            assert_close(got, want, f"N={N} d={d} {dtype} causal={causal} B={B} H={H} {order}")


@pytest.mark.parametrize("causal", [False, True])
def test_many_rounds_and_heads(sa, oracle, causal):
    """More query tiles than resident workgroups of a domain (several rounds, both directions) and
    more heads than domains (several chunks per domain)."""
    Q, K, V = workloads.make_random(1, 8, 128 * 100, 64, "f16", seed=77)   # 100 tiles per head: 2 rounds of 96
    rows = list(range(0, 128 * 100, 131)) + [128 * 100 - 1]
    want = oracle.attention(Q, K, V, 0.125, causal=causal, rows=rows)
    for order in ORDERS:
        got = run_gpu(sa, Q, K, V, 0.125, causal, order, o_dtype=torch.float32)[:, :, rows]
        assert_close(got, want, f"100 tiles causal={causal} {order}")
    Q, K, V = workloads.make_random(3, 7, 300, 128, "bf16", seed=78)      # 21 heads, parts = 8
    want = oracle.attention(Q, K, V, 0.09, causal=causal)
    for order in ORDERS:
        got = run_gpu(sa, Q, K, V, 0.09, causal, order, o_dtype=torch.float32)
        assert_close(got, want, f"21 heads causal={causal} {order}")


# ------------------------------------------------------------------ degenerate inputs
def test_scale_sign_and_zero(sa, oracle):
    Q, K, V = workloads.make_random(1, 2, 300, 64, "f16", seed=5)
    for scale in (-0.125, 0.0, 0.5, 1e-3):
        for causal in (False, True):
            want = oracle.attention(Q, K, V, scale, causal=causal)
            got = run_gpu(sa, Q, K, V, scale, causal, "sawtooth", o_dtype=torch.float32)
            assert_close(got, want, f"scale={scale} causal={causal}")
    # the same through the kernel with 64 rows per wavefront (d = 128), whose masked tiles rely on -inf scores:
    # scale = 0 and a scale below the floor of 1e-30 on scale*log2(e) must both come out as uniform attention
    Q, K, V = workloads.make_random(1, 2, 700, 128, "bf16", seed=6)
    for scale in (0.0, 1e-36, -0.09):
        for causal in (False, True):
            want = oracle.attention(Q, K, V, scale, causal=causal)
            for order in ORDERS:
                O = sa.attn_fwd_variant(Q.cuda(), K.cuda(), V.cuda(), scale=scale, causal=causal, scan_order=order,
                                        o_dtype=torch.float32, variant=sa.variant(rows_per_wavefront=64))
                torch.cuda.synchronize()
                assert_close(O.double().cpu().numpy(), want, f"wide scale={scale} causal={causal} {order}")


def test_identical_keys_uniform_attention(sa, oracle):
    Q, K, V = workloads.make_random(1, 2, 500, 128, "f16", seed=6)
    K = K[:, :, :1].expand_as(K).contiguous()
    for causal in (False, True):
        want = oracle.attention(Q, K, V, 0.1, causal=causal)
        got = run_gpu(sa, Q, K, V, 0.1, causal, "sawtooth", o_dtype=torch.float32)
        assert_close(got, want, f"identical keys causal={causal}")


def test_peaked_rows_one_hot(sa, oracle):
    """Each query matches exactly one key with a large score: P is one-hot to fp16 precision."""
    N, d = 384, 64
    g = torch.Generator("cpu").manual_seed(7)
    perm = torch.randperm(N, generator=g)
    K = torch.zeros(1, 1, N, d)
    K[0, 0, torch.arange(N), torch.arange(N) % d] = 1.0
    K[0, 0, :, :] += 0.01 * torch.randn(N, d, generator=g)
    Q = 40.0 * K[:, :, perm]
    V = torch.randn(1, 1, N, d, generator=g)
    Q, K, V = Q.half(), K.half(), V.half()
    want = oracle.attention(Q, K, V, 1.0)
    for order in ORDERS:
        got = run_gpu(sa, Q, K, V, 1.0, False, order, o_dtype=torch.float32)
        assert_close(got, want, f"peaked {order}")


@pytest.mark.parametrize("dtype,d", [("f16", 64), ("bf16", 128), ("f16", 128), ("bf16", 64)])
def test_moving_maximum_in_both_directions(sa, oracle, dtype, d):
    """Scores whose level changes from K/V tile to K/V tile by far more than the slack the kernel
    allows before it rescales (Alg. 1's running maximum has to be raised again and again), on a
    shape with two rounds per head so that the same rows' neighbours are scanned in both directions."""
    H, N = 8, 128 * 100
    g = torch.Generator("cpu").manual_seed(4242 + d)
    level = 60.0 * torch.rand(H, N // 64, generator=g)                 # per 64-key tile
    level[:, 5] = 75.0                                                 # a clear winner somewhere early
    level[:, -9] = 74.0                                                # and a runner-up near the end
    K = torch.randn(1, H, N, d, generator=g)
    K[0, :, :, 0] = level.repeat_interleave(64, dim=1)
    Q = 0.3 * torch.randn(1, H, N, d, generator=g)
    Q[0, :, :, 0] = 4.0
    V = torch.randn(1, H, N, d, generator=g)
    cast = (lambda t: t.half()) if dtype == "f16" else (lambda t: t.bfloat16())
    Q, K, V = cast(Q), cast(K), cast(V)
    rows = list(range(0, N, 517)) + [N - 1]
    for causal in (False, True):
        want = oracle.attention(Q, K, V, 1.0, causal=causal, rows=rows)
        for order in ORDERS:
            got = run_gpu(sa, Q, K, V, 1.0, causal, order, o_dtype=torch.float32)[:, :, rows]
            assert_close(got, want, f"moving maximum {dtype} d={d} causal={causal} {order}")


def test_launches_overlapping_on_two_streams(sa):
    """Launches that run at the same time share the library's per-XCD arrival counters; that may
    cost cache hits but never changes a result (each output tile is computed by one workgroup in a
    fixed order), so the outputs equal those of the same launches run one after another."""
    a = workloads.make_random(1, 24, 2048, 128, "f16", seed=31, device="cuda")
    b = workloads.make_random(2, 16, 1024, 64, "bf16", seed=32, device="cuda")
    ref_a = sa.attn_fwd(*a, scale=0.09, causal=False, scan_order="sawtooth")
    torch.cuda.synchronize()
    ref_b = sa.attn_fwd(*b, scale=0.125, causal=True, scan_order="sawtooth")
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    out_a = [torch.empty_like(ref_a) for _ in range(3)]
    out_b = [torch.empty_like(ref_b) for _ in range(3)]
    for i in range(3):
        sa.attn_fwd(*a, out_a[i], scale=0.09, causal=False, scan_order="sawtooth", stream=s1)
        sa.attn_fwd(*b, out_b[i], scale=0.125, causal=True, scan_order="sawtooth", stream=s2)
    s1.synchronize()
    s2.synchronize()
    for i in range(3):
        assert torch.equal(out_a[i], ref_a) and torch.equal(out_b[i], ref_b)


def test_large_common_shift(sa, oracle):
    """A large offset shared by all keys shifts every score of a row by the same amount."""
    Q, K, V = workloads.make_random(1, 1, 256, 64, "bf16", seed=8)
    K = (K.float() + 3.0).bfloat16()
    want = oracle.attention(Q, K, V, 0.125)
    got = run_gpu(sa, Q, K, V, 0.125, False, "sawtooth", o_dtype=torch.float32)
    assert_close(got, want, "shifted keys")


@pytest.mark.parametrize("o_dtype", [torch.float16, torch.bfloat16, torch.float32])
def test_output_dtypes_round_the_same_accumulator(sa, o_dtype):
    Q, K, V = workloads.make_random(1, 2, 300, 128, "bf16", seed=9, device="cuda")
    ref = sa.attn_fwd(Q, K, V, scale=0.1, causal=True, scan_order="cyclic", o_dtype=torch.float32)
    out = sa.attn_fwd(Q, K, V, scale=0.1, causal=True, scan_order="cyclic", o_dtype=o_dtype)
    torch.cuda.synchronize()
    assert out.dtype == o_dtype
    assert torch.equal(out, ref.to(o_dtype))   # same kernel, same order: only the final rounding differs


# ------------------------------------------------------------------ full-size workloads, sampled rows
def sample_rows(N, seed, n=48):
    g = np.random.default_rng(seed)
    fixed = [0, 1, 63, 64, 127, 128, N // 2 - 1, N // 2, N - 129, N - 128, N - 1]
    return sorted(set(fixed) | set(int(x) for x in g.integers(0, N, size=n)))


@pytest.mark.parametrize("cfg", [3, 4, 5])
def test_full_size_workloads_sampled_rows(sa, oracle, cfg):
    w = workloads.WORKLOADS[cfg]
    print("generating", w.name, flush=True)
    Q, K, V = workloads.make_qkv(w)
    Qd, Kd, Vd = Q.cuda(), K.cuda(), V.cuda()
    o_dtype = torch.float32 if w.dtype == "bf16" else torch.float16
    outs = {}
    for order in ORDERS:
        print("launch", w.name, order, flush=True)
        outs[order] = sa.attn_fwd(Qd, Kd, Vd, scale=w.scale, causal=w.causal, scan_order=order,
                                  o_dtype=o_dtype)
        torch.cuda.synchronize()
    g = np.random.default_rng(100 + cfg)
    heads = {(0, 0), (w.B - 1, w.H - 1), (0, min(8, w.H - 1)), (w.B - 1, 7 % w.H)}
    while len(heads) < 6:
        heads.add((int(g.integers(0, w.B)), int(g.integers(0, w.H))))
    rows = sample_rows(w.N, 200 + cfg)
    for (b, h) in sorted(heads):
        want = oracle.attention(Q[b:b + 1, h:h + 1], K[b:b + 1, h:h + 1], V[b:b + 1, h:h + 1],
                                w.scale, causal=w.causal, rows=rows)[0, 0]
        for order in ORDERS:
            got = outs[order][b, h][rows].double().cpu().numpy()
            e = assert_close(got, want, f"{w.name} head ({b},{h}) {order}")
            print(w.name, (b, h), order, "max-abs %.2e rel-L2 %.2e" % e, flush=True)
    # the two scan orders agree with each other everywhere (not only on the sampled rows)
    a, c = outs["cyclic"], outs["sawtooth"]
    diff = (a.float() - c.float())
    assert torch.isfinite(a.float()).all() and torch.isfinite(c.float()).all()
    max_abs = diff.abs().max().item()
    rel = (diff.double().pow(2).sum().sqrt() / a.double().pow(2).sum().sqrt()).item()
    print(w.name, "cyclic vs sawtooth: max-abs %.2e rel-L2 %.2e" % (max_abs, rel), flush=True)
    assert max_abs <= 2e-3 and rel <= 1e-3


# ------------------------------------------------------------------ the shapes the sweeps report (Sec. 3.2, Sec. 4.3)
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("B,H,N,d", [(1, 1, 131072, 64), (1, 1, 131072, 128), (8, 1, 32768, 64)])
def test_sweep_shapes_sampled_rows(sa, oracle, B, H, N, d, causal):
    """The longest points of the sequence-length and batch sweeps: one head spread over all eight XCDs with
    1024 (512) query tiles per head, several rounds per chunk, and the batch-of-eight shape.  About fifty sampled rows
    per head against the oracle, both scan orders, plus the two orders against each other on every element."""
    Q, K, V = workloads.make_random(B, H, N, d, "f16", seed=9000 + N + d)
    scale = 1.0 / math.sqrt(d)
    Qd, Kd, Vd = Q.cuda(), K.cuda(), V.cuda()
    info = sa.attn_fwd_launch_info(B, H, N, d, causal)
    assert info["q_tiles_per_head"] == -(-N // info["tile_q"]) and info["parts_per_head"] == 8 // math.gcd(B * H, 8)
    outs = {}
    for order in ORDERS:
        outs[order] = sa.attn_fwd(Qd, Kd, Vd, scale=scale, causal=causal, scan_order=order, o_dtype=torch.float32)
        torch.cuda.synchronize()
    rows = sample_rows(N, 300 + d, n=40)
    for b in sorted({0, B // 2, B - 1}):
        want = oracle.attention(Q[b:b + 1], K[b:b + 1], V[b:b + 1], scale, causal=causal, rows=rows)[0, 0]
        for order in ORDERS:
            got = outs[order][b, 0][rows].double().cpu().numpy()
            e = assert_close(got, want, f"sweep shape B{B} N{N} d{d} causal={causal} batch {b} {order}")
            print((B, H, N, d), causal, b, order, "max-abs %.2e rel-L2 %.2e" % e, flush=True)
    e = assert_close(outs["sawtooth"].double().cpu().numpy(), outs["cyclic"].double().cpu().numpy(),
                     f"sweep shape B{B} N{N} d{d} causal={causal}: sawtooth vs cyclic")


@pytest.mark.parametrize("cfg", [1, 2])
def test_scan_orders_agree_small(sa, cfg):
    w = workloads.WORKLOADS[cfg]
    Q, K, V = workloads.make_qkv(w, device="cuda")
    a = sa.attn_fwd(Q, K, V, scale=w.scale, causal=w.causal, scan_order="cyclic", o_dtype=torch.float32)
    b = sa.attn_fwd(Q, K, V, scale=w.scale, causal=w.causal, scan_order="sawtooth", o_dtype=torch.float32)
    torch.cuda.synchronize()
    e = errors(b.cpu().numpy(), a.cpu().numpy())
    assert e[0] <= 2e-3 and e[1] <= 1e-3


# ------------------------------------------------------------------ work decode and scan direction
@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("B,H,N,d", [(1, 8, 128 * 70, 128), (1, 8, 128 * 100, 64), (2, 3, 333, 128), (1, 32, 4096, 128),
                                     (1, 1, 256, 64), (1, 8, 256 * 64 + 10, 128)])
def test_device_schedule_matches_oracle(sa, B, H, N, d, causal, order):
    """Every workgroup records the query tile it took at each local iteration and the first / last
    K/V tile it visited; bit-exact against the schedule oracle (Alg. 2 + Alg. 4 per cache domain)."""
    from oracle import schedule_oracle as so
    Q, K, V = workloads.make_random(B, H, N, d, "f16", seed=21, device="cuda")
    O, trace, count = sa.attn_fwd_variant(Q, K, V, scale=0.1, causal=causal, scan_order=order, trace=True)
    O2 = sa.attn_fwd(Q, K, V, scale=0.1, causal=causal, scan_order=order)
    torch.cuda.synchronize()
    assert torch.equal(O, O2)                      # recording the schedule does not change the result
    want = so.schedule(B, H, N, causal, order, **oracle_inputs(sa.attn_fwd_launch_info(B, H, N, d, causal), d))
    trace, count = trace.cpu(), count.cpu()
    assert trace.shape[0] == len(want)
    for wg, recs in want.items():
        got = [tuple(r) for r in trace[wg, : int(count[wg])].tolist()]
        assert got == recs, f"workgroup {wg}"


# ------------------------------------------------------------------ launch variants (Alg. 2 as printed, Alg. 3, fewer slots)
VARIANTS = [dict(decode="linear"), dict(launch="grid"), dict(launch="grid", tiles_per_workgroup=1),
            dict(launch="grid", decode="linear"), dict(slots_per_domain=3), dict(decode="linear", slots_per_domain=7),
            dict(align_rounds=1), dict(align_rounds=1, slots_per_domain=2)]


@pytest.mark.parametrize("kw", VARIANTS, ids=lambda kw: "-".join(f"{k}={v}" for k, v in kw.items()))
@pytest.mark.parametrize("causal", [False, True])
def test_variants_schedule_and_output(sa, oracle, kw, causal):
    """Each variant runs the schedule its oracle lists (bit-exact records), gives the default
    schedule's output bit for bit under the cyclic order (same tiles, same direction, other
    workgroups), and stays within tolerance of the fp64 oracle under the sawtooth order."""
    from oracle import schedule_oracle as so
    var = sa.variant(**kw)
    for (B, H, N, d, dtype) in [(1, 8, 128 * 21 + 50, 64, "f16"), (2, 3, 700, 128, "bf16")]:
        Q, K, V = workloads.make_random(B, H, N, d, dtype, seed=55 + N, device="cuda")
        scale = 1.0 / math.sqrt(d)
        base = sa.attn_fwd(Q, K, V, scale=scale, causal=causal, scan_order="cyclic", o_dtype=torch.float32)
        want_O = oracle.attention(Q.cpu(), K.cpu(), V.cpu(), scale, causal=causal)
        for order in ORDERS:
            O, trace, count = sa.attn_fwd_variant(Q, K, V, scale=scale, causal=causal, scan_order=order,
                                                  o_dtype=torch.float32, variant=var, trace=True)
            torch.cuda.synchronize()
            info = sa.attn_fwd_variant_launch_info(B, H, N, d, causal, var, dtype)
            want = so.schedule(B, H, N, causal, order, **oracle_inputs(info, d, kw))
            trace, count = trace.cpu(), count.cpu()
            assert trace.shape[0] == len(want)
            for wg, recs in want.items():
                got = [tuple(r) for r in trace[wg, : int(count[wg])].tolist()]
                assert got == recs, f"workgroup {wg} {order}"
            if order == "cyclic":
                assert torch.equal(O, base)
            assert_close(O.double().cpu().numpy(), want_O, f"variant {kw} {order} causal={causal} N={N}")


def test_variants_at_full_size_agree_with_default(sa):
    """Workload 4's shape under every variant: cyclic bit-identical to the default, sawtooth within
    the summation-order difference."""
    w = workloads.WORKLOADS[4]
    Q, K, V = workloads.make_qkv(w, device="cuda")
    base = sa.attn_fwd(Q, K, V, scale=w.scale, causal=False, scan_order="cyclic")
    for kw in VARIANTS:
        var = sa.variant(**kw)
        O = sa.attn_fwd_variant(Q, K, V, scale=w.scale, causal=False, scan_order="cyclic", variant=var)
        assert torch.equal(O, base), kw
        O = sa.attn_fwd_variant(Q, K, V, scale=w.scale, causal=False, scan_order="sawtooth", variant=var)
        print(kw, assert_close(O.double().cpu().numpy(), base.double().cpu().numpy(), f"variant {kw}"))


# ------------------------------------------------------------------ 64 query rows per wavefront (d = 128)
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", ["f16", "bf16", "bf16-workspace"])
def test_wide_rows_variant_small_shapes(sa, oracle, dtype, causal):
    """256-row workgroup tiles, every length class: shorter than a tile, ragged, one and several tiles,
    both scan orders, also under the direct launch (second tile backward) and with few slots (many rounds).
    bfloat16 inputs run this kernel as they are (V converted on its way into LDS) or, given a workspace, through
    binary16 copies of K and V."""
    from oracle import schedule_oracle as so
    call = sa.attn_fwd_workspace if dtype == "bf16-workspace" else sa.attn_fwd_variant
    dtype = dtype.split("-")[0]
    for k, N in enumerate([1, 63, 64, 65, 200, 256, 257, 511, 512, 777, 1000, 2048 + 33]):
        B, H = (1, 2) if k % 2 == 0 else (2, 3)
        Q, K, V = workloads.make_random(B, H, N, 128, dtype, seed=2000 + N)
        scale = 1.0 / math.sqrt(128)
        want = oracle.attention(Q, K, V, scale, causal=causal)
        for kw in (dict(), dict(launch="grid"), dict(slots_per_domain=1)):
            var = sa.variant(rows_per_wavefront=64, **kw)
            for order in ORDERS:
                O, trace, count = call(Q.cuda(), K.cuda(), V.cuda(), scale=scale, causal=causal,
                                       scan_order=order, o_dtype=torch.float32, variant=var, trace=True)
                torch.cuda.synchronize()
                assert_close(O.double().cpu().numpy(), want, f"wide N={N} {dtype} causal={causal} {kw} {order}")
                sched = so.schedule(B, H, N, causal, order, **oracle_inputs({"tile_q": 256}, 128, kw))
                trace, count = trace.cpu(), count.cpu()
                for wg, recs in sched.items():
                    assert [tuple(r) for r in trace[wg, : int(count[wg])].tolist()] == recs, f"workgroup {wg}"


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
@pytest.mark.parametrize("scale_factor", [1.0, 8.0])
@pytest.mark.parametrize("causal", [False, True])
def test_wide_rows_moving_maximum_and_default_choice(sa, oracle, causal, scale_factor, dtype):
    """A sequence long enough that the library picks 64 rows per wavefront by itself (two rounds of 32 slots per
    head), with score levels that jump from tile to tile by far more than the slack, so that the reference
    maximum is raised again and again in both scan directions.  Every row is compared with the oracle, at the
    usual scale (scores step by up to 53) and at eight times that (steps of several hundred)."""
    H, N, d = 8, (256 * 128 if causal else 256 * 56) + 100, 128      # 129 (57) tiles of 256 rows: well-filled rounds
    scale = scale_factor / math.sqrt(d)
    assert sa.attn_fwd_launch_info(1, H, N, d, causal, dtype=dtype)["tile_q"] == 256
    g = torch.Generator("cpu").manual_seed(99)
    level = 60.0 * torch.rand(H, (N + 63) // 64, generator=g)
    level[:, 7] = 75.0
    level[:, -11] = 74.0
    K = torch.randn(1, H, N, d, generator=g)
    K[0, :, :, 0] = level.repeat_interleave(64, dim=1)[:, :N]
    Q = 3.0 * torch.randn(1, H, N, d, generator=g)
    Q[0, :, :, 0] = 8.0          # scores step by up to 8 * 75 * scale = 53 between tiles
    V = torch.randn(1, H, N, d, generator=g)
    Q, K, V = Q.to(dtype), K.to(dtype), V.to(dtype)
    # every row of two heads, sampled rows of the others
    rows = list(range(0, N, 389)) + [N - 1]
    want_all = oracle.attention(Q[:, :2], K[:, :2], V[:, :2], scale, causal=causal)
    want = oracle.attention(Q, K, V, scale, causal=causal, rows=rows)
    Qd, Kd, Vd = Q.cuda(), K.cuda(), V.cuda()
    for order in ORDERS:
        got = sa.attn_fwd(Qd, Kd, Vd, scale=scale, causal=causal, scan_order=order, o_dtype=torch.float32)
        narrow = sa.attn_fwd_variant(Qd, Kd, Vd, scale=scale, causal=causal, scan_order=order, o_dtype=torch.float32,
                                     variant=sa.variant(rows_per_wavefront=32))
        torch.cuda.synchronize()
        what = f"wide default causal={causal} x{scale_factor} {order}"
        assert_close(got.double().cpu().numpy()[:, :, rows], want, what)
        assert_close(got.double().cpu().numpy()[:, :2], want_all, what + " all rows")
        # and the two kernel shapes agree with each other on every row
        assert_close(got.double().cpu().numpy(), narrow.double().cpu().numpy(), what + " vs 32 rows")


@pytest.mark.parametrize("seed", [1, 2])
def test_wide_kernel_random_shapes_and_score_patterns(sa, oracle, seed):
    """Seeded random cases for the 64-rows-per-wavefront kernel (bf16 ones directly and through the workspace): lengths around
    the tile boundaries, few slots (many rounds), both launches and orders, any scale, and three score patterns --
    plain N(0,1), levels that jump between 64-key tiles by up to 40 score units, and a ramp that raises the maximum
    on every tile in one scan direction and never in the other."""
    rng = np.random.default_rng(seed)
    d = 128
    for case in range(30):
        dtype = str(rng.choice(["f16", "bf16", "bf16-workspace"]))
        causal = bool(rng.integers(0, 2))
        B, H = int(rng.integers(1, 3)), int(rng.integers(1, 4))
        N = int(rng.choice([rng.integers(1, 70), rng.integers(60, 400), rng.integers(250, 1400), rng.integers(1000, 3000)]))
        order = str(rng.choice(ORDERS))
        scale = float(rng.choice([1.0, 1.0, 0.25, 3.0, -1.0])) / math.sqrt(128)
        g = torch.Generator("cpu").manual_seed(int(rng.integers(0, 1 << 30)))
        Q, K, V = (torch.randn(B, H, N, d, generator=g) for _ in range(3))
        mode = int(rng.integers(0, 3))
        if mode == 1:
            level = 40.0 * torch.rand(B, H, (N + 63) // 64, generator=g)
            K[:, :, :, 0] = level.repeat_interleave(64, dim=2)[:, :, :N]
            Q[:, :, :, 0] = 6.0
        elif mode == 2:
            K[:, :, :, 1] = torch.linspace(0, 60, N)
            Q[:, :, :, 1] = 5.0 * (1 if rng.integers(0, 2) else -1)
        dt = torch.float16 if dtype == "f16" else torch.bfloat16
        Q, K, V = Q.to(dt), K.to(dt), V.to(dt)
        want = oracle.attention(Q, K, V, scale, causal=causal)
        var = sa.variant(rows_per_wavefront=64, slots_per_domain=int(rng.choice([0, 1, 2])),
                         launch=str(rng.choice(["persistent", "grid"])))
        call = sa.attn_fwd_workspace if dtype == "bf16-workspace" else sa.attn_fwd_variant
        O = call(Q.cuda(), K.cuda(), V.cuda(), scale=scale, causal=causal, scan_order=order, o_dtype=torch.float32,
                 variant=var)
        torch.cuda.synchronize()
        assert_close(O.double().cpu().numpy(), want,
                     f"case {case}: {dtype} B{B} H{H} N{N} causal={causal} {order} pattern {mode} scale {scale:.3f}")


# ------------------------------------------------------------------ bfloat16 through binary16 copies in a workspace
@pytest.mark.parametrize("causal", [False, True])
def test_workspace_path_small_shapes(sa, oracle, causal):
    """bfloat16 inputs with a workspace and 64 rows per wavefront: K and V go through binary16 copies, Q is
    converted as it is loaded.  Every length class, both scan orders, schedule as for binary16 inputs; the caller's
    tensors stay untouched; without a workspace the same request runs the kernel on the bfloat16 tensors."""
    from oracle import schedule_oracle as so
    var = sa.variant(rows_per_wavefront=64)
    for k, N in enumerate([1, 63, 64, 65, 200, 256, 257, 511, 777, 2048 + 33]):
        B, H = (1, 2) if k % 2 == 0 else (2, 3)
        Q, K, V = workloads.make_random(B, H, N, 128, "bf16", seed=3000 + N)
        scale = 1.0 / math.sqrt(128)
        want = oracle.attention(Q, K, V, scale, causal=causal)
        Qd, Kd, Vd = Q.cuda(), K.cuda(), V.cuda()
        need, info = sa.attn_fwd_workspace_bytes(B, H, N, 128, causal, var, "bf16")
        assert need == 4 * B * H * N * 128 and info["tile_q"] == 256
        ws = torch.full((need + 64,), 0x5A, dtype=torch.uint8, device="cuda")
        for order in ORDERS:
            O, trace, count = sa.attn_fwd_workspace(Qd, Kd, Vd, scale=scale, causal=causal, scan_order=order,
                                                    o_dtype=torch.float32, variant=var, trace=True, workspace=ws[:need])
            torch.cuda.synchronize()
            assert_close(O.double().cpu().numpy(), want, f"workspace N={N} causal={causal} {order}")
            sched = so.schedule(B, H, N, causal, order, **oracle_inputs(info, 128))
            trace, count = trace.cpu(), count.cpu()
            for wg, recs in sched.items():
                assert [tuple(r) for r in trace[wg, : int(count[wg])].tolist()] == recs, f"workgroup {wg}"
        assert torch.equal(Qd.cpu(), Q) and torch.equal(Kd.cpu(), K) and torch.equal(Vd.cpu(), V)
        assert bool((ws[need:] == 0x5A).all()), "wrote past the reported size"
        # the copies are the inputs rounded to binary16 (exact from 2^-14 up)
        half = ws[:need].view(torch.float16)
        assert torch.equal(half[: half.numel() // 2].view(B, H, N, 128).cpu(), K.float().half())
        assert torch.equal(half[half.numel() // 2:].view(B, H, N, 128).cpu(), V.float().half())
        big = K.float().abs() >= 2.0 ** -14
        assert torch.equal(K.float().half().float()[big], K.float()[big])
    direct = sa.attn_fwd_variant(Qd, Kd, Vd, scale=scale, causal=causal, o_dtype=torch.float32, variant=var)
    torch.cuda.synchronize()
    assert_close(direct.double().cpu().numpy(), want, f"same request without a workspace causal={causal}")
    with pytest.raises(binding.SawattnError) as e:     # too small a workspace
        sa.attn_fwd_workspace(Qd, Kd, Vd, scale=scale, causal=causal, variant=var, workspace=ws[: need - 16])
    assert e.value.code == binding.ERR_INVALID_ARG
    with pytest.raises(binding.SawattnError) as e:     # a workspace inside an input
        sa.attn_fwd_workspace(Qd, Kd, Vd, scale=scale, causal=causal, variant=var,
                              workspace=Kd.view(torch.uint8).flatten())
    assert e.value.code == binding.ERR_INVALID_ARG


def test_workspace_path_is_the_plain_path_where_it_does_not_apply(sa):
    """Short bfloat16 sequences, binary16 inputs, d = 64: the result is attn_fwd's bit for bit and the workspace is
    left alone."""
    for (B, H, N, d, dtype, causal) in ((1, 4, 1000, 128, "bf16", True), (1, 8, 256 * 40, 128, "f16", False),
                                        (2, 2, 700, 64, "bf16", False)):
        Q, K, V = workloads.make_random(B, H, N, d, dtype, seed=77, device="cuda")
        scale = 1.0 / math.sqrt(d)
        ws = torch.full((1 << 20,), 0x33, dtype=torch.uint8, device="cuda")
        a = sa.attn_fwd(Q, K, V, scale=scale, causal=causal, scan_order="sawtooth", o_dtype=torch.float32)
        b = sa.attn_fwd_workspace(Q, K, V, scale=scale, causal=causal, scan_order="sawtooth", o_dtype=torch.float32,
                                  workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(a, b) and bool((ws == 0x33).all())


def test_workspace_path_at_full_size(sa, oracle):
    """Workload 5 (bfloat16, causal, N = 32K) through the workspace, as bench.py times it: sampled rows against
    the oracle, both scan orders, and against the plain 32-row path."""
    w = workloads.WORKLOADS[5]
    Q, K, V = workloads.make_qkv(w)
    picks = [(0, 0), (w.B - 1, w.H - 1), (1, 7)]
    rows = sample_rows(w.N, 555)
    Qd, Kd, Vd = Q.cuda(), K.cuda(), V.cuda()
    need, info = sa.attn_fwd_workspace_bytes(w.B, w.H, w.N, w.d, w.causal, None, "bf16")
    assert need == 4 * Q.numel() and info["tile_q"] == 256
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    plain = sa.attn_fwd(Qd, Kd, Vd, scale=w.scale, causal=True, scan_order="sawtooth", o_dtype=torch.float32)
    wants = {(b, h): oracle.attention(Q[b:b + 1, h:h + 1], K[b:b + 1, h:h + 1], V[b:b + 1, h:h + 1], w.scale,
                                      causal=True, rows=rows)[0, 0] for (b, h) in picks}
    for order in ORDERS:
        O = sa.attn_fwd_workspace(Qd, Kd, Vd, scale=w.scale, causal=True, scan_order=order, o_dtype=torch.float32,
                                  workspace=ws)
        torch.cuda.synchronize()
        for (b, h) in picks:
            e = assert_close(O[b, h][rows].double().cpu().numpy(), wants[(b, h)], f"workload 5 workspace {order} ({b},{h})")
            print("workspace", (b, h), order, "max-abs %.2e rel-L2 %.2e" % e, flush=True)
        assert_close(O[0, :4].double().cpu().numpy(), plain[0, :4].double().cpu().numpy(), f"workspace vs plain {order}")


# ------------------------------------------------------------------ the two halves of the K/V scan at once (small problems)
@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("B,H,N,d,kw", [
    (1, 1, 256, 64, {}), (1, 8, 2048, 64, {}), (2, 3, 384, 128, {}), (1, 5, 1280, 128, {}),
    (1, 8, 2048, 64, dict(slots_per_domain=3)),              # several rounds per head: both directions
    (1, 4, 1024, 128, dict(launch="grid")), (1, 6, 640, 64, dict(decode="linear", slots_per_domain=2)),
    (1, 16, 4096, 64, {}),                                    # not what attn_fwd would pick by itself: 512 tiles
    (1, 3, 1, 64, {}), (1, 2, 63, 128, {}), (2, 2, 65, 64, {}), (1, 4, 200, 128, dict(slots_per_domain=1)),   # ragged
    (1, 7, 1000, 64, {}), (1, 2, 1989, 128, dict(slots_per_domain=2)), (1, 3, 704, 64, dict(launch="grid")),
])
def test_halved_scan_every_element(sa, oracle, B, H, N, d, kw, order, causal):
    _halved_scan_case(sa, oracle, B, H, N, d, kw, order, causal, "f16")


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("B,H,N,d,kw", [
    (1, 8, 2048, 64, {}), (2, 3, 384, 128, {}), (1, 8, 2048, 128, dict(slots_per_domain=3)), (1, 7, 1000, 64, {}),
    (1, 2, 1989, 128, dict(slots_per_domain=2)), (1, 3, 704, 64, dict(launch="grid")), (1, 3, 1, 128, {}),
])
def test_halved_scan_every_element_bf16(sa, oracle, B, H, N, d, kw, order, causal):
    """bfloat16 inputs: V of both runs goes through registers and is converted on its way into LDS."""
    _halved_scan_case(sa, oracle, B, H, N, d, kw, order, causal, "bf16")


def _halved_scan_case(sa, oracle, B, H, N, d, kw, order, causal, dtype):
    """kv_halves = 2: 64-row tiles, wavefronts 0-1 over the first half of the keys, 2-3 over the second, merged before
    the epilogue.  Every element against the oracle, the recorded schedule against the schedule oracle, and the
    single-scan kernel on the same inputs for comparison."""
    Q, K, V = workloads.make_random(B, H, N, d, dtype, seed=77 + N)
    scale = 1.0 / math.sqrt(d)
    want = oracle.attention(Q, K, V, scale, causal=causal)
    var = sa.variant(kv_halves=2, **kw)
    info = sa.attn_fwd_variant_launch_info(B, H, N, d, causal, var, dtype)
    assert info["tile_q"] == 64
    O, trace, count = sa.attn_fwd_variant(Q.cuda(), K.cuda(), V.cuda(), scale=scale, causal=causal, scan_order=order,
                                          o_dtype=torch.float32, variant=var, trace=True)
    torch.cuda.synchronize()
    assert_close(O.double().cpu().numpy(), want, f"halved scan {B},{H},{N},{d} {dtype} causal={causal} {kw} {order}")
    from oracle import schedule_oracle as so
    sched = so.schedule(B, H, N, causal, order, **oracle_inputs(info, d, kw))
    trace, count = trace.cpu(), count.cpu()
    assert trace.shape[0] == len(sched)
    for wg in range(info["grid"]):
        assert [tuple(r) for r in trace[wg, : int(count[wg])].tolist()] == sched[wg], f"workgroup {wg}"
    one = sa.attn_fwd_variant(Q.cuda(), K.cuda(), V.cuda(), scale=scale, causal=causal, scan_order=order,
                              o_dtype=torch.float32, variant=sa.variant(kv_halves=1, **kw))
    torch.cuda.synchronize()
    assert_close(O.double().cpu().numpy(), one.double().cpu().numpy(), "halved against single scan")


@pytest.mark.parametrize("d", [64, 128])
def test_halved_scan_merges_halves_with_different_maxima(sa, oracle, d):
    """Score levels that differ by tens of binades between the two halves of the keys (either way round, and
    per head), so that the merge has to rescale one partial result by a very small factor; negative scale too."""
    H, N = 6, 1024
    g = torch.Generator("cpu").manual_seed(99 + d)
    level = 40.0 * torch.rand(H, N // 64, generator=g)
    level[:3, : N // 128] += 45.0        # heads 0-2: the first half of the keys dominates
    level[3:, N // 128:] += 45.0         # heads 3-5: the second half
    K = torch.randn(1, H, N, d, generator=g)
    K[0, :, :, 0] = level.repeat_interleave(64, dim=1)
    Q = 0.3 * torch.randn(1, H, N, d, generator=g)
    Q[0, :, :, 0] = 4.0
    V = torch.randn(1, H, N, d, generator=g)
    Q, K, V = Q.half(), K.half(), V.half()
    for scale in (1.0, -0.5):
        want = oracle.attention(Q, K, V, scale, causal=False)
        for order in ORDERS:
            O = sa.attn_fwd_variant(Q.cuda(), K.cuda(), V.cuda(), scale=scale, causal=False, scan_order=order,
                                    o_dtype=torch.float32, variant=sa.variant(kv_halves=2))
            torch.cuda.synchronize()
            assert_close(O.double().cpu().numpy(), want, f"halves with different maxima d={d} scale={scale} {order}")


def test_halved_scan_is_what_the_small_workloads_run(sa):
    for cfg in (1, 2):
        w = workloads.WORKLOADS[cfg]
        assert sa.attn_fwd_launch_info(w.B, w.H, w.N, w.d, w.causal, "sawtooth", w.dtype)["tile_q"] == 64


# ------------------------------------------------------------------ Q in and O out through LDS, non-temporal
@pytest.mark.parametrize("B,H,N,d,dtype,causal,o_dtype,kw", [
    (1, 2, 1000, 64, "f16", True, torch.float16, dict()),
    (1, 2, 1000, 64, "bf16", True, torch.float32, dict()),
    (1, 3, 777, 128, "bf16", False, torch.bfloat16, dict(kv_halves=1)),
    (1, 2, 8192 + 100, 128, "f16", False, torch.float32, dict(rows_per_wavefront=64)),
    (1, 8, 2048, 64, "f16", False, torch.float16, dict(kv_halves=2)),
    (1, 3, 500, 128, "f16", True, torch.float32, dict(kv_halves=2)),
    (1, 2, 8192 + 100, 128, "bf16", True, torch.bfloat16, dict(rows_per_wavefront=64)),
    (2, 40, 3000, 64, "f16", True, torch.float16, dict()),
    (1, 24, 1111, 128, "bf16", False, torch.float32, dict(launch="grid", tiles_per_workgroup=2)),
    (2, 2, 1, 64, "f16", False, torch.float32, dict()),                 # a single row: every row of the Q tile repeats it
    (1, 3, 37, 128, "bf16", True, torch.float32, dict()),
    (1, 2, 65, 64, "f16", True, torch.float16, dict(kv_halves=1)),      # second 64-row Q tile holds one row
    (1, 2, 300, 128, "f16", False, torch.float32, dict(rows_per_wavefront=64)),   # 256-row tile, last wavefront's rows all beyond N
])
def test_streamed_q_and_o_tiles_carry_the_same_values(sa, oracle, B, H, N, d, dtype, causal, o_dtype, kw):
    """variant.qo_streaming changes the way Q tiles come in and O tiles go out (through LDS, whole lines, non-temporal)
    and nothing of what is computed: every mode bit for bit against mode 4, where each lane loads and stores its own
    pieces, in every output type and kernel shape, with ragged last tiles and several tiles per workgroup, a negative
    scale (Q's sign is flipped on the way in), sequences shorter than a tile; and mode 3 against the oracle on sampled
    rows where O is fp32."""
    Q, K, V = workloads.make_random(B, H, N, d, dtype, seed=77)
    scale = (-1.0 if N == 777 else 1.0) / math.sqrt(d)
    Qg, Kg, Vg = Q.cuda(), K.cuda(), V.cuda()
    outs = {}
    for mode in (4, 1, 2, 3, 0):
        O = torch.full((B, H, N, d), float("nan"), device="cuda", dtype=o_dtype)
        sa.attn_fwd_variant(Qg, Kg, Vg, O, scale=scale, causal=causal, scan_order="sawtooth",
                            variant=sa.variant(qo_streaming=mode, **kw))
        torch.cuda.synchronize()
        outs[mode] = O.cpu()
    for mode in (1, 2, 3, 0):
        assert torch.equal(outs[4].view(torch.uint8), outs[mode].view(torch.uint8)), f"qo_streaming={mode}"
    if o_dtype == torch.float32:
        rows = sorted(set(list(range(0, N, 53)) + [N - 1]))
        want = oracle.attention(Q, K, V, scale, causal=causal, rows=rows)
        assert_close(outs[3].double().numpy()[:, :, rows], want, f"streamed Q and O {N},{d} {dtype}")


# ------------------------------------------------------------------ short heads, several per XCD: attn_fwd launches one workgroup per tile
@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("B,H,N,d,dtype,causal", [
    (1, 128, 512, 64, "f16", False), (2, 32, 1024, 64, "bf16", True), (1, 17, 1024, 128, "f16", False),
    (1, 40, 1000, 128, "bf16", True), (3, 8, 700, 64, "f16", True), (1, 16, 4096, 64, "f16", False),
])
def test_short_heads_run_side_by_side(sa, oracle, B, H, N, d, dtype, causal, order):
    """Where a head has fewer query tiles than an XCD holds workgroups and an XCD has several heads, attn_fwd takes
    the direct launch (Alg. 3, one tile per workgroup).  Every element (sampled rows for the largest) against the
    oracle, and the recorded schedule against the schedule oracle."""
    info = sa.attn_fwd_launch_info(B, H, N, d, causal, order, dtype)
    assert info["launch"] == sa.LAUNCH_GRID and info["tiles_per_workgroup"] == 1
    Q, K, V = workloads.make_random(B, H, N, d, dtype, seed=500 + H)
    scale = 1.0 / math.sqrt(d)
    rows = None if B * H * N <= 70000 else list(range(0, N, 37)) + [N - 1]
    want = oracle.attention(Q, K, V, scale, causal=causal, rows=rows)
    O, trace, count = sa.attn_fwd_variant(Q.cuda(), K.cuda(), V.cuda(), scale=scale, causal=causal, scan_order=order,
                                          o_dtype=torch.float32, variant=None, trace=True)
    torch.cuda.synchronize()
    got = O.double().cpu().numpy()
    assert_close(got if rows is None else got[:, :, rows], want, f"short heads {B},{H},{N},{d} {dtype} causal={causal} {order}")
    from oracle import schedule_oracle as so
    sched = so.schedule(B, H, N, causal, order, **oracle_inputs(info, d))
    trace, count = trace.cpu(), count.cpu()
    assert trace.shape[0] == len(sched)
    for wg in range(info["grid"]):
        assert [tuple(r) for r in trace[wg, : int(count[wg])].tolist()] == sched[wg], f"workgroup {wg}"
    # the plain entry point runs the same thing
    O2 = sa.attn_fwd(Q.cuda(), K.cuda(), V.cuda(), scale=scale, causal=causal, scan_order=order, o_dtype=torch.float32)
    torch.cuda.synchronize()
    assert torch.equal(O, O2)


# ------------------------------------------------------------------ whatever attn_fwd picks: random shapes
@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_shapes_through_the_plain_entry_point(sa, oracle, seed):
    """Shapes drawn at random around the points where attn_fwd changes what it runs (tile height, launch, halved scan):
    every element against the oracle, both scan orders, and the launch info must describe a launch that covers all
    query tiles."""
    rng = np.random.default_rng(seed)
    kinds = set()
    for case in range(14):
        d = int(rng.choice([64, 128]))
        dtype = str(rng.choice(["f16", "bf16"]))
        causal = bool(rng.integers(0, 2))
        heads = int(rng.choice([1, 2, 3, 6, 8, 9, 16, 24, 40, 64]))
        N = int(rng.choice([64, 128, 200, 256, 384, 500, 512, 640, 1000, 1024, 1536, 2048, 3000, 4096]))
        if heads * N > 64 * 1024:
            N = max(64, (64 * 1024 // heads) // 64 * 64)
        B = 2 if heads % 2 == 0 and rng.integers(0, 2) else 1
        H = heads // B
        info = sa.attn_fwd_launch_info(B, H, N, d, causal, "sawtooth", dtype)
        kinds.add((info["tile_q"], info["launch"]))
        assert info["grid"] == info["slots"] * 8
        assert info["grid"] * info["max_local_tiles"] >= B * H * info["q_tiles_per_head"]
        Q, K, V = workloads.make_random(B, H, N, d, dtype, seed=1000 * seed + case)
        scale = float(rng.choice([1.0, 0.5, 2.0])) / math.sqrt(d)
        want = oracle.attention(Q, K, V, scale, causal=causal)
        for order in ORDERS:
            got = run_gpu(sa, Q, K, V, scale, causal, order, o_dtype=torch.float32)
            assert_close(got, want, f"random case {seed}/{case}: {B},{H},{N},{d} {dtype} causal={causal} {order} {info}")
    assert len(kinds) >= 3, kinds      # the draw reached several kinds of launch


# ------------------------------------------------------------------ the entry point that allocates nothing, replayed from a HIP graph
@pytest.mark.parametrize("B,H,N,d,dtype,causal", [
    (1, 16, 4096, 128, "f16", True),       # persistent launch, two heads per XCD: the workgroups of an XCD wait between heads
    (1, 8, 2048, 64, "f16", False),        # 64-row tiles, the two halves of the scan at once
    (1, 8, 8192, 128, "bf16", False),      # binary16 copies of K and V in the library's fixed scratch array, wide kernel
])
def test_static_entry_point_replays_from_a_graph(sa, oracle, B, H, N, d, dtype, causal):
    """attn_fwd_static is for callers that cannot allocate, graph capture among them: captured once and replayed four
    times, with eager launches of other problems and synchronisations in between and new input values before every
    replay, every replay equals the eager call on the same values bit for bit, and the first one the oracle."""
    scale = 1.0 / math.sqrt(d)
    Q, K, V = (t.cuda() for t in workloads.make_random(B, H, N, d, dtype, seed=900 + d))
    O = torch.empty(B, H, N, d, device="cuda", dtype=torch.float32)
    other = [t.cuda() for t in workloads.make_random(2, 3, 700, d, dtype, seed=5)]
    sa.attn_fwd_static(Q, K, V, O, scale=scale, causal=causal, scan_order="sawtooth")      # set-up happens here, not under capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sa.attn_fwd_static(Q, K, V, O, scale=scale, causal=causal, scan_order="sawtooth")
    torch.cuda.synchronize()
    for rep in range(4):
        fresh = [t.cuda() for t in workloads.make_random(B, H, N, d, dtype, seed=910 + rep)]
        for dst, src in zip((Q, K, V), fresh):
            dst.copy_(src)
        O.fill_(float("nan"))
        sa.attn_fwd(*other, scale=scale, causal=not causal, scan_order="cyclic")            # the program's own eager work
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = O.clone()
        want = sa.attn_fwd_static(Q, K, V, scale=scale, causal=causal, scan_order="sawtooth", o_dtype=torch.float32)
        torch.cuda.synchronize()
        assert torch.equal(got, want), f"replay {rep}: max diff {(got - want).abs().max().item():.3e}"
        if rep == 0:
            rows = list(range(0, N, 97)) + [N - 1]
            ref = oracle.attention(fresh[0].cpu(), fresh[1].cpu(), fresh[2].cpu(), scale, causal=causal, rows=rows)
            assert_close(got.double().cpu().numpy()[:, :, rows], ref, f"graph replay {B},{H},{N},{d} {dtype}")
