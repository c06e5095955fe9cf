"""Pins for the CPU oracle: what Eq. 1 (paper Sec. 2.2) and the mathematics fix, independent of
the oracle's own code.  Every test here runs without a GPU."""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch


def rnd(shape, seed, dtype=torch.float64):
    g = torch.Generator("cpu").manual_seed(seed)
    return torch.randn(shape, generator=g, dtype=torch.float64).to(dtype)


# ---------------------------------------------------------------- storage decoders
def test_f16_decoder_all_bit_patterns(oracle):
    L = oracle.lib()
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([L.attn_oracle_decode_f16(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_bf16_decoder_all_bit_patterns(oracle):
    L = oracle.lib()
    bits = torch.arange(65536, dtype=torch.int32).to(torch.int16)
    want = bits.view(torch.bfloat16).to(torch.float64).numpy()
    got = np.array([L.attn_oracle_decode_bf16(int(b) & 0xFFFF) for b in bits.tolist()])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])


# ---------------------------------------------------------------- hand example (golden fixture)
def test_hand_example_fixture(oracle):
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "eq1_hand_example.txt")
    Q = torch.eye(2, dtype=torch.float64).reshape(1, 1, 2, 2)
    V = torch.tensor([[1.0, 2.0], [3.0, 4.0]], dtype=torch.float64).reshape(1, 1, 2, 2)
    outs = {c: oracle.attention(Q, Q.clone(), V, math.log(2.0), causal=bool(c)) for c in (0, 1)}
    n = 0
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        c, r, a, b = line.split()
        want = [float(Fraction(a)), float(Fraction(b))]
        np.testing.assert_allclose(outs[int(c)][0, 0, int(r)], want, rtol=0, atol=1e-15)
        n += 1
    assert n == 4


# ---------------------------------------------------------------- invariants of the softmax
@pytest.mark.parametrize("causal", [False, True])
def test_rows_of_P_sum_to_one_and_mask(oracle, causal):
    Q, K, V = (rnd((2, 3, 97, 16), s) for s in (1, 2, 3))
    O, P, rs = oracle.attention(Q, K, V, 0.37, causal=causal, return_P=True, return_rowsum=True)
    assert np.all(P >= 0)
    np.testing.assert_allclose(P.sum(-1), 1.0, rtol=0, atol=1e-14)
    np.testing.assert_allclose(rs, 1.0, rtol=0, atol=1e-14)
    if causal:
        iu = np.triu_indices(97, k=1)
        assert np.all(P[..., iu[0], iu[1]] == 0.0)
        assert np.all(P[..., np.arange(97), np.arange(97)] > 0)
    # O is a convex combination of V rows: it equals P @ V recomputed by a library matmul
    np.testing.assert_allclose(O, np.einsum("bhij,bhjc->bhic", P, V.numpy()), rtol=0, atol=1e-14)


def test_P_matches_definition_elementwise(oracle):
    """P[i][j] = exp(s_ij) / sum_j exp(s_ij) with s = scale * <Q_i, K_j>, evaluated with Python
    floats and math.exp, one element at a time."""
    N, d, scale = 7, 3, 0.61
    Q, K, V = (rnd((1, 1, N, d), s) for s in (4, 5, 6))
    _, P = oracle.attention(Q, K, V, scale, return_P=True)
    q, k = Q[0, 0].tolist(), K[0, 0].tolist()
    for i in range(N):
        e = [math.exp(scale * sum(q[i][c] * k[j][c] for c in range(d))) for j in range(N)]
        z = sum(e)
        for j in range(N):
            assert abs(P[0, 0, i, j] - e[j] / z) < 1e-14


# ---------------------------------------------------------------- closed forms
@pytest.mark.parametrize("causal", [False, True])
def test_identical_keys_give_mean_of_values(oracle, causal):
    N, d = 53, 8
    Q, V = rnd((1, 2, N, d), 7), rnd((1, 2, N, d), 8)
    K = rnd((1, 2, 1, d), 9).expand(1, 2, N, d).contiguous()
    O = oracle.attention(Q, K, V, 0.5, causal=causal)
    v = V.numpy()
    if causal:
        want = np.cumsum(v, axis=2) / np.arange(1, N + 1)[None, None, :, None]
    else:
        want = np.broadcast_to(v.mean(axis=2, keepdims=True), v.shape)
    np.testing.assert_allclose(O, want, rtol=0, atol=1e-13)


def test_identical_keys_and_values_return_that_row(oracle):
    N, d = 40, 8
    Q = rnd((1, 1, N, d), 10)
    K = rnd((1, 1, 1, d), 11).expand(1, 1, N, d).contiguous()
    V = rnd((1, 1, 1, d), 12).expand(1, 1, N, d).contiguous()
    O = oracle.attention(Q, K, V, 1.3)
    np.testing.assert_allclose(O, V.numpy(), rtol=0, atol=1e-14)


@pytest.mark.parametrize("beta", [1.0, 3.0, 60.0])
def test_one_hot_closed_form(oracle, beta):
    """Q_i = beta*u, K_j = t_j*u with |u| = 1 and t one-hot at j*:  every row has score
    scale*beta at j* and 0 elsewhere, so O_i = (e^{s b} V_j* + sum_{j != j*} V_j)/(e^{s b}+N-1)."""
    N, d, scale, jstar = 31, 6, 0.8, 17
    u = rnd((d,), 13)
    u = u / u.norm()
    Q = (beta * u).expand(1, 1, N, d).contiguous()
    t = torch.zeros(N, dtype=torch.float64)
    t[jstar] = 1.0
    K = (t[:, None] * u[None, :]).reshape(1, 1, N, d).contiguous()
    V = rnd((1, 1, N, d), 14)
    O = oracle.attention(Q, K, V, scale)
    w = math.exp(scale * beta)
    v = V[0, 0].numpy()
    want = (w * v[jstar] + (v.sum(0) - v[jstar])) / (w + N - 1)
    np.testing.assert_allclose(O[0, 0], np.broadcast_to(want, (N, d)), rtol=0, atol=1e-13)
    if beta == 60.0:   # e^{48} swamps the rest: the output is V_j* to rounding
        np.testing.assert_allclose(O[0, 0], np.broadcast_to(v[jstar], (N, d)), rtol=0, atol=1e-12)


def test_class_lookup_large_beta(oracle):
    """Q_i = beta*e_{c(i)}, K_j = e_{c(j)}: for large beta row i averages V over its own class."""
    N, d, C = 24, 4, 4
    cls = np.arange(N) % C
    E = torch.eye(d, dtype=torch.float64)
    Q = (200.0 * E[cls]).reshape(1, 1, N, d).contiguous()
    K = E[cls].reshape(1, 1, N, d).contiguous()
    V = rnd((1, 1, N, d), 15)
    O = oracle.attention(Q, K, V, 1.0)
    v = V[0, 0].numpy()
    for i in range(N):
        np.testing.assert_allclose(O[0, 0, i], v[cls == cls[i]].mean(0), rtol=0, atol=1e-13)


def test_large_scores_need_the_max_subtraction(oracle):
    """Scores near 2000 overflow exp() unless the row maximum is removed first."""
    N, d = 9, 2
    Q = torch.full((1, 1, N, d), 100.0, dtype=torch.float64)
    K = torch.zeros((1, 1, N, d), dtype=torch.float64)
    K[0, 0, 3] = 10.0
    V = rnd((1, 1, N, d), 16)
    O = oracle.attention(Q, K, V, 1.0)
    assert np.all(np.isfinite(O))
    np.testing.assert_allclose(O[0, 0], np.broadcast_to(V[0, 0, 3].numpy(), (N, d)), atol=1e-13)


# ---------------------------------------------------------------- special cases
def test_single_key_returns_V(oracle):
    Q, K, V = (rnd((2, 2, 1, 5), s) for s in (17, 18, 19))
    np.testing.assert_array_equal(oracle.attention(Q, K, V, 0.9), V.numpy())


def test_causal_first_row_is_V0_and_last_row_is_unmasked(oracle):
    Q, K, V = (rnd((1, 2, 33, 8), s) for s in (20, 21, 22))
    Oc = oracle.attention(Q, K, V, 0.4, causal=True)
    Of = oracle.attention(Q, K, V, 0.4, causal=False)
    np.testing.assert_array_equal(Oc[:, :, 0], V[:, :, 0].numpy())
    np.testing.assert_array_equal(Oc[:, :, -1], Of[:, :, -1])
    assert np.abs(Oc[:, :, 5] - Of[:, :, 5]).max() > 1e-3


def test_causal_row_i_equals_full_attention_over_prefix(oracle):
    Q, K, V = (rnd((1, 1, 20, 4), s) for s in (23, 24, 25))
    Oc = oracle.attention(Q, K, V, 0.7, causal=True)
    for i in (0, 1, 7, 19):
        Op = oracle.attention(Q[:, :, : i + 1], K[:, :, : i + 1], V[:, :, : i + 1], 0.7)
        np.testing.assert_allclose(Oc[0, 0, i], Op[0, 0, i], rtol=0, atol=1e-15)


def test_zero_scale_is_uniform_attention(oracle):
    Q, K, V = (rnd((1, 1, 12, 4), s) for s in (26, 27, 28))
    O = oracle.attention(Q, K, V, 0.0)
    np.testing.assert_allclose(O[0, 0], np.broadcast_to(V[0, 0].numpy().mean(0), (12, 4)),
                               rtol=0, atol=1e-15)


def test_key_shift_invariance(oracle):
    """Adding one vector c to every key adds scale*<Q_i, c> to a whole score row: softmax unchanged."""
    Q, K, V = (rnd((1, 2, 45, 8), s) for s in (29, 30, 31))
    c = rnd((1, 2, 1, 8), 32)
    np.testing.assert_allclose(oracle.attention(Q, K + c, V, 0.35), oracle.attention(Q, K, V, 0.35),
                               rtol=0, atol=1e-13)


def test_joint_permutation_of_keys_and_values(oracle):
    """Non-causal attention is a sum over keys: visiting them in another order (which is all that a
    different K/V scan direction does, paper Sec. 4) leaves O unchanged."""
    Q, K, V = (rnd((1, 1, 64, 8), s) for s in (33, 34, 35))
    perm = torch.randperm(64, generator=torch.Generator("cpu").manual_seed(36))
    a = oracle.attention(Q, K, V, 0.35)
    b = oracle.attention(Q, K[:, :, perm].contiguous(), V[:, :, perm].contiguous(), 0.35)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-14)
    rev = torch.arange(63, -1, -1)
    c = oracle.attention(Q, K[:, :, rev].contiguous(), V[:, :, rev].contiguous(), 0.35)
    np.testing.assert_allclose(a, c, rtol=0, atol=1e-14)


def test_scale_is_applied_to_scores_not_to_output(oracle):
    """softmax(2s * QK^T) V == softmax(s * (2Q) K^T) V, and O is linear in V."""
    Q, K, V = (rnd((1, 1, 30, 8), s) for s in (37, 38, 39))
    a = oracle.attention(Q, K, V, 0.5)
    np.testing.assert_allclose(a, oracle.attention(2 * Q, K, V, 0.25), rtol=0, atol=1e-13)
    np.testing.assert_allclose(3 * a, oracle.attention(Q, K, 3 * V, 0.5), rtol=0, atol=1e-13)


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("causal", [False, True])
def test_brute_force_tiny_exact_dot_products(oracle, causal):
    """N <= 8, d <= 4: dot products in exact rational arithmetic, exp via math.exp, pure Python."""
    N, d, scale = 8, 4, 0.5
    Q, K, V = (rnd((1, 1, N, d), s, torch.float16) for s in (40, 41, 42))
    O = oracle.attention(Q, K, V, scale, causal=causal)
    q, k, v = (t[0, 0].double().tolist() for t in (Q, K, V))
    for i in range(N):
        vis = [j for j in range(N) if (not causal or j <= i)]
        s = {j: float(Fraction(scale) * sum(Fraction(q[i][c]) * Fraction(k[j][c]) for c in range(d)))
             for j in vis}
        m = max(s.values())
        e = {j: math.exp(s[j] - m) for j in vis}
        z = math.fsum(e.values())
        for c in range(d):
            want = math.fsum(e[j] * v[j][c] for j in vis) / z
            assert abs(O[0, 0, i, c] - want) < 1e-14


# ---------------------------------------------------------------- independent library routine
@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16, torch.float64])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("N,d", [(200, 64), (333, 128)])
def test_against_torch_sdpa_fp64(oracle, dtype, causal, N, d):
    """torch's CPU scaled_dot_product_attention in float64 is separate code computing Eq. 1."""
    Q, K, V = (rnd((2, 2, N, d), s, dtype) for s in (43, 44, 45))
    scale = 1.0 / math.sqrt(d)
    O = oracle.attention(Q, K, V, scale, causal=causal)
    ref = torch.nn.functional.scaled_dot_product_attention(
        Q.double(), K.double(), V.double(), is_causal=causal, scale=scale).numpy()
    np.testing.assert_allclose(O, ref, rtol=0, atol=2e-14)


def test_operands_are_not_interchangeable(oracle):
    """Swapping Q and K, or K and V, must change the result (guards a transposed call)."""
    Q, K, V = (rnd((1, 1, 16, 16), s) for s in (46, 47, 48))
    a = oracle.attention(Q, K, V, 0.25)
    assert np.abs(a - oracle.attention(K, Q, V, 0.25)).max() > 1e-2
    assert np.abs(a - oracle.attention(Q, V, K, 0.25)).max() > 1e-2


# ---------------------------------------------------------------- evaluation modes agree bit for bit
def test_row_subset_and_thread_count_do_not_change_bits(oracle):
    Q, K, V = (rnd((1, 2, 150, 32), s, torch.bfloat16) for s in (49, 50, 51))
    full = oracle.attention(Q, K, V, 0.2, causal=True, n_threads=1)
    full8 = oracle.attention(Q, K, V, 0.2, causal=True, n_threads=8)
    np.testing.assert_array_equal(full, full8)
    rows = [149, 0, 77, 3]
    sub = oracle.attention(Q, K, V, 0.2, causal=True, rows=rows)
    np.testing.assert_array_equal(sub, full[:, :, rows])


def test_bad_arguments_raise(oracle):
    Q = rnd((1, 1, 4, 4), 52)
    with pytest.raises(RuntimeError):
        oracle.attention(Q, Q, Q, 1.0, rows=[4])
    with pytest.raises(ValueError):
        oracle.attention(Q, Q[:, :, :2], Q, 1.0)
