"""Pins for the fp64 CPU oracle: none of these re-type the oracle's formulas.

Each test holds the oracle to something fixed outside it: published Philox
known-answer vectors, numpy's own matmul on a materialised A, closed forms
that follow from A_jk ~ N(0, 1/r) (Section 2.3, decompression paragraph:
E[A A^T] = I in this build's orientation), Theorem 2.4's envelope
(Appendix B, last display), the special cases of Algorithms 1 and 2, and
textbook properties of the Adafactor factored rule.
"""
import math
import os

import numpy as np
import pytest
from scipy import stats

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- generator
def test_philox_known_answer_vectors():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for row in rows:
        v = [int(x, 16) for x in row]
        assert oracle.philox4x32_10(v[0:4], v[4:6]) == v[6:10]


def test_counter_layout_row_quad_seed():
    # A[j, 4q..4q+3] come from counter (j_lo, q, j_hi, 0) under key (seed_lo, seed_hi):
    # a transposed (q, j) counter or a swapped key half would change the words.
    seed = 0x0123456789ABCDEF
    for j, q in [(0, 0), (5, 3), (3, 5), (2**32 + 7, 1), (123456, 63)]:
        want = oracle.philox4x32_10([j & 0xFFFFFFFF, q, j >> 32, 0],
                                    [seed & 0xFFFFFFFF, seed >> 32])
        assert oracle.raw_words(seed, j, q) == want
    assert oracle.raw_words(seed, 3, 5) != oracle.raw_words(seed, 5, 3)


def test_uniform_is_open_interval_and_fp32_exact():
    lo, hi = oracle.uniform(0), oracle.uniform(0xFFFFFFFF)
    assert lo == 2.0 ** -24 and hi == 1.0 - 2.0 ** -24
    rng = np.random.default_rng(0)
    for x in rng.integers(0, 2 ** 32, size=2000):
        u = oracle.uniform(int(x))
        assert 0.0 < u < 1.0
        assert float(np.float32(u)) == u              # exactly representable in fp32
        assert u == ((int(x) >> 9) * 2 + 1) / 2.0 ** 24
    # the low 9 bits are not used
    assert oracle.uniform(0x12345600) == oracle.uniform(0x123457FF)


def test_box_muller_pairing_and_angle():
    # z0^2 + z1^2 = -2 ln u1 and the angle of (z0, z1) is 2 pi u2: pins which word
    # feeds the radius, which the angle, and which output is cos / sin.
    seed, r = 99, 8
    for j in range(0, 50, 7):
        for q in range(2):
            x = oracle.raw_words(seed, j, q)
            z = [oracle.A_elem(seed, j, 4 * q + i, r) * math.sqrt(r) for i in range(4)]
            for (a, b, zc, zs) in [(x[0], x[1], z[0], z[1]), (x[2], x[3], z[2], z[3])]:
                u1, u2 = oracle.uniform(a), oracle.uniform(b)
                assert zc * zc + zs * zs == pytest.approx(-2.0 * math.log(u1), rel=1e-12)
                ang = (math.atan2(zs, zc) / (2 * math.pi)) % 1.0
                assert ang == pytest.approx(u2, abs=1e-12)


def test_normals_are_standard_normal():
    m, r = 4096, 64
    z = (oracle.materialise_A(2024, m, r) * math.sqrt(r)).ravel()
    N = z.size
    assert abs(z.mean()) < 4.0 / math.sqrt(N)
    assert abs(z.var() - 1.0) < 4.0 * math.sqrt(2.0 / N)
    assert abs(stats.skew(z)) < 4.0 * math.sqrt(6.0 / N)
    assert abs(stats.kurtosis(z)) < 4.0 * math.sqrt(24.0 / N)
    assert stats.kstest(z, "norm").pvalue > 1e-3
    # tails are truncated at sqrt(2*24*ln2) = 5.77 sigma by the 23-bit uniform
    assert np.abs(z).max() <= math.sqrt(2 * 24 * math.log(2)) + 1e-12


def test_entries_are_uncorrelated_within_and_across_quads():
    m, r = 8192, 16
    Z = oracle.materialise_A(7, m, r) * math.sqrt(r)
    N = m
    for (a, b) in [(0, 1), (0, 2), (1, 3), (2, 3), (3, 4), (0, 15)]:
        c = np.mean(Z[:, a] * Z[:, b])
        assert abs(c) < 4.5 / math.sqrt(N)
    c_rows = np.mean(Z[:-1, :] * Z[1:, :])
    assert abs(c_rows) < 4.5 / math.sqrt((m - 1) * r)


def test_variance_is_one_over_r_and_rank_prefix_property():
    m = 4096
    for r in (1, 3, 8, 64):
        A = oracle.materialise_A(31, m, r)
        assert A.shape == (m, r)
        assert np.mean(A * A) * r == pytest.approx(1.0, abs=5.0 * math.sqrt(2.0 / (m * r)))
    # unscaled normals do not depend on r: rank r' < r is a column prefix up to scale
    A8 = oracle.materialise_A(31, 100, 8) * math.sqrt(8)
    A3 = oracle.materialise_A(31, 100, 3) * math.sqrt(3)
    np.testing.assert_allclose(A3, A8[:, :3], rtol=1e-15)


def test_regenerated_equals_materialised_bitwise():
    seed, m, r = 555, 37, 10
    A = oracle.materialise_A(seed, m, r)
    for j in range(m):
        for k in range(r):
            assert oracle.A_elem(seed, j, k, r) == A[j, k]
    rng = np.random.default_rng(1)
    G = rng.standard_normal((6, m))
    st0 = rng.standard_normal((6, r))
    c1 = oracle.compress(G, r, seed, state=st0, a=0.7, b=0.3)
    c2 = oracle.compress(G, r, seed, state=st0, a=0.7, b=0.3, regen=True)
    assert np.array_equal(c1, c2)
    d1 = oracle.decompress(c1, m, seed, alpha=0.25)
    d2 = oracle.decompress(c1, m, seed, alpha=0.25, regen=True)
    assert np.array_equal(d1, d2)


def test_seeds_give_different_projections():
    A1 = oracle.materialise_A(1, 16, 8)
    A2 = oracle.materialise_A(2, 16, 8)
    A3 = oracle.materialise_A(1 << 32, 16, 8)       # only the high key word differs
    assert not np.allclose(A1, A2) and not np.allclose(A1, A3)
    assert np.array_equal(A1, oracle.materialise_A(1, 16, 8))


# ------------------------------------------------- brute force vs numpy matmul
SHAPES = [(4, 4, 4), (5, 7, 3), (16, 16, 8), (9, 13, 6), (1, 1, 1), (3, 16, 16), (12, 5, 20)]


@pytest.mark.parametrize("n,m,r", SHAPES)
def test_compress_decompress_transfer_brute_force(n, m, r):
    rng = np.random.default_rng(n * 1000 + m * 10 + r)
    seed, seed2 = 1234 + n, 987 + m
    A = oracle.materialise_A(seed, m, r)
    A2 = oracle.materialise_A(seed2, m, r)
    G = rng.standard_normal((n, m))
    S0 = rng.standard_normal((n, r))
    a, b, alpha = 0.9, 0.1, 1.0 / 7.0
    np.testing.assert_allclose(oracle.compress(G, r, seed, state=S0, a=a, b=b),
                               a * S0 + b * (G @ A), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(oracle.compress(G, r, seed), G @ A, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(oracle.decompress(S0, m, seed, alpha=alpha),
                               alpha * (S0 @ A.T), rtol=1e-12, atol=1e-13)
    want = (S0 @ A.T) @ A2
    lit = oracle.transfer_literal(S0, m, seed, seed2)
    re, T = oracle.transfer(S0, m, seed, seed2, return_T=True)
    np.testing.assert_allclose(lit, want, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(re, want, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(T, A.T @ A2, rtol=1e-12, atol=1e-13)
    assert np.linalg.norm(lit - re) <= 1e-12 * max(1.0, np.linalg.norm(want))
    # old and new projection are not interchangeable
    if m * r > 4:
        assert not np.allclose(oracle.transfer(S0, m, seed2, seed), want)


def test_compress_is_linear_and_additive_over_micro_steps():
    rng = np.random.default_rng(5)
    n, m, r, seed = 8, 24, 6, 42
    G1, G2 = rng.standard_normal((n, m)), rng.standard_normal((n, m))
    c = oracle.compress(2.5 * G1 - 0.5 * G2, r, seed)
    np.testing.assert_allclose(c, 2.5 * oracle.compress(G1, r, seed) - 0.5 * oracle.compress(G2, r, seed),
                               rtol=1e-12, atol=1e-13)
    acc = oracle.compress(G2, r, seed, state=oracle.compress(G1, r, seed))
    np.testing.assert_allclose(acc, oracle.compress(G1 + G2, r, seed), rtol=1e-12, atol=1e-13)


def test_state_size_closed_form():
    # state is n x r instead of n x m (Section 2.4, last paragraph); the paper's
    # GPT-3 estimate at r = 256 is 2.08 % = 256 / 12288 (Section 4).
    n, m, r = 10, 40, 4
    assert oracle.compress(np.zeros((n, m)), r, 0).shape == (n, r)
    assert round(100.0 * 256 / 12288, 2) == 2.08


# ------------------------------------- statistics over seeds (closed forms)
def _many_seeds(m, r, S, fn):
    return [fn(oracle.materialise_A(s, m, r)) for s in range(1000, 1000 + S)]


def test_unbiased_reconstruction_and_second_moments():
    # With A_jk ~ N(0,1/r):  E[x A A^T] = x;  E|xAA^T|^2 = |x|^2 (m+r+1)/r;
    # E|xAA^T - x|^2 = |x|^2 (m+1)/r  -- for r < m, r = m and r > m alike, so
    # reconstruction is NOT exact at r = m; it becomes exact only as r -> infinity.
    rng = np.random.default_rng(3)
    S = 6000
    for (m, r) in [(8, 4), (8, 8), (4, 16)]:
        x = rng.standard_normal(m)
        nx2 = float(x @ x)
        ys = np.array(_many_seeds(m, r, S, lambda A: x @ A @ A.T))
        mean = ys.mean(axis=0)
        se = ys.std(axis=0) / math.sqrt(S)
        assert np.all(np.abs(mean - x) < 5.0 * se + 1e-12)
        e2 = np.sum(ys * ys, axis=1)
        err2 = np.sum((ys - x) ** 2, axis=1)
        assert e2.mean() == pytest.approx(nx2 * (m + r + 1) / r, abs=5 * e2.std() / math.sqrt(S))
        assert err2.mean() == pytest.approx(nx2 * (m + 1) / r, abs=5 * err2.std() / math.sqrt(S))
    # r -> infinity: tiny m, huge r
    m, r = 4, 4096
    x = rng.standard_normal(m)
    rel = np.mean([np.sum((x @ A @ A.T - x) ** 2) / (x @ x)
                   for A in _many_seeds(m, r, 40, lambda A: A)])
    assert rel == pytest.approx((m + 1) / r, rel=0.5)


def test_norm_preservation_of_compression():
    # Lemma 2.3 with the 1/sqrt(r) folded into A: E|xA|^2 = |x|^2, Var = 2|x|^4/r.
    rng = np.random.default_rng(4)
    m, r, S = 12, 8, 6000
    x = rng.standard_normal(m)
    nx2 = float(x @ x)
    v = np.array(_many_seeds(m, r, S, lambda A: float(np.sum((x @ A) ** 2))))
    assert v.mean() == pytest.approx(nx2, abs=5 * v.std() / math.sqrt(S))
    assert v.var() == pytest.approx(2 * nx2 ** 2 / r, rel=0.15)


def test_transfer_second_moment():
    # E|M A_old^T A_new|_F^2 = |M|_F^2 * m / r
    rng = np.random.default_rng(6)
    n, m, r, S = 3, 10, 4, 4000
    M = rng.standard_normal((n, r))
    v = np.array([np.sum(oracle.transfer(M, m, 2 * s + 1, 2 * s + 2) ** 2) for s in range(S)])
    assert v.mean() == pytest.approx(np.sum(M * M) * m / r, abs=5 * v.std() / math.sqrt(S))


def test_theorem_2_4_envelope():
    # Appendix B, last display before the choice of r: every entry of
    # A A^T - I (paper: A^T A / r - I) is below 4 sqrt(2 log(2m/d)/r) + 8 log(2m/d)/r
    # with confidence 1 - d.
    m, r, delta = 64, 512, 0.01
    bound = 4 * math.sqrt(2 * math.log(2 * m / delta) / r) + 8 * math.log(2 * m / delta) / r
    worst = max(np.abs(A @ A.T - np.eye(m)).max() for A in _many_seeds(m, r, 20, lambda A: A))
    assert worst <= bound
    assert worst > bound / 50          # the bound is an envelope, not vacuous by orders


# ----------------------------------------------------------- Algorithm 1
def test_algorithm1_tau1_is_the_random_projection_rule():
    # tau = 1 with a fixed seed is the RP update W - eta G A A^T (Section 2.2, last display)
    rng = np.random.default_rng(8)
    n, m, r, lr, g = 6, 10, 4, 0.01, 77
    W, G = rng.standard_normal((n, m)), rng.standard_normal((n, m))
    Wn, Gt, C = oracle.algorithm1_cycle([W], [[G]], r, g, epoch=0, lr=lr)
    A = oracle.materialise_A(oracle.derive_seed(g, 0, 0), m, r)
    np.testing.assert_allclose(Wn[0], W - lr * (G @ A @ A.T), rtol=1e-12, atol=1e-13)


def test_algorithm1_scale_is_one_over_tau_and_one_seed_per_cycle():
    rng = np.random.default_rng(9)
    n, m, r, tau, g = 4, 6, 3, 5, 11
    W = rng.standard_normal((n, m))
    Gs = [rng.standard_normal((n, m)) for _ in range(tau)]
    Wn, Gt, C = oracle.algorithm1_cycle([W], [[G] for G in Gs], r, g, epoch=3, lr=0.1)
    A = oracle.materialise_A(oracle.derive_seed(g, 0, 3), m, r)
    mean_G = sum(Gs) / tau
    np.testing.assert_allclose(Gt[0], mean_G @ A @ A.T, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(C[0], sum(Gs) @ A, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(Wn[0], W - 0.1 * Gt[0], rtol=1e-12, atol=1e-13)
    # averaged over many epochs (= resampled projections) the reconstruction is the
    # arithmetic mean of the micro-step gradients: only the 1/tau scale is unbiased
    S = 3000
    acc = np.zeros((n, m))
    sq = np.zeros((n, m))
    for e in range(S):
        _, Gte, _ = oracle.algorithm1_cycle([W], [[G] for G in Gs], r, g, epoch=e, lr=0.0)
        acc += Gte[0]
        sq += Gte[0] ** 2
    mean = acc / S
    se = np.sqrt(np.maximum(sq / S - mean ** 2, 0) / S)
    assert np.all(np.abs(mean - mean_G) < 5 * se)


def test_algorithm1_new_seed_each_cycle_and_per_matrix():
    g = 5
    seeds = {oracle.derive_seed(g, l, e) for l in range(40) for e in range(40)}
    assert len(seeds) == 1600
    assert oracle.derive_seed(g, 3, 9) == oracle.derive_seed(g, 3, 9)
    x = oracle.philox4x32_10([3, 9, 0, 1], [g, 0])
    assert oracle.derive_seed(g, 3, 9) == x[0] | (x[1] << 32)
    assert oracle.derive_seed(g, 3, 9) != oracle.derive_seed(g, 9, 3)


# ----------------------------------------------------------- Algorithm 2
def test_algorithm2_without_resampling_is_plain_ema_of_projected_gradients():
    rng = np.random.default_rng(10)
    shapes, r, beta, g = [(5, 9), (3, 4)], 4, 0.9, 21
    opt = oracle.Algorithm2(shapes, r, beta, kappa=10 ** 9, global_seed=g)
    Ms = [np.zeros((n, r)) for n, _ in shapes]
    # the only resample is at t = 0 (transfer of an all-zero state): seed of epoch 1
    As = [oracle.materialise_A(oracle.derive_seed(g, l, 1), m, r) for l, (_, m) in enumerate(shapes)]
    for t in range(6):
        Gs = [rng.standard_normal(s) for s in shapes]
        ys, _ = opt.step(Gs)
        for l in range(2):
            Ms[l] = beta * Ms[l] + (1 - beta) * (Gs[l] @ As[l])
            np.testing.assert_allclose(opt.M[l], Ms[l], rtol=1e-11, atol=1e-13)
            np.testing.assert_allclose(ys[l], Ms[l] @ As[l].T, rtol=1e-11, atol=1e-13)
    assert opt.transfers == 2


def test_algorithm2_resample_schedule_and_seed_use():
    # t = 0 (mod kappa) holds at t = 0, kappa, 2 kappa, ...; the step's gradient is
    # compressed with the NEW projection and the state is carried over by the transfer.
    rng = np.random.default_rng(12)
    shapes, r, beta, kappa, g = [(4, 7)], 3, 0.5, 3, 8
    opt = oracle.Algorithm2(shapes, r, beta, kappa, g)
    M = np.zeros((4, r))
    for t in range(8):
        G = rng.standard_normal(shapes[0])
        epoch = t // kappa + 1
        A_new = oracle.materialise_A(oracle.derive_seed(g, 0, epoch), 7, r)
        if t % kappa == 0:
            A_old = oracle.materialise_A(oracle.derive_seed(g, 0, epoch - 1), 7, r)
            M = M @ A_old.T @ A_new
        M = beta * M + (1 - beta) * (G @ A_new)
        ys, _ = opt.step([G])
        np.testing.assert_allclose(opt.M[0], M, rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(ys[0], M @ A_new.T, rtol=1e-10, atol=1e-12)
        assert opt.seed_log[t][0] == oracle.derive_seed(g, 0, epoch)
    assert opt.transfers == 3                      # t = 0, 3, 6
    # config-3-like schedule: 300 steps, kappa 100 -> real transfers at t = 100, 200
    assert [t for t in range(300) if t % 100 == 0] == [0, 100, 200]


def test_algorithm2_beta_zero_is_per_step_projection():
    rng = np.random.default_rng(13)
    shapes, r, g = [(3, 8)], 4, 2
    opt = oracle.Algorithm2(shapes, r, 0.0, kappa=2, global_seed=g)
    for t in range(4):
        G = rng.standard_normal(shapes[0])
        ys, _ = opt.step([G])
        A = oracle.materialise_A(oracle.derive_seed(g, 0, t // 2 + 1), 8, r)
        np.testing.assert_allclose(ys[0], G @ A @ A.T, rtol=1e-11, atol=1e-13)


def test_algorithm2_sgd_applies_the_yield():
    rng = np.random.default_rng(14)
    shapes, r = [(3, 5)], 2
    opt = oracle.Algorithm2(shapes, r, 0.9, kappa=100, global_seed=1)
    W = rng.standard_normal(shapes[0])
    ys, Wn = opt.step([rng.standard_normal(shapes[0])], [W], lr=0.5)
    np.testing.assert_allclose(Wn[0], W - 0.5 * ys[0], rtol=1e-13, atol=1e-15)


# ------------------------------------------------- factored second moment
def test_factored_rank_one_gradient_gives_sign_update():
    # If Gt = u v^T then Gt^2 is rank one, the factored estimate is exact
    # (V = Gt^2 as eps -> 0) and U = sign(Gt): the defining property of the
    # row/column factorisation.
    rng = np.random.default_rng(15)
    n, m = 6, 9
    u, v = rng.standard_normal(n), rng.standard_normal(m)
    Gt = np.outer(u, v)
    W = rng.standard_normal((n, m))
    Wn, R, K = oracle.factored_update(W, Gt, np.zeros(n), np.zeros(m), 0.0, 1e-300, 0.0, 0.1)
    np.testing.assert_allclose(Wn, W - 0.1 * np.sign(Gt), rtol=1e-9, atol=1e-12)
    # RMS(U) = 1, so clipping at d = 1 leaves it alone and d = 0.5 halves it
    W1, _, _ = oracle.factored_update(W, Gt, np.zeros(n), np.zeros(m), 0.0, 1e-300, 1.0, 0.1)
    np.testing.assert_allclose(W1, Wn, rtol=1e-9, atol=1e-12)
    Wh, _, _ = oracle.factored_update(W, Gt, np.zeros(n), np.zeros(m), 0.0, 1e-300, 0.5, 0.1)
    np.testing.assert_allclose(Wh, W - 0.05 * np.sign(Gt), rtol=1e-9, atol=1e-12)


def test_factored_statistics_are_row_and_column_means_with_ema():
    rng = np.random.default_rng(16)
    n, m, eps1, beta2 = 5, 7, 1e-3, 0.8
    Gt = rng.standard_normal((n, m))
    R0, K0 = rng.random(n) + 0.1, rng.random(m) + 0.1
    W = np.zeros((n, m))
    Wn, R, K = oracle.factored_update(W, Gt, R0, K0, beta2, eps1, 0.0, 1.0)
    Q = Gt ** 2 + eps1
    np.testing.assert_allclose(R, beta2 * R0 + (1 - beta2) * Q.mean(axis=1), rtol=1e-13)
    np.testing.assert_allclose(K, beta2 * K0 + (1 - beta2) * Q.mean(axis=0), rtol=1e-13)
    # with beta2 = 0: sum_i R_i * m == sum_j K_j * n (both are the grand total of Q)
    _, R1, K1 = oracle.factored_update(W, Gt, R0, K0, 0.0, eps1, 0.0, 1.0)
    assert R1.sum() * m == pytest.approx(K1.sum() * n, rel=1e-13)
    # the update is -Gt / sqrt(R_i K_j / mean R)
    V = np.outer(R, K) / R.mean()
    np.testing.assert_allclose(Wn, -Gt / np.sqrt(V), rtol=1e-12)


def test_factored_constant_magnitude_gradient():
    n, m, c = 4, 6, 3.0
    rng = np.random.default_rng(17)
    Gt = c * np.sign(rng.standard_normal((n, m)))
    Wn, R, K = oracle.factored_update(np.zeros((n, m)), Gt, np.zeros(n), np.zeros(m),
                                      0.0, 0.0, 1.0, 1.0)
    np.testing.assert_allclose(R, c * c)
    np.testing.assert_allclose(K, c * c)
    np.testing.assert_allclose(Wn, -np.sign(Gt), rtol=1e-13)


# ------------------------------------------------------ the whole Adafactor step
def test_adafactor_schedules_closed_form_values():
    # rho_t = min(1e-2, 1/sqrt(t)): flat up to t = 10^4, then 1/sqrt(t);
    # beta2_t = 1 - t^-0.8: 0 at t = 1, 1 - 2^-4 at t = 32, 1 - 2^-8 at t = 1024
    assert oracle.adafactor_schedule(1) == (1e-2, 0.0)
    assert oracle.adafactor_schedule(32)[1] == pytest.approx(0.9375, rel=1e-15)
    assert oracle.adafactor_schedule(1024)[1] == pytest.approx(1 - 2.0 ** -8, rel=1e-15)
    assert oracle.adafactor_schedule(9999)[0] == 1e-2
    assert oracle.adafactor_schedule(10000)[0] == pytest.approx(1e-2, rel=1e-15)
    assert oracle.adafactor_schedule(40000)[0] == pytest.approx(5e-3, rel=1e-15)
    assert oracle.adafactor_schedule(10 ** 6)[0] == pytest.approx(1e-3, rel=1e-15)
    # beta2 increases towards 1 and never reaches it
    b = [oracle.adafactor_schedule(t)[1] for t in (1, 2, 10, 100, 10 ** 4, 10 ** 8)]
    assert all(x < y for x, y in zip(b, b[1:])) and b[-1] < 1.0


def test_rms_of_constant_and_of_unit_vectors():
    assert oracle.rms(np.full((3, 5), -4.0)) == pytest.approx(4.0, rel=1e-15)
    e = np.zeros(16)
    e[3] = 2.0
    assert oracle.rms(e) == pytest.approx(0.5, rel=1e-15)   # sqrt(4 / 16)


def test_unfactored_first_step_is_sign_descent_scaled_by_parameter_rms():
    # beta2 = 0, eps1 -> 0: V = Gt^2, U = sign(Gt), RMS(U) = 1 (no clipping at d = 1);
    # W constant = w0 has RMS |w0|, so W <- w0 - rho |w0| sign(Gt).
    rng = np.random.default_rng(21)
    n, m, w0, rho = 5, 8, -2.5, 0.01
    Gt = rng.standard_normal((n, m))
    W = np.full((n, m), w0)
    Wn, V = oracle.adafactor_step(W, Gt, V=np.zeros((n, m)), beta2=0.0, eps1=1e-300, step=rho)
    np.testing.assert_allclose(V, Gt ** 2, rtol=1e-12)
    np.testing.assert_allclose(Wn, w0 - rho * abs(w0) * np.sign(Gt), rtol=1e-12)
    # clipping threshold 0.5 halves the step, 2.0 leaves it
    Wh, _ = oracle.adafactor_step(W, Gt, V=np.zeros((n, m)), beta2=0.0, eps1=1e-300, step=rho, clip_d=0.5)
    np.testing.assert_allclose(Wh, w0 - 0.5 * rho * abs(w0) * np.sign(Gt), rtol=1e-12)
    W2, _ = oracle.adafactor_step(W, Gt, V=np.zeros((n, m)), beta2=0.0, eps1=1e-300, step=rho, clip_d=2.0)
    np.testing.assert_allclose(W2, Wn, rtol=1e-12)
    # without parameter scaling `step` is an absolute learning rate
    Wa, _ = oracle.adafactor_step(W, Gt, V=np.zeros((n, m)), beta2=0.0, eps1=1e-300, step=rho,
                                  scale_parameter=False)
    np.testing.assert_allclose(Wa, w0 - rho * np.sign(Gt), rtol=1e-12)


def test_parameter_scale_floor_eps2():
    # W = 0 has RMS 0 < eps2: the step is eps2 * rho
    rng = np.random.default_rng(22)
    Gt = rng.standard_normal((4, 6))
    Wn, _ = oracle.adafactor_step(np.zeros((4, 6)), Gt, V=np.zeros((4, 6)), beta2=0.0, eps1=1e-300,
                                  eps2=1e-3, step=0.01)
    np.testing.assert_allclose(Wn, -1e-5 * np.sign(Gt), rtol=1e-12)
    # just above the floor the RMS itself is used
    W = np.full((4, 6), 2e-3)
    Wn, _ = oracle.adafactor_step(W, Gt, V=np.zeros((4, 6)), beta2=0.0, eps1=1e-300, eps2=1e-3, step=0.01)
    np.testing.assert_allclose(Wn, 2e-3 - 2e-5 * np.sign(Gt), rtol=1e-12)


def test_unfactored_second_moment_is_elementwise_ema():
    rng = np.random.default_rng(23)
    n, m, beta2, eps1 = 3, 5, 0.7, 1e-2
    Gt = rng.standard_normal((n, m))
    V0 = rng.random((n, m)) + 0.5
    W = rng.standard_normal((n, m))
    Wn, V = oracle.adafactor_step(W, Gt, V=V0, beta2=beta2, eps1=eps1, step=0.3, clip_d=0.0,
                                  scale_parameter=False)
    for i in range(n):
        for j in range(m):
            v = 0.7 * V0[i, j] + 0.3 * (Gt[i, j] * Gt[i, j] + 1e-2)
            assert V[i, j] == pytest.approx(v, rel=1e-13)
            assert Wn[i, j] == pytest.approx(W[i, j] - 0.3 * Gt[i, j] / math.sqrt(v), rel=1e-12)


def test_factored_equals_unfactored_while_second_moment_stays_rank_one():
    # Gt_t = s_t u v^T: every Gt_t^2 lies on one rank-one ray, so the row/column factors
    # reproduce the elementwise EMA exactly (eps1 = 0) and both variants walk the same path.
    rng = np.random.default_rng(24)
    n, m = 5, 7
    u, v = rng.standard_normal(n), rng.standard_normal(m)
    Wf = Wu = rng.standard_normal((n, m))
    R, K, V = np.zeros(n), np.zeros(m), np.zeros((n, m))
    for t in range(1, 6):
        rho, beta2 = oracle.adafactor_schedule(t)
        Gt = rng.standard_normal() * np.outer(u, v)
        Wf, R, K = oracle.adafactor_step(Wf, Gt, R=R, K=K, beta2=beta2, eps1=0.0, step=rho)
        Wu, V = oracle.adafactor_step(Wu, Gt, V=V, beta2=beta2, eps1=0.0, step=rho)
        np.testing.assert_allclose(np.outer(R, K) / R.mean(), V, rtol=1e-12)
        np.testing.assert_allclose(Wf, Wu, rtol=1e-11, atol=1e-14)


def test_factored_estimate_in_row_sum_form():
    # the published form keeps row SUMS R and column SUMS C and uses R C^T / (1^T R);
    # the means kept here give the same estimate
    rng = np.random.default_rng(25)
    n, m, eps1 = 4, 9, 1e-4
    Gt = rng.standard_normal((n, m))
    W = rng.standard_normal((n, m))
    Wn, R, K = oracle.adafactor_step(W, Gt, R=np.zeros(n), K=np.zeros(m), beta2=0.0, eps1=eps1,
                                     step=0.1, clip_d=0.0, scale_parameter=False)
    Q = Gt ** 2 + eps1
    Rs, Cs = Q.sum(axis=1), Q.sum(axis=0)
    Vhat = np.outer(Rs, Cs) / Rs.sum()
    np.testing.assert_allclose(Wn, W - 0.1 * Gt / np.sqrt(Vhat), rtol=1e-12)


@pytest.mark.parametrize("factored", [True, False])
def test_relative_step_makes_the_path_scale_with_the_parameters(factored):
    # With parameter scaling and a negligible eps1 the update direction ignores the gradient's
    # scale and the step follows RMS(W): starting from c W0 with gradients g Gt_t gives c W_t.
    rng = np.random.default_rng(26)
    n, m, c, g = 6, 5, 7.0, 0.3
    W0 = rng.standard_normal((n, m))
    grads = [rng.standard_normal((n, m)) for _ in range(4)]

    def run(W, gs):
        st = dict(R=np.zeros(n), K=np.zeros(m)) if factored else dict(V=np.zeros((n, m)))
        for t, Gt in enumerate(gs, start=1):
            rho, beta2 = oracle.adafactor_schedule(t)
            out = oracle.adafactor_step(W, Gt, beta2=beta2, eps1=0.0, eps2=1e-12, step=rho, **st)
            W = out[0]
            st = dict(R=out[1], K=out[2]) if factored else dict(V=out[1])
        return W

    np.testing.assert_allclose(run(c * W0, [g * G for G in grads]), c * run(W0, grads), rtol=1e-11)


def test_adafactor_step_without_scaling_is_the_factored_rule():
    rng = np.random.default_rng(27)
    n, m = 7, 4
    W, Gt = rng.standard_normal((n, m)), rng.standard_normal((n, m))
    R0, K0 = rng.random(n) + 0.1, rng.random(m) + 0.1
    a = oracle.factored_update(W, Gt, R0, K0, 0.6, 1e-8, 1.0, 0.02)
    b = oracle.adafactor_step(W, Gt, R=R0, K=K0, beta2=0.6, eps1=1e-8, clip_d=1.0, step=0.02,
                              scale_parameter=False)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)


# ------------------------------- accumulation feeding momentum (one projection each)
def test_transfer_accumulate_is_the_matrix_product_it_names():
    rng = np.random.default_rng(31)
    n, m, r, a, b = 6, 11, 8, 0.9, 0.025
    C, M = rng.standard_normal((n, r)), rng.standard_normal((n, r))
    sc, sm = 1234, 98765
    Ac, Am = oracle.materialise_A(sc, m, r), oracle.materialise_A(sm, m, r)
    want = a * M + b * (C @ Ac.T) @ Am
    got = oracle.transfer_accumulate(M, C, m, sc, sm, a, b)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)
    # re-associated through the r x r matrix the momentum transfer uses
    np.testing.assert_allclose(got, a * M + b * oracle.transfer(C, m, sc, sm), rtol=1e-11, atol=1e-13)
    # swapping the two projections is a different result
    assert not np.allclose(got, oracle.transfer_accumulate(M, C, m, sm, sc, a, b))


def test_algorithm1_output_fed_to_algorithm2_equals_transfer_accumulate():
    # one optimizer step of "accumulate tau micro-batches (Algorithm 1), then momentum
    # (Algorithm 2)" written with the n x m intermediate, against the folded form
    rng = np.random.default_rng(32)
    n, m, r, tau, beta = 5, 9, 4, 3, 0.9
    grads = [rng.standard_normal((n, m)) for _ in range(tau)]
    sc, sm = oracle.derive_seed(5, 0, 1), oracle.derive_seed(6, 0, 1)
    C = np.zeros((n, r))
    for G in grads:
        C = oracle.compress(G, r, sc, state=C)
    Gt = oracle.decompress(C, m, sc, alpha=1.0 / tau)            # Algorithm 1's output
    M0 = rng.standard_normal((n, r))
    M_literal = oracle.compress(Gt, r, sm, state=M0, a=beta, b=1.0 - beta)   # Algorithm 2's EMA line
    M_folded = oracle.transfer_accumulate(M0, C, m, sc, sm, beta, (1.0 - beta) / tau)
    np.testing.assert_allclose(M_folded, M_literal, rtol=1e-12, atol=1e-14)


def test_accumulating_straight_into_the_momentum_is_algorithm2_on_the_mean_gradient():
    # With one projection for both, linearity lets the EMA absorb the micro-batches one by
    # one: M <- beta M + ((1-beta)/tau) G_1 A, then M <- M + ((1-beta)/tau) G_i A, which is
    # Algorithm 2's EMA line applied to the exact mean gradient.
    rng = np.random.default_rng(33)
    n, m, r, tau, beta, seed = 4, 10, 8, 4, 0.8, 77
    grads = [rng.standard_normal((n, m)) for _ in range(tau)]
    M0 = rng.standard_normal((n, r))
    M = M0
    for i, G in enumerate(grads):
        M = oracle.compress(G, r, seed, state=M, a=beta if i == 0 else 1.0, b=(1.0 - beta) / tau)
    want = oracle.compress(sum(grads) / tau, r, seed, state=M0, a=beta, b=1.0 - beta)
    np.testing.assert_allclose(M, want, rtol=1e-12, atol=1e-14)


def test_projection_entries_match_the_stored_fixture():
    # regression pin of the generator as a whole (the fixture is written by
    # tests/golden/make_golden.py from the oracle alone)
    rows = [l for l in open(os.path.join(GOLDEN, "projection_entries.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) == 5
    for line in rows:
        head, vals = line.split(":")
        seed, row, r = (int(x) for x in head.split())
        want = [float.fromhex(v) for v in vals.split()]
        got = [oracle.A_elem(seed, row, k, r) for k in range(8)]
        # (to a few ulps: the host's libm may pick another code path for log / sin / cos)
        assert got == pytest.approx(want, rel=1e-14, abs=0)
        # and the same numbers through the matrix route for rows that fit
        if row < 20000:
            A = oracle.materialise_A(seed, row + 1, r)
            assert list(A[row, :8]) == got


# ---- compressed EMA of another statistic (closing remark of Section 2.4, "Sublinear memory momentum"): the second moment

def test_mapped_compress_is_the_matrix_product_of_the_squares():
    rng = np.random.default_rng(61)
    n, m, r, seed = 9, 37, 8, 4242
    G, S0 = rng.standard_normal((n, m)), rng.standard_normal((n, r))
    A = oracle.materialise_A(seed, m, r)
    got = oracle.compress_mapped(G, r, seed, "square", state=S0, a=0.75, b=0.25)
    np.testing.assert_allclose(got, 0.75 * S0 + 0.25 * (G * G) @ A, rtol=0, atol=1e-12)
    # the sign of G cannot matter, and the identity map is plain compression
    np.testing.assert_array_equal(oracle.compress_mapped(-G, r, seed, "square", state=S0, a=0.75, b=0.25), got)
    np.testing.assert_array_equal(oracle.compress_mapped(G, r, seed, "identity"), oracle.compress(G, r, seed))
    with pytest.raises(ValueError):
        oracle.compress_mapped(G, r, seed, "cube")


def test_compressed_second_moment_ema_decompresses_to_the_ema_without_bias():
    # V_T = sum_t beta2^(T-t) (1 - beta2) G_t^2 ; its compressed form under one projection, decompressed
    # and averaged over many independent projections, must approach V_T (E[A A^T] = I), and a single
    # projection must be off by the relative error sqrt((m + 1) / r) that any n x m matrix suffers
    rng = np.random.default_rng(62)
    n, m, r, beta2, T = 6, 40, 8, 0.9, 5
    Gs = [rng.standard_normal((n, m)) for _ in range(T)]
    V = np.zeros((n, m))
    for G in Gs:
        V = beta2 * V + (1 - beta2) * G * G
    trials, acc, err2 = 3000, np.zeros((n, m)), 0.0
    for k in range(trials):
        seed = oracle.derive_seed(99, 0, k)
        S = np.zeros((n, r))
        for G in Gs:
            S = oracle.compress_mapped(G, r, seed, "square", state=S, a=beta2, b=1 - beta2)
        est = oracle.decompress(S, m, seed)
        acc += est
        err2 += np.linalg.norm(est - V) ** 2
    mean = acc / trials
    assert np.linalg.norm(mean - V) / np.linalg.norm(V) < 4 * np.sqrt((m + 1) / r / trials)
    assert err2 / trials / np.linalg.norm(V) ** 2 == pytest.approx((m + 1) / r, rel=0.1)
