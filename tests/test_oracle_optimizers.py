"""Pins of the oracle's other optimisers (active / separable CMA-ES, plain (mu, lambda)-ES, ARS): all CPU.

Each test ties a function to something it does not compute itself: a hand-derived closed form, a property
the method's publication states, or an already pinned function in the special case where the two coincide."""
import math

import numpy as np
import pytest

import oracle as orc


def _state(n, rng, diagonal=False):
    st = orc.cma_state_init(n, 0.32, rng.standard_normal(n))
    if diagonal:
        d = rng.uniform(0.5, 2.0, n)
        st.B, st.D, st.C = np.eye(n), d, np.diag(d * d)
    else:
        Q, _ = np.linalg.qr(rng.standard_normal((n, n)))
        d = rng.uniform(0.5, 2.0, n)
        st.B, st.D, st.C = Q, d, (Q * (d * d)[None, :]) @ Q.T
    st.p_sigma = 0.1 * rng.standard_normal(n)
    st.p_c = 0.1 * rng.standard_normal(n)
    st.t = 3
    return st


# ---------------------------------------------------------------- active CMA-ES
def test_active_weights_lambda_4_by_hand():
    # w'_i = ln(2.5 / i): the two positive ones sum to ln(2.5 * 1.25) = ln 3.125, the negative ones keep the
    # ratio ln(5/6) : ln(5/8)
    c = orc.active_cma_constants(50, 4)
    assert c.mu == 2 and c.weights.shape == (4,)
    assert c.weights[0] == pytest.approx(math.log(2.5) / math.log(3.125), rel=1e-14)
    assert c.weights[1] == pytest.approx(math.log(1.25) / math.log(3.125), rel=1e-14)
    assert c.weights[2] < 0 and c.weights[3] < 0
    assert c.weights[2] / c.weights[3] == pytest.approx(math.log(5 / 6) / math.log(5 / 8), rel=1e-13)
    assert c.mu_eff == pytest.approx(1.0 / (c.weights[0] ** 2 + c.weights[1] ** 2), rel=1e-14)


@pytest.mark.parametrize("n,lam", [(40, 12), (200, 32), (1792, 96)])
def test_active_weights_make_the_decay_vanish(n, lam):
    # tutorial, below Eq. (53): with the sum of negative weights set by alpha_mu = 1 + c_1 / c_mu the factor
    # 1 - c_1 - c_mu sum(w) in front of C is exactly one; in these dimensions alpha_mu is the smallest bound
    c = orc.active_cma_constants(n, lam)
    assert c.weights[:c.mu].sum() == pytest.approx(1.0, abs=1e-14)
    assert np.all(np.diff(c.weights) <= 1e-18)
    assert 1.0 - c.c_1 - c.c_mu * c.weights.sum() == pytest.approx(1.0, abs=1e-13)


def test_active_weights_small_n_take_the_positive_definite_bound():
    # n = 2, lambda = 12: (1 - c_1 - c_mu) / (n c_mu) is the smallest of the three bounds, and with it the worst
    # case of the update (every ||C^-1/2 y||^2 rescaled to n) leaves a non-negative factor in front of C
    c = orc.active_cma_constants(2, 12)
    neg = -c.weights[c.mu:].sum()
    assert neg > 0.5
    assert neg == pytest.approx((1.0 - c.c_1 - c.c_mu) / (2 * c.c_mu), rel=1e-12)
    assert neg < 1.0 + c.c_1 / c.c_mu
    assert 1.0 - c.c_1 - c.c_mu - c.c_mu * 2 * neg >= -1e-15
    # lambda = 64 in two dimensions: c_1 + c_mu = 1 already, nothing is left for negative weights
    c = orc.active_cma_constants(2, 64)
    assert c.c_1 + c.c_mu == pytest.approx(1.0, abs=1e-15) and np.all(c.weights[c.mu:] == 0.0)


@pytest.mark.parametrize("lam", [4, 9, 32])
def test_active_update_moves_mean_paths_and_step_like_the_positive_variant(lam):
    rng = np.random.default_rng(7)
    st = _state(11, rng)
    seeds = rng.integers(0, 2 ** 32, lam, dtype=np.uint64)
    F = rng.standard_normal(lam).astype(np.float32)
    a, oa = orc.cma_update_active(st, seeds, F)
    p, op = orc.cma_update(st, seeds, F)
    assert np.array_equal(oa, op)
    for name in ("m", "p_sigma", "p_c"):
        np.testing.assert_allclose(getattr(a, name), getattr(p, name), rtol=1e-13, atol=1e-15)
    assert a.sigma == pytest.approx(p.sigma, rel=1e-14) and a.t == p.t == st.t + 1


def test_active_update_trace_identity_on_the_identity_state():
    # C = I: a positive candidate adds w ||z||^2 to the trace of the rank-mu term, a negative one exactly w n
    n, lam = 6, 10
    rng = np.random.default_rng(3)
    st = orc.cma_state_init(n, 0.5)
    seeds = rng.integers(0, 2 ** 32, lam, dtype=np.uint64)
    F = rng.standard_normal(lam).astype(np.float32)
    new, order = orc.cma_update_active(st, seeds, F)
    c = orc.active_cma_constants(n, lam)
    h = new.extra["h_sigma"]
    decay = 1.0 - c.c_1 - c.c_mu * c.weights.sum() + (1 - h) * c.c_1 * c.c_c * (2 - c.c_c)
    R = (new.C - decay * st.C - c.c_1 * np.outer(new.p_c, new.p_c)) / c.c_mu
    z2 = [float(np.sum(orc.normals_from_seed(int(seeds[k]), n).astype(np.float64) ** 2)) for k in order]
    expect = sum(c.weights[i] * z2[i] for i in range(c.mu)) + n * c.weights[c.mu:].sum()
    assert np.trace(R) == pytest.approx(expect, rel=1e-10)
    np.testing.assert_allclose(R, R.T, atol=1e-15)


def test_active_update_is_stationary_under_random_selection():
    # rewards independent of the candidates: E[C_new - c_1 p_c p_c^T] = (1 - c_1) C (the negative weights take
    # out of the expectation exactly what the decay factor leaves in); the rare stalled generation (h_sigma = 0)
    # has its extra c_1 c_c (2 - c_c) C taken off first
    n, lam, trials = 4, 10, 2500
    rng = np.random.default_rng(11)
    st = _state(n, rng)
    st.p_sigma[:] = 0.0
    st.t = 1000
    c = orc.active_cma_constants(n, lam)
    acc = np.zeros((trials, n, n))
    for i in range(trials):
        seeds = rng.integers(0, 2 ** 32, lam, dtype=np.uint64)
        new, _ = orc.cma_update_active(st, seeds, rng.standard_normal(lam).astype(np.float32))
        acc[i] = new.C - c.c_1 * np.outer(new.p_c, new.p_c) - (1.0 - new.extra["h_sigma"]) * c.c_1 * c.c_c * (2.0 - c.c_c) * st.C
    mean, err = acc.mean(axis=0), acc.std(axis=0) / math.sqrt(trials)
    assert np.all(np.abs(mean - (1.0 - c.c_1) * st.C) < 4.5 * err + 1e-12)
    # and the test has teeth: without the negative weights the same average sits well above
    assert c.c_mu * abs(c.weights[c.mu:].sum()) * np.abs(st.C).max() > 10 * err.max()


def test_active_update_keeps_the_covariance_positive_definite():
    n, lam = 2, 12
    rng = np.random.default_rng(5)
    st = _state(n, rng)
    for g in range(200):
        seeds = rng.integers(0, 2 ** 32, lam, dtype=np.uint64)
        st, _ = orc.cma_update_active(st, seeds, rng.standard_normal(lam).astype(np.float32))
        assert np.linalg.eigvalsh((st.C + st.C.T) / 2).min() > 0
        lamb, B = np.linalg.eigh((st.C + st.C.T) / 2)
        st.B, st.D = B, np.sqrt(lamb)


# ---------------------------------------------------------------- separable CMA-ES
def test_sep_cma_is_the_full_update_when_n_is_one():
    # (n + 2) / 3 = 1: nothing distinguishes the two
    rng = np.random.default_rng(2)
    full = orc.cma_state_init(1, 0.32, [0.3])
    sep = orc.sep_cma_init(1, 0.32, [0.3])
    for g in range(5):
        seeds = rng.integers(0, 2 ** 32, 6, dtype=np.uint64)
        F = rng.standard_normal(6).astype(np.float32)
        th_f, _ = orc.sample_candidates(full.m, full.sigma, full.B, full.D, seeds)
        th_s, _ = orc.sep_cma_sample(sep, seeds)
        np.testing.assert_allclose(th_s, th_f, rtol=1e-14)
        full, _ = orc.cma_update(full, seeds, F)
        full.B, full.D = np.eye(1), np.sqrt(np.diag(full.C))
        sep, _ = orc.sep_cma_update(sep, seeds, F)
        assert sep.c_diag[0] == pytest.approx(full.C[0, 0], rel=1e-13)
        assert sep.sigma == pytest.approx(full.sigma, rel=1e-14) and sep.m[0] == pytest.approx(full.m[0], rel=1e-13)


def test_sep_cma_learning_rates():
    n, lam = 100, 16
    c, c_1, c_mu = orc.sep_cma_constants(n, lam)
    assert c_1 == pytest.approx(34.0 * c.c_1, rel=1e-15) and c_mu == pytest.approx(34.0 * c.c_mu, rel=1e-15)
    c, c_1, c_mu = orc.sep_cma_constants(2, 400)       # many candidates in two dimensions: the caps bind
    assert 0 < c_1 <= 1 and c_1 + c_mu <= 1 + 1e-15


def test_sep_cma_matches_the_diagonal_of_the_full_update_term_by_term():
    # on a diagonal state the full update's vectors are the separable ones, and its matrix terms, read on the
    # diagonal and re-weighted with the separable learning rates, give the separable covariance
    n, lam = 9, 12
    rng = np.random.default_rng(4)
    full = _state(n, rng, diagonal=True)
    sep = orc.SepState(n=n, t=full.t, sigma=full.sigma, m=full.m.copy(), p_sigma=full.p_sigma.copy(), p_c=full.p_c.copy(),
                       c_diag=np.diag(full.C).copy())
    seeds = rng.integers(0, 2 ** 32, lam, dtype=np.uint64)
    F = rng.standard_normal(lam).astype(np.float32)
    f, of = orc.cma_update(full, seeds, F)
    s, os_ = orc.sep_cma_update(sep, seeds, F)
    assert np.array_equal(of, os_)
    for name in ("m", "p_sigma", "p_c"):
        np.testing.assert_allclose(getattr(s, name), getattr(f, name), rtol=1e-13, atol=1e-15)
    assert s.sigma == pytest.approx(f.sigma, rel=1e-14)
    c, c_1, c_mu = orc.sep_cma_constants(n, lam)
    h = f.extra["h_sigma"]
    corr = (1 - h) * c.c_c * (2 - c.c_c)
    rank_mu_diag = (np.diag(f.C) - (1 - c.c_1 - c.c_mu + c.c_1 * corr) * np.diag(full.C) - c.c_1 * f.p_c ** 2) / c.c_mu
    expect = (1 - c_1 - c_mu + c_1 * corr) * np.diag(full.C) + c_1 * f.p_c ** 2 + c_mu * rank_mu_diag
    np.testing.assert_allclose(s.c_diag, expect, rtol=1e-11)


def test_sep_cma_converges_on_an_axis_parallel_ellipsoid():
    n, lam = 20, 12
    rng = np.random.default_rng(9)
    scale = 10.0 ** np.linspace(0, 2, n)
    st = orc.sep_cma_init(n, 0.5, np.ones(n))
    f0 = float(np.sum((scale * st.m) ** 2))
    for g in range(300):
        seeds = rng.integers(0, 2 ** 32, lam, dtype=np.uint64)
        theta, _ = orc.sep_cma_sample(st, seeds)
        st, _ = orc.sep_cma_update(st, seeds, (-np.sum((scale[None, :] * theta) ** 2, axis=1)).astype(np.float32))
    assert float(np.sum((scale * st.m) ** 2)) < 1e-6 * f0
    # the learnt axis lengths follow the inverse scales
    ratio = np.sqrt(st.c_diag) * scale
    assert ratio.max() / ratio.min() < 30.0


# ---------------------------------------------------------------- plain (mu, lambda)-ES
@pytest.mark.parametrize("lam", [2, 3])
def test_es_update_is_the_cma_mean_step_when_mu_is_one(lam):
    rng = np.random.default_rng(1)
    n = 7
    st = orc.cma_state_init(n, 0.4, rng.standard_normal(n))
    seeds = rng.integers(0, 2 ** 32, lam, dtype=np.uint64)
    F = rng.standard_normal(lam).astype(np.float32)
    full, order = orc.cma_update(st, seeds, F)
    m_new, order_es = orc.es_update(st.m, st.sigma, seeds, F)
    assert np.array_equal(order, order_es)
    np.testing.assert_allclose(m_new, full.m, rtol=1e-14)


def test_es_update_brute_force():
    n, lam = 5, 6
    m = np.arange(n, dtype=np.float64)
    seeds = [10, 11, 12, 13, 14, 15]
    F = np.array([0.1, 0.9, 0.5, 0.9, -1.0, 0.7], np.float32)      # best three: 1, 3 (tie, lower index first), 5
    theta, Z = orc.es_sample(m, 0.25, seeds)
    for k in range(lam):
        np.testing.assert_array_equal(theta[k], m + 0.25 * orc.normals_from_seed(seeds[k], n).astype(np.float64))
    m_new, order = orc.es_update(m, 0.25, seeds, F)
    assert list(order[:3]) == [1, 3, 5]
    np.testing.assert_allclose(m_new, (theta[1] + theta[3] + theta[5]) / 3.0, rtol=1e-15)


# ---------------------------------------------------------------- ARS
def test_ars_single_pair_closed_form():
    # N = b = 1: the standard deviation of {r+, r-} is |r+ - r-| / 2, so the step is 2 alpha sign(r+ - r-) z
    n = 6
    m = np.linspace(-1, 1, n)
    z = orc.normals_from_seed(77, n).astype(np.float64)
    theta, Z = orc.ars_sample(m, 0.05, [77])
    np.testing.assert_array_equal(theta[0], m + 0.05 * z)
    np.testing.assert_array_equal(theta[1], m - 0.05 * z)
    up, _ = orc.ars_update(m, [77], np.array([3.0, 1.0], np.float32), alpha=0.02, b=1)
    np.testing.assert_allclose(up, m + 0.04 * z, rtol=1e-14)
    down, _ = orc.ars_update(m, [77], np.array([1.0, 3.0], np.float32), alpha=0.02, b=1)
    np.testing.assert_allclose(down, m - 0.04 * z, rtol=1e-14)
    same, _ = orc.ars_update(m, [77], np.array([2.0, 2.0], np.float32), alpha=0.02, b=1)
    np.testing.assert_array_equal(same, m)


def test_ars_invariances():
    n, N, b = 8, 6, 4
    rng = np.random.default_rng(6)
    m = rng.standard_normal(n)
    seeds = rng.integers(0, 2 ** 32, N, dtype=np.uint64)
    r = rng.integers(-8, 9, 2 * N).astype(np.float32)
    base, order = orc.ars_update(m, seeds, r, 0.1, b)
    shifted, _ = orc.ars_update(m, seeds, r + 16.0, 0.1, b)          # exact in fp32 for these integers
    scaled, _ = orc.ars_update(m, seeds, 4.0 * r, 0.1, b)
    np.testing.assert_allclose(shifted, base, rtol=1e-13)
    np.testing.assert_allclose(scaled, base, rtol=1e-13)
    swapped = r.reshape(N, 2)[:, ::-1].reshape(-1).copy()
    mirrored, order_sw = orc.ars_update(m, seeds, swapped, 0.1, b)
    assert np.array_equal(order, order_sw)
    np.testing.assert_allclose(mirrored - m, -(base - m), rtol=1e-13)
    # only the b best directions count: a discarded pair may change freely
    worst = order[-1]
    r2 = r.copy()
    r2[2 * worst], r2[2 * worst + 1] = r.min() - 1.0, r.min() - 5.0
    np.testing.assert_array_equal(orc.ars_update(m, seeds, r2, 0.1, b)[0], base)


def test_ars_follows_the_gradient_of_a_linear_reward():
    # r(theta) = g . theta: the step is (2 alpha nu / s_R) (1/N) sum (g . z_j) z_j, which tends to a positive multiple of g
    n, N = 4, 400
    rng = np.random.default_rng(8)
    g = np.array([1.0, -2.0, 0.5, 3.0])
    m = np.zeros(n)
    seeds = rng.integers(0, 2 ** 32, N, dtype=np.uint64)
    theta, _ = orc.ars_sample(m, 0.1, seeds)
    new, _ = orc.ars_update(m, seeds, (theta @ g).astype(np.float32), alpha=0.05, b=N)
    step = new - m
    assert step @ g / (np.linalg.norm(step) * np.linalg.norm(g)) > 0.97


# ---------------------------------------------------------------- stalled step (h_sigma = 0) of the two other CMA kinds
def test_active_update_stalled_branch_keeps_the_rank_one_mass():
    # as for the positive-weight update: with C = p_c p_c^T and h_sigma = 0 the c_1 terms cancel,
    # C' = (1 - c_mu sum w) C + c_mu sum_i w~_i y_i y_i^T, negative weights rescaled by n / |z_i|^2
    n, lam = 3, 8
    rng = np.random.default_rng(31)
    st = orc.cma_state_init(n, 0.32, rng.standard_normal(n))
    st.p_c = rng.standard_normal(n)
    st.C = np.outer(st.p_c, st.p_c)
    st.p_sigma = np.array([90.0, 0.0, 0.0])
    st.t = 4
    seeds = list(range(60, 60 + lam))
    F = rng.standard_normal(lam)
    new, order = orc.cma_update_active(st, seeds, F)
    c = orc.active_cma_constants(n, lam)
    assert new.extra["h_sigma"] == 0.0
    np.testing.assert_allclose(new.p_c, (1.0 - c.c_c) * st.p_c, rtol=1e-15)
    Z = np.stack([orc.normals_from_seed(s, n) for s in seeds]).astype(np.float64)
    ranked = sorted(range(lam), key=lambda i: -F[i])
    expect = (1.0 - c.c_mu * c.weights.sum()) * st.C
    for i, k in enumerate(ranked):
        w = c.weights[i] if i < c.mu else c.weights[i] * n / float(Z[k] @ Z[k])
        expect += c.c_mu * w * np.outer(Z[k], Z[k])
    np.testing.assert_allclose(new.C, expect, rtol=1e-12, atol=1e-15)


def test_sep_update_stalled_branch_keeps_the_rank_one_mass():
    n, lam = 5, 6
    rng = np.random.default_rng(32)
    st = orc.sep_cma_init(n, 0.32, rng.standard_normal(n))
    st.p_c = rng.standard_normal(n)
    st.c_diag = st.p_c ** 2
    st.p_sigma = np.zeros(n)
    st.p_sigma[1] = 200.0
    st.t = 7
    seeds = list(range(70, 70 + lam))
    F = rng.standard_normal(lam)
    new, order = orc.sep_cma_update(st, seeds, F)
    c, c_1, c_mu = orc.sep_cma_constants(n, lam)
    assert new.extra["h_sigma"] == 0.0
    np.testing.assert_allclose(new.p_c, (1.0 - c.c_c) * st.p_c, rtol=1e-15)
    Z = np.stack([orc.normals_from_seed(s, n) for s in seeds]).astype(np.float64)
    ranked = sorted(range(lam), key=lambda i: -F[i])
    expect = (1.0 - c_mu) * st.c_diag
    for i in range(c.mu):
        expect += c_mu * c.weights[i] * st.c_diag * Z[ranked[i]] ** 2          # y = sqrt(c_diag) z
    np.testing.assert_allclose(new.c_diag, expect, rtol=1e-12)
