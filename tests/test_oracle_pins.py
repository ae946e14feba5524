"""Pins of the CPU oracle against facts that do not come from the oracle itself (all CPU)."""
import math
import os

import numpy as np
import pytest

import essa_workloads as wl
import oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- Philox / normals
def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for row in rows:
        v = [int(x, 16) for x in row]
        out = orc.philox4x32_10(v[0:4], v[4:6])
        assert [int(x) for x in out] == v[6:10]


def test_philox_is_a_bijection_per_key_on_a_small_counter_set():
    ctr = np.zeros((4096, 4), np.uint32)
    ctr[:, 0] = np.arange(4096)
    out = orc.philox4x32_10(ctr, np.tile(np.array([[5, 0]], np.uint32), (4096, 1)))
    assert len({tuple(r) for r in out.tolist()}) == 4096


def test_seed_stream_layout():
    # block c of candidate `seed` is Philox(counter=(c,0,0,0), key=(seed,0))
    w = orc.philox_words_for_seed(123, 5)
    assert [int(x) for x in w[3]] == [int(x) for x in orc.philox4x32_10([3, 0, 0, 0], [123, 0])]


def test_normals_range_and_moments():
    z = orc.normals_from_seed(2025, 1_000_000).astype(np.float64)
    assert np.abs(z).max() <= math.sqrt(-2.0 * math.log(2.0 ** -25)) + 1e-6   # 24-bit uniforms bound |z|
    assert abs(z.mean()) < 4e-3
    assert abs(z.var() - 1.0) < 6e-3
    assert abs((z ** 4).mean() - 3.0) < 5e-2
    assert abs((z ** 3).mean()) < 2e-2
    # the two members of a Box-Muller pair are uncorrelated, and so are neighbours across pairs
    assert abs(np.mean(z[0::2] * z[1::2])) < 4e-3
    assert abs(np.mean(z[1:-1:2] * z[2::2])) < 4e-3


def test_box_muller_pair_geometry():
    # (z0,z1) = rho (cos, sin): radius from word 0, angle from word 1 -- catches swapped words / sin-cos
    w = orc.philox_words_for_seed(9, 64)
    z = orc.normals_from_seed(9, 256).astype(np.float64).reshape(64, 4)
    u = orc.uniform24(w)
    for a, b in ((0, 1), (2, 3)):
        rho2 = z[:, a] ** 2 + z[:, b] ** 2
        np.testing.assert_allclose(rho2, -2.0 * np.log(u[:, a]), rtol=1e-5)
        ang = np.mod(np.arctan2(z[:, b], z[:, a]), 2 * np.pi)
        np.testing.assert_allclose(ang, 2 * np.pi * u[:, b], atol=2e-5)


def test_same_seed_same_candidate_and_prefix_property():
    a = orc.normals_from_seed(77, 1000)
    b = orc.normals_from_seed(77, 1000)
    assert np.array_equal(a, b)
    assert np.array_equal(orc.normals_from_seed(77, 10), a[:10])       # surplus discarded, not reshuffled
    assert not np.array_equal(orc.normals_from_seed(78, 1000), a)


# ---------------------------------------------------------------- sampler transform
def test_sampler_identity_and_diagonal():
    n, seeds = 50, [1, 2, 3]
    m = np.linspace(-1, 1, n)
    th, Z = orc.sample_candidates(m, 0.32, np.eye(n), np.ones(n), seeds)
    np.testing.assert_allclose(th, m[None] + 0.32 * Z.astype(np.float64), rtol=0, atol=1e-15)
    d = np.linspace(0.5, 2.0, n)
    th, Z = orc.sample_candidates(m, 0.1, np.eye(n), d, seeds)
    np.testing.assert_allclose(th, m[None] + 0.1 * d[None] * Z, atol=1e-15)


def test_sampler_rotation_norm_and_covariance():
    n = 6
    Q, d = wl.random_covariance_basis(n, 1)
    Q, d = Q.astype(np.float64), d.astype(np.float64)
    m = np.arange(n, dtype=np.float64)
    seeds = list(range(1, 20001))
    th, Z = orc.sample_candidates(m, 0.5, Q, d, seeds)
    np.testing.assert_allclose(np.linalg.norm(th - m, axis=1), 0.5 * np.linalg.norm(d[None] * Z, axis=1), rtol=1e-6)
    C = Q @ np.diag(d ** 2) @ Q.T
    emp = np.cov((th - m).T, bias=True)
    assert np.max(np.abs(emp - 0.25 * C)) < 0.06 * np.max(np.abs(0.25 * C))
    # not the transposed basis: column j of B is the axis scaled by d_j
    th1, Z1 = orc.sample_candidates(np.zeros(n), 1.0, Q, d, [5])
    np.testing.assert_allclose(th1[0], sum(Q[:, j] * d[j] * Z1[0, j] for j in range(n)), atol=1e-12)


# ---------------------------------------------------------------- theta -> sigma
def test_search_dimension_closed_form():
    assert orc.sigma_map_dim(28 * 4, 8, 1.0) == 1792        # "d ~ 1.8K" for the 7B model at r = 8
    assert orc.sigma_map_dim(28 * 4, 16, 1.0) == 3584
    assert orc.sigma_map_dim(4, 8, 0.1) == 0                 # rounding down leaves nothing trainable
    assert orc.sigma_map_dim(4, 16, 0.5) == 4 * 2 * 8


def test_theta_to_sigma_layout_and_top_alpha():
    P, r, K = 3, 4, 2
    sA0 = np.arange(P * r, dtype=np.float64).reshape(P, r) + 100
    sB0 = np.arange(P * r, dtype=np.float64).reshape(P, r) + 200
    th = np.arange(K * P * 2 * r, dtype=np.float64).reshape(K, -1) / 1000
    sA, sB = orc.theta_to_sigma(th, sA0, sB0, 1.0)
    assert sA[1, 2, 3] == sA0[2, 3] + th[1, 2 * 8 + 3]
    assert sB[1, 2, 3] == sB0[2, 3] + th[1, 2 * 8 + 4 + 3]
    # zero offset gives the fine-tuned model back
    sA, sB = orc.theta_to_sigma(np.zeros((K, P * 2 * r)), sA0, sB0, 1.0)
    assert np.array_equal(sA[0], sA0) and np.array_equal(sB[1], sB0)
    # alpha = 0.5: only the first two of each factor move
    th = np.ones((K, P * 2 * 2))
    sA, sB = orc.theta_to_sigma(th, sA0, sB0, 0.5)
    assert np.array_equal(sA[0, :, :2], sA0[:, :2] + 1) and np.array_equal(sA[0, :, 2:], sA0[:, 2:])
    with pytest.raises(ValueError):
        orc.theta_to_sigma(np.zeros((K, 0)), sA0, sB0, 0.1)


# ---------------------------------------------------------------- quantised formats
def test_int4_pack_roundtrip_and_dequant():
    g = np.random.default_rng(0)
    q = g.integers(0, 16, size=(5, 256), dtype=np.uint8)
    assert np.array_equal(orc.unpack_int4(orc.pack_int4(q)), q)
    p = orc.pack_int4(q)
    assert p[0, 0] == q[0, 0] | (q[0, 1] << 4)
    s = g.uniform(0.001, 0.01, (5, 2)).astype(np.float16)
    z = g.uniform(6, 9, (5, 2)).astype(np.float16)
    W = orc.dequant_int4(p, s, z)
    assert W[3, 130] == float(s[3, 1]) * (float(q[3, 130]) - float(z[3, 1]))
    assert W[0, 127] == float(s[0, 0]) * (float(q[0, 127]) - float(z[0, 0]))


def test_int8_dequant():
    q = np.array([[1, -2], [3, 127]], np.int8)
    s = np.array([0.5, 0.25], np.float32)
    assert np.array_equal(orc.dequant_int8(q, s), np.array([[0.5, -1.0], [0.75, 31.75]]))


# ---------------------------------------------------------------- forward
def _tiny(seed=0, d_in=24, d_out=20, r=4, K=3, rows=5):
    g = np.random.default_rng(seed)
    W = g.standard_normal((d_out, d_in))
    A = g.standard_normal((r, d_in)) / math.sqrt(d_in)
    B = g.standard_normal((d_out, r)) * 0.1
    X = g.standard_normal((K * rows, d_in))
    r2c = wl.row2cand_contiguous(K, rows)
    return W, A, B, X, r2c, g


def test_forward_own_singular_values_give_W_plus_BA():
    W, A, B, X, r2c, _ = _tiny()
    f = orc.thin_svd_factors(A, B)
    K = 3
    Y = orc.svdlora_forward(W, f, X, r2c, np.tile(f["S_A"], (K, 1)), np.tile(f["S_B"], (K, 1)))
    np.testing.assert_allclose(Y, X @ W.T + (X @ A.T) @ B.T, rtol=1e-12, atol=1e-12)   # unfactored A, B


def test_forward_zero_sigma_gives_base_layer():
    W, A, B, X, r2c, _ = _tiny(1)
    f = orc.thin_svd_factors(A, B)
    z = np.zeros((3, 4))
    s = np.tile(f["S_A"], (3, 1))
    np.testing.assert_allclose(orc.svdlora_forward(W, f, X, r2c, z, np.tile(f["S_B"], (3, 1))), X @ W.T, atol=1e-13)
    np.testing.assert_allclose(orc.svdlora_forward(W, f, X, r2c, s, z), X @ W.T, atol=1e-13)


def test_forward_brute_force_loops():
    W, A, B, X, r2c, g = _tiny(2, d_in=7, d_out=6, r=2, K=2, rows=2)
    f = orc.thin_svd_factors(A, B)
    sA, sB = g.standard_normal((2, 2)), g.standard_normal((2, 2))
    Y = orc.svdlora_forward(W, f, X, r2c, sA, sB)
    UA, VA, UB, VB = f["U_A"], f["V_A"], f["U_B"], f["V_B"]
    for i in range(X.shape[0]):
        k = r2c[i]
        for o in range(W.shape[0]):
            acc = 0.0
            for j in range(W.shape[1]):
                w = W[o, j]
                for a in range(2):          # (B_k A_k)[o,j] = sum_ab UB[o,b] sB[b] (VB^T UA)[b,a] sA[a] VA[j,a]
                    for b in range(2):
                        core = sum(VB[t, b] * UA[t, a] for t in range(2))
                        w += UB[o, b] * sB[k, b] * core * sA[k, a] * VA[j, a]
                acc += w * X[i, j]
            assert abs(acc - Y[i, o]) < 1e-12


def test_forward_linearity_permutation_and_candidate_order():
    W, A, B, X, r2c, g = _tiny(3)
    f = orc.thin_svd_factors(A, B)
    sA1, sA2, sB = g.standard_normal((3, 4)), g.standard_normal((3, 4)), g.standard_normal((3, 4))
    base = X @ W.T
    l1 = orc.svdlora_forward(W, f, X, r2c, sA1, sB) - base
    l2 = orc.svdlora_forward(W, f, X, r2c, sA2, sB) - base
    l12 = orc.svdlora_forward(W, f, X, r2c, sA1 + 2 * sA2, sB) - base
    np.testing.assert_allclose(l12, l1 + 2 * l2, atol=1e-12)
    np.testing.assert_allclose(orc.svdlora_forward(W, f, X, r2c, sA1, sB, lora_only=True), l1, atol=1e-12)
    perm = g.permutation(X.shape[0])
    Yp = orc.svdlora_forward(W, f, X[perm], r2c[perm], sA1, sB)
    np.testing.assert_allclose(Yp, orc.svdlora_forward(W, f, X, r2c, sA1, sB)[perm], atol=1e-13)
    # renaming candidates (with their sigma rows) does not change any row's output
    ren = np.array([2, 0, 1])
    inv = np.argsort(ren)
    Yr = orc.svdlora_forward(W, f, X, ren[r2c], sA1[inv], sB[inv])
    np.testing.assert_allclose(Yr, orc.svdlora_forward(W, f, X, r2c, sA1, sB), atol=1e-13)
    # the sampled-rows evaluation is the same function
    rows = np.array([0, 7, 14])
    np.testing.assert_allclose(orc.svdlora_forward_rows(W, f, X, r2c, sA1, sB, rows),
                               orc.svdlora_forward(W, f, X, r2c, sA1, sB)[rows], atol=1e-13)


def test_forward_c1_against_dense_formula_with_quantised_base():
    p = wl.make_projection("q", 512, 512, 8, "int8")
    f = orc.thin_svd_factors(p.A, p.B)
    X = wl.make_x_f32(64, 512)
    r2c = wl.row2cand_contiguous(4, 16)
    Wd = orc.dequant_int8(p.Wq, p.scales)
    K = 4
    Y = orc.svdlora_forward(Wd, f, X, r2c, np.tile(f["S_A"], (K, 1)), np.tile(f["S_B"], (K, 1)))
    ref = X.astype(np.float64) @ (p.Wq.astype(np.float64) * p.scales.astype(np.float64)[:, None]).T \
        + (X.astype(np.float64) @ p.A.astype(np.float64).T) @ p.B.astype(np.float64).T
    np.testing.assert_allclose(Y, ref, rtol=1e-11, atol=1e-11)


def test_w8a8_quantiser_and_accumulators():
    g = np.random.default_rng(4)
    X = g.standard_normal((6, 40)).astype(np.float32)
    X[2] = 0
    q, s = orc.quantize_rows_int8(X)
    assert q.dtype == np.int8 and np.all(np.abs(q) <= 127)
    assert np.all(q[2] == 0) and s[2] == 0
    assert np.all(np.max(np.abs(q[[0, 1, 3, 4, 5]]), axis=1) == 127)           # the largest entry maps to +-127
    assert np.max(np.abs(q * s[:, None] - X)) <= 0.5 * s.max() * 1.0001
    Wq = g.integers(-127, 128, size=(9, 40), dtype=np.int8)
    acc = orc.int8_accumulators(q, Wq)
    assert acc[1, 3] == sum(int(q[1, j]) * int(Wq[3, j]) for j in range(40))
    # worst case stays inside int32: 127*127*8192 < 2^31
    assert 127 * 127 * 8192 < 2 ** 31


def test_round_to_bf16():
    x = np.array([1.0, 1.00390625, 1.01171875, -3.1415926, 0.0, 1e-3, 65280.0, 255.5])
    got = orc.round_to_bf16(x)
    assert np.array_equal(got, wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(x.astype(np.float32))).astype(np.float64))
    assert got[1] == 1.0 and got[2] == 1.015625 and got[7] == 256.0


def test_reward_definition():
    Y = np.array([[1.0, 2.0], [3.0, 4.0], [5.0, 6.0]])
    v = np.array([1.0, -1.0])
    F = orc.reward_accumulate(np.zeros(3), Y, v, np.array([0, 0, 1]), 3)
    assert F[0] == -1.0 and F[1] == -1.0 and math.isnan(F[2])
    F2 = orc.reward_accumulate(F, Y, v, np.array([0, 0, 1]), 3)
    assert F2[0] == -2.0


# ---------------------------------------------------------------- ranking and CMA-ES
def test_rank_rules():
    assert list(orc.rank_desc_stable([1.0, 3.0, 2.0])) == [1, 2, 0]
    assert list(orc.rank_desc_stable([5.0] * 4)) == [0, 1, 2, 3]
    assert list(orc.rank_desc_stable([1.0, float("nan"), 2.0, float("-inf")])) == [2, 0, 1, 3]
    assert list(orc.rank_desc_stable([float("inf"), 1.0, float("inf")])) == [0, 2, 1]
    g = np.random.default_rng(5)
    F = g.integers(0, 5, 40).astype(np.float32)
    o = orc.rank_desc_stable(F)
    assert sorted(o) == list(range(40))
    assert list(o) == sorted(range(40), key=lambda i: (-F[i], i))


def test_cma_constants_closed_form():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "cma_constants.txt")) if l.strip() and not l.startswith("#")]
    for row in rows:
        n, lam, mu = int(row[0]), int(row[1]), int(row[2])
        c = orc.cma_constants(n, lam)
        assert c.mu == mu
        got = [c.weights[0], c.weights[-1], c.mu_eff, c.c_sigma, c.d_sigma, c.c_c, c.c_1, c.c_mu, c.chi_n]
        for g_, want in zip(got, row[3:]):
            if want == "nan":
                continue
            digits = len(want.split("e")[0].replace(".", "").lstrip("0"))
            tol = max(2e-6, 0.6 * 10.0 ** (1 - digits))
            assert abs(g_ - float(want)) <= tol * abs(float(want)), (g_, want)
        assert abs(c.weights.sum() - 1.0) < 1e-14
        assert np.all(np.diff(c.weights) < 0)


def _toy_update(n=6, lam=8, seed0=100, rewards=None, m0=None):
    st = orc.cma_state_init(n, 0.32, m0)
    seeds = list(range(seed0, seed0 + lam))
    if rewards is None:
        rewards = np.random.default_rng(1).standard_normal(lam)
    return st, seeds, np.asarray(rewards, np.float64)


def test_cma_first_update_closed_forms():
    st, seeds, F = _toy_update()
    new, order = orc.cma_update(st, seeds, F)
    c = orc.cma_constants(6, 8)
    Z = np.stack([orc.normals_from_seed(s, 6) for s in seeds]).astype(np.float64)
    best = sorted(range(8), key=lambda i: -F[i])[:4]
    assert list(order[:4]) == best
    z_w = sum(c.weights[i] * Z[best[i]] for i in range(4))
    np.testing.assert_allclose(new.p_sigma, math.sqrt(c.c_sigma * (2 - c.c_sigma) * c.mu_eff) * z_w, atol=1e-14)
    np.testing.assert_allclose(new.m, 0.32 * z_w, atol=1e-14)                  # B = D = I, m0 = 0
    assert np.allclose(new.C, new.C.T, atol=1e-15)
    assert new.t == 1
    expect_sigma = 0.32 * math.exp(c.c_sigma / c.d_sigma * (np.linalg.norm(new.p_sigma) / c.chi_n - 1))
    assert abs(new.sigma - expect_sigma) < 1e-15
    # C: decay + rank-one + rank-mu, each term recomputed with loops
    h = new.extra["h_sigma"]
    assert h == 1.0
    pc = math.sqrt(c.c_c * (2 - c.c_c) * c.mu_eff) * z_w
    Cexp = (1 - c.c_1 - c.c_mu) * np.eye(6) + c.c_1 * np.outer(pc, pc)
    for i in range(4):
        Cexp += c.c_mu * c.weights[i] * np.outer(Z[best[i]], Z[best[i]])
    np.testing.assert_allclose(new.C, Cexp, atol=1e-14)


def test_cma_invariances():
    st, seeds, F = _toy_update()
    a, _ = orc.cma_update(st, seeds, F)
    # monotone transform of the rewards: only the order matters
    b, _ = orc.cma_update(st, seeds, np.exp(F) * 3 + 1)
    assert np.array_equal(a.C, b.C) and a.sigma == b.sigma and np.array_equal(a.m, b.m)
    # translation of the mean: same C, sigma, paths; shifted mean
    shift = np.arange(6.0)
    st2, _, _ = _toy_update(m0=shift)
    c2, _ = orc.cma_update(st2, seeds, F)
    np.testing.assert_allclose(c2.m - shift, a.m, atol=1e-15)
    assert np.array_equal(c2.C, a.C) and c2.sigma == a.sigma
    # minimising -F picks the opposite end
    d, od = orc.cma_update(st, seeds, -F)
    assert not np.array_equal(d.m, a.m)
    # identical steps for all candidates: mean moves by sigma*y, when every seed is the same
    e, _ = orc.cma_update(st, [42] * 8, F)
    np.testing.assert_allclose(e.m, 0.32 * orc.normals_from_seed(42, 6).astype(np.float64), atol=1e-15)


def test_cma_uses_basis_for_y_and_B_only_for_p_sigma():
    n = 5
    Q, d = wl.random_covariance_basis(n, 3)
    st = orc.cma_state_init(n, 0.5)
    st.B, st.D = Q.astype(np.float64), d.astype(np.float64)
    st.C = st.B @ np.diag(st.D ** 2) @ st.B.T
    seeds, F = [3, 4, 5, 6], np.array([0.1, 0.4, 0.3, 0.2])
    new, order = orc.cma_update(st, seeds, F)
    c = orc.cma_constants(n, 4)
    Z = np.stack([orc.normals_from_seed(s, n) for s in seeds]).astype(np.float64)
    zw = c.weights[0] * Z[1] + c.weights[1] * Z[2]
    np.testing.assert_allclose(new.m, 0.5 * st.B @ (st.D * zw), atol=1e-14)
    np.testing.assert_allclose(new.p_sigma, math.sqrt(c.c_sigma * (2 - c.c_sigma) * c.mu_eff) * (st.B @ zw), atol=1e-14)
    # sampling and update agree on what a candidate is: theta_k - m = sigma * y_k
    th, _ = orc.sample_candidates(st.m, st.sigma, st.B, st.D, seeds)
    yw = c.weights[0] * th[1] + c.weights[1] * th[2]
    np.testing.assert_allclose(new.m, yw, atol=1e-14)


@pytest.mark.parametrize("cond", [1.0, 100.0])
def test_cma_converges_on_quadratics(cond):
    """Textbook behaviour: maximising -sum(a_i x_i^2) drives the mean to 0 (sphere and ellipsoid)."""
    n, lam = 8, 12
    a = cond ** (np.arange(n) / (n - 1))
    st = orc.cma_state_init(n, 0.32, np.full(n, 1.0))
    f0 = float(np.sum(a * st.m ** 2))
    seed = 1
    for gen in range(260):
        seeds = list(range(seed, seed + lam))
        seed += lam
        th, _ = orc.sample_candidates(st.m, st.sigma, st.B, st.D, seeds)
        F = -np.sum(a[None] * th ** 2, axis=1)
        st, _ = orc.cma_update(st, seeds, F)
        w, V = np.linalg.eigh((st.C + st.C.T) / 2)         # the eigen refresh sits outside the hot path
        st.B, st.D = V, np.sqrt(np.maximum(w, 1e-30))
    assert float(np.sum(a * st.m ** 2)) < 1e-8 * f0


# ------------------------------------------------------------------------------------------------
# eigendecomposition of the covariance (tutorial Sec. B.2: C = B D^2 B^T)
# ------------------------------------------------------------------------------------------------
def test_refresh_basis_closed_form_2x2():
    """[[a, b], [b, c]]: eigenvalues (a+c)/2 -+ sqrt(((a-c)/2)^2 + b^2), eigenvector angle atan2(2b, a-c)/2."""
    a, b, c = 3.0, 0.8, 1.5
    B, D = orc.cma_refresh_basis(np.array([[a, b], [b, c]]))
    mid, rad = (a + c) / 2, math.hypot((a - c) / 2, b)
    np.testing.assert_allclose(D ** 2, [mid - rad, mid + rad], rtol=1e-14)
    phi = 0.5 * math.atan2(2 * b, a - c)                      # direction of the larger eigenvalue
    big = B[:, 1] * np.sign(B[0, 1])
    np.testing.assert_allclose(big, [math.cos(phi), math.sin(phi)], atol=1e-14)
    assert abs(B[:, 0] @ B[:, 1]) < 1e-15


def test_refresh_basis_diagonal_and_known_spectrum():
    d2 = np.array([4.0, 0.25, 9.0, 1.0])
    B, D = orc.cma_refresh_basis(np.diag(d2))
    np.testing.assert_allclose(D, np.sqrt(np.sort(d2)), rtol=1e-15)
    np.testing.assert_allclose(np.abs(B), np.eye(4)[:, np.argsort(d2)], atol=1e-15)        # a permutation of the axes
    # a known orthogonal basis and spectrum are recovered: eigenvalues exactly, eigenvectors up to sign
    n = 24
    Q, d = wl.random_covariance_basis(n, 11)
    Q, d = np.linalg.qr(Q.astype(np.float64))[0], d.astype(np.float64)     # orthonormal to fp64 round-off
    C = (Q * d ** 2) @ Q.T
    B, D = orc.cma_refresh_basis(C)
    order = np.argsort(d)
    np.testing.assert_allclose(D, d[order], rtol=1e-10)
    np.testing.assert_allclose(np.abs(np.sum(B * Q[:, order], axis=0)), 1.0, atol=1e-8)
    # the defining identities
    np.testing.assert_allclose((B * D ** 2) @ B.T, (C + C.T) / 2, atol=1e-12)
    np.testing.assert_allclose(B.T @ B, np.eye(n), atol=1e-12)
    # an asymmetric round-off in C does not matter (it is symmetrised), a slightly negative eigenvalue is clamped
    B2, D2 = orc.cma_refresh_basis(C + 1e-9 * np.triu(np.ones((n, n)), 1))
    np.testing.assert_allclose(D2, D, rtol=1e-6)
    _, D3 = orc.cma_refresh_basis(np.array([[1.0, 1.0 + 1e-12], [1.0 + 1e-12, 1.0]]))
    assert D3[0] == 0.0 and abs(D3[1] ** 2 - 2.0) < 1e-9


def test_refresh_basis_keeps_the_sampling_distribution():
    """Sampling through the refreshed (B, D) draws from N(m, sigma^2 C): the covariance of B D z is C, and a state whose
    C moved away from its old basis samples differently before and after the refresh."""
    n = 6
    g = np.random.default_rng(0)
    M = g.standard_normal((n, n))
    C = M @ M.T + 0.1 * np.eye(n)
    B, D = orc.cma_refresh_basis(C)
    T = B * D                                                 # y = T z
    np.testing.assert_allclose(T @ T.T, C, atol=1e-12)
    th, z = orc.sample_candidates(np.zeros(n), 1.0, B, D, [5])
    np.testing.assert_allclose(th[0], T @ z[0], atol=1e-5)


# ---------------------------------------------------------------- W8A8 composition, stalled CMA-ES update
def test_w8a8_forward_hand_worked_case():
    # One row x = (1, -0.3, 0.26): amax = 1, codes rint(127 x) = (127, -38, 33) worked by hand.  Wq = [[1, 2, 3],
    # [-4, 5, -6]] gives the integer sums 127 - 76 + 99 = 150 and -508 - 190 - 198 = -896; with channel scales
    # (0.5, 0.25) the base term is (150 / 127 * 0.5, -896 / 127 * 0.25).  The rank-1 update A = (0, 10, 0),
    # B = (1, 2)^T at its own singular values adds B A x = 10 * (-0.3) * (1, 2) on the UNQUANTISED x (on the codes it
    # would be 10 * (-38 / 127) * (1, 2), 0.008 away).
    Wq = np.array([[1, 2, 3], [-4, 5, -6]], np.int8)
    ws = np.array([0.5, 0.25], np.float32)
    A = np.array([[0.0, 10.0, 0.0]])
    B = np.array([[1.0], [2.0]])
    f = orc.thin_svd_factors(A, B)
    assert f["S_A"][0] == pytest.approx(10.0) and f["S_B"][0] == pytest.approx(math.sqrt(5.0))
    X = np.array([[1.0, -0.3, 0.26]], np.float32)
    y = orc.svdlora_forward_w8a8(Wq, ws, f, X, np.zeros(1, np.int32), f["S_A"][None], f["S_B"][None])
    expect = np.array([150.0 / 127.0 * 0.5 - 3.0, -896.0 / 127.0 * 0.25 - 6.0])
    np.testing.assert_allclose(y[0], expect, rtol=1e-6)
    assert np.abs(y[0] - (expect + 10 * (0.3 - 38 / 127) * np.array([1.0, 2.0]))).max() > 5e-3   # not the LoRA-on-codes reading
    # sigma = 0 leaves the base term alone
    y0 = orc.svdlora_forward_w8a8(Wq, ws, f, X, np.zeros(1, np.int32), np.zeros((1, 1)), f["S_B"][None])
    np.testing.assert_allclose(y0[0], expect + np.array([3.0, 6.0]), rtol=1e-6)


def test_w8a8_forward_within_the_quantisation_bound_of_the_exact_forward():
    # |x^ - x| <= s_i / 2 per entry, so the W8A8 output sits within (s_i / 2) sum_j |W_deq[o, j]| of the exact forward,
    # element by element; and it is not the exact forward (the rounding is really there).  A dropped channel scale,
    # a dropped row scale or a transposed operand leaves the bound by orders of magnitude.
    p = wl.make_projection("t", 96, 40, 4, "int8", layer=2)
    W = orc.dequant_int8(p.Wq, p.scales)
    f = orc.thin_svd_factors(p.A, p.B)
    K, R = 3, 17
    g = np.random.default_rng(8)
    sA = (f["S_A"][None] + 0.05 * g.standard_normal((K, 4))).astype(np.float32)
    sB = (f["S_B"][None] + 0.05 * g.standard_normal((K, 4))).astype(np.float32)
    _, xv = wl.make_x_bf16(R, 96, x_id=33)
    r2c = g.integers(0, K, R).astype(np.int32)
    y8 = orc.svdlora_forward_w8a8(p.Wq, p.scales, f, xv, r2c, sA, sB)
    y = orc.svdlora_forward(W, f, xv, r2c, sA, sB)
    s = np.abs(xv).max(axis=1).astype(np.float64) / 127.0
    bound = 0.5 * s[:, None] * np.abs(W).sum(axis=1)[None, :]
    assert np.all(np.abs(y8 - y) <= bound * (1 + 1e-6) + 1e-12)
    assert np.abs(y8 - y).max() > 1e-3 * bound.max()
    # statistically the error is that of uniform rounding noise: rms about s sqrt(sum_j W^2 / 12)
    pred = s[:, None] * np.sqrt((W * W).sum(axis=1) / 12.0)[None, :]
    ratio = np.sqrt(np.mean((y8 - y) ** 2)) / np.sqrt(np.mean(pred ** 2))
    assert 0.7 < ratio < 1.3


def _stalled_state(n, rng, t=5):
    """C = p_c p_c^T, B = D = I, |p_sigma| far above the stall threshold (1.4 + 2 / (n + 1)) chi_n."""
    st = orc.cma_state_init(n, 0.32, rng.standard_normal(n))
    st.p_c = rng.standard_normal(n)
    st.C = np.outer(st.p_c, st.p_c)
    st.p_sigma = np.zeros(n)
    st.p_sigma[0] = 50.0 * math.sqrt(n)
    st.t = t
    return st


def test_cma_update_stalled_branch_closed_form():
    # Tutorial, Eqs. (45)-(47): when |p_sigma| is too long, h_sigma = 0 drops the y_w term from p_c, and the factor of
    # C gains c_1 c_c (2 - c_c).  Because (1 - c_c)^2 + c_c (2 - c_c) = 1, a state with C = p_c p_c^T then keeps all its
    # rank-one mass: C' = (1 - c_mu) C + c_mu sum_i w_i y_i y_i^T, with no c_1 in it.  A wrong sign or factor in the
    # stall term, or a p_c that still takes y_w, breaks the identity.
    n, lam = 3, 8
    rng = np.random.default_rng(21)
    st = _stalled_state(n, rng)
    seeds = list(range(40, 40 + lam))
    F = rng.standard_normal(lam)
    new, order = orc.cma_update(st, seeds, F)
    c = orc.cma_constants(n, lam)
    assert new.extra["h_sigma"] == 0.0
    np.testing.assert_allclose(new.p_c, (1.0 - c.c_c) * st.p_c, rtol=1e-15)
    Z = np.stack([orc.normals_from_seed(s, n) for s in seeds]).astype(np.float64)       # B = D = I: y = z
    best = sorted(range(lam), key=lambda i: -F[i])[:c.mu]
    expect = (1.0 - c.c_mu) * st.C
    for i in range(c.mu):
        for a in range(n):
            for b in range(n):
                expect[a, b] += c.c_mu * c.weights[i] * Z[best[i], a] * Z[best[i], b]
    np.testing.assert_allclose(new.C, expect, rtol=1e-12, atol=1e-15)
    # the same step written out term by term with loops (decay, rank one, rank mu)
    decay = 1.0 - c.c_1 - c.c_mu + c.c_1 * c.c_c * (2.0 - c.c_c)
    loops = np.zeros((n, n))
    for a in range(n):
        for b in range(n):
            loops[a, b] = decay * st.C[a, b] + c.c_1 * (1 - c.c_c) ** 2 * st.p_c[a] * st.p_c[b]
            for i in range(c.mu):
                loops[a, b] += c.c_mu * c.weights[i] * Z[best[i], a] * Z[best[i], b]
    np.testing.assert_allclose(new.C, loops, rtol=1e-12, atol=1e-15)
    # mean and step size do not look at the flag
    z_w = sum(c.weights[i] * Z[best[i]] for i in range(c.mu))
    np.testing.assert_allclose(new.m, st.m + 0.32 * z_w, rtol=1e-13)
    ps = (1 - c.c_sigma) * st.p_sigma + math.sqrt(c.c_sigma * (2 - c.c_sigma) * c.mu_eff) * z_w
    assert new.sigma == pytest.approx(0.32 * math.exp(c.c_sigma / c.d_sigma * (np.linalg.norm(ps) / c.chi_n - 1)), rel=1e-13)
    assert new.sigma > 0.32                                       # a long path lengthens the step
    # with the path just short enough the flag is 1 again and p_c takes y_w
    st.p_sigma[0] = 0.5
    alive, _ = orc.cma_update(st, seeds, F)
    assert alive.extra["h_sigma"] == 1.0
    np.testing.assert_allclose(alive.p_c, (1 - c.c_c) * st.p_c + math.sqrt(c.c_c * (2 - c.c_c) * c.mu_eff) * z_w, rtol=1e-13)


def test_cma_stall_threshold_from_the_hand_evaluated_constants():
    # n = 16, lambda = 4 with the golden constants: the flag flips where |p_sigma| / sqrt(1 - (1 - c_sigma)^(2 (t + 1)))
    # crosses (1.4 + 2 / 17) chi_n.  p_sigma is chosen so that the NEW path has a given length: with all rewards equal and
    # the old path along e_0, p_sigma' = (1 - c_sigma) p_sigma + const z_w.
    rows = [l.split() for l in open(os.path.join(GOLDEN, "cma_constants.txt")) if l.strip() and not l.startswith("#")]
    row = [r for r in rows if r[0] == "16" and r[1] == "4"][0]
    c_sigma, chi_n = float(row[6]), float(row[11])
    n, lam, t = 16, 4, 2
    thr = (1.4 + 2.0 / 17.0) * chi_n * math.sqrt(1.0 - (1.0 - c_sigma) ** (2 * (t + 1)))
    seeds = [3, 4, 5, 6]
    F = np.array([4.0, 3.0, 2.0, 1.0])
    st = orc.cma_state_init(n, 0.32)
    st.t = t
    base, _ = orc.cma_update(st, seeds, F)                        # p_sigma = 0: the new path is the z_w term alone
    step = base.p_sigma
    for target, flag in ((0.98 * thr, 1.0), (1.02 * thr, 0.0)):
        # |(1 - c_sigma) a e_0 + step| = target  ->  a from the quadratic
        q = 1.0 - c_sigma
        bq, cq = 2 * q * step[0], float(step @ step) - target ** 2
        a = (-bq + math.sqrt(bq * bq - 4 * q * q * cq)) / (2 * q * q)
        st.p_sigma = np.zeros(n)
        st.p_sigma[0] = a
        new, _ = orc.cma_update(st, seeds, F)
        assert new.extra["ps_norm"] == pytest.approx(target, rel=1e-5)
        assert new.extra["h_sigma"] == flag
