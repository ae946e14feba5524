"""GPU parity of the other optimisers on the seed sampler (active / separable CMA-ES, plain (mu, lambda)-ES, ARS):
the HIP library through its C ABI binding against the CPU oracle, generation after generation on the same seeds
and rewards.  Rankings are bit-exact; states are held to the fp32 bar of the main update (rms 1e-5, max 1e-4
relative to the whole tensor)."""
import math

import numpy as np
import pytest
import torch

import essa_workloads as wl
import oracle as orc
from helpers import seeds_dev, to_dev

pytestmark = pytest.mark.gpu

FP32_RMS, FP32_MAX = 1e-5, 1e-4


@pytest.fixture(scope="module")
def ctx(essa):
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = essa.Context(0)
    yield c
    c.close()


def _say(msg):
    print(msg, flush=True)


def _close(a, b, what):
    e_max, e_rms = orc.rel_errors(np.asarray(a, np.float64), np.asarray(b, np.float64))
    assert e_rms <= FP32_RMS and e_max <= FP32_MAX, (what, e_max, e_rms)
    return e_max, e_rms


# ------------------------------------------------------------------------------------------------ active CMA-ES
@pytest.mark.parametrize("n,K,gens", [(16, 4, 3), (50, 13, 3), (257, 24, 2), (130, 42, 2), (2, 12, 3), (2, 64, 2), (1792, 96, 2)])
def test_active_cma_update(essa, ctx, n, K, gens):
    _say("active update n=%d K=%d" % (n, K))
    Q, d = wl.random_covariance_basis(n, basis_id=2000 + n)
    g = np.random.default_rng(n + K)
    m0 = g.standard_normal(n).astype(np.float32)
    C0 = (Q.astype(np.float64) * d.astype(np.float64) ** 2) @ Q.astype(np.float64).T
    C0 = ((C0 + C0.T) / 2).astype(np.float32)
    cma = essa.CmaState(ctx, n, 0.32, m0, kind=essa.OPT_ACTIVE_CMA)
    z = np.zeros(n, np.float32)
    cma.import_blob(essa.CmaState.pack_blob(n, 0, 0.32, m0, z, z, d, C0, Q, kind=essa.OPT_ACTIVE_CMA))
    st = orc.cma_state_init(n, np.float32(0.32), m0)
    st.B, st.D, st.C = Q.astype(np.float64), d.astype(np.float64), C0.astype(np.float64)
    seed = 7
    for gen in range(gens):
        seeds = list(range(seed, seed + K))
        seed += K
        F = g.standard_normal(K).astype(np.float32)
        F[0] = F[K - 1]
        order = torch.empty(K, dtype=torch.int32, device="cuda")
        essa.essa_cmaes_update(ctx, cma, seeds_dev(seeds), to_dev(F), order)
        st, ref_order = orc.cma_update_active(st, seeds, F)
        assert np.array_equal(order.cpu().numpy(), ref_order)
        exp = cma.export()
        assert exp["t"] == st.t and exp["kind"] == essa.OPT_ACTIVE_CMA
        for name in ("m", "p_sigma", "p_c", "C"):
            e = _close(exp[name], getattr(st, name), name)
            _say("  gen %d %s: %.2g/%.2g" % (gen, name, *e))
        assert abs(exp["sigma"] - st.sigma) / st.sigma <= 1e-5
        assert np.array_equal(exp["C"], exp["C"].T)
    # the tolerance can tell the two variants apart: the positive-weight update from the same state lands elsewhere
    plain, _ = orc.cma_update(st, seeds, F)
    act, _ = orc.cma_update_active(st, seeds, F)
    assert orc.rel_errors(plain.C, act.C)[1] > 50 * FP32_RMS or n > 60 or K == 64
    cma.close()


def test_active_cma_samples_like_the_default_kind(essa, ctx):
    n, K = 96, 10
    Q, d = wl.random_covariance_basis(n, basis_id=5)
    a = essa.CmaState(ctx, n, 0.32, None, kind=essa.OPT_ACTIVE_CMA)
    b = essa.CmaState(ctx, n, 0.32, None)
    for c in (a, b):
        c.set_basis(to_dev(Q), to_dev(d))
    ta, tb = torch.empty(K, n, device="cuda"), torch.empty(K, n, device="cuda")
    essa.essa_sample_candidates(ctx, a, seeds_dev(range(K)), ta, None)
    essa.essa_sample_candidates(ctx, b, seeds_dev(range(K)), tb, None)
    assert torch.equal(ta, tb)
    sweeps, off = a.refresh_basis(ctx)          # the matrix kinds share the eigendecomposition
    assert sweeps >= 1 and off <= 1e-7
    a.close()
    b.close()


# ------------------------------------------------------------------------------------------------ separable CMA-ES
@pytest.mark.parametrize("n,K,gens", [(1, 6, 4), (16, 4, 4), (257, 24, 3), (130, 42, 3), (3584, 64, 3), (100003, 32, 2)])
def test_sep_cma_generations(essa, ctx, n, K, gens):
    """sample -> update -> sample ...: the update refreshes the axis lengths itself, so the loop closes on the device."""
    _say("sep-CMA n=%d K=%d" % (n, K))
    g = np.random.default_rng(n * 3 + K)
    m0 = g.standard_normal(n).astype(np.float32)
    cd0 = g.uniform(0.25, 4.0, n).astype(np.float32)
    d0 = np.sqrt(cd0.astype(np.float64)).astype(np.float32)
    cma = essa.CmaState(ctx, n, 0.32, m0, kind=essa.OPT_SEP_CMA)
    z = np.zeros(n, np.float32)
    cma.import_blob(essa.CmaState.pack_blob(n, 0, 0.32, m0, z, z, d0, cd0, kind=essa.OPT_SEP_CMA))
    st = orc.sep_cma_init(n, np.float32(0.32), m0)
    st.c_diag = cd0.astype(np.float64)
    seed = 11
    for gen in range(gens):
        seeds = list(range(seed, seed + K))
        seed += K
        theta = torch.empty(K, n, device="cuda")
        zs = torch.empty(K, n, device="cuda")
        essa.essa_sample_candidates(ctx, cma, seeds_dev(seeds), theta, zs)
        ref_theta, ref_z = orc.sep_cma_sample(st, seeds)
        assert np.all(np.abs(zs.cpu().numpy() - ref_z) <= 2e-6 + 2e-6 * np.abs(ref_z))
        _close(theta.cpu().numpy(), ref_theta, "theta")
        F = g.standard_normal(K).astype(np.float32)
        F[1] = F[K - 1]
        order = torch.empty(K, dtype=torch.int32, device="cuda")
        essa.essa_cmaes_update(ctx, cma, seeds_dev(seeds), to_dev(F), order)
        st, ref_order = orc.sep_cma_update(st, seeds, F)
        assert np.array_equal(order.cpu().numpy(), ref_order)
        exp = cma.export()
        assert exp["t"] == st.t and exp["kind"] == essa.OPT_SEP_CMA
        for name in ("m", "p_sigma", "p_c", "c_diag"):
            e = _close(exp[name], getattr(st, name), name)
            _say("  gen %d %s: %.2g/%.2g" % (gen, name, *e))
        _close(exp["D"], np.sqrt(st.c_diag), "D")
        assert abs(exp["sigma"] - st.sigma) / st.sigma <= 1e-5
    cma.close()


# ------------------------------------------------------------------------------------------------ plain (mu, lambda)-ES
@pytest.mark.parametrize("n,K,gens", [(7, 2, 3), (50, 13, 3), (3584, 96, 3), (100003, 24, 2)])
def test_plain_es_generations(essa, ctx, n, K, gens):
    _say("ES n=%d K=%d" % (n, K))
    g = np.random.default_rng(n + 5 * K)
    m0 = g.standard_normal(n).astype(np.float32)
    cma = essa.CmaState(ctx, n, 0.05, m0, kind=essa.OPT_ES)
    m = m0.astype(np.float64)
    sigma = float(np.float32(0.05))
    seed = 3
    for gen in range(gens):
        seeds = list(range(seed, seed + K))
        seed += K
        theta = torch.empty(K, n, device="cuda")
        essa.essa_sample_candidates(ctx, cma, seeds_dev(seeds), theta, None)
        ref_theta, _ = orc.es_sample(m, sigma, seeds)
        _close(theta.cpu().numpy(), ref_theta, "theta")
        F = g.standard_normal(K).astype(np.float32)
        F[0] = F[K - 1]
        if gen == 1 and K > 4:
            F[2] = np.nan
        order = torch.empty(K, dtype=torch.int32, device="cuda")
        essa.essa_cmaes_update(ctx, cma, seeds_dev(seeds), to_dev(F), order)
        m, ref_order = orc.es_update(m, sigma, seeds, F)
        assert np.array_equal(order.cpu().numpy(), ref_order)
        exp = cma.export()
        assert exp["t"] == gen + 1 and exp["sigma"] == np.float32(0.05) and exp["kind"] == essa.OPT_ES
        e = _close(exp["m"], m, "m")
        # the step itself, not only the mean it lands on
        _say("  gen %d m: %.2g/%.2g" % (gen, *e))
    cma.close()


def test_plain_es_step_is_resolved(essa, ctx):
    """A mean far from the origin: the step sigma * mean(z) must still come out to fp32 accuracy of the sum."""
    n, K = 4096, 32
    m0 = np.full(n, 3.0, np.float32)
    cma = essa.CmaState(ctx, n, 0.01, m0, kind=essa.OPT_ES)
    seeds = list(range(100, 100 + K))
    F = np.random.default_rng(0).standard_normal(K).astype(np.float32)
    essa.essa_cmaes_update(ctx, cma, seeds_dev(seeds), to_dev(F), None)
    ref, _ = orc.es_update(m0.astype(np.float64), float(np.float32(0.01)), seeds, F)
    got = cma.export()["m"].astype(np.float64)
    assert np.all(np.abs(got - ref) <= 2.4e-7)       # half an ulp of 3.0 in fp32
    cma.close()


# ------------------------------------------------------------------------------------------------ ARS
@pytest.mark.parametrize("n,N,b,gens", [(6, 1, 1, 2), (50, 7, 3, 3), (3584, 48, 48, 2), (3584, 48, 16, 2), (100003, 12, 5, 2)])
def test_ars_generations(essa, ctx, n, N, b, gens):
    _say("ARS n=%d N=%d b=%d" % (n, N, b))
    g = np.random.default_rng(n + N + b)
    m0 = g.standard_normal(n).astype(np.float32)
    alpha, nu = 0.02, 0.03
    cma = essa.CmaState(ctx, n, nu, m0, kind=essa.OPT_ARS, ars_alpha=alpha, ars_top=b)
    m = m0.astype(np.float64)
    seed = 21
    for gen in range(gens):
        seeds = list(range(seed, seed + N))
        seed += N
        theta = torch.empty(2 * N, n, device="cuda")
        zs = torch.empty(2 * N, n, device="cuda")
        essa.essa_sample_candidates(ctx, cma, seeds_dev(seeds), theta, zs)
        ref_theta, ref_z = orc.ars_sample(m, float(np.float32(nu)), seeds)
        _close(theta.cpu().numpy(), ref_theta, "theta")
        zg = zs.cpu().numpy()
        assert np.array_equal(zg[0::2], -zg[1::2])
        assert np.all(np.abs(zg[0::2] - ref_z) <= 2e-6 + 2e-6 * np.abs(ref_z))
        F = g.standard_normal(2 * N).astype(np.float32)
        if N > 2:
            F[2], F[3] = F[1], F[0]                    # two directions with the same key
        order = torch.empty(N, dtype=torch.int32, device="cuda")
        essa.essa_cmaes_update(ctx, cma, seeds_dev(seeds), to_dev(F), order)
        m_new, ref_order = orc.ars_update(m, seeds, F, float(np.float32(alpha)), b)
        assert np.array_equal(order.cpu().numpy(), ref_order)
        exp = cma.export()
        assert exp["t"] == gen + 1 and exp["kind"] == essa.OPT_ARS
        _close(exp["m"], m_new, "m")
        e = orc.rel_errors(exp["m"].astype(np.float64) - m, m_new - m)
        _say("  gen %d step: %.2g/%.2g" % (gen, *e))
        if n <= 4000:
            assert e[1] <= 1e-4                        # the step itself (m is fp32: its rounding limits this)
        m = m_new
    cma.close()


def test_ars_degenerate_rewards_leave_the_mean(essa, ctx):
    n, N = 64, 4
    m0 = np.linspace(-1, 1, n).astype(np.float32)
    cma = essa.CmaState(ctx, n, 0.1, m0, kind=essa.OPT_ARS, ars_alpha=0.5, ars_top=2)
    for F in (np.zeros(2 * N, np.float32),                                   # s_R = 0
              np.array([1, 2, np.nan, 3, 0, 0, 0, 0], np.float32),           # a NaN among the rewards used
              np.array([np.inf, 2, 1, 3, 0, 0, 0, 0], np.float32)):
        essa.essa_cmaes_update(ctx, cma, seeds_dev(range(N)), to_dev(F), None)
        assert np.array_equal(cma.export()["m"], m0)
        assert np.array_equal(orc.ars_update(m0.astype(np.float64), list(range(N)), F, 0.5, 2)[0], m0.astype(np.float64))
    # a NaN in a discarded direction does not matter
    F = np.array([1, 2, 5, 3, np.nan, 0, 0, -1], np.float32)
    essa.essa_cmaes_update(ctx, cma, seeds_dev(range(N)), to_dev(F), None)
    ref, _ = orc.ars_update(m0.astype(np.float64), list(range(N)), F, float(np.float32(0.5)), 2)
    _close(cma.export()["m"], ref, "m")
    cma.close()


# ------------------------------------------------------------------------------------------------ shared behaviour
def test_kinds_without_a_matrix_refuse_basis_calls_and_resume_from_blobs(essa, ctx):
    n, K = 40, 8
    g = np.random.default_rng(1)
    for kind, kw in ((essa.OPT_SEP_CMA, {}), (essa.OPT_ES, {}), (essa.OPT_ARS, dict(ars_alpha=0.1, ars_top=3))):
        Fs = [g.standard_normal(K).astype(np.float32) for _ in range(4)]
        nseeds = K // 2 if kind == essa.OPT_ARS else K

        def run(resume):
            cma = essa.CmaState(ctx, n, 0.2, None, kind=kind, **kw)
            for gen in range(4):
                if resume and gen == 2:
                    blob = cma.export_blob()
                    cma.close()
                    cma = essa.CmaState(ctx, n, 1.0, None, kind=kind, **kw)
                    cma.import_blob(blob)
                essa.essa_cmaes_update(ctx, cma, seeds_dev(range(gen * K, gen * K + nseeds)), to_dev(Fs[gen]), None)
            out = cma.export_blob()
            cma.close()
            return out

        a, b, c = run(False), run(False), run(True)
        assert a == b and a == c
        assert len(a) == 24 + 5 * n * 4
        cma = essa.CmaState(ctx, n, 0.2, None, kind=kind, **kw)
        with pytest.raises(essa.EssaError):
            cma.set_basis(torch.eye(n, device="cuda"), torch.ones(n, device="cuda"))
        with pytest.raises(essa.EssaError):
            cma.refresh_basis(ctx)
        other = essa.CmaState(ctx, n, 0.2, None, kind=essa.OPT_SEP_CMA if kind != essa.OPT_SEP_CMA else essa.OPT_ES)
        with pytest.raises(essa.EssaError):
            other.import_blob(a)                       # a blob of another kind
        other.close()
        cma.close()
    with pytest.raises(essa.EssaError):
        essa.CmaState(ctx, n, 0.2, None, kind=essa.OPT_ARS, ars_alpha=0.0, ars_top=3)
    with pytest.raises(essa.EssaError):
        essa.CmaState(ctx, n, 0.2, None, kind=7)
    ars = essa.CmaState(ctx, n, 0.2, None, kind=essa.OPT_ARS, ars_alpha=0.1, ars_top=5)
    with pytest.raises(essa.EssaError):                # fewer pairs than directions to keep
        essa.essa_cmaes_update(ctx, ars, seeds_dev(range(4)), to_dev(np.zeros(8, np.float32)), None)
    ars.close()


def test_optimizer_generation_records_and_replays(essa, ctx):
    """A recorded sample + update of each kind replays to the same bits as the eager calls."""
    n, K = 300, 12
    for kind, kw in ((essa.OPT_ACTIVE_CMA, {}), (essa.OPT_SEP_CMA, {}), (essa.OPT_ES, {}), (essa.OPT_ARS, dict(ars_alpha=0.1, ars_top=4))):
        nseeds = K // 2 if kind == essa.OPT_ARS else K
        seeds = seeds_dev(range(50, 50 + nseeds))
        F = to_dev(np.random.default_rng(kind).standard_normal(K).astype(np.float32))
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            c2 = essa.Context(0, stream=side)
            eager = essa.CmaState(c2, n, 0.3, None, kind=kind, **kw)
            rec = essa.CmaState(c2, n, 0.3, None, kind=kind, **kw)
            th_e, th_r = torch.empty(K, n, device="cuda"), torch.empty(K, n, device="cuda")
            # warm-up: sizes the scratch and uploads the weights, then back to the initial state
            blob = rec.export_blob()
            essa.essa_sample_candidates(c2, rec, seeds, th_r, None)
            essa.essa_cmaes_update(c2, rec, seeds, F, None)
            rec.import_blob(blob)
            c2.graph_begin()
            essa.essa_sample_candidates(c2, rec, seeds, th_r, None)
            essa.essa_cmaes_update(c2, rec, seeds, F, None)
            graph = c2.graph_end()
            for rep in range(3):
                graph.launch()
                essa.essa_sample_candidates(c2, eager, seeds, th_e, None)
                essa.essa_cmaes_update(c2, eager, seeds, F, None)
                c2.synchronize()
                assert torch.equal(th_e, th_r), (kind, rep)
                assert eager.export_blob() == rec.export_blob(), (kind, rep)
            graph.close()
            eager.close()
            rec.close()
            c2.close()


# ------------------------------------------------------------------------------------------------ stalled steps, delta C
@pytest.mark.parametrize("kind_name,n,K", [("active", 16, 12), ("active", 50, 13), ("sep", 16, 4), ("sep", 257, 24)])
def test_stalled_step_of_the_other_cma_kinds(essa, ctx, kind_name, n, K):
    """|p_sigma| far above the threshold (h_sigma = 0) for the active and the separable update: p_c without y_w, the
    factor of C (of its diagonal) with the extra c_1 c_c (2 - c_c)."""
    _say("stalled %s n=%d K=%d" % (kind_name, n, K))
    g = np.random.default_rng(n + K)
    m0 = g.standard_normal(n).astype(np.float32)
    p_sigma = (8.0 * g.standard_normal(n)).astype(np.float32)
    p_c = g.standard_normal(n).astype(np.float32)
    seeds = list(range(3, 3 + K))
    F = g.standard_normal(K).astype(np.float32)
    if kind_name == "active":
        Q, d = wl.random_covariance_basis(n, basis_id=4000 + n)
        C0 = (Q.astype(np.float64) * d.astype(np.float64) ** 2) @ Q.astype(np.float64).T
        C0 = ((C0 + C0.T) / 2).astype(np.float32)
        cma = essa.CmaState(ctx, n, 0.32, m0, kind=essa.OPT_ACTIVE_CMA)
        cma.import_blob(essa.CmaState.pack_blob(n, 6, 0.32, m0, p_sigma, p_c, d, C0, Q, kind=essa.OPT_ACTIVE_CMA))
        st = orc.cma_state_init(n, np.float32(0.32), m0)
        st.B, st.D, st.C = Q.astype(np.float64), d.astype(np.float64), C0.astype(np.float64)
        st.p_sigma, st.p_c, st.t = p_sigma.astype(np.float64), p_c.astype(np.float64), 6
        essa.essa_cmaes_update(ctx, cma, seeds_dev(seeds), to_dev(F), None)
        new, _ = orc.cma_update_active(st, seeds, F)
        names = ("m", "p_sigma", "p_c", "C")
    else:
        cd0 = g.uniform(0.25, 4.0, n).astype(np.float32)
        d0 = np.sqrt(cd0.astype(np.float64)).astype(np.float32)
        cma = essa.CmaState(ctx, n, 0.32, m0, kind=essa.OPT_SEP_CMA)
        cma.import_blob(essa.CmaState.pack_blob(n, 6, 0.32, m0, p_sigma, p_c, d0, cd0, kind=essa.OPT_SEP_CMA))
        st = orc.sep_cma_init(n, np.float32(0.32), m0)
        st.c_diag, st.p_sigma, st.p_c, st.t = cd0.astype(np.float64), p_sigma.astype(np.float64), p_c.astype(np.float64), 6
        essa.essa_cmaes_update(ctx, cma, seeds_dev(seeds), to_dev(F), None)
        new, _ = orc.sep_cma_update(st, seeds, F)
        names = ("m", "p_sigma", "p_c", "c_diag")
    assert new.extra["h_sigma"] == 0.0
    exp = cma.export()
    for name in names:
        e = _close(exp[name], getattr(new, name), name)
        _say("  %s: %.2g/%.2g" % (name, *e))
    assert abs(exp["sigma"] - new.sigma) / new.sigma <= 1e-5
    cma.close()


def test_active_update_full_grid_delta_c(essa, ctx):
    """n = 1792, K = 96 with negative weights: the covariance kernel's change of C against the oracle's, resolved below
    the bar on C itself (an element is stored to within a rounding of its own size)."""
    n, K = 1792, 96
    Q, d = wl.random_covariance_basis(n, basis_id=2000 + n)
    g = np.random.default_rng(78)
    m0 = g.standard_normal(n).astype(np.float32)
    C0 = (Q.astype(np.float64) * d.astype(np.float64) ** 2) @ Q.astype(np.float64).T
    C0 = ((C0 + C0.T) / 2).astype(np.float32)
    p_sigma = (0.3 * g.standard_normal(n)).astype(np.float32)
    p_c = (Q.astype(np.float64) @ (d * g.standard_normal(n))).astype(np.float32)
    cma = essa.CmaState(ctx, n, 0.32, m0, kind=essa.OPT_ACTIVE_CMA)
    cma.import_blob(essa.CmaState.pack_blob(n, 30, 0.32, m0, p_sigma, p_c, d, C0, Q, kind=essa.OPT_ACTIVE_CMA))
    st = orc.cma_state_init(n, np.float32(0.32), m0)
    st.B, st.D, st.C = Q.astype(np.float64), d.astype(np.float64), C0.astype(np.float64)
    st.p_sigma, st.p_c, st.t = p_sigma.astype(np.float64), p_c.astype(np.float64), 30
    seeds = list(range(900, 900 + K))
    F = g.standard_normal(K).astype(np.float32)
    essa.essa_cmaes_update(ctx, cma, seeds_dev(seeds), to_dev(F), None)
    new, _ = orc.cma_update_active(st, seeds, F)
    exp = cma.export()
    dC = exp["C"].astype(np.float64) - C0.astype(np.float64)
    dref = new.C - st.C
    err = np.abs(dC - dref)
    bound = 1.05 * 2.0 ** -23 * np.abs(new.C) + 2e-5 * np.abs(dref).max()
    assert np.all(err <= bound), float((err / bound).max())
    e_max, e_rms = orc.rel_errors(dC, dref)
    _say("active n=1792: delta C rel err max %.3g rms %.3g" % (e_max, e_rms))
    assert e_rms <= 1e-2
    # teeth: the positive-weight update's change from the same state is far outside that bar
    plain, _ = orc.cma_update(st, seeds, F)
    assert orc.rel_errors(plain.C - st.C, dref)[1] > 5e-2
    cma.close()
