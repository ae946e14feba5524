"""GPU parity: the HIP library (through its C ABI binding) against the CPU oracle on the same seeded inputs.

Tolerances (relative to the whole reference tensor: max|d|/max|ref| and ||d||/||ref||):
  bit-exact      Philox words, int8 activation codes, int32 accumulators, ranking
  fp32 paths     rms 1e-5, max 1e-4   (tiny config, sampler, update)
  bf16 inputs    rms 1e-3, max 2e-2   (the stated bar) for bf16 outputs.  With fp32 outputs the same kernels are
                 held to tighter bars that follow from their arithmetic:
                   exact-product paths (ESSA_COMPUTE_BF16, generic kernel): rms 2e-5, max 2e-4 (fp32 accumulation,
                   bf16 head+tail operands in the rank-r term);
                   default int8-limb path: rms 2e-4, max 2e-3 -- each activation is rounded to a grid of
                   amax_row/32639, a uniform error of rms amax/113064, i.e. about 3e-5 of the output for N(0,1) rows.
"""
import math

import numpy as np
import pytest
import torch

import essa_workloads as wl
import oracle as orc
from helpers import bf16_dev, bf16_host, candidate_sigmas, gpu_proj, oracle_proj, sample_rows, seeds_dev, to_dev

pytestmark = pytest.mark.gpu

FP32_RMS, FP32_MAX = 1e-5, 1e-4
BF16_RMS, BF16_MAX = 1e-3, 2e-2
EXACT_RMS, EXACT_MAX = 2e-5, 2e-4
LIMB_RMS, LIMB_MAX = 2e-4, 2e-3


@pytest.fixture(scope="module")
def ctx(essa):
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = essa.Context(0)
    yield c
    c.close()


def _say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------------------------------------ sampler
def test_philox_words_bit_exact(essa, ctx):
    seeds = [0, 1, 2, 0xFFFFFFFF, 20250704]
    nb = 1000
    out = torch.empty(len(seeds) * nb * 4, dtype=torch.int32, device="cuda")
    essa.essa_philox_words(ctx, seeds_dev(seeds), nb, out)
    got = out.cpu().numpy().view(np.uint32).reshape(len(seeds), nb, 4)
    for i, s in enumerate(seeds):
        assert np.array_equal(got[i], orc.philox_words_for_seed(s, nb)), "seed %d" % s


@pytest.mark.parametrize("n,K", [(16, 4), (50, 3), (257, 70), (96, 42), (64, 400), (3584, 64)])
def test_sample_candidates(essa, ctx, n, K):
    _say("sample n=%d K=%d" % (n, K))
    Q, d = wl.random_covariance_basis(n, basis_id=n)
    m0 = np.linspace(-1, 1, n).astype(np.float32)
    cma = essa.CmaState(ctx, n, 0.32, m0)
    cma.set_basis(to_dev(Q), to_dev(d))
    seeds = list(range(1, K + 1))
    theta = torch.empty(K, n, device="cuda")
    z = torch.empty(K, n, device="cuda")
    essa.essa_sample_candidates(ctx, cma, seeds_dev(seeds), theta, z)
    theta2 = torch.empty_like(theta)
    essa.essa_sample_candidates(ctx, cma, seeds_dev(seeds), theta2, None)
    ref_theta, ref_z = orc.sample_candidates(m0, np.float32(0.32), Q, d, seeds)
    zg = z.cpu().numpy()
    assert np.all(np.abs(zg - ref_z) <= 2e-6 + 2e-6 * np.abs(ref_z))
    assert np.mean(zg == ref_z) > 0.999          # fp64 Box-Muller on both sides: almost always the same float
    e_max, e_rms = orc.rel_errors(theta.cpu().numpy(), ref_theta)
    assert e_rms <= FP32_RMS and e_max <= FP32_MAX, (e_max, e_rms)
    assert torch.equal(theta, theta2)            # same seed, same candidate, bit for bit
    # a candidate does not depend on who else is in the call
    one = torch.empty(1, n, device="cuda")
    essa.essa_sample_candidates(ctx, cma, seeds_dev([seeds[-1]]), one, None)
    assert torch.equal(one[0], theta[-1])
    cma.close()


def test_sample_identity_basis_is_exact(essa, ctx):
    n, K = 64, 5
    cma = essa.CmaState(ctx, n, 0.5, None)
    theta = torch.empty(K, n, device="cuda")
    z = torch.empty(K, n, device="cuda")
    essa.essa_sample_candidates(ctx, cma, seeds_dev([9, 8, 7, 6, 5]), theta, z)
    assert torch.equal(theta, 0.5 * z)
    cma.close()


def test_theta_to_sigma(essa, ctx):
    P, r, K = 6, 16, 5
    g = np.random.default_rng(0)
    sA0 = g.uniform(0.5, 2, (P, r)).astype(np.float32)
    sB0 = g.uniform(0.5, 2, (P, r)).astype(np.float32)
    for n_top in (16, 8, 1):
        th = g.standard_normal((K, P * 2 * n_top)).astype(np.float32)
        sA = torch.empty(K, P, r, device="cuda")
        sB = torch.empty(K, P, r, device="cuda")
        essa.essa_theta_to_sigma(ctx, n_top, to_dev(sA0), to_dev(sB0), to_dev(th), sA, sB)
        rA, rB = orc.theta_to_sigma(th, sA0, sB0, n_top / r)
        assert np.array_equal(sA.cpu().numpy(), rA.astype(np.float32))
        assert np.array_equal(sB.cpu().numpy(), rB.astype(np.float32))
    with pytest.raises(essa.EssaError):
        essa.essa_theta_to_sigma(ctx, 0, to_dev(sA0), to_dev(sB0), to_dev(np.zeros((K, 1), np.float32)),
                                 torch.empty(K, P, r, device="cuda"), torch.empty(K, P, r, device="cuda"))


# ------------------------------------------------------------------------------------------------ forward
def test_forward_c1_tiny_fp32(essa, ctx):
    """Configuration 1 as stated: 512x512 int8, r=8, K=4 candidates from seeds through the sampler."""
    p = wl.make_projection("q", 512, 512, 8, "int8")
    W, f = oracle_proj(p)
    gp = gpu_proj(essa, ctx, p)
    gA, gB = gp.spectrum()
    np.testing.assert_allclose(gA, f["S_A"], rtol=2e-6)
    np.testing.assert_allclose(gB, f["S_B"], rtol=2e-6)
    # sigma_k = sigma_0 (1 + 0.1 z): sampler with m = 0, step 0.1, B = I, D = own spectrum, then offsets
    n, K = 16, 4
    D = np.concatenate([f["S_A"], f["S_B"]]).astype(np.float32)
    cma = essa.CmaState(ctx, n, 0.1, None)
    cma.set_basis(to_dev(np.eye(n, dtype=np.float32)), to_dev(D))
    seeds = [1, 2, 3, 4]
    theta = torch.empty(K, n, device="cuda")
    essa.essa_sample_candidates(ctx, cma, seeds_dev(seeds), theta, None)
    sA = torch.empty(K, 1, 8, device="cuda")
    sB = torch.empty(K, 1, 8, device="cuda")
    essa.essa_theta_to_sigma(ctx, 8, to_dev(f["S_A"][None].astype(np.float32)), to_dev(f["S_B"][None].astype(np.float32)), theta, sA, sB)
    ref_theta, _ = orc.sample_candidates(np.zeros(n), np.float32(0.1), np.eye(n), D, seeds)
    rA, rB = orc.theta_to_sigma(ref_theta, f["S_A"][None].astype(np.float32), f["S_B"][None].astype(np.float32), 1.0)
    np.testing.assert_allclose(sA.cpu().numpy(), rA, rtol=1e-5)
    X = wl.make_x_f32(64, 512)
    r2c = wl.row2cand_contiguous(4, 16)
    Y = torch.empty(64, 512, device="cuda")
    essa.essa_svdlora_forward(ctx, gp, to_dev(X), to_dev(r2c), sA[:, 0, :], sB[:, 0, :], Y)
    ref = orc.svdlora_forward(W, f, X, r2c, rA[:, 0, :], rB[:, 0, :])
    e_max, e_rms = orc.rel_errors(Y.cpu().numpy(), ref)
    _say("c1 err max %.3g rms %.3g" % (e_max, e_rms))
    assert e_rms <= FP32_RMS and e_max <= FP32_MAX
    cma.close()
    gp.close()


@pytest.mark.parametrize("quant,d_in,d_out,r,K,R", [
    ("int8", 320, 200, 8, 7, 203),       # ragged rows and columns, five k-tiles
    ("int8", 1024, 384, 16, 5, 640),     # several 128x128 tiles
    ("int8", 512, 256, 32, 3, 65),
    ("int8", 328, 96, 4, 2, 9),          # d_in not a multiple of 16: generic kernel
    ("int4", 384, 200, 16, 6, 130),
    ("int4", 1024, 512, 32, 9, 300),
])
def test_forward_small_shapes_bf16(essa, ctx, quant, d_in, d_out, r, K, R):
    _say("forward %s d_in=%d d_out=%d r=%d K=%d R=%d" % (quant, d_in, d_out, r, K, R))
    p = wl.make_projection("t", d_in, d_out, r, quant, layer=3, proj=1)
    W, f = oracle_proj(p)
    gp = gpu_proj(essa, ctx, p)
    sA, sB = candidate_sigmas(f, K, 0.05)
    xb, xv = wl.make_x_bf16(R, d_in, x_id=7)
    g = np.random.default_rng(1)
    r2c = g.integers(0, K, R).astype(np.int32)
    r2c[r2c == K - 1] = 0                                  # one candidate owns no row
    ref = orc.svdlora_forward(W, f, xv, r2c, sA, sB)
    Xd, rd, sAd, sBd = bf16_dev(xb), to_dev(r2c), to_dev(sA), to_dev(sB)
    Y32 = torch.empty(R, d_out, device="cuda")
    base = xv.astype(np.float64) @ W.T
    ref_l = orc.svdlora_forward(W, f, xv, r2c, sA, sB, lora_only=True)
    own_A = to_dev(np.tile(f["S_A"].astype(np.float32), (K, 1)))
    own_B = to_dev(np.tile(f["S_B"].astype(np.float32), (K, 1)))
    ref_own = base + (xv.astype(np.float64) @ p.A.astype(np.float64).T) @ p.B.astype(np.float64).T
    # the default path rounds activations to 16-bit fixed point; ESSA_COMPUTE_BF16 and the generic kernel are exact in
    # the products
    variants = [(0, LIMB_RMS, LIMB_MAX), (essa.COMPUTE_BF16, EXACT_RMS, EXACT_MAX)] if d_in % 16 == 0 else [(0, EXACT_RMS, EXACT_MAX)]
    for fl, t_rms, t_max in variants:
        essa.essa_svdlora_forward(ctx, gp, Xd, rd, sAd, sBd, Y32, fl)
        e_max, e_rms = orc.rel_errors(Y32.cpu().numpy(), ref)
        _say("  flags %d fp32 out: max %.3g rms %.3g" % (fl, e_max, e_rms))
        assert e_rms <= t_rms and e_max <= t_max
        Y16 = torch.empty(R, d_out, device="cuda", dtype=torch.bfloat16)
        essa.essa_svdlora_forward(ctx, gp, Xd, rd, sAd, sBd, Y16, fl)
        e_max, e_rms = orc.rel_errors(bf16_host(Y16), orc.round_to_bf16(ref))
        _say("  flags %d bf16 out: max %.3g rms %.3g" % (fl, e_max, e_rms))
        assert e_rms <= BF16_RMS and e_max <= BF16_MAX
        # the rank-r term alone (never touched by the activation rounding) and the base alone
        essa.essa_svdlora_forward(ctx, gp, Xd, rd, sAd, sBd, Y32, fl | essa.LORA_ONLY)
        e_max, e_rms = orc.rel_errors(Y32.cpu().numpy(), ref_l)
        _say("  flags %d lora only: max %.3g rms %.3g" % (fl, e_max, e_rms))
        assert e_rms <= 1e-4 and e_max <= 1e-3
        essa.essa_svdlora_forward(ctx, gp, Xd, rd, sAd, sBd, Y32, fl | essa.BASE_ONLY)
        e_max, e_rms = orc.rel_errors(Y32.cpu().numpy(), base)
        assert e_rms <= t_rms and e_max <= t_max
        # sigma = 0 reproduces the base layer; own spectrum reproduces W + BA of the unfactored factors
        z = torch.zeros(K, r, device="cuda")
        essa.essa_svdlora_forward(ctx, gp, Xd, rd, z, sBd, Y32, fl)
        assert orc.rel_errors(Y32.cpu().numpy(), base)[1] <= t_rms
        essa.essa_svdlora_forward(ctx, gp, Xd, rd, own_A, own_B, Y32, fl)
        assert orc.rel_errors(Y32.cpu().numpy(), ref_own)[1] <= t_rms
    gp.close()


def test_forward_edge_cases(essa, ctx):
    p = wl.make_projection("t", 256, 128, 8, "int8", layer=5)
    W, f = oracle_proj(p)
    gp = gpu_proj(essa, ctx, p)
    sA, sB = candidate_sigmas(f, 1, 0.05)
    # R = 1, K = 1
    xb, xv = wl.make_x_bf16(1, 256, x_id=3)
    Y = torch.empty(1, 128, device="cuda")
    essa.essa_svdlora_forward(ctx, gp, bf16_dev(xb), to_dev(np.zeros(1, np.int32)), to_dev(sA), to_dev(sB), Y)
    e_max, e_rms = orc.rel_errors(Y.cpu().numpy(), orc.svdlora_forward(W, f, xv, np.zeros(1, np.int32), sA, sB))
    assert e_rms <= LIMB_RMS
    # R = 0 is a no-op
    essa.essa_svdlora_forward(ctx, gp, torch.empty(0, 256, device="cuda", dtype=torch.bfloat16), torch.empty(0, dtype=torch.int32, device="cuda"),
                              to_dev(sA), to_dev(sB), torch.empty(0, 128, device="cuda"))
    # argument errors are reported, not launched
    with pytest.raises(essa.EssaError):
        essa.essa_svdlora_forward(ctx, gp, bf16_dev(xb), to_dev(np.zeros(1, np.int32)), to_dev(sA), to_dev(sB), Y, 0x80)
    with pytest.raises(essa.EssaError):
        essa.essa_svdlora_forward(ctx, gp, bf16_dev(xb), to_dev(np.zeros(1, np.int32)), to_dev(sA), to_dev(sB), Y, essa.LORA_ONLY | essa.BASE_ONLY)
    gp.close()
    # population sizes and ranks from the paper's sweeps that are not powers of two
    for K, r in ((24, 2), (42, 4), (400, 8)):
        p = wl.make_projection("t", 128, 64, r, "int8", layer=6)
        W, f = oracle_proj(p)
        gp = gpu_proj(essa, ctx, p)
        sA, sB = candidate_sigmas(f, K, 0.05)
        xb, xv = wl.make_x_bf16(K, 128, x_id=4)
        r2c = np.arange(K, dtype=np.int32)[::-1].copy()
        Y = torch.empty(K, 64, device="cuda")
        essa.essa_svdlora_forward(ctx, gp, bf16_dev(xb), to_dev(r2c), to_dev(sA), to_dev(sB), Y)
        e_max, e_rms = orc.rel_errors(Y.cpu().numpy(), orc.svdlora_forward(W, f, xv, r2c, sA, sB))
        assert e_rms <= LIMB_RMS, (K, r, e_rms)
        gp.close()


def test_forward_row_permutation_and_strided_sigma(essa, ctx):
    p = wl.make_projection("t", 512, 192, 16, "int8", layer=7)
    W, f = oracle_proj(p)
    gp = gpu_proj(essa, ctx, p)
    K, R = 6, 150
    sA, sB = candidate_sigmas(f, K, 0.05)
    xb, xv = wl.make_x_bf16(R, 512, x_id=5)
    r2c = wl.row2cand_contiguous(K, 25)
    perm = np.random.default_rng(2).permutation(R)
    Y1 = torch.empty(R, 192, device="cuda")
    Y2 = torch.empty(R, 192, device="cuda")
    # sigma handed over as a slice of a [K, P, r] tensor
    big_A = torch.zeros(K, 3, 16, device="cuda")
    big_B = torch.zeros(K, 3, 16, device="cuda")
    big_A[:, 1, :] = to_dev(sA)
    big_B[:, 1, :] = to_dev(sB)
    essa.essa_svdlora_forward(ctx, gp, bf16_dev(xb), to_dev(r2c), big_A[:, 1, :], big_B[:, 1, :], Y1)
    essa.essa_svdlora_forward(ctx, gp, bf16_dev(xb[perm]), to_dev(r2c[perm]), to_dev(sA), to_dev(sB), Y2)
    assert torch.equal(Y1[torch.from_numpy(perm).cuda()], Y2)      # a row's result does not depend on where it sits
    e_max, e_rms = orc.rel_errors(Y1.cpu().numpy(), orc.svdlora_forward(W, f, xv, r2c, sA, sB))
    assert e_rms <= LIMB_RMS
    gp.close()


def test_w8a8_bit_exact_and_forward(essa, ctx):
    p = wl.make_projection("t", 448, 200, 16, "int8", layer=8)
    W, f = oracle_proj(p)
    gp = gpu_proj(essa, ctx, p)
    K, R = 4, 131
    xb, xv = wl.make_x_bf16(R, 448, x_id=6)
    xv[5] = 0
    xb[5] = 0
    xq = torch.empty(R, 448, dtype=torch.int8, device="cuda")
    xs = torch.empty(R, device="cuda")
    acc = torch.empty(R, 200, dtype=torch.int32, device="cuda")
    essa.essa_w8a8_accumulators(ctx, gp, bf16_dev(xb), xq, xs, acc)
    rq, rs = orc.quantize_rows_int8(xv)
    assert np.array_equal(xq.cpu().numpy(), rq)
    assert np.array_equal(xs.cpu().numpy(), rs)
    assert np.array_equal(acc.cpu().numpy().astype(np.int64), orc.int8_accumulators(rq, p.Wq))
    sA, sB = candidate_sigmas(f, K, 0.05)
    r2c = np.random.default_rng(3).integers(0, K, R).astype(np.int32)
    Y = torch.empty(R, 200, device="cuda")
    essa.essa_svdlora_forward(ctx, gp, bf16_dev(xb), to_dev(r2c), to_dev(sA), to_dev(sB), Y, essa.COMPUTE_W8A8)
    ref = orc.svdlora_forward_w8a8(p.Wq, p.scales, f, xv, r2c, sA, sB)
    e_max, e_rms = orc.rel_errors(Y.cpu().numpy(), ref)
    _say("w8a8 fp32 out: max %.3g rms %.3g" % (e_max, e_rms))
    assert e_rms <= 2e-5 and e_max <= 2e-4
    Yb = torch.empty(R, 200, device="cuda", dtype=torch.bfloat16)
    essa.essa_svdlora_forward(ctx, gp, bf16_dev(xb), to_dev(r2c), to_dev(sA), to_dev(sB), Yb, essa.COMPUTE_W8A8)
    e_max, e_rms = orc.rel_errors(bf16_host(Yb), orc.round_to_bf16(ref))
    assert e_rms <= BF16_RMS and e_max <= BF16_MAX
    gp.close()


def _layer_case(essa, ctx, cfg, layer, n_cands_checked, rows_per_cand_checked, flags=0):
    """One layer of a configuration at its full shape, q/k/v sharing X and o with its own, grouped launch."""
    projs = wl.make_layer(cfg.hidden, cfg.kv, cfg.r, cfg.quant, layer)
    K, R = cfg.K, cfg.R
    r2c = wl.row2cand_interleaved(K, cfg.rows_per_cand, layer) if cfg.interleaved else wl.row2cand_contiguous(K, cfg.rows_per_cand)
    xb1, xv1 = wl.make_x_bf16(R, cfg.hidden, x_id=2 * layer)
    xb2, xv2 = wl.make_x_bf16(R, cfg.hidden, x_id=2 * layer + 1)
    X1, X2, rd = bf16_dev(xb1), bf16_dev(xb2), to_dev(r2c)
    gps, items, outs, refs = [], [], [], []
    cands = list(range(K)) if n_cands_checked >= K else sorted(np.random.default_rng(layer).choice(K, n_cands_checked, replace=False).tolist())
    rows = np.arange(R) if (n_cands_checked >= K and rows_per_cand_checked >= cfg.rows_per_cand) else sample_rows(r2c, cands, rows_per_cand_checked, seed=layer)
    for pi, p in enumerate(projs):
        W, f = oracle_proj(p)
        sA, sB = candidate_sigmas(f, K, cfg.sigma_step, pert_id=layer * 4 + pi)
        gp = gpu_proj(essa, ctx, p)
        Y = torch.empty(R, p.d_out, device="cuda", dtype=torch.bfloat16)
        X, xv = (X2, xv2) if p.name == "o" else (X1, xv1)
        items.append((gp, X, rd, to_dev(sA), to_dev(sB), Y))
        gps.append(gp)
        outs.append(Y)
        if flags & essa.COMPUTE_W8A8:
            ref = orc.svdlora_forward_w8a8(p.Wq, p.scales, f, xv[rows], r2c[rows], sA, sB)
        else:
            ref = orc.svdlora_forward_rows(W, f, xv, r2c, sA, sB, rows)
        refs.append(orc.round_to_bf16(ref))
        _say("  oracle done for %s.%s (%d rows)" % (cfg.name, p.name, len(rows)))
    essa.essa_svdlora_forward_group(ctx, items, flags)
    torch.cuda.synchronize()
    rows_t = torch.from_numpy(rows).cuda()
    for p, Y, ref in zip(projs, outs, refs):
        e_max, e_rms = orc.rel_errors(bf16_host(Y[rows_t]), ref)
        _say("  %s.%s: max %.3g rms %.3g" % (cfg.name, p.name, e_max, e_rms))
        assert e_rms <= BF16_RMS and e_max <= BF16_MAX, (p.name, e_max, e_rms)
        assert torch.isfinite(Y.float()).all()
    # grouped and single launches agree bit for bit
    gp, X, rd_, a_, b_, Y = items[1]
    Y1 = torch.empty_like(Y)
    essa.essa_svdlora_forward(ctx, gp, X, rd_, a_, b_, Y1, flags)
    assert torch.equal(Y, Y1)
    for gp in gps:
        gp.close()


def test_forward_c2_full_layer(essa, ctx):
    _say("c2: 7B-shaped decode layer, all rows against the oracle")
    _layer_case(essa, ctx, wl.CONFIGS["c2_7b_decode"], layer=0, n_cands_checked=32, rows_per_cand_checked=8)


def test_forward_c2_full_layer_w8a8(essa, ctx):
    _say("c2 W8A8")
    _layer_case(essa, ctx, wl.CONFIGS["c2_7b_decode"], layer=1, n_cands_checked=32, rows_per_cand_checked=8, flags=1)


def test_forward_c3_prefill_sampled(essa, ctx):
    _say("c3: 32B-shaped prefill layer, sampled rows of 6 candidates")
    _layer_case(essa, ctx, wl.CONFIGS["c3_32b_prefill"], layer=0, n_cands_checked=6, rows_per_cand_checked=6)


def test_forward_c5_layer_sampled(essa, ctx):
    _say("c5: one 7B-shaped layer at the 32768 rows of the full iteration, sampled rows of 5 candidates")
    _layer_case(essa, ctx, wl.CONFIGS["c5_7b_es_iter"], layer=2, n_cands_checked=5, rows_per_cand_checked=6)


def test_forward_c4_int4_interleaved_sampled(essa, ctx):
    _say("c4: 72B-shaped int4 decode layer, interleaved rows, sampled candidates")
    _layer_case(essa, ctx, wl.CONFIGS["c4_72b_decode"], layer=0, n_cands_checked=5, rows_per_cand_checked=4)


# ------------------------------------------------------------------------------------------------ reward, ranking, update
def test_reward_accumulate(essa, ctx):
    g = np.random.default_rng(4)
    R, d, K = 300, 96, 7
    Yb = wl.f32_to_bf16_bits(g.standard_normal((R, d)).astype(np.float32))
    v = g.standard_normal(d).astype(np.float32)
    r2c = g.integers(0, K - 1, R).astype(np.int32)          # candidate K-1 has no rows
    F = torch.zeros(K, device="cuda")
    essa.essa_reward_accumulate(ctx, bf16_dev(Yb), to_dev(v), to_dev(r2c), F)
    essa.essa_reward_accumulate(ctx, bf16_dev(Yb), to_dev(v), to_dev(r2c), F)
    ref = orc.reward_accumulate(np.zeros(K), wl.bf16_bits_to_f32(Yb), v, r2c, K)
    ref = orc.reward_accumulate(ref, wl.bf16_bits_to_f32(Yb), v, r2c, K)
    got = F.cpu().numpy()
    assert math.isnan(got[K - 1]) and math.isnan(ref[K - 1])
    np.testing.assert_allclose(got[:K - 1], ref[:K - 1], rtol=1e-5, atol=1e-6)
    # several outputs in one call: same sum as one call per output, whatever their widths
    Y2 = wl.f32_to_bf16_bits(g.standard_normal((R, 41)).astype(np.float32))
    v2 = g.standard_normal(41).astype(np.float32)
    F = torch.zeros(K, device="cuda")
    essa.essa_reward_accumulate_group(ctx, [bf16_dev(Yb), bf16_dev(Y2)], [to_dev(v), to_dev(v2)], to_dev(r2c), F)
    ref2 = orc.reward_accumulate(orc.reward_accumulate(np.zeros(K), wl.bf16_bits_to_f32(Yb), v, r2c, K), wl.bf16_bits_to_f32(Y2), v2, r2c, K)
    np.testing.assert_allclose(F.cpu().numpy()[:K - 1], ref2[:K - 1], rtol=1e-5, atol=1e-6)
    Y32 = g.standard_normal((R, d)).astype(np.float32)
    F = torch.zeros(K, device="cuda")
    essa.essa_reward_accumulate(ctx, to_dev(Y32), to_dev(v), to_dev(r2c), F)
    np.testing.assert_allclose(F.cpu().numpy()[:K - 1], orc.reward_accumulate(np.zeros(K), Y32, v, r2c, K)[:K - 1], rtol=1e-5, atol=1e-6)


def _reward_bound(Yref, v, r2c, K, rel):
    """|dF_k| allowed when Y carries a relative row error `rel`: rel * mean_i ||Y_i|| * ||v|| (Cauchy-Schwarz per row)."""
    norms = np.linalg.norm(Yref, axis=1)
    out = np.zeros(K)
    for k in range(K):
        sel = r2c == k
        out[k] = rel * norms[sel].mean() * np.linalg.norm(v) if sel.any() else 0.0
    return out


@pytest.mark.parametrize("quant,x_fp32", [("int8", False), ("int4", False), ("int8", True)])
def test_forward_reward_fused(essa, ctx, quant, x_fp32):
    """Forward with the reward share added in the same launches, two 'layers' accumulated into one set of rows,
    against the oracle's forward -> round -> reward chain."""
    d_in, r, K, R = 256, 8, 5, 150
    d_outs = [200, 72] if not x_fp32 else [96, 40]
    _say("fused reward %s x_fp32=%s" % (quant, x_fp32))
    g = np.random.default_rng(11)
    r2c = g.integers(0, K - 1, R).astype(np.int32)          # candidate K-1 owns no row
    rd = to_dev(r2c)
    nblk = 2 * sum((d + essa.REWARD_BLOCK - 1) // essa.REWARD_BLOCK for d in d_outs)
    rowpart = torch.full((nblk + 1, R), float("nan"), device="cuda")       # one spare block that must stay untouched
    b0 = 0
    F_ref = np.zeros(K)
    bound = np.zeros(K)
    F_sep = torch.zeros(K, device="cuda")
    keep = []
    for layer in range(2):
        items, vs, Ys = [], [], []
        for pi, d_out in enumerate(d_outs):
            p = wl.make_projection("t", d_in, d_out, r, quant, layer=layer, proj=pi)
            W, f = oracle_proj(p)
            gp = gpu_proj(essa, ctx, p)
            sA, sB = candidate_sigmas(f, K, 0.05, pert_id=layer * 2 + pi)
            if x_fp32:
                xv = wl.make_x_f32(R, d_in, x_id=layer)
                Xd = to_dev(xv)
                Y = torch.empty(R, d_out, device="cuda")
            else:
                xb, xv = wl.make_x_bf16(R, d_in, x_id=layer)
                Xd = bf16_dev(xb)
                Y = torch.empty(R, d_out, device="cuda", dtype=torch.bfloat16)
            v = wl.reward_vector(d_out, layer, pi)
            ref = orc.svdlora_forward(W, f, xv, r2c, sA, sB)
            Yr = ref if x_fp32 else orc.round_to_bf16(ref)
            F_ref = orc.reward_accumulate(F_ref, Yr, v, r2c, K)
            bound += _reward_bound(Yr, v, r2c, K, 1e-4 if x_fp32 else 2e-3)
            items.append((gp, Xd, rd, to_dev(sA), to_dev(sB), Y))
            vs.append(to_dev(v))
            Ys.append(Y)
            keep.append(gp)
        grp = essa.ForwardGroup(items, vs)
        b0 = essa.essa_svdlora_forward_reward_group(ctx, grp, None, rowpart, b0)
        essa.essa_reward_accumulate_group(ctx, Ys, vs, rd, F_sep)
    assert b0 == nblk
    with pytest.raises(essa.EssaError):                                   # a block range past the buffer is refused
        essa.essa_svdlora_forward_reward_group(ctx, grp, None, rowpart, nblk)
    F = torch.zeros(K, device="cuda")
    essa.essa_reward_finish(ctx, rowpart, nblk, rd, F)
    got, sep = F.cpu().numpy(), F_sep.cpu().numpy()
    assert not torch.isnan(rowpart[:nblk]).any() and torch.isnan(rowpart[nblk]).all()
    assert math.isnan(got[K - 1]) and math.isnan(F_ref[K - 1])
    _say("  max |dF| %.3g (bound %.3g), vs two-pass GPU reward %.3g" % (np.abs(got[:K - 1] - F_ref[:K - 1]).max(), bound[:K - 1].min(),
                                                                       np.abs(got[:K - 1] - sep[:K - 1]).max()))
    assert np.all(np.abs(got[:K - 1] - F_ref[:K - 1]) <= bound[:K - 1])
    # same Y, same definition: the fused sum and the two-pass sum differ by fp32 summation order only
    np.testing.assert_allclose(got[:K - 1], sep[:K - 1], rtol=2e-5, atol=2e-6)
    # fixed summation order: a second run gives the same bits
    part2 = torch.empty(nblk // 2, R, device="cuda")
    part3 = torch.empty(nblk // 2, R, device="cuda")
    essa.essa_svdlora_forward_reward_group(ctx, grp, None, part2)
    essa.essa_svdlora_forward_reward_group(ctx, grp, None, part3)
    assert torch.equal(part2, part3) and torch.equal(part2, rowpart[nblk // 2:nblk])
    F2, F3 = torch.zeros(K, device="cuda"), torch.zeros(K, device="cuda")
    essa.essa_reward_finish(ctx, rowpart, nblk, rd, F2)
    essa.essa_reward_finish(ctx, rowpart, nblk, rd, F3)
    assert torch.equal(F2[:K - 1], F3[:K - 1]) and torch.equal(F2[:K - 1], F[:K - 1])
    for gp in keep:
        gp.close()


def test_forward_large_row_count_tile(essa, ctx):
    """Row counts in the thousands take the 128 x 256 tile: ragged rows and channels (the last tile's second half lies
    past d_out), both output types, one and two limbs, and the reward partials of every 128-channel block."""
    d_in, d_out, r, K, R = 192, 15400, 16, 7, 2050
    _say("large-R tile: d_in=%d d_out=%d R=%d" % (d_in, d_out, R))
    p = wl.make_projection("t", d_in, d_out, r, "int8", layer=5, proj=2)
    W, f = oracle_proj(p)
    gp = gpu_proj(essa, ctx, p)
    sA, sB = candidate_sigmas(f, K, 0.05)
    xb, xv = wl.make_x_bf16(R, d_in, x_id=11)
    r2c = np.random.default_rng(2).integers(0, K, R).astype(np.int32)
    ref = orc.svdlora_forward(W, f, xv, r2c, sA, sB)
    Xd, rd, sAd, sBd = bf16_dev(xb), to_dev(r2c), to_dev(sA), to_dev(sB)
    Y32 = torch.empty(R, d_out, device="cuda")
    essa.essa_svdlora_forward(ctx, gp, Xd, rd, sAd, sBd, Y32)
    e_max, e_rms = orc.rel_errors(Y32.cpu().numpy(), ref)
    _say("  fp32 out: max %.3g rms %.3g" % (e_max, e_rms))
    assert e_rms <= LIMB_RMS and e_max <= LIMB_MAX
    Y16 = torch.empty(R, d_out, device="cuda", dtype=torch.bfloat16)
    v = wl.reward_vector(d_out, 5, 2)
    nblk = (d_out + essa.REWARD_BLOCK - 1) // essa.REWARD_BLOCK
    rowpart = torch.full((nblk + 1, R), float("nan"), device="cuda")
    grp = essa.ForwardGroup([(gp, Xd, rd, sAd, sBd, Y16)], [to_dev(v)])
    assert essa.essa_svdlora_forward_reward_group(ctx, grp, None, rowpart) == nblk
    ref16 = orc.round_to_bf16(ref)
    e_max, e_rms = orc.rel_errors(bf16_host(Y16), ref16)
    _say("  bf16 out: max %.3g rms %.3g" % (e_max, e_rms))
    assert e_rms <= BF16_RMS and e_max <= BF16_MAX
    assert not torch.isnan(rowpart[:nblk]).any() and torch.isnan(rowpart[nblk]).all()
    F = torch.zeros(K, device="cuda")
    essa.essa_reward_finish(ctx, rowpart, nblk, rd, F)
    F_ref = orc.reward_accumulate(np.zeros(K), ref16, v, r2c, K)
    assert np.all(np.abs(F.cpu().numpy() - F_ref) <= _reward_bound(ref16, v, r2c, K, 2e-3))
    # the rank-r term and the base alone, and the one-limb mode against its own oracle
    essa.essa_svdlora_forward(ctx, gp, Xd, rd, sAd, sBd, Y32, essa.LORA_ONLY)
    e_max, e_rms = orc.rel_errors(Y32.cpu().numpy(), orc.svdlora_forward(W, f, xv, r2c, sA, sB, lora_only=True))
    assert e_rms <= 1e-4 and e_max <= 1e-3
    # at this size the prep kernel finishes the rank-space vectors itself (one workgroup over all K slices); a few rows
    # alone take the other route (shares per K slice, added up by the GEMM): the same bits in the rank-r term
    for sub in (slice(0, 40), slice(R - 35, R)):
        n = sub.stop - sub.start
        Ysub = torch.empty(n, d_out, device="cuda")
        essa.essa_svdlora_forward(ctx, gp, Xd[sub].contiguous(), rd[sub].contiguous(), sAd, sBd, Ysub, essa.LORA_ONLY)
        assert torch.equal(Ysub, Y32[sub])
    essa.essa_svdlora_forward(ctx, gp, Xd, rd, sAd, sBd, Y32, essa.COMPUTE_W8A8)
    e_max, e_rms = orc.rel_errors(Y32.cpu().numpy(), orc.svdlora_forward_w8a8(p.Wq, p.scales, f, xv, r2c, sA, sB))
    _say("  w8a8: max %.3g rms %.3g" % (e_max, e_rms))
    assert e_rms <= EXACT_RMS and e_max <= EXACT_MAX
    gp.close()


def test_forward_int4_wide_tile(essa, ctx):
    """4-bit weights with enough rows and channels for the 64 x 256 tile: ragged rows (the last row tile is partly
    empty) and channels (the last tile's blocks past d_out), both ranks paddings, both output types, the reward partials
    of every 128-channel block, the rank-r term and the base alone; and the same rows through the narrow tiles (a single
    small launch) give the same bits."""
    d_in, d_out, R = 256, 8232, 500                      # 258 blocks of 32 channels -> 33 column tiles x 8 row tiles
    for r, K in ((8, 5), (32, 9)):
        _say("int4 wide tile: d_in=%d d_out=%d R=%d r=%d" % (d_in, d_out, R, r))
        p = wl.make_projection("t", d_in, d_out, r, "int4", layer=6, proj=r)
        W, f = oracle_proj(p)
        gp = gpu_proj(essa, ctx, p)
        sA, sB = candidate_sigmas(f, K, 0.05)
        xb, xv = wl.make_x_bf16(R, d_in, x_id=12)
        r2c = np.random.default_rng(3).integers(0, K, R).astype(np.int32)
        ref = orc.svdlora_forward(W, f, xv, r2c, sA, sB)
        Xd, rd, sAd, sBd = bf16_dev(xb), to_dev(r2c), to_dev(sA), to_dev(sB)
        Y32 = torch.empty(R, d_out, device="cuda")
        essa.essa_svdlora_forward(ctx, gp, Xd, rd, sAd, sBd, Y32)
        e_max, e_rms = orc.rel_errors(Y32.cpu().numpy(), ref)
        _say("  fp32 out: max %.3g rms %.3g" % (e_max, e_rms))
        assert e_rms <= LIMB_RMS and e_max <= LIMB_MAX
        Y16 = torch.empty(R, d_out, device="cuda", dtype=torch.bfloat16)
        v = wl.reward_vector(d_out, 6, 1)
        nblk = (d_out + essa.REWARD_BLOCK - 1) // essa.REWARD_BLOCK
        rowpart = torch.full((nblk + 1, R), float("nan"), device="cuda")
        grp = essa.ForwardGroup([(gp, Xd, rd, sAd, sBd, Y16)], [to_dev(v)])
        assert essa.essa_svdlora_forward_reward_group(ctx, grp, None, rowpart) == nblk
        ref16 = orc.round_to_bf16(ref)
        e_max, e_rms = orc.rel_errors(bf16_host(Y16), ref16)
        _say("  bf16 out: max %.3g rms %.3g" % (e_max, e_rms))
        assert e_rms <= BF16_RMS and e_max <= BF16_MAX
        assert not torch.isnan(rowpart[:nblk]).any() and torch.isnan(rowpart[nblk]).all()
        F = torch.zeros(K, device="cuda")
        essa.essa_reward_finish(ctx, rowpart, nblk, rd, F)
        F_ref = orc.reward_accumulate(np.zeros(K), ref16, v, r2c, K)
        assert np.all(np.abs(F.cpu().numpy() - F_ref) <= _reward_bound(ref16, v, r2c, K, 2e-3))
        essa.essa_svdlora_forward(ctx, gp, Xd, rd, sAd, sBd, Y32, essa.LORA_ONLY)
        e_max, e_rms = orc.rel_errors(Y32.cpu().numpy(), orc.svdlora_forward(W, f, xv, r2c, sA, sB, lora_only=True))
        assert e_rms <= 1e-4 and e_max <= 1e-3
        essa.essa_svdlora_forward(ctx, gp, Xd, rd, sAd, sBd, Y32, essa.BASE_ONLY)
        e_max, e_rms = orc.rel_errors(Y32.cpu().numpy(), xv.astype(np.float64) @ W.T)
        assert e_rms <= LIMB_RMS and e_max <= LIMB_MAX
        # 40 of the rows alone: too few tiles for the wide kernel, so the 64 x 128 tiles take them -- same bits
        sub = slice(123, 163)
        Ysub = torch.empty(40, d_out, device="cuda", dtype=torch.bfloat16)
        essa.essa_svdlora_forward(ctx, gp, Xd[sub].contiguous(), rd[sub].contiguous(), sAd, sBd, Ysub)
        assert torch.equal(Ysub, Y16[sub])
        gp.close()


def test_forward_int4_wide_tile_mixed_heights(essa, ctx):
    """4-bit weights, 9 x 58 = 522 tiles of 64 x 256 on 512 places: the last 64 rows of every column go in 32-row tiles
    instead (ragged: 570 rows, the last 32-row tile holds 26; the last column tile ends inside a 32-channel block).
    Both outputs, the reward partials, and rows from either kind of tile alone through the narrow tiles: same bits."""
    d_in, d_out, R, r, K = 256, 14824, 570, 16, 7
    _say("int4 wide tile, mixed heights: d_in=%d d_out=%d R=%d" % (d_in, d_out, R))
    p = wl.make_projection("t", d_in, d_out, r, "int4", layer=8, proj=1)
    W, f = oracle_proj(p)
    gp = gpu_proj(essa, ctx, p)
    sA, sB = candidate_sigmas(f, K, 0.05)
    xb, xv = wl.make_x_bf16(R, d_in, x_id=14)
    r2c = np.random.default_rng(5).integers(0, K, R).astype(np.int32)
    ref = orc.svdlora_forward(W, f, xv, r2c, sA, sB)
    Xd, rd, sAd, sBd = bf16_dev(xb), to_dev(r2c), to_dev(sA), to_dev(sB)
    Y32 = torch.empty(R, d_out, device="cuda")
    essa.essa_svdlora_forward(ctx, gp, Xd, rd, sAd, sBd, Y32)
    e_max, e_rms = orc.rel_errors(Y32.cpu().numpy(), ref)
    _say("  fp32 out: max %.3g rms %.3g" % (e_max, e_rms))
    assert e_rms <= LIMB_RMS and e_max <= LIMB_MAX
    Y16 = torch.empty(R, d_out, device="cuda", dtype=torch.bfloat16)
    v = wl.reward_vector(d_out, 8, 1)
    nblk = (d_out + essa.REWARD_BLOCK - 1) // essa.REWARD_BLOCK
    rowpart = torch.full((nblk + 1, R), float("nan"), device="cuda")
    grp = essa.ForwardGroup([(gp, Xd, rd, sAd, sBd, Y16)], [to_dev(v)])
    assert essa.essa_svdlora_forward_reward_group(ctx, grp, None, rowpart) == nblk
    ref16 = orc.round_to_bf16(ref)
    e_max, e_rms = orc.rel_errors(bf16_host(Y16), ref16)
    _say("  bf16 out: max %.3g rms %.3g" % (e_max, e_rms))
    assert e_rms <= BF16_RMS and e_max <= BF16_MAX
    assert not torch.isnan(rowpart[:nblk]).any() and torch.isnan(rowpart[nblk]).all()
    F = torch.zeros(K, device="cuda")
    essa.essa_reward_finish(ctx, rowpart, nblk, rd, F)
    F_ref = orc.reward_accumulate(np.zeros(K), ref16, v, r2c, K)
    assert np.all(np.abs(F.cpu().numpy() - F_ref) <= _reward_bound(ref16, v, r2c, K, 2e-3))
    for sub in (slice(100, 140), slice(500, 540), slice(R - 30, R)):      # 64-row tiles, both kinds, 32-row tiles
        n = sub.stop - sub.start
        Ysub = torch.empty(n, d_out, device="cuda", dtype=torch.bfloat16)
        essa.essa_svdlora_forward(ctx, gp, Xd[sub].contiguous(), rd[sub].contiguous(), sAd, sBd, Ysub)
        assert torch.equal(Ysub, Y16[sub])
    gp.close()


@pytest.mark.parametrize("quant,d_in,d_out,r", [
    ("int8", 592, 72, 8),        # two trips of 64 chunks per row, the second one ragged
    ("int8", 3600, 40, 16),      # eight trips, two chunks in the last one
    ("int8", 6160, 40, 32),      # wider than 4096: two rows per workgroup at this row count too
    ("int4", 640, 264, 8),       # group sums: five real groups, three in the zero padding
])
def test_forward_rows_in_thousands_prep(essa, ctx, quant, d_in, d_out, r):
    """From 2048 rows on, activation rows up to 4096 wide are quantised one wave per row: ragged row count (the last
    workgroup's waves past the last row do nothing), row widths that end inside a trip of 64 chunks, both weight formats;
    and a few of the rows alone (quantised two rows per workgroup) give the same bits."""
    K, R = 6, 2051
    _say("rows in thousands: %s d_in=%d d_out=%d r=%d R=%d" % (quant, d_in, d_out, r, R))
    p = wl.make_projection("t", d_in, d_out, r, quant, layer=7, proj=3)
    W, f = oracle_proj(p)
    gp = gpu_proj(essa, ctx, p)
    sA, sB = candidate_sigmas(f, K, 0.05)
    xb, xv = wl.make_x_bf16(R, d_in, x_id=13)
    xb[5] = 0                                              # a row of zeros: unit 0, all limbs 0
    xv[5] = 0
    r2c = np.random.default_rng(4).integers(0, K, R).astype(np.int32)
    ref = orc.svdlora_forward(W, f, xv, r2c, sA, sB)
    Xd, rd, sAd, sBd = bf16_dev(xb), to_dev(r2c), to_dev(sA), to_dev(sB)
    Y32 = torch.empty(R, d_out, device="cuda")
    essa.essa_svdlora_forward(ctx, gp, Xd, rd, sAd, sBd, Y32)
    e_max, e_rms = orc.rel_errors(Y32.cpu().numpy(), ref)
    _say("  fp32 out: max %.3g rms %.3g" % (e_max, e_rms))
    assert e_rms <= LIMB_RMS and e_max <= LIMB_MAX
    assert torch.count_nonzero(Y32[5]).item() == 0
    if quant == "int8":
        essa.essa_svdlora_forward(ctx, gp, Xd, rd, sAd, sBd, Y32, essa.COMPUTE_W8A8)
        e_max, e_rms = orc.rel_errors(Y32.cpu().numpy(), orc.svdlora_forward_w8a8(p.Wq, p.scales, f, xv, r2c, sA, sB))
        _say("  w8a8: max %.3g rms %.3g" % (e_max, e_rms))
        assert e_rms <= EXACT_RMS and e_max <= EXACT_MAX
    Y16 = torch.empty(R, d_out, device="cuda", dtype=torch.bfloat16)
    essa.essa_svdlora_forward(ctx, gp, Xd, rd, sAd, sBd, Y16)
    e_max, e_rms = orc.rel_errors(bf16_host(Y16), orc.round_to_bf16(ref))
    assert e_rms <= BF16_RMS and e_max <= BF16_MAX
    for sub in (slice(0, 40), slice(R - 37, R)):
        n = sub.stop - sub.start
        Ysub = torch.empty(n, d_out, device="cuda", dtype=torch.bfloat16)
        essa.essa_svdlora_forward(ctx, gp, Xd[sub].contiguous(), rd[sub].contiguous(), sAd, sBd, Ysub)
        assert torch.equal(Ysub, Y16[sub])
    gp.close()


def test_forward_paper_sweep_values_mixed_group(essa, ctx):
    """The population sizes, ranks and alpha of the paper's sweeps (Appendix, hyperparameter study: K in 24..400, r down to
    2, alpha < 1) in ONE grouped launch with mixed ranks and mixed weight formats: candidates sampled from seeds, only the
    top floor(alpha r) singular values of each factor moved, rows of the K = 42 candidates interleaved."""
    K, rows_per, d_in = 42, 3, 256
    R = K * rows_per
    specs = [("int8", 200, 2), ("int4", 96, 4), ("int8", 328, 16), ("int4", 160, 32)]        # (format, d_out, rank)
    alpha = 0.5
    r2c = wl.row2cand_interleaved(K, rows_per, 3)
    xb, xv = wl.make_x_bf16(R, d_in, x_id=21)
    Xd, rd = bf16_dev(xb), to_dev(r2c)
    items, refs, gps = [], [], []
    for pi, (quant, d_out, r) in enumerate(specs):
        p = wl.make_projection("t", d_in, d_out, r, quant, layer=9, proj=pi)
        W, f = oracle_proj(p)
        gp = gpu_proj(essa, ctx, p)
        n_top = max(1, int(alpha * r))
        n = 2 * n_top
        # theta from seeds through the sampler (identity basis, step 0.05), then the top-alpha map, on both sides
        cma = essa.CmaState(ctx, n, 0.05, None)
        seeds = list(range(100 * pi + 1, 100 * pi + 1 + K))
        theta = torch.empty(K, n, device="cuda")
        essa.essa_sample_candidates(ctx, cma, seeds_dev(seeds), theta, None)
        sA = torch.empty(K, 1, r, device="cuda")
        sB = torch.empty(K, 1, r, device="cuda")
        sftA, sftB = f["S_A"][None].astype(np.float32), f["S_B"][None].astype(np.float32)
        essa.essa_theta_to_sigma(ctx, n_top, to_dev(sftA), to_dev(sftB), theta, sA, sB)
        ref_theta, _ = orc.sample_candidates(np.zeros(n), np.float32(0.05), np.eye(n), np.ones(n), seeds)
        rA, rB = orc.theta_to_sigma(ref_theta, sftA, sftB, n_top / r)
        assert np.array_equal(sA.cpu().numpy()[:, 0, n_top:], np.tile(sftA[0, n_top:], (K, 1)))      # the tail stays frozen
        np.testing.assert_allclose(sA.cpu().numpy(), rA, rtol=1e-5, atol=1e-7)
        refs.append(orc.round_to_bf16(orc.svdlora_forward(W, f, xv, r2c, rA[:, 0, :], rB[:, 0, :])))
        items.append((gp, Xd, rd, sA[:, 0, :], sB[:, 0, :], torch.empty(R, d_out, device="cuda", dtype=torch.bfloat16)))
        gps.append(gp)
        cma.close()
    essa.essa_svdlora_forward_group(ctx, items)
    for (quant, d_out, r), it, ref in zip(specs, items, refs):
        e_max, e_rms = orc.rel_errors(bf16_host(it[5]), ref)
        _say("  %s d_out=%d r=%d: max %.3g rms %.3g" % (quant, d_out, r, e_max, e_rms))
        assert e_rms <= BF16_RMS and e_max <= BF16_MAX
    # the same items one by one give the same bits
    for it in items:
        Y1 = torch.empty_like(it[5])
        essa.essa_svdlora_forward(ctx, it[0], it[1], it[2], it[3], it[4], Y1)
        assert torch.equal(Y1, it[5])
    for gp in gps:
        gp.close()


@pytest.mark.parametrize("K", [1, 4, 32, 64, 128, 400, 1024])
def test_rank_bit_exact(essa, ctx, K):
    g = np.random.default_rng(K)
    F = g.integers(0, max(2, K // 3), K).astype(np.float32)      # many ties
    if K >= 4:
        F[1] = np.nan
        F[2] = np.inf
        F[3] = -np.inf
    order = torch.empty(K, dtype=torch.int32, device="cuda")
    essa.essa_rank_rewards(ctx, to_dev(F), order)
    assert np.array_equal(order.cpu().numpy(), orc.rank_desc_stable(F))
    F = g.standard_normal(K).astype(np.float32)
    essa.essa_rank_rewards(ctx, to_dev(F), order)
    assert np.array_equal(order.cpu().numpy(), orc.rank_desc_stable(F))


def _state_errors(exp, ref):
    out = {}
    for name in ("m", "p_sigma", "p_c", "C"):
        out[name] = orc.rel_errors(exp[name], getattr(ref, name))
    out["sigma"] = abs(exp["sigma"] - ref.sigma) / ref.sigma
    return out


@pytest.mark.parametrize("n,K,gens", [(16, 4, 3), (50, 13, 3), (257, 24, 2), (120, 36, 2), (130, 42, 2), (200, 400, 2), (3584, 64, 2)])
def test_cmaes_update(essa, ctx, n, K, gens):
    _say("update n=%d K=%d" % (n, K))
    Q, d = wl.random_covariance_basis(n, basis_id=1000 + n)
    g = np.random.default_rng(n)
    m0 = g.standard_normal(n).astype(np.float32)
    C0 = (Q.astype(np.float64) * d.astype(np.float64) ** 2) @ Q.astype(np.float64).T
    C0 = ((C0 + C0.T) / 2).astype(np.float32)
    cma = essa.CmaState(ctx, n, 0.32, m0)
    z = np.zeros(n, np.float32)
    cma.import_blob(essa.CmaState.pack_blob(n, 0, 0.32, m0, z, z, d, C0, Q))
    st = orc.cma_state_init(n, np.float32(0.32), m0)
    st.B, st.D, st.C = Q.astype(np.float64), d.astype(np.float64), C0.astype(np.float64)
    seed = 1
    for gen in range(gens):
        seeds = list(range(seed, seed + K))
        seed += K
        F = g.standard_normal(K).astype(np.float32)
        F[0] = F[K - 1]                                        # a tie
        order = torch.empty(K, dtype=torch.int32, device="cuda")
        essa.essa_cmaes_update(ctx, cma, seeds_dev(seeds), to_dev(F), order)
        st, ref_order = orc.cma_update(st, seeds, F)
        assert np.array_equal(order.cpu().numpy(), ref_order)
        exp = cma.export()
        errs = _state_errors(exp, st)
        _say("  gen %d: %s" % (gen, {k: (("%.2g/%.2g" % v) if isinstance(v, tuple) else "%.2g" % v) for k, v in errs.items()}))
        assert exp["t"] == st.t
        for name in ("m", "p_sigma", "p_c", "C"):
            assert errs[name][1] <= FP32_RMS and errs[name][0] <= FP32_MAX, (name, errs[name])
        assert errs["sigma"] <= 1e-5
        assert np.array_equal(exp["C"], exp["C"].T)            # exactly symmetric
    cma.close()


def test_cmaes_update_is_reproducible_and_resumable(essa, ctx):
    n, K = 96, 10
    g = np.random.default_rng(5)
    Fs = [g.standard_normal(K).astype(np.float32) for _ in range(4)]

    def run(import_after=None):
        cma = essa.CmaState(ctx, n, 0.32, None)
        for gen in range(4):
            if import_after is not None and gen == 2:
                blob = cma.export_blob()
                cma.close()
                cma = essa.CmaState(ctx, n, 1.0, None)
                cma.import_blob(blob)
            essa.essa_cmaes_update(ctx, cma, seeds_dev(range(gen * K, gen * K + K)), to_dev(Fs[gen]), None)
        out = cma.export_blob()
        cma.close()
        return out

    a, b, c = run(), run(), run(import_after=2)
    assert a == b          # every worker performs the same update, bit for bit
    assert a == c          # export -> import -> continue equals the uninterrupted run
    # NaN rewards rank last and never reach the state
    cma = essa.CmaState(ctx, n, 0.32, None)
    F = Fs[0].copy()
    F[3] = np.nan
    essa.essa_cmaes_update(ctx, cma, seeds_dev(range(K)), to_dev(F), None)
    e = cma.export()
    assert np.isfinite(e["C"]).all() and np.isfinite(e["m"]).all() and math.isfinite(e["sigma"])
    with pytest.raises(essa.EssaError):
        cma.import_blob(a[:-4])
    with pytest.raises(essa.EssaError):
        essa.essa_cmaes_update(ctx, cma, seeds_dev([1]), to_dev(np.zeros(1, np.float32)), None)
    cma.close()


def test_full_iteration_small(essa, ctx):
    """A whole generation (configuration 5's structure at a small size): seeds -> theta -> sigma -> all
    projections -> reward -> update, each stage against the oracle; the update is fed the oracle's rewards
    on both sides so that a near-tie cannot flip the comparison."""
    layers, hidden, kv, r, K, rows_per = 2, 256, 64, 8, 6, 10
    P = layers * 4
    n = P * 2 * r
    R = K * rows_per
    projs = [p for l in range(layers) for p in wl.make_layer(hidden, kv, r, "int8", layer=20 + l)]
    orcs = [oracle_proj(p) for p in projs]
    gps = [gpu_proj(essa, ctx, p) for p in projs]
    sft_A = np.stack([f["S_A"] for _, f in orcs]).astype(np.float32)
    sft_B = np.stack([f["S_B"] for _, f in orcs]).astype(np.float32)
    Q, d = wl.random_covariance_basis(n, basis_id=77)
    d = (d * 0.05).astype(np.float32)
    cma = essa.CmaState(ctx, n, 0.32, None)
    C0 = ((Q.astype(np.float64) * d.astype(np.float64) ** 2) @ Q.astype(np.float64).T).astype(np.float32)
    zero = np.zeros(n, np.float32)
    cma.import_blob(essa.CmaState.pack_blob(n, 0, 0.32, zero, zero, zero, d, C0, Q))
    st = orc.cma_state_init(n, np.float32(0.32))
    st.B, st.D, st.C = Q.astype(np.float64), d.astype(np.float64), C0.astype(np.float64)
    seeds = list(range(1, K + 1))
    xb, xv = wl.make_x_bf16(R, hidden, x_id=99)
    r2c = wl.row2cand_contiguous(K, rows_per)
    Xd, rd = bf16_dev(xb), to_dev(r2c)
    # GPU pipeline
    theta = torch.empty(K, n, device="cuda")
    essa.essa_sample_candidates(ctx, cma, seeds_dev(seeds), theta, None)
    sA = torch.empty(K, P, r, device="cuda")
    sB = torch.empty(K, P, r, device="cuda")
    essa.essa_theta_to_sigma(ctx, r, to_dev(sft_A), to_dev(sft_B), theta, sA, sB)
    F = torch.zeros(K, device="cuda")
    Ys = []
    for l in range(layers):
        items = []
        for pi in range(4):
            j = l * 4 + pi
            Y = torch.empty(R, projs[j].d_out, device="cuda", dtype=torch.bfloat16)
            items.append((gps[j], Xd, rd, sA[:, j, :], sB[:, j, :], Y))
            Ys.append(Y)
        essa.essa_svdlora_forward_group(ctx, items)
        for pi in range(4):
            j = l * 4 + pi
            essa.essa_reward_accumulate(ctx, Ys[j], to_dev(wl.reward_vector(projs[j].d_out, 20 + l, pi)), rd, F)
    # oracle pipeline
    ref_theta, _ = orc.sample_candidates(np.zeros(n), np.float32(0.32), Q, d, seeds)
    rA, rB = orc.theta_to_sigma(ref_theta, sft_A, sft_B, 1.0)
    refF = np.zeros(K)
    for j, (W, f) in enumerate(orcs):
        ref = orc.round_to_bf16(orc.svdlora_forward(W, f, xv, r2c, rA[:, j, :], rB[:, j, :]))
        e_max, e_rms = orc.rel_errors(bf16_host(Ys[j]), ref)
        assert e_rms <= BF16_RMS and e_max <= BF16_MAX
        refF = orc.reward_accumulate(refF, ref, wl.reward_vector(projs[j].d_out, 20 + j // 4, j % 4), r2c, K)
    e_max, e_rms = orc.rel_errors(F.cpu().numpy(), refF)
    _say("full iteration: reward err max %.3g rms %.3g" % (e_max, e_rms))
    assert e_rms <= 1e-3
    refF32 = refF.astype(np.float32)
    essa.essa_cmaes_update(ctx, cma, seeds_dev(seeds), to_dev(refF32), None)
    st, _ = orc.cma_update(st, seeds, refF32)
    errs = _state_errors(cma.export(), st)
    for name in ("m", "p_sigma", "p_c", "C"):
        assert errs[name][1] <= FP32_RMS and errs[name][0] <= FP32_MAX, (name, errs[name])
    for gp in gps:
        gp.close()
    cma.close()


def test_recorded_generation_replays_bit_exact(essa):
    """A whole generation recorded once as a graph and replayed with new seeds: every replay leaves the same bits as the
    same generation run call by call (rewards and the whole search state), with eager work between the replays."""
    layers, hidden, kv, r, K, rows_per = 2, 256, 64, 8, 6, 10
    P, R = layers * 4, K * rows_per
    n = P * 2 * r
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        c2 = essa.Context(0, stream=side)
        projs = [p for l in range(layers) for p in wl.make_layer(hidden, kv, r, "int8", layer=30 + l)]
        gps = [gpu_proj(essa, c2, p) for p in projs]
        spec = [gp.spectrum() for gp in gps]
        sft_A = to_dev(np.stack([a for a, _ in spec]))
        sft_B = to_dev(np.stack([b for _, b in spec]))
        Q, d = wl.random_covariance_basis(n, basis_id=78)
        d = (d * 0.05).astype(np.float32)
        C0 = ((Q.astype(np.float64) * d.astype(np.float64) ** 2) @ Q.astype(np.float64).T).astype(np.float32)
        zero = np.zeros(n, np.float32)
        blob0 = essa.CmaState.pack_blob(n, 0, 0.32, zero, zero, zero, d, C0, Q)
        cma = essa.CmaState(c2, n, 0.32, None)
        xb, _ = wl.make_x_bf16(R, hidden, x_id=98)
        Xd, rd = bf16_dev(xb), to_dev(wl.row2cand_contiguous(K, rows_per))
        seeds = torch.zeros(K, dtype=torch.int32, device="cuda")
        theta = torch.empty(K, n, device="cuda")
        sA = torch.empty(K, P, r, device="cuda")
        sB = torch.empty(K, P, r, device="cuda")
        F = torch.zeros(K, device="cuda")
        groups = []
        for l in range(layers):
            items = [(gps[l * 4 + pi], Xd, rd, sA[:, l * 4 + pi, :], sB[:, l * 4 + pi, :],
                      torch.empty(R, projs[l * 4 + pi].d_out, device="cuda", dtype=torch.bfloat16)) for pi in range(4)]
            vs = [to_dev(wl.reward_vector(projs[l * 4 + pi].d_out, 30 + l, pi)) for pi in range(4)]
            groups.append(essa.ForwardGroup(items, vs))
        rowpart = torch.empty(sum(g.blocks for g in groups), R, device="cuda")

        def generation():
            essa.essa_sample_candidates(c2, cma, seeds, theta, None)
            essa.essa_theta_to_sigma(c2, r, sft_A, sft_B, theta, sA, sB)
            F.zero_()
            b = 0
            for g in groups:
                b = essa.essa_svdlora_forward_reward_group(c2, g, None, rowpart, b)
            essa.essa_reward_finish(c2, rowpart, b, rd, F)
            essa.essa_cmaes_update(c2, cma, seeds, F, None)

        seed_sets = [seeds_dev(range(1 + 10 * g, 1 + 10 * g + K)) for g in range(3)]
        cma.import_blob(blob0)
        eager = []
        for sset in seed_sets:
            seeds.copy_(sset)
            generation()
            side.synchronize()
            eager.append((F.clone(), cma.export()))
        # record (nothing runs), then replay from the same starting state
        cma.import_blob(blob0)
        c2.graph_begin()
        generation()
        graph = c2.graph_end()
        for sset, (F_ref, st_ref) in zip(seed_sets, eager):
            seeds.copy_(sset)
            graph.launch()
            side.synchronize()
            assert torch.equal(F, F_ref)
            st = cma.export()
            assert st["t"] == st_ref["t"] and st["sigma"] == st_ref["sigma"]
            for name in ("m", "p_sigma", "p_c", "C"):
                assert np.array_equal(st[name], st_ref[name]), name
            assert math.isfinite(float(rowpart.sum().item()))            # eager work between the replays
        # a call that would have to grow the scratch while recording is refused, and the recording survives it
        bigX = torch.zeros(4096, hidden, device="cuda", dtype=torch.bfloat16)
        bigY = torch.empty(4096, projs[0].d_out, device="cuda", dtype=torch.bfloat16)
        big_r2c = torch.zeros(4096, dtype=torch.int32, device="cuda")
        c2.graph_begin()
        with pytest.raises(essa.EssaError):
            essa.essa_svdlora_forward(c2, gps[0], bigX, big_r2c, sA[:, 0, :], sB[:, 0, :], bigY)
        essa.essa_theta_to_sigma(c2, r, sft_A, sft_B, theta, sA, sB)
        c2.graph_end().close()
        graph.close()
        for gp in gps:
            gp.close()
        cma.close()
        side.synchronize()
        c2.close()


@pytest.mark.parametrize("n", [2, 40, 64, 100, 257])
def test_refresh_basis(essa, ctx, n):
    """C -> (B, D) on the device against the oracle's eigendecomposition: eigenvalues, the defining identities, and the
    eigenvectors themselves where the spectrum separates them (each is defined up to sign)."""
    _say("refresh basis n=%d" % n)
    Q, d = wl.random_covariance_basis(n, basis_id=500 + n)
    g = np.random.default_rng(n)
    Qd = np.linalg.qr(Q.astype(np.float64))[0]
    C = ((Qd * d.astype(np.float64) ** 2) @ Qd.T).astype(np.float32)
    C = ((C + C.T) / 2).astype(np.float32)
    cma = essa.CmaState(ctx, n, 0.32, None)
    z = np.zeros(n, np.float32)
    cma.import_blob(essa.CmaState.pack_blob(n, 3, 0.5, z, z, z, np.ones(n, np.float32), C, np.eye(n, dtype=np.float32)))
    sweeps, off = cma.refresh_basis(ctx)
    _say("  %d sweeps, off %.2g" % (sweeps, off))
    st = cma.export()
    B, D = st["B"].astype(np.float64), st["D"].astype(np.float64)
    assert np.array_equal(st["C"], C) and st["t"] == 3                      # nothing else of the state moves
    Bref, Dref = orc.cma_refresh_basis(C)
    order = np.argsort(D)
    np.testing.assert_allclose(D[order], Dref, rtol=2e-6, atol=1e-7 * Dref.max())
    C64 = C.astype(np.float64)
    assert np.abs((B * D ** 2) @ B.T - C64).max() <= 2e-6 * np.abs(C64).max()
    assert np.abs(B.T @ B - np.eye(n)).max() <= 2e-6
    # eigenvectors, up to sign, where the neighbouring eigenvalues are at least 1 % away
    lam = Dref ** 2
    gap = np.minimum(np.diff(lam, prepend=-np.inf), np.diff(lam, append=np.inf)) / lam
    sel = gap > 1e-2
    dots = np.abs(np.sum(B[:, order] * Bref, axis=0))
    assert sel.sum() >= 1 and np.all(dots[sel] >= 1 - 1e-4)
    # sampling goes through the new basis: candidates follow the oracle's theta = m + sigma B (D z) with the device's B, D
    seeds = [5, 6, 7]
    theta = torch.empty(3, n, device="cuda")
    essa.essa_sample_candidates(ctx, cma, seeds_dev(seeds), theta, None)
    ref_theta, _ = orc.sample_candidates(np.zeros(n), np.float32(0.5), B, D, seeds)
    e_max, e_rms = orc.rel_errors(theta.cpu().numpy(), ref_theta)
    assert e_rms <= FP32_RMS and e_max <= FP32_MAX
    # a second refresh starts from the basis just found: nothing left to rotate, the same decomposition
    sweeps2, _ = cma.refresh_basis(ctx)
    st2 = cma.export()
    assert sweeps2 == 1
    np.testing.assert_allclose(st2["D"], st["D"], rtol=1e-6)
    assert np.abs(np.abs(np.sum(st2["B"].astype(np.float64) * B, axis=0)) - 1).max() <= 1e-5
    # same input, same bits: a fresh state (cold start) repeats the first result exactly
    cma3 = essa.CmaState(ctx, n, 0.32, None)
    cma3.import_blob(essa.CmaState.pack_blob(n, 3, 0.5, z, z, z, np.ones(n, np.float32), C, np.eye(n, dtype=np.float32)))
    cma3.refresh_basis(ctx)
    st3 = cma3.export()
    assert np.array_equal(st3["B"], st["B"]) and np.array_equal(st3["D"], st["D"])
    cma3.close()
    cma.close()


def test_refresh_basis_closes_the_loop(essa, ctx):
    """Generations of sampling and update with the basis refreshed every third one, device against oracle: every refresh
    is a valid factorisation of both sides' C, the candidates agree generation after generation, and a refresh that
    starts from the previous basis needs few sweeps."""
    n, K = 48, 12
    g = np.random.default_rng(9)
    cma = essa.CmaState(ctx, n, 0.3, None)
    st = orc.cma_state_init(n, np.float32(0.3))
    seed, warm_sweeps = 1, []
    for gen in range(12):
        seeds = list(range(seed, seed + K))
        seed += K
        theta = torch.empty(K, n, device="cuda")
        essa.essa_sample_candidates(ctx, cma, seeds_dev(seeds), theta, None)
        ref_theta, _ = orc.sample_candidates(st.m, st.sigma, st.B, st.D, seeds)
        e_max, e_rms = orc.rel_errors(theta.cpu().numpy(), ref_theta)
        assert e_rms <= 2e-5 and e_max <= 2e-4, (gen, e_max, e_rms)
        F = (-np.sum((ref_theta - 0.5) ** 2, axis=1)).astype(np.float32)          # a quadratic to climb, same rewards both sides
        essa.essa_cmaes_update(ctx, cma, seeds_dev(seeds), to_dev(F), None)
        st, _ = orc.cma_update(st, seeds, F)
        if gen % 3 == 2:
            sweeps, _ = cma.refresh_basis(ctx)
            if gen > 2:
                warm_sweeps.append(sweeps)
            _, Dref = orc.cma_refresh_basis(st.C)
            e = cma.export()
            B, D = e["B"].astype(np.float64), e["D"].astype(np.float64)
            assert np.abs((B * D ** 2) @ B.T - e["C"]).max() <= 5e-6 * np.abs(e["C"]).max()
            assert np.abs((B * D ** 2) @ B.T - st.C).max() <= 1e-4 * np.abs(st.C).max()          # ... and of the oracle's C
            np.testing.assert_allclose(np.sort(D), Dref, rtol=1e-4)
            # B D z depends on the signs and the order of the eigenvectors, which the decomposition leaves open: from here
            # on the oracle samples through the device's factorisation (just checked to be one of its own C)
            st.B, st.D = B, D
    _say("  warm refreshes took %s sweeps" % warm_sweeps)
    errs = _state_errors(cma.export(), st)
    for name in ("m", "C"):
        assert errs[name][1] <= 1e-4, (name, errs[name])
    cma.close()


# ------------------------------------------------------------------------------------------------ outliers, non-finite rows
@pytest.mark.parametrize("quant,d_in,d_out,r", [("int8", 3584, 256, 16), ("int4", 8192, 128, 32), ("int8", 512, 96, 8)])
def test_forward_outlier_rows_default_path(essa, ctx, quant, d_in, d_out, r):
    """Rows of the kind real hidden states have: one channel at 20x, 60x and 1000x the row's rms (it sets the fixed-point
    unit of the whole row), rows of tiny values, a row of zeros.  Bars, each row judged against its own output (a
    tensor-wide ratio would let the rows with the largest outputs speak for all):
      fp32 outputs   rms 1e-3, max 2e-2 (the stated bar) for every row: the rounding noise of a row on the 16-bit grid is
                     e_i = amax_i sqrt(d_in) / (32639 sqrt(12) |x_i|) of its output, at most sqrt(d_in) / 113064 (8e-4 at
                     d_in = 8192) whatever the row holds;
      bf16 outputs   compared after rounding both sides to bf16, a relative error e flips the rounding of a share
                     0.8 e / ulp of the elements by one ulp (2^-8 .. 2^-7 of the element), i.e. rms sqrt(0.8 e 2^-7.5):
                     inside 1e-3 up to e = 2.3e-4 (a largest entry of about 27 x rms at d_in = 3584), 1.3e-3 .. 1.7e-3 for
                     the single-outlier rows beyond.  Such rows meet 1e-3 in the exact-product mode (ESSA_COMPUTE_BF16)."""
    K, R = 4, 90
    _say("outlier rows %s d_in=%d" % (quant, d_in))
    p = wl.make_projection("t", d_in, d_out, r, quant, layer=11, proj=2)
    W, f = oracle_proj(p)
    gp = gpu_proj(essa, ctx, p)
    sA, sB = candidate_sigmas(f, K, 0.05)
    x = wl.make_x_f32(R, d_in, x_id=31)
    g = np.random.default_rng(6)
    for i in range(0, 40):                                  # rows 0..19: one 60x channel, 20..39: one 1000x channel
        x[i, g.integers(0, d_in)] = (60.0 if i < 20 else 1000.0) * (1 if i % 2 else -1)
    x[40:50] *= 1e-20                                       # tiny rows
    x[50] = 0.0
    x[51] *= 1e-32                                          # below 2^-100: the base term treats it as a row of zeros
    for i in range(52, 90):                                 # rows 52..89: one 20x channel
        x[i, g.integers(0, d_in)] = 20.0 * (1 if i % 2 else -1)
    xb = wl.f32_to_bf16_bits(x)
    xv = wl.bf16_bits_to_f32(xb)
    r2c = g.integers(0, K, R).astype(np.int32)
    ref = orc.svdlora_forward(W, f, xv, r2c, sA, sB)
    Xd, rd, sAd, sBd = bf16_dev(xb), to_dev(r2c), to_dev(sA), to_dev(sB)
    Y32 = torch.empty(R, d_out, device="cuda")
    essa.essa_svdlora_forward(ctx, gp, Xd, rd, sAd, sBd, Y32)
    Y16 = torch.empty(R, d_out, device="cuda", dtype=torch.bfloat16)
    essa.essa_svdlora_forward(ctx, gp, Xd, rd, sAd, sBd, Y16)
    got32, got16, ref16 = Y32.cpu().numpy().astype(np.float64), bf16_host(Y16), orc.round_to_bf16(ref)
    worst32 = 0.0
    e_pred = np.zeros(R)
    for i in range(R):
        if i in (50, 51):
            continue
        xi = xv[i].astype(np.float64)
        e_pred[i] = np.abs(xi).max() * math.sqrt(d_in) / (32639.0 * math.sqrt(12.0) * np.linalg.norm(xi))
        assert e_pred[i] <= math.sqrt(d_in) / 113064.0 * (1 + 1e-9)
        e_max, e_rms = orc.rel_errors(got32[i], ref[i])
        worst32 = max(worst32, e_rms)
        assert e_rms <= BF16_RMS and e_max <= BF16_MAX, ("fp32 out", i, e_max, e_rms)
        assert e_rms <= 1.5 * e_pred[i] + 2e-5, ("fp32 out against the predicted noise", i, e_rms, e_pred[i])
    _say("  worst row rms, fp32 out: %.3g" % worst32)
    # bf16 outputs by class of rows (one row's 100-odd outputs are too few to judge a rate of rounding flips)
    classes = {"60x": np.r_[0:20], "1000x": np.r_[20:40], "20x and tiny": np.r_[40:50, 52:90]}
    for name, rows in classes.items():
        e = float(np.sqrt(np.mean(e_pred[rows] ** 2)))
        bar16 = max(BF16_RMS, 1.2 * math.sqrt(0.8 * e * 2.0 ** -7.5))
        per_row = [orc.rel_errors(got16[i], ref16[i]) for i in rows]
        rms16 = float(np.sqrt(np.mean([v[1] ** 2 for v in per_row])))
        _say("  bf16 out, rows with %s: rms of the rows' relative errors %.3g (predicted noise %.3g, bar %.3g)" % (name, rms16, e, bar16))
        assert rms16 <= bar16 and max(v[0] for v in per_row) <= BF16_MAX, (name, rms16, bar16)
        if name == "20x and tiny":
            assert bar16 == BF16_RMS                        # this class meets the stated bar as it is
    assert np.count_nonzero(got32[50]) == 0
    base51 = xv[51].astype(np.float64) @ W.T
    assert np.abs(got32[51] - (ref[51] - base51)).max() <= 1e-3 * np.abs(ref[51] - base51).max() + 1e-38   # rank-r term only
    # the exact-product mode has no such rounding: every row at the stated bar in bf16 outputs, far inside it in fp32
    essa.essa_svdlora_forward(ctx, gp, Xd, rd, sAd, sBd, Y32, essa.COMPUTE_BF16)
    essa.essa_svdlora_forward(ctx, gp, Xd, rd, sAd, sBd, Y16, essa.COMPUTE_BF16)
    got, got16 = Y32.cpu().numpy().astype(np.float64), bf16_host(Y16)
    for i in range(50):
        assert orc.rel_errors(got[i], ref[i])[1] <= EXACT_RMS * 5, i
    for name, rows in classes.items():
        per_row = [orc.rel_errors(got16[i], ref16[i]) for i in rows]
        rms16 = float(np.sqrt(np.mean([v[1] ** 2 for v in per_row])))
        assert rms16 <= BF16_RMS and max(v[0] for v in per_row) <= BF16_MAX, ("exact mode, bf16 out", name, rms16)
    gp.close()


@pytest.mark.parametrize("quant", ["int8", "int4"])
def test_forward_nonfinite_rows_give_nan_rows(essa, ctx, quant):
    """A NaN or an Inf in an activation row: that row of the output is NaN where W_deq x + B_k A_k x is non-finite in every
    element, and no other row moves (default path, one-limb mode, exact-product mode; rows in the same tile as the bad ones)."""
    d_in, d_out, r, K, R = 512, 160, 8, 3, 45
    p = wl.make_projection("t", d_in, d_out, r, quant, layer=12, proj=1)
    W, f = oracle_proj(p)
    gp = gpu_proj(essa, ctx, p)
    sA, sB = candidate_sigmas(f, K, 0.05)
    xb, xv = wl.make_x_bf16(R, d_in, x_id=32)
    clean = bf16_dev(xb.copy())
    xb[3, 17] = 0x7FC0                                      # NaN
    xb[9, 400] = 0x7F80                                     # +Inf
    xb[40, 0] = 0xFF80                                      # -Inf
    bad = [3, 9, 40]
    good = [i for i in range(R) if i not in bad]
    xv = wl.bf16_bits_to_f32(xb)
    r2c = np.random.default_rng(7).integers(0, K, R).astype(np.int32)
    with np.errstate(invalid="ignore", over="ignore"):
        ref = orc.svdlora_forward(W, f, xv, r2c, sA, sB)
    # the exact result of such a row is non-finite in every element (NaN for a NaN, an infinity of either sign -- or NaN
    # against a zero weight -- for an Inf); the library reports the whole row as NaN
    assert np.isnan(ref[3]).all() and not np.isfinite(ref[bad]).any() and np.isfinite(ref[good]).all()
    rd, sAd, sBd = to_dev(r2c), to_dev(sA), to_dev(sB)
    modes = [0, essa.COMPUTE_BF16] + ([essa.COMPUTE_W8A8] if quant == "int8" else [])
    for fl in modes:
        Y, Yc = torch.empty(R, d_out, device="cuda"), torch.empty(R, d_out, device="cuda")
        essa.essa_svdlora_forward(ctx, gp, bf16_dev(xb), rd, sAd, sBd, Y, fl)
        essa.essa_svdlora_forward(ctx, gp, clean, rd, sAd, sBd, Yc, fl)
        got = Y.cpu().numpy()
        assert np.isnan(got[bad]).all(), fl
        assert np.array_equal(got[good], Yc.cpu().numpy()[good]), fl
    gp.close()


# ------------------------------------------------------------------------------------------------ int32 sums at full shapes
def test_w8a8_accumulators_bit_exact_full_shapes(essa, ctx):
    """The raw int32 sums of the production kernels at the sizes they run at: the decode tile at the 7B q projection
    (256 x 3584 x 3584) and the 128 x 256 tile of row counts in the thousands (4100 x 1024 x 4100, ragged in rows and
    channels).  Sampled rows against the oracle's integer sums, every element against the same sums taken in fp64 (exact:
    they stay below 2^53)."""
    for d_in, d_out, R, layer in ((3584, 3584, 256, 0), (1024, 4100, 4100, 13)):
        _say("int32 sums d_in=%d d_out=%d R=%d" % (d_in, d_out, R))
        p = wl.make_projection("q", d_in, d_out, 16, "int8", layer=layer)
        gp = gpu_proj(essa, ctx, p)
        xb, xv = wl.make_x_bf16(R, d_in, x_id=40 + layer)
        xq = torch.empty(R, d_in, dtype=torch.int8, device="cuda")
        xs = torch.empty(R, device="cuda")
        acc = torch.empty(R, d_out, dtype=torch.int32, device="cuda")
        essa.essa_w8a8_accumulators(ctx, gp, bf16_dev(xb), xq, xs, acc)
        rq, rs = orc.quantize_rows_int8(xv)
        assert np.array_equal(xq.cpu().numpy(), rq) and np.array_equal(xs.cpu().numpy(), rs)
        got = acc.cpu().numpy()
        rows = np.unique(np.concatenate([[0, 1, 31, 32, 63, 64, 127, 128, R - 1], np.random.default_rng(layer).integers(0, R, 24)]))
        assert np.array_equal(got[rows].astype(np.int64), orc.int8_accumulators(rq[rows], p.Wq))
        full = rq.astype(np.float64) @ p.Wq.astype(np.float64).T
        assert np.array_equal(got.astype(np.float64), full)
        gp.close()


# ------------------------------------------------------------------------------------------------ update: stall, delta C
def _cma_pair(essa, ctx, n, kind, Q, d, C0, m0, p_sigma, p_c, t, sigma=0.32):
    cma = essa.CmaState(ctx, n, sigma, m0, kind=kind)
    cma.import_blob(essa.CmaState.pack_blob(n, t, sigma, m0, p_sigma, p_c, d, C0, Q, kind=kind))
    st = orc.cma_state_init(n, np.float32(sigma), m0)
    st.B, st.D, st.C = Q.astype(np.float64), d.astype(np.float64), C0.astype(np.float64)
    st.p_sigma, st.p_c, st.t = p_sigma.astype(np.float64), p_c.astype(np.float64), t
    return cma, st


@pytest.mark.parametrize("n,K", [(16, 4), (50, 13), (130, 42)])
def test_cmaes_update_stalled_step(essa, ctx, n, K):
    """A state whose conjugate path is far too long (h_sigma = 0): p_c must not take y_w and the factor of C gains
    c_1 c_c (2 - c_c); then a second generation from the state that leaves, whatever its flag is."""
    _say("stalled update n=%d K=%d" % (n, K))
    Q, d = wl.random_covariance_basis(n, basis_id=3000 + n)
    g = np.random.default_rng(n)
    m0 = g.standard_normal(n).astype(np.float32)
    C0 = (Q.astype(np.float64) * d.astype(np.float64) ** 2) @ Q.astype(np.float64).T
    C0 = ((C0 + C0.T) / 2).astype(np.float32)
    p_sigma = (8.0 * g.standard_normal(n)).astype(np.float32)          # |p_sigma| = 8 sqrt(n), threshold about 1.5 sqrt(n)
    p_c = g.standard_normal(n).astype(np.float32)
    cma, st = _cma_pair(essa, ctx, n, essa.OPT_CMA, Q, d, C0, m0, p_sigma, p_c, t=9)
    seed = 1
    for gen in range(2):
        seeds = list(range(seed, seed + K))
        seed += K
        F = g.standard_normal(K).astype(np.float32)
        essa.essa_cmaes_update(ctx, cma, seeds_dev(seeds), to_dev(F), None)
        prev = st
        st, _ = orc.cma_update(st, seeds, F)
        if gen == 0:
            assert st.extra["h_sigma"] == 0.0
            c = orc.cma_constants(n, K)
            np.testing.assert_allclose(st.p_c, (1 - c.c_c) * prev.p_c, rtol=1e-14)
        errs = _state_errors(cma.export(), st)
        _say("  gen %d (h_sigma %g): %s" % (gen, st.extra["h_sigma"], {k: (("%.2g/%.2g" % v) if isinstance(v, tuple) else "%.2g" % v) for k, v in errs.items()}))
        for name in ("m", "p_sigma", "p_c", "C"):
            assert errs[name][1] <= FP32_RMS and errs[name][0] <= FP32_MAX, (name, errs[name])
        assert errs["sigma"] <= 1e-5
    cma.close()


def _delta_c_check(exp_C, C_old32, st_new, st_old, what):
    """C' - C on the device against the oracle's.  In fp32 one update at n in the thousands moves C by a few 1e-6 of its
    diagonal, less than the bar on C itself; the difference is resolved because an element is stored to within one
    rounding of its own size: |err_ij| <= 2^-23 |C_ij| (two roundings at most) + 2e-5 of the largest change."""
    dC = exp_C.astype(np.float64) - C_old32.astype(np.float64)
    dref = st_new.C - st_old.C
    err = np.abs(dC - dref)
    bound = 1.05 * 2.0 ** -23 * np.abs(st_new.C) + 2e-5 * np.abs(dref).max()
    assert np.all(err <= bound), (what, float((err / bound).max()))
    e_max, e_rms = orc.rel_errors(dC, dref)
    _say("  %s: delta C rel err max %.3g rms %.3g (|dC| rms %.3g of |C| rms %.3g)" % (what, e_max, e_rms, np.sqrt(np.mean(dref ** 2)), np.sqrt(np.mean(st_new.C ** 2))))
    assert e_rms <= 1e-2, (what, e_rms)
    return e_rms


def test_cmaes_update_full_size_delta_c(essa, ctx):
    """n = 3584, K = 64 (the full iteration's search state): the covariance kernel's whole grid, judged on what it adds."""
    n, K = 3584, 64
    Q, d = wl.random_covariance_basis(n, basis_id=1000 + n)
    g = np.random.default_rng(77)
    m0 = g.standard_normal(n).astype(np.float32)
    C0 = (Q.astype(np.float64) * d.astype(np.float64) ** 2) @ Q.astype(np.float64).T
    C0 = ((C0 + C0.T) / 2).astype(np.float32)
    p_sigma = (0.3 * g.standard_normal(n)).astype(np.float32)
    p_c = (Q.astype(np.float64) @ (d * g.standard_normal(n))).astype(np.float32)       # a path of the stationary size, ~ N(0, C)
    cma, st = _cma_pair(essa, ctx, n, essa.OPT_CMA, Q, d, C0, m0, p_sigma, p_c, t=40)
    seeds = list(range(500, 500 + K))
    F = g.standard_normal(K).astype(np.float32)
    essa.essa_cmaes_update(ctx, cma, seeds_dev(seeds), to_dev(F), None)
    new, _ = orc.cma_update(st, seeds, F)
    assert new.extra["h_sigma"] == 1.0
    exp = cma.export()
    _delta_c_check(exp["C"], C0, new, st, "cma n=3584")
    assert np.array_equal(exp["C"], exp["C"].T)
    # the comparison has teeth: without the rank-one term, or without the decay, the oracle's own change is far outside
    c = orc.cma_constants(n, K)
    dref = new.C - st.C
    assert orc.rel_errors(dref - c.c_1 * np.outer(new.p_c, new.p_c), dref)[1] > 5e-2
    assert orc.rel_errors(dref + (c.c_1 + c.c_mu) * st.C, dref)[1] > 5e-2
    for name in ("m", "p_sigma", "p_c"):
        e = orc.rel_errors(exp[name], getattr(new, name))
        assert e[1] <= FP32_RMS and e[0] <= FP32_MAX, (name, e)
    cma.close()


def test_refresh_basis_full_size(essa, ctx):
    """The eigendecomposition at the size the search state has (n = 3584): eigenvalues against the oracle's, the defining
    identities, and candidates drawn through the new basis."""
    n = 3584
    Q, d = wl.random_covariance_basis(n, basis_id=500 + n)
    Qd = Q.astype(np.float64)
    C = ((Qd * d.astype(np.float64) ** 2) @ Qd.T)
    C = ((C + C.T) / 2).astype(np.float32)
    cma = essa.CmaState(ctx, n, 0.32, None)
    z = np.zeros(n, np.float32)
    cma.import_blob(essa.CmaState.pack_blob(n, 3, 0.5, z, z, z, np.ones(n, np.float32), C, np.eye(n, dtype=np.float32)))
    _say("refresh basis n=%d ..." % n)
    sweeps, off = cma.refresh_basis(ctx)
    _say("  %d sweeps, off %.2g" % (sweeps, off))
    st = cma.export()
    B, D = st["B"].astype(np.float64), st["D"].astype(np.float64)
    assert np.array_equal(st["C"], C)
    _, Dref = orc.cma_refresh_basis(C)
    np.testing.assert_allclose(np.sort(D), Dref, rtol=3e-6, atol=1e-7 * Dref.max())
    C64 = C.astype(np.float64)
    assert np.abs((B * D ** 2) @ B.T - C64).max() <= 4e-6 * np.abs(C64).max()
    assert np.abs(B.T @ B - np.eye(n)).max() <= 4e-6
    seeds = [5, 6, 7]
    theta = torch.empty(3, n, device="cuda")
    essa.essa_sample_candidates(ctx, cma, seeds_dev(seeds), theta, None)
    ref_theta, _ = orc.sample_candidates(np.zeros(n), np.float32(0.5), B, D, seeds)
    e_max, e_rms = orc.rel_errors(theta.cpu().numpy(), ref_theta)
    assert e_rms <= FP32_RMS and e_max <= FP32_MAX
    cma.close()


# ------------------------------------------------------------------------------------------------ boundary rules
def test_validate_flag_checks_row2cand_on_the_host(essa, ctx):
    p = wl.make_projection("t", 256, 64, 8, "int8", layer=14)
    _, f = oracle_proj(p)
    gp = gpu_proj(essa, ctx, p)
    K, R = 3, 20
    sA, sB = candidate_sigmas(f, K, 0.05)
    xb, _ = wl.make_x_bf16(R, 256, x_id=41)
    r2c = np.random.default_rng(1).integers(0, K, R).astype(np.int32)
    Y = torch.full((R, 64), 7.0, device="cuda")
    essa.essa_svdlora_forward(ctx, gp, bf16_dev(xb), to_dev(r2c), to_dev(sA), to_dev(sB), Y, essa.VALIDATE)
    good = Y.clone()
    for bad_value in (K, -1, 1 << 20):
        bad = r2c.copy()
        bad[R - 2] = bad_value
        Y.fill_(7.0)
        with pytest.raises(essa.EssaError) as ei:
            essa.essa_svdlora_forward(ctx, gp, bf16_dev(xb), to_dev(bad), to_dev(sA), to_dev(sB), Y, essa.VALIDATE)
        assert ei.value.code == 1 and "row2cand[%d]" % (R - 2) in str(ei.value)
        assert torch.all(Y == 7.0)                          # nothing was launched
    # the flag changes nothing else
    Y2 = torch.empty_like(Y)
    essa.essa_svdlora_forward(ctx, gp, bf16_dev(xb), to_dev(r2c), to_dev(sA), to_dev(sB), Y2)
    assert torch.equal(Y2, good)
    gp.close()


def test_graph_lifetime_rules(essa):
    """While a recorded graph is alive its context neither moves the scratch (a larger problem is refused, not served from
    a new buffer the graph does not know) nor re-uploads the update's weights for another population size; destroying the
    graph lifts both; a graph whose context is gone refuses to launch."""
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        c2 = essa.Context(0, stream=side)
        p = wl.make_projection("t", 256, 64, 8, "int8", layer=15)
        _, f = oracle_proj(p)
        gp = gpu_proj(essa, c2, p)
        K = 3
        sA, sB = candidate_sigmas(f, K, 0.05)
        sAd, sBd = to_dev(sA), to_dev(sB)

        def fwd(R):
            xb, _ = wl.make_x_bf16(R, 256, x_id=42)
            Y = torch.empty(R, 64, device="cuda")
            essa.essa_svdlora_forward(c2, gp, bf16_dev(xb), to_dev(np.zeros(R, np.int32)), sAd, sBd, Y)
            return Y

        n = 24
        cma = essa.CmaState(c2, n, 0.3, None)
        seeds8, F8 = seeds_dev(range(8)), to_dev(np.arange(8, dtype=np.float32))
        essa.essa_cmaes_update(c2, cma, seeds8, F8, None)
        small_X, _ = wl.make_x_bf16(16, 256, x_id=43)
        Xs, Ys, r0 = bf16_dev(small_X), torch.empty(16, 64, device="cuda"), to_dev(np.zeros(16, np.int32))
        essa.essa_svdlora_forward(c2, gp, Xs, r0, sAd, sBd, Ys)
        side.synchronize()
        want = Ys.clone()
        c2.graph_begin()
        essa.essa_svdlora_forward(c2, gp, Xs, r0, sAd, sBd, Ys)
        essa.essa_cmaes_update(c2, cma, seeds8, F8, None)
        graph = c2.graph_end()
        with pytest.raises(essa.EssaError) as ei:                       # needs far more scratch than any call before
            fwd(20000)
        assert ei.value.code == 6
        with pytest.raises(essa.EssaError) as ei:                       # another population size: other weights
            essa.essa_cmaes_update(c2, cma, seeds_dev(range(12)), to_dev(np.arange(12, dtype=np.float32)), None)
        assert ei.value.code == 6
        Ys.zero_()
        graph.launch()                                                   # the graph still works on the memory it knows
        side.synchronize()
        assert torch.equal(Ys, want)
        graph.close()
        assert fwd(20000).shape[0] == 20000                              # ... and without it both calls go through
        essa.essa_cmaes_update(c2, cma, seeds_dev(range(12)), to_dev(np.arange(12, dtype=np.float32)), None)
        side.synchronize()
        c2.graph_begin()
        essa.essa_svdlora_forward(c2, gp, Xs, r0, sAd, sBd, Ys)
        orphan = c2.graph_end()
        gp.close()
        cma.close()
        c2.close()
        with pytest.raises(essa.EssaError):
            orphan.launch()
        orphan.close()


# ------------------------------------------------------------------------------------------------ row counts up to 64
@pytest.mark.parametrize("d_in,d_out,r,K", [(320, 200, 8, 5), (3584, 264, 16, 7), (1024, 72, 32, 3), (5120, 136, 16, 4)])
def test_forward_small_row_counts_stream_kernel(essa, ctx, d_in, d_out, r, K):
    """Up to 64 rows on int8 weights take the kernel that splits K over the waves of a 32-channel workgroup, with one
    block of 32 rows or two: one row, a few rows, one full block, one row more (two blocks), two full blocks, and one row
    more (the 32-row tiles again); ragged channels; both output types; the one-limb mode; the rank-r term and the base
    alone; the fused reward (a pass of its own behind this kernel); and the rows of a larger call (64-row tiles, K split in
    halves) give the same bits in fp32 and bf16.  The 5120-wide case has more chunks per wave than the kernel asks weights for
    at once (a second bunch)."""
    _say("small row counts d_in=%d d_out=%d r=%d" % (d_in, d_out, r))
    p = wl.make_projection("t", d_in, d_out, r, "int8", layer=18, proj=r % 4)
    W, f = oracle_proj(p)
    gp = gpu_proj(essa, ctx, p)
    sA, sB = candidate_sigmas(f, K, 0.05)
    sAd, sBd = to_dev(sA), to_dev(sB)
    Rbig = 150
    xb, xv = wl.make_x_bf16(Rbig, d_in, x_id=60)
    xb[2] = 0
    xv[2] = 0
    r2c = np.random.default_rng(8).integers(0, K, Rbig).astype(np.int32)
    Xd, rd = bf16_dev(xb), to_dev(r2c)
    ref = orc.svdlora_forward(W, f, xv, r2c, sA, sB)
    ref8 = orc.svdlora_forward_w8a8(p.Wq, p.scales, f, xv, r2c, sA, sB)
    big32 = torch.empty(Rbig, d_out, device="cuda")
    big16 = torch.empty(Rbig, d_out, device="cuda", dtype=torch.bfloat16)
    essa.essa_svdlora_forward(ctx, gp, Xd, rd, sAd, sBd, big32)           # 150 rows: the 64-row tiles
    essa.essa_svdlora_forward(ctx, gp, Xd, rd, sAd, sBd, big16)
    v = wl.reward_vector(d_out, 18, 0)
    nblk = (d_out + essa.REWARD_BLOCK - 1) // essa.REWARD_BLOCK
    for R in (1, 8, 31, 32, 33, 48, 64, 65):
        for start in (0, Rbig - R):
            sub = slice(start, start + R)
            Xs, rs = Xd[sub].contiguous(), rd[sub].contiguous()
            Y32 = torch.empty(R, d_out, device="cuda")
            Y16 = torch.empty(R, d_out, device="cuda", dtype=torch.bfloat16)
            essa.essa_svdlora_forward(ctx, gp, Xs, rs, sAd, sBd, Y32)
            essa.essa_svdlora_forward(ctx, gp, Xs, rs, sAd, sBd, Y16)
            assert torch.equal(Y32, big32[sub]) and torch.equal(Y16, big16[sub]), (R, start)
            e_max, e_rms = orc.rel_errors(Y32.cpu().numpy(), ref[sub])
            assert e_rms <= LIMB_RMS and e_max <= LIMB_MAX, (R, start, e_max, e_rms)
            if R > 4:
                e_max, e_rms = orc.rel_errors(bf16_host(Y16), orc.round_to_bf16(ref[sub]))
                assert e_rms <= 2 * BF16_RMS and e_max <= BF16_MAX, (R, start, e_max, e_rms)   # few elements: see the whole-tensor check below
            essa.essa_svdlora_forward(ctx, gp, Xs, rs, sAd, sBd, Y32, essa.COMPUTE_W8A8)
            e_max, e_rms = orc.rel_errors(Y32.cpu().numpy(), ref8[sub])
            assert e_rms <= EXACT_RMS and e_max <= EXACT_MAX, ("w8a8", R, start, e_max, e_rms)
            essa.essa_svdlora_forward(ctx, gp, Xs, rs, sAd, sBd, Y32, essa.LORA_ONLY)
            e_max, e_rms = orc.rel_errors(Y32.cpu().numpy(), orc.svdlora_forward(W, f, xv[sub], r2c[sub], sA, sB, lora_only=True))
            assert e_rms <= 1e-4 and e_max <= 1e-3, ("lora only", R, start)
            essa.essa_svdlora_forward(ctx, gp, Xs, rs, sAd, sBd, Y32, essa.BASE_ONLY)
            e_max, e_rms = orc.rel_errors(Y32.cpu().numpy(), xv[sub].astype(np.float64) @ W.T)
            assert e_rms <= LIMB_RMS and e_max <= LIMB_MAX, ("base only", R, start)
            # the fused reward: the partials of every 128-channel block, same bits as those of the larger call's rows
            rowpart = torch.full((nblk + 1, R), float("nan"), device="cuda")
            grp = essa.ForwardGroup([(gp, Xs, rs, sAd, sBd, Y16)], [to_dev(v)])
            assert essa.essa_svdlora_forward_reward_group(ctx, grp, None, rowpart) == nblk
            assert torch.equal(Y16, big16[sub])
            assert not torch.isnan(rowpart[:nblk]).any() and torch.isnan(rowpart[nblk]).all()
            yv = bf16_host(Y16)
            for b in range(nblk):
                want = yv[:, 128 * b:128 * (b + 1)] @ v[128 * b:128 * (b + 1)].astype(np.float64)
                np.testing.assert_allclose(rowpart[b].cpu().numpy(), want, rtol=2e-5, atol=1e-5 * np.abs(want).max())
    e_max, e_rms = orc.rel_errors(bf16_host(big16), orc.round_to_bf16(ref))
    assert e_rms <= BF16_RMS and e_max <= BF16_MAX
    gp.close()


@pytest.mark.parametrize("specs", [[(200, 16, 25), (96, 8, 25), (328, 32, 10), (64, 4, 32)],
                                   [(200, 16, 25), (96, 8, 25), (328, 32, 50), (64, 4, 64)]], ids=["one_row_block", "two_row_blocks"])
def test_forward_small_row_counts_grouped_mixed_rows(essa, ctx, specs):
    """A grouped call whose items ((d_out, rank, rows)) have different small row counts and ranks, q/k/v-like sharing of one
    X between two items: rows past an item's own count are never loaded, also when the group as a whole takes two row
    blocks per workgroup and an item fills only the first; each item alone gives the same bits."""
    d_in, K = 768, 6
    rows = sorted({R for _, _, R in specs})
    xs = {R: wl.make_x_bf16(R, d_in, x_id=70 + R) for R in rows}
    r2cs = {R: np.random.default_rng(R).integers(0, K, R).astype(np.int32) for R in rows}
    Xd = {R: bf16_dev(xs[R][0]) for R in xs}
    rd = {R: to_dev(r2cs[R]) for R in xs}
    items, refs, gps = [], [], []
    for pi, (d_out, r, R) in enumerate(specs):
        p = wl.make_projection("t", d_in, d_out, r, "int8", layer=19, proj=pi)
        W, f = oracle_proj(p)
        gp = gpu_proj(essa, ctx, p)
        sA, sB = candidate_sigmas(f, K, 0.05, pert_id=pi)
        items.append((gp, Xd[R], rd[R], to_dev(sA), to_dev(sB), torch.empty(R, d_out, device="cuda")))
        refs.append(orc.svdlora_forward(W, f, xs[R][1], r2cs[R], sA, sB))
        gps.append(gp)
    essa.essa_svdlora_forward_group(ctx, items)
    for it, ref in zip(items, refs):
        e_max, e_rms = orc.rel_errors(it[5].cpu().numpy(), ref)
        assert e_rms <= LIMB_RMS and e_max <= LIMB_MAX, (e_max, e_rms)
        Y1 = torch.empty_like(it[5])
        essa.essa_svdlora_forward(ctx, it[0], it[1], it[2], it[3], it[4], Y1)
        assert torch.equal(Y1, it[5])
    for gp in gps:
        gp.close()
