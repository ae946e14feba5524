"""Shared plumbing of the GPU parity tests: moving seeded inputs to the device and to the oracle."""
import numpy as np
import torch

import essa_workloads as wl
import oracle as orc


def to_dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def bf16_dev(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()


def bf16_host(t):
    """bf16 GPU tensor -> fp64 numpy (exact)."""
    return wl.bf16_bits_to_f32(t.cpu().view(torch.int16).numpy().view(np.uint16)).astype(np.float64)


def seeds_dev(seeds):
    return torch.from_numpy(np.asarray(seeds, dtype=np.uint32).view(np.int32).copy()).cuda()


def gpu_proj(essa, ctx, p: wl.Projection):
    quant = essa.QUANT_INT8_PERCH if p.quant == "int8" else essa.QUANT_INT4_G128
    return essa.Projection(ctx, p.Wq, p.scales, p.zeros, p.A, p.B, quant)


def oracle_proj(p: wl.Projection):
    """(W_deq fp64, SVD factors) of a projection, by the oracle's own routines."""
    W = orc.dequant_int8(p.Wq, p.scales) if p.quant == "int8" else orc.dequant_int4(p.Wq, p.scales, p.zeros)
    return W, orc.thin_svd_factors(p.A, p.B)


def candidate_sigmas(f, K, step, pert_id=0):
    """sigma_k = own spectrum + step * N(0,1), rounded to fp32 (what both sides are given)."""
    r = f["S_A"].shape[0]
    dA, dB = wl.sigma_perturbation(K, 1, r, step, pert_id)
    sA = (f["S_A"][None, :] + dA[:, 0, :]).astype(np.float32)
    sB = (f["S_B"][None, :] + dB[:, 0, :]).astype(np.float32)
    return sA, sB


def sample_rows(row2cand, cands, per_cand, seed=0):
    """first, last and a few pseudo-random rows of each listed candidate."""
    g = np.random.default_rng(seed)
    rows = []
    for k in cands:
        idx = np.nonzero(row2cand == k)[0]
        if idx.size == 0:
            continue
        pick = {int(idx[0]), int(idx[-1])}
        pick.update(int(x) for x in g.choice(idx, size=min(per_cand, idx.size), replace=False))
        rows.extend(sorted(pick))
    return np.array(rows, dtype=np.int64)
