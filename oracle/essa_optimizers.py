"""Plain fp64 CPU oracle of the other rank-based optimisers that run on the ESSA sampler.

TEST INFRASTRUCTURE ONLY (same rules as essa_oracle.py: no code shared with the HIP library, never
imported by it, never tuned for speed).

The paper's ablation "Alternative gradient-free optimizers" names plain isotropic (mu, lambda)-ES and ARS
beside CMA-ES, on the same SFT-seeded search space and the same per-step budget of candidate evaluations,
with step sizes tuned per optimiser; it defines none of them.  Its main text leaves the CMA-ES variant to a
library's defaults.  The readings taken here, each from the method's own publication:

* active CMA-ES: the (mu/mu_w, lambda)-CMA-ES of Hansen's tutorial (arXiv:1604.00772) with the negative
  recombination weights of its Table 1 / Eqs. (49)-(58) in the rank-mu term, rescaled per candidate as in
  Eq. (46)-(47) so that the covariance stays positive definite.
* separable CMA-ES: Ros & Hansen, "A simple modification in CMA-ES achieving linear time and space
  complexity" (PPSN 2008): only the diagonal of C is kept and updated, the two covariance learning rates are
  multiplied by (n + 2) / 3.
* plain isotropic (mu/mu_I, lambda)-ES (Beyer & Schwefel 2002, intermediate recombination, comma selection):
  C = I, a fixed step size, the new mean is the plain average of the mu = floor(lambda / 2) best candidates.
* ARS: Mania, Guy & Recht, "Simple random search of static linear policies is competitive for reinforcement
  learning" (NeurIPS 2018), Algorithm 1 in its V1-t form (there are no states to normalise here): antithetic
  pairs m +- nu z_j, the b directions with the largest max(r+, r-), the step divided by the standard deviation
  of the 2b rewards used.

Pins (tests/test_oracle_optimizers.py, CPU): hand-computed weights for lambda = 4; the mean / path / step-size
updates of the active variant against the pinned positive-weight update; neutral-selection stationarity of the
active rank-mu term (Monte Carlo); separable CMA against the full update on a diagonal state and n = 1
identity; (mu, lambda)-ES against the mu = 1 case of the pinned update and a brute-force average; ARS closed
form for one pair, invariance to shifting and scaling the rewards, antisymmetry.  Against the implementations
the paper ran (unnamed libraries) all four are PARITY UNPINNED.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

from .essa_oracle import CmaState, cma_constants, normals_from_seed, rank_desc_stable

__all__ = [
    "ActiveConstants", "active_cma_constants", "cma_update_active",
    "SepState", "sep_cma_init", "sep_cma_constants", "sep_cma_sample", "sep_cma_update",
    "es_sample", "es_update", "ars_sample", "ars_update",
]


# ----------------------------------------------------------------------------
# Active CMA-ES (Hansen's tutorial, Table 1 and Eqs. (46)-(47), (49)-(58))
# ----------------------------------------------------------------------------
@dataclass
class ActiveConstants:
    n: int
    lam: int
    mu: int
    weights: np.ndarray        # all lambda of them, best first; the first mu sum to one, the rest are <= 0
    mu_eff: float
    c_sigma: float
    d_sigma: float
    c_c: float
    c_1: float
    c_mu: float
    chi_n: float


def active_cma_constants(n: int, lam: int) -> ActiveConstants:
    """Default strategy parameters with negative weights.  c_sigma, d_sigma, c_c, c_1 and the positive weights
    are those of the positive-weight variant; c_mu carries the tutorial's extra 1/4 in its numerator (Eq. 58),
    and the negative weights are scaled to sum to -min(alpha_mu, alpha_mueff, alpha_posdef) (Eqs. 50-53)."""
    base = cma_constants(n, lam)
    mu = base.mu
    wp = np.array([math.log((lam + 1) / 2.0) - math.log(i) for i in range(1, lam + 1)], dtype=np.float64)
    pos, neg = wp[:mu], wp[mu:]
    mu_eff = float(pos.sum() ** 2 / np.sum(pos * pos))
    neg_sum = float(np.sum(np.abs(neg)))
    mu_eff_neg = float(neg.sum() ** 2 / np.sum(neg * neg)) if neg_sum > 0 else 0.0
    c_1 = base.c_1
    c_mu = min(1.0 - c_1, 2.0 * (0.25 + mu_eff + 1.0 / mu_eff - 2.0) / ((n + 2.0) ** 2 + mu_eff))
    alpha_mu = 1.0 + c_1 / c_mu
    alpha_mueff = 1.0 + 2.0 * mu_eff_neg / (mu_eff + 2.0)
    alpha_posdef = (1.0 - c_1 - c_mu) / (n * c_mu)
    w = np.empty(lam, dtype=np.float64)
    w[:mu] = pos / pos.sum()
    w[mu:] = (min(alpha_mu, alpha_mueff, alpha_posdef) / neg_sum) * neg if neg_sum > 0 else 0.0
    return ActiveConstants(n, lam, mu, w, mu_eff, base.c_sigma, base.d_sigma, base.c_c, c_1, c_mu, base.chi_n)


def cma_update_active(st: CmaState, seeds, rewards) -> tuple[CmaState, np.ndarray]:
    """One generation with negative weights in the rank-mu term.  Mean, both paths and the step size use the
    mu best candidates only.  A candidate with a negative weight enters the covariance with
    w * n / ||C^{-1/2} y||^2, and C^{-1/2} y = B D^{-1} B^T (B D z) = B z has the length of z."""
    lam = len(seeds)
    c = active_cma_constants(st.n, lam)
    order = rank_desc_stable(rewards)
    Z = np.stack([normals_from_seed(int(s), st.n) for s in seeds]).astype(np.float64)
    Y = (st.B @ (st.D[:, None] * Z.T)).T
    Zs, Ys = Z[order], Y[order]                              # best first
    wpos = c.weights[:c.mu]
    z_w = wpos @ Zs[:c.mu]
    y_w = wpos @ Ys[:c.mu]
    m = st.m + st.sigma * y_w
    p_sigma = (1.0 - c.c_sigma) * st.p_sigma + math.sqrt(c.c_sigma * (2.0 - c.c_sigma) * c.mu_eff) * (st.B @ z_w)
    ps_norm = float(np.linalg.norm(p_sigma))
    h_sigma = 1.0 if ps_norm / math.sqrt(1.0 - (1.0 - c.c_sigma) ** (2 * (st.t + 1))) < (1.4 + 2.0 / (st.n + 1.0)) * c.chi_n else 0.0
    p_c = (1.0 - c.c_c) * st.p_c + h_sigma * math.sqrt(c.c_c * (2.0 - c.c_c) * c.mu_eff) * y_w
    w_eff = c.weights.copy()
    for i in range(c.mu, lam):
        w_eff[i] = c.weights[i] * st.n / float(Zs[i] @ Zs[i])
    rank_mu = (Ys.T * w_eff[None, :]) @ Ys
    decay = 1.0 - c.c_1 - c.c_mu * float(c.weights.sum()) + (1.0 - h_sigma) * c.c_1 * c.c_c * (2.0 - c.c_c)
    C = decay * st.C + c.c_1 * np.outer(p_c, p_c) + c.c_mu * rank_mu
    sigma = st.sigma * math.exp((c.c_sigma / c.d_sigma) * (ps_norm / c.chi_n - 1.0))
    new = CmaState(n=st.n, t=st.t + 1, sigma=sigma, m=m, p_sigma=p_sigma, p_c=p_c, C=C, B=st.B, D=st.D,
                   extra=dict(h_sigma=h_sigma, ps_norm=ps_norm, decay=decay, rank_mu=rank_mu))
    return new, order


# ----------------------------------------------------------------------------
# Separable CMA-ES (Ros & Hansen 2008)
# ----------------------------------------------------------------------------
@dataclass
class SepState:
    n: int
    t: int
    sigma: float
    m: np.ndarray
    p_sigma: np.ndarray
    p_c: np.ndarray
    c_diag: np.ndarray         # diagonal of C
    extra: dict = field(default_factory=dict)


def sep_cma_init(n: int, sigma0: float, m0=None) -> SepState:
    return SepState(n=n, t=0, sigma=float(sigma0), m=np.zeros(n) if m0 is None else np.asarray(m0, np.float64).copy(),
                    p_sigma=np.zeros(n), p_c=np.zeros(n), c_diag=np.ones(n))


def sep_cma_constants(n: int, lam: int):
    """The positive-weight defaults with both covariance learning rates times (n + 2) / 3, kept inside
    c_1 <= 1 and c_1 + c_mu <= 1."""
    c = cma_constants(n, lam)
    f = (n + 2.0) / 3.0
    c_1 = min(1.0, c.c_1 * f)
    c_mu = min(1.0 - c_1, c.c_mu * f)
    return c, c_1, c_mu


def sep_cma_sample(st: SepState, seeds):
    """theta_k = m + sigma * sqrt(c_diag) * z_k."""
    Z = np.stack([normals_from_seed(int(s), st.n) for s in seeds]) if len(seeds) else np.zeros((0, st.n), np.float32)
    d = np.sqrt(st.c_diag)
    return st.m[None, :] + st.sigma * d[None, :] * Z.astype(np.float64), Z


def sep_cma_update(st: SepState, seeds, rewards) -> tuple[SepState, np.ndarray]:
    lam = len(seeds)
    c, c_1, c_mu = sep_cma_constants(st.n, lam)
    order = rank_desc_stable(rewards)
    Z = np.stack([normals_from_seed(int(s), st.n) for s in seeds]).astype(np.float64)
    d = np.sqrt(st.c_diag)
    Y = d[None, :] * Z
    sel = order[:c.mu]
    z_w = c.weights @ Z[sel]
    y_w = c.weights @ Y[sel]
    m = st.m + st.sigma * y_w
    p_sigma = (1.0 - c.c_sigma) * st.p_sigma + math.sqrt(c.c_sigma * (2.0 - c.c_sigma) * c.mu_eff) * z_w
    ps_norm = float(np.linalg.norm(p_sigma))
    h_sigma = 1.0 if ps_norm / math.sqrt(1.0 - (1.0 - c.c_sigma) ** (2 * (st.t + 1))) < (1.4 + 2.0 / (st.n + 1.0)) * c.chi_n else 0.0
    p_c = (1.0 - c.c_c) * st.p_c + h_sigma * math.sqrt(c.c_c * (2.0 - c.c_c) * c.mu_eff) * y_w
    c_diag = (1.0 - c_1 - c_mu + (1.0 - h_sigma) * c_1 * c.c_c * (2.0 - c.c_c)) * st.c_diag \
        + c_1 * p_c * p_c + c_mu * (c.weights @ (Y[sel] * Y[sel]))
    sigma = st.sigma * math.exp((c.c_sigma / c.d_sigma) * (ps_norm / c.chi_n - 1.0))
    new = SepState(n=st.n, t=st.t + 1, sigma=sigma, m=m, p_sigma=p_sigma, p_c=p_c, c_diag=c_diag,
                   extra=dict(h_sigma=h_sigma, ps_norm=ps_norm))
    return new, order


# ----------------------------------------------------------------------------
# Plain isotropic (mu/mu_I, lambda)-ES
# ----------------------------------------------------------------------------
def es_sample(m, sigma, seeds):
    """theta_k = m + sigma z_k."""
    m = np.asarray(m, np.float64)
    Z = np.stack([normals_from_seed(int(s), m.shape[0]) for s in seeds]) if len(seeds) else np.zeros((0, m.shape[0]), np.float32)
    return m[None, :] + float(sigma) * Z.astype(np.float64), Z


def es_update(m, sigma, seeds, rewards):
    """New mean = average of the mu = floor(lambda / 2) best candidates; sigma does not change."""
    m = np.asarray(m, np.float64)
    lam = len(seeds)
    mu = lam // 2
    order = rank_desc_stable(rewards)
    theta, _ = es_sample(m, sigma, seeds)
    return theta[order[:mu]].mean(axis=0), order


# ----------------------------------------------------------------------------
# ARS (Mania, Guy & Recht 2018, Algorithm 1, V1-t)
# ----------------------------------------------------------------------------
def ars_sample(m, nu, seeds):
    """2N candidates from N seeds: theta_{2j} = m + nu z_j, theta_{2j+1} = m - nu z_j."""
    m = np.asarray(m, np.float64)
    n = m.shape[0]
    theta = np.empty((2 * len(seeds), n), dtype=np.float64)
    Z = np.empty((len(seeds), n), dtype=np.float32)
    for j, s in enumerate(seeds):
        Z[j] = normals_from_seed(int(s), n)
        theta[2 * j] = m + float(nu) * Z[j].astype(np.float64)
        theta[2 * j + 1] = m - float(nu) * Z[j].astype(np.float64)
    return theta, Z


def ars_update(m, seeds, rewards, alpha: float, b: int):
    """m + alpha / (b s_R) sum over the b best directions of (r+ - r-) z, directions ordered by max(r+, r-)
    (larger first, ties by index, NaN as -inf), s_R the standard deviation (divisor 2b) of the 2b rewards of
    those directions.  s_R = 0 (all of them equal) leaves the mean where it is.  Returns (m_new, direction order)."""
    m = np.asarray(m, np.float64)
    r = np.asarray(rewards, dtype=np.float32).astype(np.float64)
    N = len(seeds)
    if r.shape[0] != 2 * N or not (1 <= b <= N):
        raise ValueError("rewards must hold one pair per seed and 1 <= b <= N")
    r = np.where(np.isnan(r), -np.inf, r)
    key = np.maximum(r[0::2], r[1::2])
    order = rank_desc_stable(key.astype(np.float32))
    top = order[:b]
    used = np.concatenate([r[2 * top], r[2 * top + 1]])
    if not np.all(np.isfinite(used)):
        return m.copy(), order
    s_R = float(np.sqrt(np.mean((used - used.mean()) ** 2)))
    if s_R == 0.0:
        return m.copy(), order
    step = np.zeros_like(m)
    for j in top:
        step += (r[2 * j] - r[2 * j + 1]) * normals_from_seed(int(seeds[j]), m.shape[0]).astype(np.float64)
    return m + (float(alpha) / (b * s_R)) * step, order
