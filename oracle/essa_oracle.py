"""Plain, slow, fp64 CPU oracle of the ESSA hot path (arXiv 2507.04453).

TEST INFRASTRUCTURE ONLY: only tests/, __graft_entry__.smoke() and bench.py's
cpu_baseline leg may import it.  It shares no code with the HIP library, does
not import it, and is never tuned for speed.

What the paper fixes and what is a reading of it
------------------------------------------------
* Method section, "LoRA + SVD parameterization": every attention matrix W0
  (m x n) carries a LoRA update dW = B A, B (m x r), A (r x n).  Each factor is
  SVD-decomposed, A = U_A S_A V_A^T and B = U_B S_B V_B^T, the bases are frozen
  and only (a top-alpha fraction of) the singular values move.
* Algorithm 1, candidate-reconstruction step: a candidate rebuilds
  A' = U_A diag(s_A + d_A) V_A^T, B' likewise, and uses W' = W + B' A'.
  `candidate_weight` / `svdlora_forward` are that definition written out: the
  dense W' is formed per candidate in fp64 and applied to that candidate's rows.
* Method section, "Evolutionary optimization": the search vector theta holds
  the singular-value offsets; CMA-ES draws a population from N(m, s^2 C),
  workers regenerate any member from a seed, and (m, s, C) is updated from the
  reward ranking (Algorithm 1, last two steps of the loop).

The paper does not say which random generator, which seed-to-normal map, which
CMA-ES variant or which quantised formats are used.  The readings taken here:
Philox4x32-10 (Salmon et al., SC'11) keyed by the 32-bit seed, Box-Muller on
24-bit uniforms, the (mu/mu_w, lambda)-CMA-ES of Hansen's tutorial
(arXiv:1604.00772) with its default constants and positive weights, int8
symmetric per-output-channel weights and int4 asymmetric group-128 weights.

Pins (tests/test_oracle_*.py, all CPU): Philox known-answer blocks of the
published algorithm; moment / range checks of the normals; closed-form CMA-ES
constants; forward invariants (own singular values give W + B A from the
unfactored factors, zero singular values give the base layer, brute-force
dense products on tiny shapes, linearity, row permutation); CMA-ES invariants
and convergence on sphere / ellipsoid; the stalled step (h_sigma = 0) against a closed form
(with C = p_c p_c^T the update is (1 - c_mu) C + c_mu sum w_i y_i y_i^T) and the threshold that
decides it; the W8A8 composition against a hand-worked 2 x 3 case and within its quantisation bound
of the fp64 forward; the eigendecomposition against closed forms (2 x 2, diagonal,
known spectrum) and its defining identities.  The exact CMA-ES variant the paper ran
(an external library's defaults) cannot be checked here: against that library
the update is PARITY UNPINNED; it is pinned to the tutorial's equations only.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

__all__ = [
    "philox4x32_10", "philox_words_for_seed", "normals_from_seed", "uniform24",
    "sample_candidates", "sigma_map_dim", "theta_to_sigma",
    "dequant_int8", "dequant_int4", "pack_int4", "unpack_int4",
    "thin_svd_factors", "candidate_weight", "svdlora_forward", "svdlora_forward_rows",
    "quantize_rows_int8", "int8_accumulators", "svdlora_forward_w8a8",
    "round_to_bf16", "reward_accumulate", "rank_desc_stable",
    "CmaConstants", "cma_constants", "CmaState", "cma_state_init", "cma_update", "cma_refresh_basis",
    "rel_errors",
]

# ----------------------------------------------------------------------------
# Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
# as 1, 2, 3", SC'11).  Reading of "workers share a random-number stream and
# regenerate a population member from a seed" (Method, Evolutionary optimization).
# ----------------------------------------------------------------------------
_PHILOX_M0 = np.uint64(0xD2511F53)
_PHILOX_M1 = np.uint64(0xCD9E8D57)
_PHILOX_W0 = 0x9E3779B9
_PHILOX_W1 = 0xBB67AE85
_MASK32 = np.uint64(0xFFFFFFFF)


def philox4x32_10(counter, key):
    """Ten Philox rounds.  counter: (..., 4) uint32, key: (..., 2) uint32 -> (..., 4) uint32."""
    c = np.asarray(counter, dtype=np.uint64) & _MASK32
    k = np.asarray(key, dtype=np.uint64) & _MASK32
    c0, c1, c2, c3 = (c[..., i].copy() for i in range(4))
    k0, k1 = k[..., 0].copy(), k[..., 1].copy()
    for rnd in range(10):
        if rnd > 0:
            k0 = (k0 + np.uint64(_PHILOX_W0)) & _MASK32
            k1 = (k1 + np.uint64(_PHILOX_W1)) & _MASK32
        p0 = _PHILOX_M0 * c0          # 32x32 -> 64 bit product, fits uint64
        p1 = _PHILOX_M1 * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & _MASK32
        hi1, lo1 = p1 >> np.uint64(32), p1 & _MASK32
        c0, c1, c2, c3 = (hi1 ^ c1 ^ k0), lo1, (hi0 ^ c3 ^ k1), lo0
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def philox_words_for_seed(seed: int, n_blocks: int) -> np.ndarray:
    """Blocks 0..n_blocks-1 of the stream of one candidate: key (seed, 0), counter (c, 0, 0, 0)."""
    ctr = np.zeros((n_blocks, 4), dtype=np.uint32)
    ctr[:, 0] = np.arange(n_blocks, dtype=np.uint32)
    key = np.zeros((n_blocks, 2), dtype=np.uint32)
    key[:, 0] = np.uint32(seed & 0xFFFFFFFF)
    return philox4x32_10(ctr, key)


def uniform24(w: np.ndarray) -> np.ndarray:
    """32-bit word -> uniform in (0,1): ((w >> 8) + 0.5) * 2^-24, exact in fp64."""
    return ((np.asarray(w, dtype=np.uint32) >> np.uint32(8)).astype(np.float64) + 0.5) * (2.0 ** -24)


def normals_from_seed(seed: int, n: int) -> np.ndarray:
    """z[4c + l], l = 0..3, from block c: (w0,w1)->(z0,z1), (w2,w3)->(z2,z3) by Box-Muller.

    rho = sqrt(-2 ln u_a), z_a = rho cos(2 pi u_b), z_b = rho sin(2 pi u_b); evaluated in
    fp64, rounded once to fp32.  A surplus beyond n is discarded.
    """
    nb = (n + 3) // 4
    w = philox_words_for_seed(seed, nb)
    u = uniform24(w)
    z = np.empty((nb, 4), dtype=np.float64)
    for a, b in ((0, 1), (2, 3)):
        rho = np.sqrt(-2.0 * np.log(u[:, a]))
        ang = 2.0 * np.pi * u[:, b]
        z[:, a] = rho * np.cos(ang)
        z[:, b] = rho * np.sin(ang)
    return z.reshape(-1)[:n].astype(np.float32)


def sample_candidates(m, sigma, B, D, seeds):
    """theta_k = m + sigma * B (D * z_k), z_k from seed k  (population drawn from N(m, sigma^2 C),
    C = B D^2 B^T; Method, Evolutionary optimization).  Returns (Theta[K,n] fp64, Z[K,n] fp32)."""
    m = np.asarray(m, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    D = np.asarray(D, dtype=np.float64)
    n = m.shape[0]
    Z = np.stack([normals_from_seed(int(s), n) for s in seeds]) if len(seeds) else np.zeros((0, n), np.float32)
    theta = np.empty((len(seeds), n), dtype=np.float64)
    for k in range(len(seeds)):
        theta[k] = m + float(sigma) * (B @ (D * Z[k].astype(np.float64)))
    return theta, Z


# ----------------------------------------------------------------------------
# theta <-> singular values (Algorithm 1, SVD-init step and reconstruction step;
# Figure 1: one contiguous slice of theta per LoRA matrix).
# ----------------------------------------------------------------------------
def sigma_map_dim(P: int, r: int, alpha: float) -> int:
    """Search dimension: P adapted matrices x 2 factors x floor(alpha r) exposed values."""
    ka = int(math.floor(alpha * r + 1e-9))
    return P * 2 * ka


def theta_to_sigma(theta, sigma_sft_A, sigma_sft_B, alpha: float = 1.0):
    """sA[k,p,j] = sft_A[p,j] + theta[k, p*2ka + j] for j < ka = floor(alpha r), unchanged beyond;
    sB[k,p,j] = sft_B[p,j] + theta[k, p*2ka + ka + j].  Order inside theta: projection-major
    (layer, then q,k,v,o), factor A before factor B, singular values in descending order."""
    theta = np.asarray(theta, dtype=np.float64)
    sA0 = np.asarray(sigma_sft_A, dtype=np.float64)
    sB0 = np.asarray(sigma_sft_B, dtype=np.float64)
    P, r = sA0.shape
    ka = int(math.floor(alpha * r + 1e-9))
    if ka <= 0:
        raise ValueError("floor(alpha*r) = 0: no trainable singular value")
    K = theta.shape[0]
    if theta.shape[1] != P * 2 * ka:
        raise ValueError("theta has the wrong width")
    sA = np.broadcast_to(sA0, (K, P, r)).copy()
    sB = np.broadcast_to(sB0, (K, P, r)).copy()
    for p in range(P):
        base = p * 2 * ka
        sA[:, p, :ka] += theta[:, base:base + ka]
        sB[:, p, :ka] += theta[:, base + ka:base + 2 * ka]
    return sA, sB


# ----------------------------------------------------------------------------
# Quantised base weights.  The paper only says INT8 / INT4 (Introduction; precision
# study); formats are this build's reading.
# ----------------------------------------------------------------------------
def dequant_int8(q, scale):
    """W[o,j] = scale[o] * q[o,j]; q int8, scale fp32 per output channel."""
    return np.asarray(scale, dtype=np.float32).astype(np.float64)[:, None] * np.asarray(q, dtype=np.int8).astype(np.float64)


def pack_int4(q):
    """q[o,j] in 0..15 -> bytes [o, j/2], low nibble = even j."""
    q = np.asarray(q, dtype=np.uint8)
    assert q.shape[1] % 2 == 0 and q.max(initial=0) <= 15
    return (q[:, 0::2] | (q[:, 1::2] << 4)).astype(np.uint8)


def unpack_int4(packed):
    p = np.asarray(packed, dtype=np.uint8)
    q = np.empty((p.shape[0], p.shape[1] * 2), dtype=np.uint8)
    q[:, 0::2] = p & 0xF
    q[:, 1::2] = p >> 4
    return q


def dequant_int4(packed, scale_f16, zero_f16, group: int = 128):
    """W[o,j] = s[o,g] (q[o,j] - z[o,g]), g = j // group; s, z stored as fp16."""
    q = unpack_int4(packed).astype(np.float64)
    s = np.asarray(scale_f16, dtype=np.float16).astype(np.float64)
    z = np.asarray(zero_f16, dtype=np.float16).astype(np.float64)
    return np.repeat(s, group, axis=1) * (q - np.repeat(z, group, axis=1))


# ----------------------------------------------------------------------------
# SVD-parameterised LoRA forward (Method, LoRA + SVD parameterization; Algorithm 1,
# reconstruction step).
# ----------------------------------------------------------------------------
def thin_svd_factors(A, B):
    """Thin SVDs A = U_A S_A V_A^T (r x d_in) and B = U_B S_B V_B^T (d_out x r), fp64,
    singular values descending.  Returns dict with U_A[r,r], S_A[r], V_A[d_in,r], U_B[d_out,r],
    S_B[r], V_B[r,r]."""
    A = np.asarray(A, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    UA, SA, VAt = np.linalg.svd(A, full_matrices=False)
    UB, SB, VBt = np.linalg.svd(B, full_matrices=False)
    return dict(U_A=UA, S_A=SA, V_A=VAt.T.copy(), U_B=UB, S_B=SB, V_B=VBt.T.copy())


def candidate_weight(W_deq, f, sA_k, sB_k):
    """W' = W + (U_B diag(sB) V_B^T)(U_A diag(sA) V_A^T), dense fp64."""
    A_k = (f["U_A"] * np.asarray(sA_k, np.float64)[None, :]) @ f["V_A"].T
    B_k = (f["U_B"] * np.asarray(sB_k, np.float64)[None, :]) @ f["V_B"].T
    return np.asarray(W_deq, np.float64) + B_k @ A_k


def svdlora_forward(W_deq, f, X, row2cand, sA, sB, lora_only=False, base_only=False):
    """y_i = W'_{row2cand[i]} x_i with fp64 accumulation.  X[R,d_in], sA/sB [K,r] -> Y[R,d_out] fp64."""
    X = np.asarray(X, dtype=np.float64)
    row2cand = np.asarray(row2cand)
    W_deq = np.asarray(W_deq, np.float64)
    Y = np.zeros((X.shape[0], W_deq.shape[0]), dtype=np.float64)
    for k in np.unique(row2cand):
        rows = np.nonzero(row2cand == k)[0]
        if base_only:
            Wk = W_deq
        else:
            Wk = candidate_weight(W_deq, f, sA[k], sB[k])
            if lora_only:
                Wk = Wk - W_deq
        Y[rows] = X[rows] @ Wk.T
    return Y


def svdlora_forward_rows(W_deq, f, X, row2cand, sA, sB, rows):
    """The same definition evaluated only on the listed rows (full-size sampled parity)."""
    rows = np.asarray(rows)
    return svdlora_forward(W_deq, f, np.asarray(X)[rows], np.asarray(row2cand)[rows], sA, sB)


def quantize_rows_int8(X):
    """Per-row dynamic int8 activation quantisation, decided in fp32 (the kernel's precision):
    amax = max|x|, inv = 127/amax, q = rint(x*inv) (ties to even), scale = amax/127."""
    X = np.asarray(X, dtype=np.float32)
    amax = np.max(np.abs(X), axis=1).astype(np.float32)
    safe = np.where(amax > 0, amax, np.float32(1.0)).astype(np.float32)
    inv = (np.float32(127.0) / safe).astype(np.float32)
    q = np.rint((X * inv[:, None]).astype(np.float32))
    q = np.clip(q, -127, 127).astype(np.int8)
    scale = np.where(amax > 0, (amax / np.float32(127.0)).astype(np.float32), np.float32(0.0)).astype(np.float32)
    q[amax == 0] = 0
    return q, scale


def int8_accumulators(Xq, Wq):
    """acc[i,o] = sum_j Xq[i,j] Wq[o,j] in exact integer arithmetic (int64)."""
    return np.asarray(Xq, np.int64) @ np.asarray(Wq, np.int64).T


def svdlora_forward_w8a8(Wq, w_scale, f, X, row2cand, sA, sB):
    """W8A8 mode: base term on the quantised activations, LoRA term on the unquantised ones:
    y_i = s_i * w_scale * (Wq . xq_i) + B_k A_k x_i."""
    Xq, xs = quantize_rows_int8(X)
    acc = int8_accumulators(Xq, Wq).astype(np.float64)
    base = acc * xs.astype(np.float64)[:, None] * np.asarray(w_scale, np.float32).astype(np.float64)[None, :]
    zeroW = np.zeros((np.asarray(Wq).shape[0], np.asarray(Wq).shape[1]))
    return base + svdlora_forward(zeroW, f, X, row2cand, sA, sB)


def round_to_bf16(x):
    """Round fp64 to the nearest bfloat16 value (8-bit significand, ties to even), returned as fp64."""
    x = np.asarray(x, dtype=np.float64)
    mant, exp = np.frexp(x)                       # x = mant * 2^exp, 0.5 <= |mant| < 1
    return np.ldexp(np.rint(mant * 256.0), exp - 8)


def reward_accumulate(F, Y, v, row2cand, K):
    """Synthetic reward: F[k] += < mean of the rows of Y owned by candidate k , v >.
    A candidate without rows gets NaN (0/0)."""
    Y = np.asarray(Y, np.float64)
    v = np.asarray(v, np.float64)
    row2cand = np.asarray(row2cand)
    d = Y @ v
    out = np.array(F, dtype=np.float64, copy=True)
    for k in range(K):
        rows = row2cand == k
        cnt = int(rows.sum())
        out[k] += (d[rows].sum() / cnt) if cnt else float("nan")
    return out


# ----------------------------------------------------------------------------
# Ranking and the CMA-ES update (Algorithm 1: each worker performs the same update).
# ----------------------------------------------------------------------------
def rank_desc_stable(F):
    """order[i] = index of the i-th best candidate; larger reward first, equal rewards keep
    ascending candidate index, NaN counts as -inf."""
    F = np.asarray(F, dtype=np.float32).astype(np.float64)
    key = np.where(np.isnan(F), -np.inf, F)
    K = key.shape[0]
    order = np.empty(K, dtype=np.int32)
    for i in range(K):
        better = int(np.sum(key > key[i]) + np.sum((key == key[i]) & (np.arange(K) < i)))
        order[better] = i
    return order


@dataclass
class CmaConstants:
    n: int
    lam: int
    mu: int
    weights: np.ndarray
    mu_eff: float
    c_sigma: float
    d_sigma: float
    c_c: float
    c_1: float
    c_mu: float
    chi_n: float


def cma_constants(n: int, lam: int) -> CmaConstants:
    """Default strategy parameters of the (mu/mu_w, lambda)-CMA-ES, positive weights only."""
    mu = lam // 2
    w = np.array([math.log((lam + 1) / 2.0) - math.log(i) for i in range(1, mu + 1)], dtype=np.float64)
    w = w / w.sum()
    mu_eff = 1.0 / float(np.sum(w * w))
    c_sigma = (mu_eff + 2.0) / (n + mu_eff + 5.0)
    d_sigma = 1.0 + 2.0 * max(0.0, math.sqrt((mu_eff - 1.0) / (n + 1.0)) - 1.0) + c_sigma
    c_c = (4.0 + mu_eff / n) / (n + 4.0 + 2.0 * mu_eff / n)
    c_1 = 2.0 / ((n + 1.3) ** 2 + mu_eff)
    c_mu = min(1.0 - c_1, 2.0 * (mu_eff - 2.0 + 1.0 / mu_eff) / ((n + 2.0) ** 2 + mu_eff))
    chi_n = math.sqrt(n) * (1.0 - 1.0 / (4.0 * n) + 1.0 / (21.0 * n * n))
    return CmaConstants(n, lam, mu, w, mu_eff, c_sigma, d_sigma, c_c, c_1, c_mu, chi_n)


@dataclass
class CmaState:
    n: int
    t: int
    sigma: float
    m: np.ndarray
    p_sigma: np.ndarray
    p_c: np.ndarray
    C: np.ndarray
    B: np.ndarray
    D: np.ndarray
    extra: dict = field(default_factory=dict)


def cma_state_init(n: int, sigma0: float, m0=None) -> CmaState:
    return CmaState(n=n, t=0, sigma=float(sigma0),
                    m=np.zeros(n) if m0 is None else np.asarray(m0, np.float64).copy(),
                    p_sigma=np.zeros(n), p_c=np.zeros(n), C=np.eye(n), B=np.eye(n), D=np.ones(n))


def cma_update(st: CmaState, seeds, rewards) -> tuple[CmaState, np.ndarray]:
    """One generation of the update, from seeds and scalar rewards only.  B, D are not refreshed."""
    lam = len(seeds)
    c = cma_constants(st.n, lam)
    order = rank_desc_stable(rewards)
    Z = np.stack([normals_from_seed(int(s), st.n) for s in seeds]).astype(np.float64)
    Y = (st.B @ (st.D[:, None] * Z.T)).T                     # y_k = B D z_k
    sel = order[:c.mu]
    z_w = c.weights @ Z[sel]
    y_w = c.weights @ Y[sel]
    m = st.m + st.sigma * y_w
    p_sigma = (1.0 - c.c_sigma) * st.p_sigma + math.sqrt(c.c_sigma * (2.0 - c.c_sigma) * c.mu_eff) * (st.B @ z_w)
    ps_norm = float(np.linalg.norm(p_sigma))
    h_sigma = 1.0 if ps_norm / math.sqrt(1.0 - (1.0 - c.c_sigma) ** (2 * (st.t + 1))) < (1.4 + 2.0 / (st.n + 1.0)) * c.chi_n else 0.0
    p_c = (1.0 - c.c_c) * st.p_c + h_sigma * math.sqrt(c.c_c * (2.0 - c.c_c) * c.mu_eff) * y_w
    rank_mu = (Y[sel].T * c.weights[None, :]) @ Y[sel]
    C = (1.0 - c.c_1 - c.c_mu + (1.0 - h_sigma) * c.c_1 * c.c_c * (2.0 - c.c_c)) * st.C \
        + c.c_1 * np.outer(p_c, p_c) + c.c_mu * rank_mu
    sigma = st.sigma * math.exp((c.c_sigma / c.d_sigma) * (ps_norm / c.chi_n - 1.0))
    new = CmaState(n=st.n, t=st.t + 1, sigma=sigma, m=m, p_sigma=p_sigma, p_c=p_c, C=C, B=st.B, D=st.D,
                   extra=dict(h_sigma=h_sigma, ps_norm=ps_norm, z_w=z_w, y_w=y_w))
    return new, order


def cma_refresh_basis(C):
    """Eigendecomposition of the covariance, C = B diag(D^2) B^T (the decomposition step of the (mu/mu_w,
    lambda)-CMA-ES in Hansen's tutorial, arXiv:1604.00772, Sec. B.2 "C -> B D^2 B^T"; Algorithm 1 of the paper keeps
    (m, sigma, C) and samples through this factorisation).  C is symmetrised first, as the tutorial does; eigenvalues
    below zero (round-off of a positive semi-definite matrix) are clamped to zero.  Returns (B, D) with the
    eigenvalues ascending; the columns of B are orthonormal eigenvectors, each defined up to sign (and up to a
    rotation inside an eigenspace of repeated eigenvalues)."""
    C = np.asarray(C, dtype=np.float64)
    if C.ndim != 2 or C.shape[0] != C.shape[1]:
        raise ValueError("C must be square")
    lam, B = np.linalg.eigh((C + C.T) / 2.0)
    return B, np.sqrt(np.maximum(lam, 0.0))


def rel_errors(y, ref):
    """(max|y-ref| / max|ref|, ||y-ref||_2 / ||ref||_2) over the whole tensor."""
    y = np.asarray(y, np.float64)
    ref = np.asarray(ref, np.float64)
    den_max = float(np.max(np.abs(ref))) if ref.size else 0.0
    den_rms = float(np.linalg.norm(ref))
    d = y - ref
    e_max = float(np.max(np.abs(d))) if d.size else 0.0
    e_rms = float(np.linalg.norm(d))
    return (e_max / den_max if den_max > 0 else e_max, e_rms / den_rms if den_rms > 0 else e_rms)
