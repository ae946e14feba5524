// Eigendecomposition of the search covariance on the device: C = B diag(D^2) B^T
// (decomposition step of the (mu/mu_w, lambda)-CMA-ES, Hansen's tutorial arXiv:1604.00772 Sec. B.2; the paper's
// Algorithm 1 keeps (m, sigma, C) and samples through this factorisation).
//
// Method: one-sided block Jacobi in fp64.  A = C V is kept column by column (At[c][:] = column c of A), V starts as the
// identity.  Columns are grouped in blocks of 32; a sweep visits every pair of blocks once (round-robin tournament,
// nblk/2 disjoint pairs per round, nblk-1 rounds).  For a pair the 64 x 64 Gram matrix G = P^T P of its 64-column
// panel P is formed, diagonalised by a small two-sided Jacobi solver in LDS (G -> Q^T G Q), and the panel of A and of
// V is multiplied by Q.  When all columns of A are orthogonal, they are lambda_c v_c: V holds the eigenvectors and
// lambda_c = v_c^T a_c.  Every sum runs in a fixed order, so the result is the same bits on every run.
#include "essa_internal.h"
#include <cstring>

namespace {

constexpr int EB = 32;             // columns per block
constexpr int EP = 2 * EB;         // columns per panel
constexpr int ER = 64;             // rows per LDS chunk
constexpr int EPITCH = ER + 1;     // LDS pitch (doubles)
typedef __attribute__((ext_vector_type(4))) double f64x4;

// round-robin tournament over nblk players (nblk even): the p-th pair of round `round`
__device__ __forceinline__ void pair_of(int nblk, int round, int p, int& I, int& J) {
    const int m = nblk - 1;
    if (p == 0) { I = m; J = round % m; }
    else { I = (round + p) % m; J = (round - p + m) % m; }
    if (I > J) { const int t = I; I = J; J = t; }
}

__device__ __forceinline__ int panel_col(int I, int J, int c) { return c < EB ? I * EB + c : J * EB + (c - EB); }

// 1 / sqrt(x) for a normal x: the hardware's estimate and two Newton steps y <- y (3/2 - x/2 y^2)
__device__ __forceinline__ double rsqrt_newton(double x) {
    double y = __builtin_amdgcn_rsq(x);
    const double hx = 0.5 * x;
    y = y * fma(-hx * y, y, 1.5);
    y = y * fma(-hx * y, y, 1.5);
    return y;
}

// Cs[c][r] = (C[c][r] + C[r][c]) / 2 in fp64, zero beyond n; on a cold start also Vt = identity
__global__ __launch_bounds__(256) void eig_init_kernel(const float* __restrict__ C, int n, int ld, double* __restrict__ Cs, double* __restrict__ Vt,
                                                      int cold) {
    const int c = blockIdx.x;
    for (int r = threadIdx.x; r < ld; r += 256) {
        double a = 0.0;
        if (c < n && r < n) a = 0.5 * ((double)C[(size_t)c * n + r] + (double)C[(size_t)r * n + c]);
        Cs[(size_t)c * ld + r] = a;
        if (cold) Vt[(size_t)c * ld + r] = (r == c) ? 1.0 : 0.0;
    }
}

// At = Vt * Cs (row c of At = column c of A = C V; C symmetric): 64 x 64 output tiles, K chunks of 16
__global__ __launch_bounds__(256) void eig_matmul_kernel(const double* __restrict__ Vt, const double* __restrict__ Cs, int ld, double* __restrict__ At) {
    __shared__ double Va[64][17], Cb[16][65];
    const int c0 = blockIdx.y * 64, r0 = blockIdx.x * 64, tid = threadIdx.x;
    const int tc = tid >> 4, tr = tid & 15;
    double acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;
    for (int k0 = 0; k0 < ld; k0 += 16) {
        for (int idx = tid; idx < 64 * 16; idx += 256) {
            Va[idx >> 4][idx & 15] = Vt[(size_t)(c0 + (idx >> 4)) * ld + k0 + (idx & 15)];
            Cb[idx >> 6][idx & 63] = Cs[(size_t)(k0 + (idx >> 6)) * ld + r0 + (idx & 63)];
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            double a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = Va[4 * tc + i][k]; b[i] = Cb[k][4 * tr + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fma(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) At[(size_t)(c0 + 4 * tc + i) * ld + r0 + 4 * tr + j] = acc[i][j];
}

// Gram matrix of a panel over one slice of the rows: Gpart[pair][slice][a][b] = sum_r P[r][a] P[r][b]
__global__ __launch_bounds__(256) void eig_gram_kernel(const double* __restrict__ At, int ld, int n, int nblk, int round, int chunks_per_slice,
                                                      double* __restrict__ Gpart) {
    __shared__ double T[EP][EPITCH];
    const int pair = blockIdx.x, slice = blockIdx.y, S = gridDim.y, tid = threadIdx.x;
    int I, J;
    pair_of(nblk, round, pair, I, J);
    // fp64 MFMA 16x16x4: wave w owns rows 16w .. 16w+15 of G (all four 16-column blocks).  Operand element (i, k) and (k, j)
    // sit in lane i + 16 k resp. j + 16 k; with A[i][k] = P[r0 + k][16w + i] and B[k][j] = P[r0 + k][16jb + j] both operands
    // are T[column][row] read at [16 x + lane % 16][rr + lane / 16].  Accumulator element v of a lane is G[16w + 4 v +
    // lane / 16][16jb + lane % 16] (the fp64 form's own order: not that of the fp32 16x16x4).  (The vector and the matrix unit have the same fp64 rate on this chip; the MFMA needs a sixth of
    // the LDS reads per product.)
    const int wave = tid >> 6, lane = tid & 63, l16 = lane & 15, kq = lane >> 4;
    f64x4 acc[4];
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) acc[jb] = (f64x4){0.0, 0.0, 0.0, 0.0};
    for (int ch = 0; ch < chunks_per_slice; ++ch) {
        const int r0 = (slice * chunks_per_slice + ch) * ER;
        if (r0 >= n) break;                                    // uniform for the workgroup
        for (int idx = tid; idx < EP * ER; idx += 256) {
            const int c = idx >> 6, rr = idx & 63, row = r0 + rr;
            T[c][rr] = row < n ? At[(size_t)panel_col(I, J, c) * ld + row] : 0.0;
        }
        __syncthreads();
#pragma unroll 4
        for (int rr = 0; rr < ER; rr += 4) {
            double f[4];
#pragma unroll
            for (int jb = 0; jb < 4; ++jb) f[jb] = T[16 * jb + l16][rr + kq];
            const double a = T[16 * wave + l16][rr + kq];      // (one of the four above; read again rather than selected)
#pragma unroll
            for (int jb = 0; jb < 4; ++jb) acc[jb] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, f[jb], acc[jb], 0, 0, 0);
        }
        __syncthreads();
    }
    double* out = Gpart + ((size_t)pair * S + slice) * EP * EP;
#pragma unroll
    for (int jb = 0; jb < 4; ++jb)
#pragma unroll
        for (int v = 0; v < 4; ++v) out[(16 * wave + 4 * v + kq) * EP + 16 * jb + l16] = acc[jb][v];
}

// Diagonalises the 64 x 64 Gram matrix of every panel: cyclic two-sided Jacobi in LDS, 32 disjoint rotations per step
// (round-robin over the 64 indices), 63 steps per sweep.  With the 32 rotations J_k of a step known, the 2 x 2 block of G
// at (rows of pair k, columns of pair l) becomes J_k^T block J_l independently of all other blocks: one thread per block
// (1024 threads), two barriers per step.  Q (the product of the rotations) goes to Qout; the largest
// |G[a][b]| / sqrt(G[a][a] G[b][b]) met before rotating goes to offmax (as the bits of a non-negative float, so that an
// integer maximum orders them).
constexpr int SMALL_NT = 1024;
__global__ __launch_bounds__(SMALL_NT) void eig_small_kernel(const double* __restrict__ Gpart, int S, double* __restrict__ Qout,
                                                            unsigned* __restrict__ offmax, unsigned* __restrict__ rotated, int max_inner,
                                                            double inner_tol) {
    extern __shared__ __attribute__((aligned(16))) double dyn_small[];       // two 64 x 65 matrices: more than the static limit
    double (*G)[EPITCH] = reinterpret_cast<double (*)[EPITCH]>(dyn_small);
    double (*Q)[EPITCH] = reinterpret_cast<double (*)[EPITCH]>(dyn_small + EP * EPITCH);
    __shared__ double cs[EB][2];
    __shared__ int pq[EB][2];
    __shared__ double red[SMALL_NT / 64];
    __shared__ int again, did;                                 // did: some rotation of this panel was not the identity
    const int pair = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) did = 0;
    const double* src = Gpart + (size_t)pair * S * EP * EP;
    for (int idx = tid; idx < EP * EP; idx += SMALL_NT) {
        double g = src[idx];
        for (int s = 1; s < S; ++s) g += src[(size_t)s * EP * EP + idx];
        G[idx >> 6][idx & 63] = g;
        Q[idx >> 6][idx & 63] = (idx >> 6) == (idx & 63) ? 1.0 : 0.0;
    }
    __syncthreads();
    for (int sweep = 0; sweep < max_inner; ++sweep) {
        // how far from diagonal (relative); the first measure is the panel's contribution to the outer test
        double m = 0.0;
        for (int idx = tid; idx < EP * EP; idx += SMALL_NT) {
            const int a = idx >> 6, b = idx & 63;
            if (a < b) {
                const double d = G[a][a] * G[b][b];
                if (d > 0.0) m = fmax(m, fabs(G[a][b]) / sqrt(d));
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) m = fmax(m, __shfl_xor(m, off, 64));
        if (lane == 0) red[wave] = m;
        __syncthreads();
        if (tid == 0) {
            double t = red[0];
            for (int w = 1; w < SMALL_NT / 64; ++w) t = fmax(t, red[w]);
            if (sweep == 0) atomicMax(offmax, __float_as_uint((float)t));
            again = t > inner_tol;
        }
        __syncthreads();
        if (!again) break;
        for (int step = 0; step < EP - 1; ++step) {
            if (tid < EB) {
                int p, q;
                pair_of(EP, step, tid, p, q);
                const double gpq = G[p][q], gpp = G[p][p], gqq = G[q][q];
                double c = 1.0, s = 0.0;
                if (fabs(gpq) > 1e-300 && gpq * gpq > (inner_tol * inner_tol) * fabs(gpp * gqq)) {
                    // t = tan(phi) = sign(a) b / (|a| + sqrt(a^2 + b^2)) with a = gqq - gpp, b = 2 gpq (the tutorial form with
                    // theta = a / b, multiplied through by |b|), c = 1 / sqrt(1 + t^2), s = t c.  These 32 threads are the
                    // critical path of a step, so the square roots and the division are the hardware's reciprocal (square
                    // root) estimates with Newton steps: c to full precision (c^2 + s^2 = c^2 (1 + t^2) = 1 to rounding whatever
                    // t is, which is what keeps Q orthogonal); an error in t only moves the angle by its relative size.
                    const double a = gqq - gpp, b = 2.0 * gpq, h2 = a * a + b * b;
                    double t;
                    if (h2 > 1e-280 && h2 < 1e280) {
                        const double den = fabs(a) + h2 * rsqrt_newton(h2);
                        double r = __builtin_amdgcn_rcp(den);
                        r = fma(fma(-den, r, 1.0), r, r);
                        r = fma(fma(-den, r, 1.0), r, r);
                        t = (a >= 0.0 ? b : -b) * r;
                    } else {
                        const double theta = a / b;
                        t = (theta >= 0.0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
                    }
                    c = rsqrt_newton(fma(t, t, 1.0));
                    s = t * c;
                    if (s != 0.0) did = 1;
                }
                pq[tid][0] = p; pq[tid][1] = q;
                cs[tid][0] = c; cs[tid][1] = s;
            }
            __syncthreads();
            {
                // block (k, l) of G: rows (p_k, q_k), columns (p_l, q_l)
                const int k = tid >> 5, l = tid & 31;
                const int pk = pq[k][0], qk = pq[k][1], pl = pq[l][0], ql = pq[l][1];
                const double ck = cs[k][0], sk = cs[k][1], cl = cs[l][0], sl = cs[l][1];
                const double a = G[pk][pl], b = G[pk][ql], c = G[qk][pl], d = G[qk][ql];
                const double a1 = cl * a - sl * b, b1 = sl * a + cl * b, c1 = cl * c - sl * d, d1 = sl * c + cl * d;
                G[pk][pl] = ck * a1 - sk * c1;
                G[qk][pl] = sk * a1 + ck * c1;
                G[pk][ql] = ck * b1 - sk * d1;
                G[qk][ql] = sk * b1 + ck * d1;
                // columns (p_l, q_l) of Q, rows 2k and 2k + 1
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const int i = 2 * k + e;
                    const double qp = Q[i][pl], qq = Q[i][ql];
                    Q[i][pl] = cl * qp - sl * qq;
                    Q[i][ql] = sl * qp + cl * qq;
                }
            }
            __syncthreads();
        }
    }
    // a panel that needed no rotation has Q = I exactly: the update kernel skips it (no traffic at all for its columns)
    if (tid == 0) rotated[pair] = (unsigned)did;
    if (!did) return;                                          // uniform: did was last written before the last barrier
    double* out = Qout + (size_t)pair * EP * EP;
    for (int idx = tid; idx < EP * EP; idx += SMALL_NT) out[idx] = Q[idx >> 6][idx & 63];
}

// panel <- panel * Q for A (blockIdx.z = 0) and V (blockIdx.z = 1); a workgroup loads Q once and takes UCH chunks of 64 rows
constexpr int UCH = 4;
__global__ __launch_bounds__(256) void eig_update_kernel(double* __restrict__ At, double* __restrict__ Vt, int ld, int n, int nblk, int round,
                                                        const double* __restrict__ Qin, const unsigned* __restrict__ rotated) {
    extern __shared__ __attribute__((aligned(16))) double dyn_upd[];
    double (*T)[EPITCH] = reinterpret_cast<double (*)[EPITCH]>(dyn_upd);
    double (*Qs)[EPITCH] = reinterpret_cast<double (*)[EPITCH]>(dyn_upd + EP * EPITCH);
    const int pair = blockIdx.x, tid = threadIdx.x;
    if (rotated[pair] == 0) return;                            // Q = I: nothing to do (uniform for the workgroup)
    double* M = blockIdx.z == 0 ? At : Vt;
    int I, J;
    pair_of(nblk, round, pair, I, J);
    const double* qsrc = Qin + (size_t)pair * EP * EP;
    for (int idx = tid; idx < EP * EP; idx += 256) Qs[idx >> 6][idx & 63] = qsrc[idx];      // Qs[c][c'] = Q[c][c']
    // fp64 MFMA 16x16x4: wave w owns rows 16w .. 16w+15 of the chunk for all 64 new columns.  out[c'][row] = sum_c Q[c][c']
    // T[c][row]: A[i][k] = Q[kk + k][16ib + i], B[k][j] = T[kk + k][16w + j]; accumulator element v of a lane is new column
    // 16ib + 4 v + lane / 16 at row 16w + lane % 16.
    const int wave = tid >> 6, lane = tid & 63, l16 = lane & 15, kq = lane >> 4;
    for (int ch = 0; ch < UCH; ++ch) {
        const int r0 = (blockIdx.y * UCH + ch) * ER;
        if (r0 >= n) break;                                    // uniform for the workgroup
        __syncthreads();                                       // Q is in place / the previous chunk's tile has been read
        for (int idx = tid; idx < EP * ER; idx += 256) {
            const int c = idx >> 6, rr = idx & 63, row = r0 + rr;
            T[c][rr] = row < n ? M[(size_t)panel_col(I, J, c) * ld + row] : 0.0;
        }
        __syncthreads();
        f64x4 acc[4];
#pragma unroll
        for (int ib = 0; ib < 4; ++ib) acc[ib] = (f64x4){0.0, 0.0, 0.0, 0.0};
#pragma unroll 4
        for (int kk = 0; kk < EP; kk += 4) {
            const double b = T[kk + kq][16 * wave + l16];
#pragma unroll
            for (int ib = 0; ib < 4; ++ib) acc[ib] = __builtin_amdgcn_mfma_f64_16x16x4f64(Qs[kk + kq][16 * ib + l16], b, acc[ib], 0, 0, 0);
        }
        const int row = r0 + 16 * wave + l16;
        if (row < n) {
#pragma unroll
            for (int ib = 0; ib < 4; ++ib)
#pragma unroll
                for (int v = 0; v < 4; ++v) M[(size_t)panel_col(I, J, 16 * ib + 4 * v + kq) * ld + row] = acc[ib][v];
        }
    }
}

// lambda_c = v_c^T a_c (A = C V), D_c = sqrt(max(lambda_c, 0)), B[r][c] = V[r][c]
__global__ __launch_bounds__(256) void eig_finish_kernel(const double* __restrict__ At, const double* __restrict__ Vt, int ld, int n,
                                                        float* __restrict__ B, float* __restrict__ D) {
    __shared__ double red[256];
    const int c = blockIdx.x, tid = threadIdx.x;
    double s = 0.0;
    for (int r = tid; r < n; r += 256) {
        const double v = Vt[(size_t)c * ld + r];
        s = fma(v, At[(size_t)c * ld + r], s);
        B[(size_t)r * n + c] = (float)v;
    }
    red[tid] = s;
    __syncthreads();
    for (int st = 128; st > 0; st >>= 1) {
        if (tid < st) red[tid] += red[tid + st];
        __syncthreads();
    }
    if (tid == 0) D[c] = (float)sqrt(fmax(red[0], 0.0));
}

__global__ void eig_clear_kernel(unsigned* flag) { *flag = 0u; }

}  // namespace

namespace essa_k {

size_t eig_basis_bytes(int n) {
    const size_t npad = (size_t)(n + EP - 1) / EP * EP;
    return npad * npad * sizeof(double);
}

size_t eig_workspace_bytes(int n) {
    const size_t npad = (size_t)(n + EP - 1) / EP * EP, ld = npad, npairs = npad / EP;
    const size_t S = 8;
    return 2 * npad * ld * sizeof(double) + npairs * S * EP * EP * sizeof(double) + npairs * EP * EP * sizeof(double) + 256 + npairs * sizeof(unsigned);
}

hipError_t eig_refresh(hipStream_t st, const float* C, int n, void* ws, double* Vt, int warm, int max_sweeps, float tol, float* B, float* D,
                       int* sweeps_done, float* off_final) {
    const int npad = (n + EP - 1) / EP * EP, ld = npad, nblk = npad / EB, npairs = nblk / 2;
    const int chunks = (n + ER - 1) / ER;
    const int S = 8, chunks_per_slice = (chunks + S - 1) / S;
    double* At = (double*)ws;
    double* Cs = At + (size_t)npad * ld;
    double* Gpart = Cs + (size_t)npad * ld;
    double* Q = Gpart + (size_t)npairs * S * EP * EP;
    unsigned* flag = (unsigned*)(Q + (size_t)npairs * EP * EP);
    unsigned* rotated = flag + 64;                             // [npairs], behind the 256 bytes of the flag
    constexpr size_t two_mats = (size_t)2 * EP * EPITCH * sizeof(double);
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(eig_small_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)two_mats);
        if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(eig_update_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)two_mats);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    // A = C V: with the basis of the last refresh (kept in fp64) the columns of A start out nearly orthogonal and the
    // iteration is in its quadratic phase from the first sweep; on a cold start V = I and A = C
    hipLaunchKernelGGL(eig_init_kernel, dim3(npad), dim3(256), 0, st, C, n, ld, Cs, Vt, warm ? 0 : 1);
    hipLaunchKernelGGL(eig_matmul_kernel, dim3(npad / 64, npad / 64), dim3(256), 0, st, Vt, Cs, ld, At);
    // a pair of columns whose cosine is a hundredth of the caller's tolerance or less is left alone (and a panel with only such
    // pairs costs no update): the outer test cannot tell the difference, and an unchanged C costs one pass of Gram matrices
    const double inner_tol = tol > 1e-13f ? 0.01 * (double)tol : 1e-15;
    int sweep = 0;
    float off = 0.f;
    for (; sweep < max_sweeps; ++sweep) {
        hipLaunchKernelGGL(eig_clear_kernel, dim3(1), dim3(1), 0, st, flag);
        for (int round = 0; round < nblk - 1; ++round) {
            hipLaunchKernelGGL(eig_gram_kernel, dim3(npairs, S), dim3(256), 0, st, At, ld, n, nblk, round, chunks_per_slice, Gpart);
            hipLaunchKernelGGL(eig_small_kernel, dim3(npairs), dim3(SMALL_NT), two_mats, st, Gpart, S, Q, flag, rotated, 4, inner_tol);
            hipLaunchKernelGGL(eig_update_kernel, dim3(npairs, (chunks + UCH - 1) / UCH, 2), dim3(256), two_mats, st, At, Vt, ld, n, nblk, round, Q, rotated);
        }
        unsigned bits = 0;
        hipError_t e = hipMemcpyAsync(&bits, flag, sizeof bits, hipMemcpyDeviceToHost, st);
        if (e != hipSuccess) return e;
        e = hipStreamSynchronize(st);
        if (e != hipSuccess) return e;
        std::memcpy(&off, &bits, sizeof off);
        if (off <= tol) { ++sweep; break; }      // the sweep that measured `off` has also rotated: it counts
    }
    hipLaunchKernelGGL(eig_finish_kernel, dim3(n), dim3(256), 0, st, At, Vt, ld, n, B, D);
    if (sweeps_done) *sweeps_done = sweep;
    if (off_final) *off_final = off;
    return hipGetLastError();
}

}  // namespace essa_k
