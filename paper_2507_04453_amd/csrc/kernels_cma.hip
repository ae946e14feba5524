// Ranking and the rank-weighted update of (m, sigma, C)  (paper: Algorithm 1, "each worker
// reconstructs the same population and performs one CMA-ES update").  Equations follow Hansen's
// tutorial (arXiv:1604.00772).  All reductions run in a fixed order without atomics, so replicated
// workers stay bit-identical.
#include "essa_internal.h"

namespace {

// order[#candidates that beat i] = i.  j beats i when F_j > F_i, or F_j == F_i and j < i.  NaN -> -inf.
__global__ __launch_bounds__(1024) void rank_kernel(const float* __restrict__ F, int K, int32_t* __restrict__ order) {
    __shared__ float key[1024];
    const int i = threadIdx.x;
    if (i < K) {
        const float f = F[i];
        key[i] = (f != f) ? -INFINITY : f;
    }
    __syncthreads();
    if (i < K) {
        const float mine = key[i];
        int better = 0;
        for (int j = 0; j < K; ++j) {
            const float o = key[j];
            better += (o > mine) || (o == mine && j < i);
        }
        order[better] = i;
    }
}

// z_w[l] = sum_i w[i] Z[i, l], summed for i = 0..mu-1 in fp64;  out_z = z_w,  out_dz = D * z_w.
__global__ void weighted_rowsum_kernel(const float* __restrict__ Z, const float* __restrict__ w, const float* __restrict__ D, int mu,
                                       int n, float* __restrict__ out_z, float* __restrict__ out_dz) {
    const int l = blockIdx.x * blockDim.x + threadIdx.x;
    if (l >= n) return;
    double acc = 0.0;
    for (int i = 0; i < mu; ++i) acc += (double)w[i] * (double)Z[(size_t)i * n + l];
    const float zw = (float)acc;
    out_z[l] = zw;
    out_dz[l] = D[l] * zw;
}

__device__ __forceinline__ double block_sum_1024(double v, double* sh) {
    // fixed binary tree over 1024 slots
    sh[threadIdx.x] = v;
    __syncthreads();
    for (int s = 512; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) sh[threadIdx.x] += sh[threadIdx.x + s];
        __syncthreads();
    }
    const double r = sh[0];
    __syncthreads();
    return r;
}

// One workgroup.  BY rows 0..ny-1 are y_{i:lambda} = B D z_{i:lambda}, row ny is B z_w, row ny+1 is y_w = B D z_w
// (the weighted mean of the mu best y_i, taken before the product with B because that product is linear).
__global__ __launch_bounds__(1024) void cma_vectors_kernel(essa_k::cma_consts c, const float* __restrict__ w, const float* __restrict__ BY,
                                                          float* __restrict__ m, float* __restrict__ p_sigma, float* __restrict__ p_c,
                                                          essa_cma_scalars* __restrict__ sc) {
    __shared__ double sh[1024];
    const int n = c.n, mu = c.ny;
    const float sigma = sc->sigma;
    const int t = sc->t;
    const double cs = c.c_sigma, cc = c.c_c, mueff = c.mu_eff;
    const float ps_coef = (float)sqrt(cs * (2.0 - cs) * mueff);
    double part = 0.0;
    for (int l = threadIdx.x; l < n; l += 1024) {
        const float ps = (1.0f - c.c_sigma) * p_sigma[l] + ps_coef * BY[(size_t)mu * n + l];
        p_sigma[l] = ps;
        part += (double)ps * (double)ps;
    }
    const double ps_norm = sqrt(block_sum_1024(part, sh));
    const double denom = sqrt(1.0 - pow(1.0 - cs, 2.0 * (double)(t + 1)));
    const float h_sigma = (ps_norm / denom < (1.4 + 2.0 / ((double)n + 1.0)) * (double)c.chi_n) ? 1.0f : 0.0f;
    const float pc_coef = h_sigma * (float)sqrt(cc * (2.0 - cc) * mueff);
    for (int l = threadIdx.x; l < n; l += 1024) {
        const float yw = BY[(size_t)(mu + 1) * n + l];
        m[l] += sigma * yw;
        p_c[l] = (1.0f - c.c_c) * p_c[l] + pc_coef * yw;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        sc->sigma = (float)((double)sigma * exp((cs / (double)c.d_sigma) * (ps_norm / (double)c.chi_n - 1.0)));
        sc->t = t + 1;
        sc->h_sigma = h_sigma;
        sc->ps_norm = (float)ps_norm;
    }
}

// C <- a C + c_1 p_c p_c^T + c_mu sum_i w_i y_i y_i^T on one 64x64 tile per workgroup.
// Every rank-one term enters as (s sqrt|coef| v)(sqrt|coef| v)^T, s the sign of its weight, so that C stays exactly
// symmetric.  A negative weight (tutorial, Eq. 46-47) is first rescaled by n / |C^-1/2 y|^2 = n / |z|^2.
constexpr int CV_T = 64, CV_CH = 32;
__global__ __launch_bounds__(256) void cma_cov_kernel(essa_k::cma_consts c, const float* __restrict__ w, const float* __restrict__ BY,
                                                     const float* __restrict__ p_c, const essa_cma_scalars* __restrict__ sc,
                                                     const float* __restrict__ zn2, float* __restrict__ C) {
    __shared__ __attribute__((aligned(16))) float Vi[CV_CH][CV_T], Vj[CV_CH][CV_T];
    __shared__ float coef[CV_CH], csign[CV_CH];
    const int n = c.n, mu = c.ny;
    const int i0 = blockIdx.y * CV_T, j0 = blockIdx.x * CV_T;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    float acc[4][4] = {};
    // the tile of C is asked for first: it comes from HBM while the rank-one terms are added up
    const int j = j0 + tx * 4;
    const bool vec = (n % 4 == 0) && j + 3 < n;
    float4 cold[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const int i = i0 + ty * 4 + x;
        cold[x] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (vec && i < n) cold[x] = *reinterpret_cast<const float4*>(C + (size_t)i * n + j);
    }
    const int nvec = mu + 1;   // vector mu is p_c with coefficient c_1
    for (int v0 = 0; v0 < nvec; v0 += CV_CH) {
        __syncthreads();
        if (threadIdx.x < CV_CH) {
            const int v = v0 + threadIdx.x;
            float wv = v < mu ? w[v] : 0.f;
            if (wv < 0.f) wv = wv * (float)n / zn2[v];
            coef[threadIdx.x] = v < mu ? sqrtf(c.c_mu * fabsf(wv)) : (v == mu ? sqrtf(c.c_1) : 0.f);
            csign[threadIdx.x] = wv < 0.f ? -1.f : 1.f;
        }
        __syncthreads();
        for (int idx = threadIdx.x; idx < CV_CH * CV_T; idx += 256) {
            const int vv = idx / CV_T, e = idx % CV_T, v = v0 + vv;
            float a = 0.f, b = 0.f;
            if (v < nvec) {
                const float* src = v < mu ? BY + (size_t)v * n : p_c;
                if (i0 + e < n) a = csign[vv] * (coef[vv] * src[i0 + e]);
                if (j0 + e < n) b = coef[vv] * src[j0 + e];
            }
            Vi[vv][e] = a;
            Vj[vv][e] = b;
        }
        __syncthreads();
        const int lim = min(CV_CH, nvec - v0);
        for (int vv = 0; vv < lim; ++vv) {
            const float4 a = *reinterpret_cast<const float4*>(&Vi[vv][ty * 4]);
            const float4 b = *reinterpret_cast<const float4*>(&Vj[vv][tx * 4]);
            const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
            for (int x = 0; x < 4; ++x)
#pragma unroll
                for (int y = 0; y < 4; ++y) acc[x][y] = fmaf(av[x], bv[y], acc[x][y]);
        }
    }
    const float hs = sc->h_sigma;
    const float decay = 1.0f - c.c_1 - c.c_mu * c.w_sum + (1.0f - hs) * c.c_1 * c.c_c * (2.0f - c.c_c);
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const int i = i0 + ty * 4 + x;
        if (i >= n) continue;
        if (vec) {
            float4* p = reinterpret_cast<float4*>(C + (size_t)i * n + j);
            float4 cv = cold[x];
            cv.x = decay * cv.x + acc[x][0];
            cv.y = decay * cv.y + acc[x][1];
            cv.z = decay * cv.z + acc[x][2];
            cv.w = decay * cv.w + acc[x][3];
            *p = cv;
        } else {
#pragma unroll
            for (int y = 0; y < 4; ++y)
                if (j + y < n) C[(size_t)i * n + j + y] = decay * C[(size_t)i * n + j + y] + acc[x][y];
        }
    }
}

// out[j] = |Z[j, :]|^2.  One workgroup per row, fp64, fixed tree.
__global__ __launch_bounds__(1024) void row_norms2_kernel(const float* __restrict__ Z, int n, float* __restrict__ out) {
    __shared__ double sh[1024];
    const float* z = Z + (size_t)blockIdx.x * n;
    double part = 0.0;
    for (int l = threadIdx.x; l < n; l += 1024) part += (double)z[l] * (double)z[l];
    const double tot = block_sum_1024(part, sh);
    if (threadIdx.x == 0) out[blockIdx.x] = (float)tot;
}

// Separable CMA-ES (Ros & Hansen 2008): the covariance update read on the diagonal, with its own learning rates
// (already in c.c_1, c.c_mu), and the axis lengths that the next generation samples with.
__global__ void sep_cov_kernel(essa_k::cma_consts c, const float* __restrict__ w, const float* __restrict__ Y, const float* __restrict__ p_c,
                               const essa_cma_scalars* __restrict__ sc, float* __restrict__ Cd, float* __restrict__ D) {
    const int l = blockIdx.x * blockDim.x + threadIdx.x;
    if (l >= c.n) return;
    double acc = 0.0;
    for (int i = 0; i < c.mu; ++i) {
        const double y = (double)Y[(size_t)i * c.n + l];
        acc += (double)w[i] * y * y;
    }
    const float hs = sc->h_sigma;
    const float decay = 1.0f - c.c_1 - c.c_mu + (1.0f - hs) * c.c_1 * c.c_c * (2.0f - c.c_c);
    const float pc = p_c[l];
    const float v = decay * Cd[l] + c.c_1 * pc * pc + c.c_mu * (float)acc;
    Cd[l] = v;
    D[l] = sqrtf(fmaxf(v, 0.f));
}

// m[l] += scale * sum_j coef_j Z[j, l]; generation counter bumped by the first thread.
__global__ void mean_step_kernel(const float* __restrict__ Z, const float* __restrict__ coef, double uniform, int J, int n,
                                 essa_cma_scalars* __restrict__ sc, int use_sigma, float* __restrict__ m) {
    const int l = blockIdx.x * blockDim.x + threadIdx.x;
    if (l < n) {
        double acc = 0.0;
        for (int j = 0; j < J; ++j) acc += (coef ? (double)coef[j] : uniform) * (double)Z[(size_t)j * n + l];
        const double scale = use_sigma ? (double)sc->sigma : 1.0;
        m[l] = (float)((double)m[l] + scale * acc);
    }
    if (l == 0) sc->t = sc->t + 1;
}

// ARS (Mania, Guy & Recht 2018, Algorithm 1): directions ordered by max(r+, r-), the step's coefficients for the b best.
__global__ __launch_bounds__(1024) void ars_prepare_kernel(const float* __restrict__ r, int N, int b, float alpha, int32_t* __restrict__ order,
                                                          float* __restrict__ coef) {
    __shared__ float key[1024];
    __shared__ int ord[1024];
    __shared__ double sh[1024];
    const int j = threadIdx.x;
    float rp = 0.f, rm = 0.f;
    if (j < N) {
        rp = r[2 * j];
        rm = r[2 * j + 1];
        if (rp != rp) rp = -INFINITY;
        if (rm != rm) rm = -INFINITY;
        key[j] = fmaxf(rp, rm);
    }
    __syncthreads();
    if (j < N) {
        const float mine = key[j];
        int better = 0;
        for (int o = 0; o < N; ++o) better += (key[o] > mine) || (key[o] == mine && o < j);
        ord[better] = j;
        order[better] = j;
    }
    __syncthreads();
    // thread i < b owns direction ord[i]
    double a = 0.0, d = 0.0;
    int bad = 0;
    if (j < b) {
        const int dir = ord[j];
        float p = r[2 * dir], q = r[2 * dir + 1];
        if (p != p) p = -INFINITY;
        if (q != q) q = -INFINITY;
        bad = !(isfinite(p) && isfinite(q));
        a = bad ? 0.0 : (double)p + (double)q;
        d = bad ? 0.0 : (double)p - (double)q;
    }
    const double nbad = block_sum_1024((double)bad, sh);
    const double mean = block_sum_1024(a, sh) / (2.0 * b);
    double dev = 0.0;
    if (j < b && !bad) {
        const int dir = ord[j];
        const double p = (double)r[2 * dir] - mean, q = (double)r[2 * dir + 1] - mean;
        dev = p * p + q * q;
    }
    const double var = block_sum_1024(dev, sh) / (2.0 * b);
    const double sR = sqrt(var);
    if (j < b) coef[j] = (nbad > 0.0 || !(sR > 0.0)) ? 0.f : (float)((double)alpha * d / ((double)b * sR));
}

}  // namespace

namespace essa_k {

hipError_t rank_rewards(hipStream_t st, const float* F, int K, int32_t* order) {
    hipLaunchKernelGGL(rank_kernel, dim3(1), dim3(1024), 0, st, F, K, order);
    return hipGetLastError();
}

hipError_t cma_build_rhs(hipStream_t st, const uint32_t* seeds, int32_t* order, const float* rewards, const float* w, const cma_consts& c,
                         const float* D, float* S, float* Z) {
    hipError_t e = rewards ? normals_scaled(st, seeds, nullptr, c.ny, c.n, D, S, Z, rewards, c.K, order)
                           : normals_scaled(st, seeds, order, c.ny, c.n, D, S, Z);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(weighted_rowsum_kernel, dim3((c.n + 255) / 256), dim3(256), 0, st, Z, w, D, c.mu, c.n, S + (size_t)c.ny * c.n,
                       S + (size_t)(c.ny + 1) * c.n);
    return hipGetLastError();
}

hipError_t cma_vectors(hipStream_t st, const cma_consts& c, const float* w, const float* BY, float* m, float* p_sigma,
                       float* p_c, essa_cma_scalars* sc) {
    hipLaunchKernelGGL(cma_vectors_kernel, dim3(1), dim3(1024), 0, st, c, w, BY, m, p_sigma, p_c, sc);
    return hipGetLastError();
}

hipError_t cma_covariance(hipStream_t st, const cma_consts& c, const float* w, const float* BY, const float* p_c,
                          const essa_cma_scalars* sc, const float* zn2, float* C) {
    dim3 grid((c.n + CV_T - 1) / CV_T, (c.n + CV_T - 1) / CV_T);
    hipLaunchKernelGGL(cma_cov_kernel, grid, dim3(256), 0, st, c, w, BY, p_c, sc, zn2, C);
    return hipGetLastError();
}

hipError_t row_norms2(hipStream_t st, const float* Z, int J, int n, float* out) {
    hipLaunchKernelGGL(row_norms2_kernel, dim3(J), dim3(1024), 0, st, Z, n, out);
    return hipGetLastError();
}

hipError_t sep_covariance(hipStream_t st, const cma_consts& c, const float* w, const float* Y, const float* p_c,
                          const essa_cma_scalars* sc, float* Cd, float* D) {
    hipLaunchKernelGGL(sep_cov_kernel, dim3((c.n + 255) / 256), dim3(256), 0, st, c, w, Y, p_c, sc, Cd, D);
    return hipGetLastError();
}

hipError_t mean_step(hipStream_t st, const float* Z, const float* coef, double uniform, int J, int n, essa_cma_scalars* sc,
                     int use_sigma, float* m) {
    hipLaunchKernelGGL(mean_step_kernel, dim3((n + 255) / 256), dim3(256), 0, st, Z, coef, uniform, J, n, sc, use_sigma, m);
    return hipGetLastError();
}

hipError_t ars_prepare(hipStream_t st, const float* rewards, int N, int b, float alpha, int32_t* order, float* coef) {
    hipLaunchKernelGGL(ars_prepare_kernel, dim3(1), dim3(1024), 0, st, rewards, N, b, alpha, order, coef);
    return hipGetLastError();
}

}  // namespace essa_k
