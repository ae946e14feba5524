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

// One workgroup.  BY rows 0..mu-1 are y_{i:lambda} = B D z_{i:lambda}, row mu is B z_w, row mu+1 is y_w = B D z_w
// (the weighted mean of the y_i, taken before the product with B because that product is linear).
__global__ __launch_bounds__(1024) void cma_vectors_kernel(essa_k::cma_consts c, const float* __restrict__ w, const float* __restrict__ BY,
                                                          float* __restrict__ m, float* __restrict__ p_sigma, float* __restrict__ p_c,
                                                          essa_cma_scalars* __restrict__ sc) {
    __shared__ double sh[1024];
    const int n = c.n, mu = c.mu;
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
// Every rank-one term enters as (sqrt(coef) v)(sqrt(coef) v)^T so that C stays exactly symmetric.
constexpr int CV_T = 64, CV_CH = 32;
__global__ __launch_bounds__(256) void cma_cov_kernel(essa_k::cma_consts c, const float* __restrict__ w, const float* __restrict__ BY,
                                                     const float* __restrict__ p_c, const essa_cma_scalars* __restrict__ sc,
                                                     float* __restrict__ C) {
    __shared__ __attribute__((aligned(16))) float Vi[CV_CH][CV_T], Vj[CV_CH][CV_T];
    __shared__ float coef[CV_CH];
    const int n = c.n, mu = c.mu;
    const int i0 = blockIdx.y * CV_T, j0 = blockIdx.x * CV_T;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    float acc[4][4] = {};
    const int nvec = mu + 1;   // vector mu is p_c with coefficient c_1
    for (int v0 = 0; v0 < nvec; v0 += CV_CH) {
        __syncthreads();
        if (threadIdx.x < CV_CH) {
            const int v = v0 + threadIdx.x;
            coef[threadIdx.x] = v < mu ? sqrtf(c.c_mu * w[v]) : (v == mu ? sqrtf(c.c_1) : 0.f);
        }
        __syncthreads();
        for (int idx = threadIdx.x; idx < CV_CH * CV_T; idx += 256) {
            const int vv = idx / CV_T, e = idx % CV_T, v = v0 + vv;
            float a = 0.f, b = 0.f;
            if (v < nvec) {
                const float* src = v < mu ? BY + (size_t)v * n : p_c;
                if (i0 + e < n) a = coef[vv] * src[i0 + e];
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
    const float decay = 1.0f - c.c_1 - c.c_mu + (1.0f - hs) * c.c_1 * c.c_c * (2.0f - c.c_c);
    const int j = j0 + tx * 4;
    const bool vec = (n % 4 == 0) && j + 3 < n;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const int i = i0 + ty * 4 + x;
        if (i >= n) continue;
        if (vec) {
            float4* p = reinterpret_cast<float4*>(C + (size_t)i * n + j);
            float4 cv = *p;
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

}  // namespace

namespace essa_k {

hipError_t rank_rewards(hipStream_t st, const float* F, int K, int32_t* order) {
    hipLaunchKernelGGL(rank_kernel, dim3(1), dim3(1024), 0, st, F, K, order);
    return hipGetLastError();
}

hipError_t cma_build_rhs(hipStream_t st, const uint32_t* seeds, const int32_t* order, const float* w, const cma_consts& c,
                         const float* D, float* S, float* Z) {
    hipError_t e = normals_scaled(st, seeds, order, c.mu, c.n, D, S, Z);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(weighted_rowsum_kernel, dim3((c.n + 255) / 256), dim3(256), 0, st, Z, w, D, c.mu, c.n, S + (size_t)c.mu * c.n,
                       S + (size_t)(c.mu + 1) * c.n);
    return hipGetLastError();
}

hipError_t cma_vectors(hipStream_t st, const cma_consts& c, const float* w, const float* BY, float* m, float* p_sigma,
                       float* p_c, essa_cma_scalars* sc) {
    hipLaunchKernelGGL(cma_vectors_kernel, dim3(1), dim3(1024), 0, st, c, w, BY, m, p_sigma, p_c, sc);
    return hipGetLastError();
}

hipError_t cma_covariance(hipStream_t st, const cma_consts& c, const float* w, const float* BY, const float* p_c,
                          const essa_cma_scalars* sc, float* C) {
    dim3 grid((c.n + CV_T - 1) / CV_T, (c.n + CV_T - 1) / CV_T);
    hipLaunchKernelGGL(cma_cov_kernel, grid, dim3(256), 0, st, c, w, BY, p_c, sc, C);
    return hipGetLastError();
}

}  // namespace essa_k
