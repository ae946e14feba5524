// Seed -> candidate sampling kernels (paper: Method, "Evolutionary optimization"; Algorithm 1,
// "sample candidate offsets from shared seeds"), the theta -> singular-value scatter, and the skinny
// fp32 product with the covariance basis that both the sampler and the update use.
#include "essa_internal.h"

typedef __attribute__((ext_vector_type(16))) float f32x16;

namespace {

// Philox4x32-10 of Salmon et al. (SC'11): ten rounds of two 32x32->64 multiplies and xors, the key
// bumped by the Weyl constants between rounds.
__device__ __forceinline__ uint4 philox4x32_10(uint4 c, uint2 k) {
    const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int rnd = 0; rnd < 10; ++rnd) {
        if (rnd > 0) { k.x += W0; k.y += W1; }
        const uint32_t hi0 = __umulhi(M0, c.x), lo0 = M0 * c.x;
        const uint32_t hi1 = __umulhi(M1, c.z), lo1 = M1 * c.z;
        c = make_uint4(hi1 ^ c.y ^ k.x, lo1, hi0 ^ c.w ^ k.y, lo0);
    }
    return c;
}

// Box-Muller on 24-bit uniforms, evaluated in fp64 and rounded once to fp32 so that the value does
// not depend on the accuracy of fp32 log / sincos near u = 1.
__device__ __forceinline__ void box_muller(uint32_t wa, uint32_t wb, float& za, float& zb) {
    const double ua = ((double)(wa >> 8) + 0.5) * 0x1p-24;
    const double ub = ((double)(wb >> 8) + 0.5) * 0x1p-24;
    const double rho = sqrt(-2.0 * log(ua));
    double s, c;
    sincospi(2.0 * ub, &s, &c);
    za = (float)(rho * c);
    zb = (float)(rho * s);
}

__global__ void philox_words_kernel(const uint32_t* __restrict__ seeds, int K, int n_blocks, uint32_t* __restrict__ out) {
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long long)K * n_blocks) return;
    const int k = (int)(idx / n_blocks), c = (int)(idx % n_blocks);
    const uint4 w = philox4x32_10(make_uint4((uint32_t)c, 0u, 0u, 0u), make_uint2(seeds[k], 0u));
    reinterpret_cast<uint4*>(out)[idx] = w;
}

// S[j, l] = D[l] * z_{cand(j)}[l],  cand(j) = sel ? sel[j] : j ; optional copy of z itself.
// With rank_F the selection is the ranking of rank_K <= 256 rewards (larger first, ties by index, NaN last), which every
// workgroup works out for itself in LDS -- a few hundred comparisons instead of a kernel launch of its own; the first
// workgroup also writes it to rank_order.
__global__ __launch_bounds__(256) void normals_scaled_kernel(const uint32_t* __restrict__ seeds, const int32_t* __restrict__ sel, int J, int n,
                                                            const float* __restrict__ D, float* __restrict__ S, float* __restrict__ z_out,
                                                            const float* __restrict__ rank_F, int rank_K, int32_t* __restrict__ rank_order) {
    __shared__ float key[256];
    __shared__ int ord[256];
    if (rank_F) {
        const int i = threadIdx.x;
        if (i < rank_K) {
            const float f = rank_F[i];
            key[i] = (f != f) ? -INFINITY : f;
        }
        __syncthreads();
        if (i < rank_K) {
            const float mine = key[i];
            int better = 0;
            for (int j = 0; j < rank_K; ++j) {
                const float o = key[j];
                better += (o > mine) || (o == mine && j < i);
            }
            ord[better] = i;
            if (blockIdx.x == 0 && rank_order) rank_order[better] = i;
        }
        __syncthreads();
    }
    const int nb = (n + 3) / 4;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long long)J * nb) return;
    const int j = (int)(idx / nb), c = (int)(idx % nb);
    const int cand = rank_F ? ord[j] : (sel ? sel[j] : j);
    const uint4 w = philox4x32_10(make_uint4((uint32_t)c, 0u, 0u, 0u), make_uint2(seeds[cand], 0u));
    float z[4];
    box_muller(w.x, w.y, z[0], z[1]);
    box_muller(w.z, w.w, z[2], z[3]);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int l = 4 * c + e;
        if (l < n) {
            S[(size_t)j * n + l] = D ? D[l] * z[e] : z[e];
            if (z_out) z_out[(size_t)j * n + l] = z[e];
        }
    }
}

// Distributions with a diagonal covariance: theta[k, l] = m[l] + s_k sigma d[l] z[l] (d = 1 without D).  With
// pairs, candidates 2j and 2j + 1 mirror each other around m on the direction of seed j (ARS, Algorithm 1).
__global__ void sample_diag_kernel(const uint32_t* __restrict__ seeds, int K, int n, const float* __restrict__ m,
                                   const float* __restrict__ D, const essa_cma_scalars* __restrict__ sc, int pairs,
                                   float* __restrict__ theta, float* __restrict__ z_out) {
    const int nb = (n + 3) / 4;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long long)K * nb) return;
    const int k = (int)(idx / nb), c = (int)(idx % nb);
    const uint32_t seed = pairs ? seeds[k >> 1] : seeds[k];
    const float sgn = (pairs && (k & 1)) ? -1.0f : 1.0f;
    const uint4 w = philox4x32_10(make_uint4((uint32_t)c, 0u, 0u, 0u), make_uint2(seed, 0u));
    float z[4];
    box_muller(w.x, w.y, z[0], z[1]);
    box_muller(w.z, w.w, z[2], z[3]);
    const float sigma = sc->sigma;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int l = 4 * c + e;
        if (l < n) {
            const float zs = sgn * z[e];
            theta[(size_t)k * n + l] = m[l] + (D ? sigma * D[l] : sigma) * zs;
            if (z_out) z_out[(size_t)k * n + l] = zs;
        }
    }
}

__global__ void theta_to_sigma_kernel(int P, int r, int n_top, const float* __restrict__ sftA, const float* __restrict__ sftB,
                                      const float* __restrict__ theta, int K, float* __restrict__ sA, float* __restrict__ sB) {
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long total = (long long)K * P * r;
    if (idx >= total) return;
    const int j = (int)(idx % r), p = (int)((idx / r) % P), k = (int)(idx / ((long long)r * P));
    const size_t n = (size_t)P * 2 * n_top;
    float a = sftA[p * r + j], b = sftB[p * r + j];
    if (j < n_top) {
        a += theta[k * n + (size_t)p * 2 * n_top + j];
        b += theta[k * n + (size_t)p * 2 * n_top + n_top + j];
    }
    sA[idx] = a;
    sB[idx] = b;
}

// Out[j, i] = bias[i] + scale * sum_l S[j,l] * B[i,l]        (fp32 MFMA 16x16x4)
// One workgroup = 16 rows of B x (16 * JB) rows of S.  Its 8 waves interleave over chunks of 16 columns (a lane
// loads four consecutive floats of its row, which feed four MFMA steps) and their partial tiles are summed
// through LDS in a fixed order (bit-reproducible).  B is read exactly once when J <= 16 * JB.
constexpr int SG_WAVES = 8;
constexpr int SG_BUNCH = 14;         // chunks of B a wave asks for at once (n = 3584: 28 chunks per wave, two bunches)
constexpr int SG_AHEAD = 4;          // chunks of S in flight ahead of their MFMAs
typedef __attribute__((ext_vector_type(4))) float f32x4;
template <bool ALIGNED, int JB>
__global__ __launch_bounds__(SG_WAVES * 64) void skinny_gemm_nt_kernel(const float* __restrict__ S, int J, const float* __restrict__ B,
                                                                      int n, const float* __restrict__ bias,
                                                                      const essa_cma_scalars* __restrict__ sc, int use_sigma,
                                                                      float* __restrict__ Out) {
    __shared__ __attribute__((aligned(16))) float red[SG_WAVES][JB][4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i0 = blockIdx.x * 16, j0 = blockIdx.y * 16 * JB;
    const int l16 = lane & 15, kq = lane >> 4;
    const int i = i0 + l16;
    f32x4 acc[JB];
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) acc[jb] = (f32x4){0.f, 0.f, 0.f, 0.f};
    const int nchunks = (n + 15) / 16;
    auto load4 = [&](const float* base, int row, int rows, int l) {
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (row < rows) {
            if (ALIGNED) {
                if (l < n) v = *reinterpret_cast<const f32x4*>(base + (size_t)row * n + l);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (l + e < n) v[e] = base[(size_t)row * n + l + e];
            }
        }
        return v;
    };
    // A wave walks its chunks (wave, wave + 8, ...) in ascending order.
    if constexpr (ALIGNED) {
        // Buffer loads: a row or a chunk past the end is an offset outside the descriptor and comes back as zeros, so there
        // is no branch around any load and the compiler can count them.  The B fragments of SG_BUNCH chunks are asked for
        // together and the S fragments then stream past them a few chunks ahead of their MFMAs: a CU's loads complete in
        // order, B comes from HBM and S out of the L2, and S loads spread evenly between B loads would all move at HBM
        // latency.  (n <= 16384 on this path: both matrices stay below the descriptor's 2 GB.)
        typedef __amdgpu_buffer_rsrc_t rsrc_t;
        constexpr uint32_t OUT_OF_RANGE = 0x80000000u;
        const rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(B), 0, (uint32_t)n * (uint32_t)n * 4u, 0x00020000);
        const rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(S), 0, (uint32_t)J * (uint32_t)n * 4u, 0x00020000);
        const uint32_t brow = (uint32_t)i * (uint32_t)n * 4u;                    // i >= n: beyond the descriptor
        uint32_t srow[JB];
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) srow[jb] = (uint32_t)(j0 + 16 * jb + l16) * (uint32_t)n * 4u;
        auto ld = [&](rsrc_t r, uint32_t row_off, int chunk) {
            const int l = chunk * 16 + 4 * kq;
            const uint32_t off = l < n ? row_off + (uint32_t)l * 4u : OUT_OF_RANGE;
            const auto v = __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
            f32x4 f;
            __builtin_memcpy(&f, &v, 16);
            return f;
        };
        for (int base = wave; base < nchunks; base += SG_BUNCH * SG_WAVES) {
            f32x4 a[SG_BUNCH], sv[SG_AHEAD][JB];
#pragma unroll
            for (int u = 0; u < SG_BUNCH; ++u) a[u] = ld(rb, brow, base + u * SG_WAVES);
            __builtin_amdgcn_sched_barrier(0);              // left alone, the compiler moves every load down to its first use
#pragma unroll
            for (int u = 0; u < SG_AHEAD; ++u)
#pragma unroll
                for (int jb = 0; jb < JB; ++jb) sv[u][jb] = ld(rs, srow[jb], base + u * SG_WAVES);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < SG_BUNCH; ++u) {
                f32x4 cur[JB];
#pragma unroll
                for (int jb = 0; jb < JB; ++jb) cur[jb] = sv[u % SG_AHEAD][jb];
                if (u + SG_AHEAD < SG_BUNCH) {
#pragma unroll
                    for (int jb = 0; jb < JB; ++jb) sv[u % SG_AHEAD][jb] = ld(rs, srow[jb], base + (u + SG_AHEAD) * SG_WAVES);
                }
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int jb = 0; jb < JB; ++jb) acc[jb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u][e], cur[jb][e], acc[jb], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    } else {
        for (int ch0 = wave; ch0 < nchunks; ch0 += 2 * SG_WAVES) {
            // two chunks per trip: all their loads are issued before the first MFMA
            f32x4 a[2], sv[2][JB];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int l = (ch0 + u * SG_WAVES) * 16 + 4 * kq;      // past the end: l >= n, everything loads as zero
                a[u] = load4(B, i, n, l);
#pragma unroll
                for (int jb = 0; jb < JB; ++jb) sv[u][jb] = load4(S, j0 + 16 * jb + l16, J, l);
            }
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int jb = 0; jb < JB; ++jb) acc[jb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u][e], sv[u][jb][e], acc[jb], 0, 0, 0);
        }
    }
#pragma unroll
    for (int jb = 0; jb < JB; ++jb)
#pragma unroll
        for (int q = 0; q < 4; ++q) red[wave][jb][q][lane] = acc[jb][q];
    __syncthreads();
    const float scale = use_sigma ? sc->sigma : 1.0f;
    for (int idx = threadIdx.x; idx < JB * 4 * 64; idx += SG_WAVES * 64) {
        const int ln = idx & 63, q = (idx >> 6) & 3, jb = idx >> 8;
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < SG_WAVES; ++w) sum += red[w][jb][q][ln];
        // accumulator element q of lane ln: row (of B) 4*(ln/16) + q, column (of S) ln%16
        const int ii = i0 + 4 * (ln >> 4) + q;
        const int jj = j0 + 16 * jb + (ln & 15);
        if (ii < n && jj < J) Out[(size_t)jj * n + ii] = (bias ? bias[ii] : 0.f) + scale * sum;
    }
}

}  // namespace

namespace essa_k {

hipError_t philox_words(hipStream_t st, const uint32_t* seeds, int K, int n_blocks, uint32_t* out) {
    const long long total = (long long)K * n_blocks;
    hipLaunchKernelGGL(philox_words_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, seeds, K, n_blocks, out);
    return hipGetLastError();
}

hipError_t normals_scaled(hipStream_t st, const uint32_t* seeds, const int32_t* sel, int J, int n, const float* D, float* S,
                          float* z_out, const float* rank_F, int rank_K, int32_t* rank_order) {
    const long long total = (long long)J * ((n + 3) / 4);
    hipLaunchKernelGGL(normals_scaled_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, seeds, sel, J, n, D, S, z_out, rank_F,
                       rank_K, rank_order);
    return hipGetLastError();
}

hipError_t sample_diag(hipStream_t st, const uint32_t* seeds, int K, int n, const float* m, const float* D,
                       const essa_cma_scalars* sc, int pairs, float* theta, float* z_out) {
    const long long total = (long long)K * ((n + 3) / 4);
    hipLaunchKernelGGL(sample_diag_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, seeds, K, n, m, D, sc, pairs, theta,
                       z_out);
    return hipGetLastError();
}

template <int JB>
static void launch_skinny(hipStream_t st, const float* S, int J, const float* B, int n, const float* bias, const essa_cma_scalars* sc,
                          int use_sigma, float* Out) {
    dim3 grid((n + 15) / 16, (J + 16 * JB - 1) / (16 * JB));
    if (n % 4 == 0)
        hipLaunchKernelGGL((skinny_gemm_nt_kernel<true, JB>), grid, dim3(SG_WAVES * 64), 0, st, S, J, B, n, bias, sc, use_sigma, Out);
    else
        hipLaunchKernelGGL((skinny_gemm_nt_kernel<false, JB>), grid, dim3(SG_WAVES * 64), 0, st, S, J, B, n, bias, sc, use_sigma, Out);
}

hipError_t skinny_gemm_nt(hipStream_t st, const float* S, int J, const float* B, int n, const float* bias,
                          const essa_cma_scalars* sc, int use_sigma, float* Out) {
    if (J <= 16) launch_skinny<1>(st, S, J, B, n, bias, sc, use_sigma, Out);
    else if (J <= 32) launch_skinny<2>(st, S, J, B, n, bias, sc, use_sigma, Out);
    else launch_skinny<4>(st, S, J, B, n, bias, sc, use_sigma, Out);
    return hipGetLastError();
}

hipError_t theta_to_sigma(hipStream_t st, int P, int r, int n_top, const float* sftA, const float* sftB, const float* theta,
                          int K, float* sA, float* sB) {
    const long long total = (long long)K * P * r;
    hipLaunchKernelGGL(theta_to_sigma_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, P, r, n_top, sftA, sftB, theta,
                       K, sA, sB);
    return hipGetLastError();
}

}  // namespace essa_k
