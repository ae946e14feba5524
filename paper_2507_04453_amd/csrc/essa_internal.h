// Internal declarations shared by the host glue and the kernel launchers of libessa.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <string>
#include <vector>

#include "essa.h"

// ---- error reporting ---------------------------------------------------------------------------
essa_status essa_fail(essa_status code, const char* fmt, ...);
#define ESSA_HIP(call)                                                                             \
    do {                                                                                           \
        hipError_t e_ = (call);                                                                    \
        if (e_ != hipSuccess)                                                                      \
            return essa_fail(ESSA_ERR_HIP, "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_),  \
                             __FILE__, __LINE__);                                                  \
    } while (0)
#define ESSA_TRY(expr)                  \
    do {                                \
        essa_status s_ = (expr);        \
        if (s_ != ESSA_OK) return s_;   \
    } while (0)

// ---- objects -----------------------------------------------------------------------------------
struct essa_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    void* ws = nullptr;        // scratch, grown on demand
    size_t ws_bytes = 0;
    bool profiling = false;    // bracket GEMM launches with events
    std::vector<hipEvent_t> ev;   // pairs (start, stop)
    size_t ev_used = 0;
    bool capturing = false;    // between essa_graph_begin and essa_graph_end: no allocation, no synchronisation, no events
    std::vector<struct essa_graph*> graphs;   // recorded graphs that are still alive: their launches hold pointers into ws
};
struct essa_graph {
    essa_ctx* ctx = nullptr;   // null once the context is gone: the graph can then only be destroyed
    int device = 0;
    hipStream_t stream = nullptr;
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
};
essa_status essa_ws_reserve(essa_ctx* ctx, size_t bytes);
// One projection's forward on a scratch buffer the caller brings (no allocation of any kind): the body of the entry
// point for callers that cannot allocate.
essa_status essa_forward_on_scratch(essa_ctx* ctx, const essa_fwd_item* item, int x_dtype, int y_dtype, unsigned flags, void* scratch,
                                    size_t scratch_bytes, const char* who);

struct essa_proj {
    essa_ctx* ctx = nullptr;   // identity check only; never dereferenced after creation
    int device = 0;
    hipStream_t stream = nullptr;
    int d_in = 0, d_out = 0, r = 0;
    int rp = 0;                // rank padded to 16 or 32 (zero columns)
    int quant = 0;
    int groups = 0;            // d_in / 128 for int4, 0 for int8
    void* Wq = nullptr;        // int8 [d_out,d_in]  |  packed nibbles [d_out,d_in/2]
    float* scale = nullptr;    // int8: [d_out]      |  int4: [d_out,groups]
    float* zero = nullptr;     // int4: [d_out,groups] (quantised units), else null
    float* VA32 = nullptr;     // [d_in, rp]   V_A, fp32, zero padded
    uint16_t* VA16 = nullptr;  // [rp, d_in]   V_A^T, bf16 (rows = singular directions)
    float* UB32 = nullptr;     // [d_out, rp]
    uint16_t* UB16 = nullptr;  // [d_out, 2, rp]  bf16 head and tail of U_B
    float* M = nullptr;        // [rp, rp]     V_B^T U_A, zero padded
    // fast path (int8 weights): weights tiled for direct-to-register MFMA operand loads, and V_A^T as bf16
    int8_t* Wt = nullptr;      // [d_in_pad/32][n_blocks][2][32][16]: block (kc,nb), half h, channel n, 16 consecutive k
    int d_in_pad = 0;          // d_in rounded up to 512 (zero weights beyond d_in)
    int n_blocks = 0;          // ceil(d_out / 32)
    uint16_t* VAp = nullptr;   // [ceil(d_in/16)][2*rp/32][64][8] bf16: heads (rows 0..rp-1) and tails (rp..2rp-1) of V_A's columns, MFMA-operand tiles
    // 4-bit weights on the fast path: Wt holds nibbles ([d_in_pad/64][n_blocks][2][32][16] bytes: byte j of lane
    // (h, n) = columns 64p+16h+j (low nibble) and 64p+32+16h+j (high nibble) of channel n)
    float* St = nullptr;       // [d_in_pad/128][n_blocks*32] group scales, group major
    uint16_t* SZ16 = nullptr;  // [n_blocks*32][2][Gp] bf16 head and tail of -scale*zero
    int Gp = 0;                // groups rounded up to 16
    std::vector<float> sA, sB; // own singular values, host copies
};

struct essa_cma_scalars {      // lives on the device, updated by kernels only
    float sigma;
    int32_t t;
    float h_sigma;             // last update's stall flag (diagnostic)
    float ps_norm;             // last update's |p_sigma|
};

struct essa_cma {
    essa_ctx* ctx = nullptr;   // identity check only; never dereferenced after creation
    int device = 0;
    hipStream_t stream = nullptr;
    int n = 0;
    int kind = 0;              // essa_optimizer; kinds >= ESSA_OPT_SEP_CMA have no C and no B
    float ars_alpha = 0.f;
    int ars_top = 0;
    float *m = nullptr, *p_sigma = nullptr, *p_c = nullptr, *D = nullptr, *C = nullptr, *B = nullptr;
    float* Cdiag = nullptr;    // [n] diagonal of C (kinds without a matrix)
    essa_cma_scalars* sc = nullptr;
    float* weights = nullptr;  // device [mu] (active CMA: [K]) for weights_K
    int weights_K = 0;
    double* eigV = nullptr;    // the basis of the last eigendecomposition in fp64 (allocated by the first refresh)
    bool eigV_valid = false;   // false after the basis was set from outside: the next refresh starts from the identity
};

// ---- host-side setup helpers ----------------------------------------------------------------------
// Thin SVD of a tall matrix G (m x r, row-major, m >= r) by one-sided Jacobi in fp64:
// G = U diag(s) V^T, s descending.  U: m x r, V: r x r (row-major).
void essa_host_thin_svd(const double* G, int m, int r, double* U, double* s, double* V);

// ---- launchers (each checks nothing: callers validated the arguments) -----------------------------
namespace essa_k {
hipError_t philox_words(hipStream_t st, const uint32_t* seeds, int K, int n_blocks, uint32_t* out);
// S[k, :] = D * z_k (z optionally stored too)
// rank_F: null, or rank_K <= 256 rewards whose ranking (written to rank_order as well) replaces sel
constexpr int kRankInKernelMax = 256;
hipError_t normals_scaled(hipStream_t st, const uint32_t* seeds, const int32_t* sel /*null or [J]*/, int J, int n,
                          const float* D /*null = 1*/, float* S, float* z_out, const float* rank_F = nullptr, int rank_K = 0,
                          int32_t* rank_order = nullptr);
// theta[k, l] = m[l] + s_k sigma (D ? D[l] : 1) z[l];  pairs: candidate k uses seeds[k / 2] and s_k = +1, -1, else seeds[k], +1
hipError_t sample_diag(hipStream_t st, const uint32_t* seeds, int K, int n, const float* m, const float* D,
                       const essa_cma_scalars* sc, int pairs, float* theta, float* z_out);
// Out[j, i] = bias[i] + scale * sum_l S[j,l] B[i,l]; scale = use_sigma ? sc->sigma : 1; bias may be null
hipError_t skinny_gemm_nt(hipStream_t st, const float* S, int J, const float* B, int n, const float* bias,
                          const essa_cma_scalars* sc, int use_sigma, float* Out);
hipError_t theta_to_sigma(hipStream_t st, int P, int r, int n_top, const float* sftA, const float* sftB,
                          const float* theta, int K, float* sA, float* sB);
hipError_t rank_rewards(hipStream_t st, const float* F, int K, int32_t* order);
// C (n x n, fp32, symmetric) -> B (eigenvectors in columns), D (square roots of the eigenvalues); ws: eig_workspace_bytes(n).
// Synchronises the stream once per sweep (the convergence measure comes back to the host).
// Vt: the basis in fp64 (eig_basis_bytes(n)), kept by the state from one refresh to the next; warm = it holds the last result.
size_t eig_workspace_bytes(int n);
size_t eig_basis_bytes(int n);
hipError_t eig_refresh(hipStream_t st, const float* C, int n, void* ws, double* Vt, int warm, int max_sweeps, float tol, float* B, float* D,
                       int* sweeps_done, float* off_final);

struct cma_consts {
    int n, K, mu;
    int ny;                    // rows of y in BY: mu, or K when the worse half enters the covariance with negative weights
    float mu_eff, c_sigma, d_sigma, c_c, c_1, c_mu, chi_n;
    float w_sum;               // sum of the ny weights (1 without negative weights)
};
// S rows 0..ny-1 = D*z_sel, row ny = z_w (the mu positive weights applied), row ny+1 = D*z_w; needs order
// rewards non-null: the ranking is taken inside (c.K <= kRankInKernelMax) and written to order; else order is read
hipError_t cma_build_rhs(hipStream_t st, const uint32_t* seeds, int32_t* order, const float* rewards, const float* w,
                         const cma_consts& c, const float* D, float* S, float* Z /*[ny,n] scratch*/);
hipError_t cma_vectors(hipStream_t st, const cma_consts& c, const float* w, const float* BY /*[ny+2,n]*/,
                       float* m, float* p_sigma, float* p_c, essa_cma_scalars* sc);
// zn2: [ny] squared lengths of the sorted z (read for negative weights only), or null
hipError_t cma_covariance(hipStream_t st, const cma_consts& c, const float* w, const float* BY, const float* p_c,
                          const essa_cma_scalars* sc, const float* zn2, float* C);
// out[j] = |Z[j, :]|^2, fp64 sum in a fixed order
hipError_t row_norms2(hipStream_t st, const float* Z, int J, int n, float* out);
// diagonal covariance: Cd <- decay Cd + c_1 p_c^2 + c_mu sum_i w_i y_i^2, D <- sqrt(Cd)   (Y rows 0..mu-1)
hipError_t sep_covariance(hipStream_t st, const cma_consts& c, const float* w, const float* Y, const float* p_c,
                          const essa_cma_scalars* sc, float* Cd, float* D);
// m[l] += scale * sum_j coef_j Z[j, l] (fp64 sum, j ascending); coef null = uniform; scale = use_sigma ? sigma : 1; then t += 1
hipError_t mean_step(hipStream_t st, const float* Z, const float* coef, double uniform, int J, int n, essa_cma_scalars* sc,
                     int use_sigma, float* m);
// ARS: ranks the N directions by max(r+, r-), order[N] best first, coef[b] = alpha (r+ - r-) / (b s_R) or zeros
hipError_t ars_prepare(hipStream_t st, const float* rewards, int N, int b, float alpha, int32_t* order, float* coef);

// columns of one K slice of the prep kernel's rank-space partial sums: never more than 8 slices up to d_in = 8192
constexpr int prep_slice_cols(int d_in) { return d_in <= 4096 ? 512 : 1024; }
constexpr int prep_slices(int d_in) { return (d_in + prep_slice_cols(d_in) - 1) / prep_slice_cols(d_in); }

struct fwd_item {              // one projection of a grouped forward, device pointers only
    const void* X;
    const int32_t* row2cand;
    const float* sigmaA;
    const float* sigmaB;
    void* Y;
    long long sigma_stride;
    int R, K;
    // projection
    int d_in, d_out, r, rp, quant, groups;
    const void* Wq;
    const float* scale;
    const float* zero;
    const float* VA32;
    const uint16_t* VA16;
    const float* UB32;
    const uint16_t* UB16;
    const float* M;
    // scratch of this item
    float* U32;                // [R, rp]  fp32 rank-space vector u_i
    uint16_t* U16;             // [R, 2, rp]  bf16 head and tail of u_i
    float* xsum;               // [R, max(groups,1)] group sums of x (int4) / unused
    int8_t* Xq;                // [R, d_in] (W8A8)
    float* xscale;             // [R]      (W8A8)
    // fast path
    const int8_t* Wt;
    const uint16_t* VAp;
    int d_in_pad, n_blocks;
    int8_t* Xh;                // [R rounded up to 256, d_in_pad] high limb (or the single int8 code)
    int8_t* Xl;                // same, low limb
    float* xdelta;             // [R] value of one unit of the fixed-point row
    int x_owner;               // 1: this item's rows are quantised by the prep kernel (first user of that X)
    const float* St;
    const uint16_t* SZ16;
    int Gp;
    uint16_t* XS16;            // [R][2][Gp] bf16 head and tail of delta_i * (sum of the row's fixed-point activations over a group)
    float* Tpart;              // [R rounded up to 32][rp][8] the K slices' shares of sA_c * (V_A^T x); slots past tslices hold zeros
    int tslices;               // prep_slices(d_in)
    float* SBrow;              // [R, rp] the row's candidate's sigma_B (gathered by the prep kernel)
    // fused reward (optional)
    const float* rv;           // [d_out] reward vector, or null
    float* rowpart;            // [ceil(d_out / 128)][R] partial <Y, v> over blocks of 128 output channels
};
hipError_t forward_group(hipStream_t st, const fwd_item* items, int n_items, int x_dtype, int y_dtype,
                         unsigned flags, hipEvent_t ev_start, hipEvent_t ev_stop);
hipError_t w8a8_accumulators(hipStream_t st, const fwd_item& it, int x_dtype, int32_t* acc_out);
// fast path for int8 weights x bf16 activations (kernels_stream.hip)
hipError_t forward_stream(hipStream_t st, const fwd_item* items, int n_items, int y_dtype, unsigned flags,
                          hipEvent_t ev_start, hipEvent_t ev_stop);
hipError_t w8a8_accumulators_stream(hipStream_t st, const fwd_item& it, int32_t* acc_out);
// rowpart[b][i] = <Y_g[i, 128 b ..], v_g[128 b ..]> for the items that carry a reward vector (any forward path)
hipError_t rowdot_blocks(hipStream_t st, const fwd_item* items, int n_items, int y_dtype);
// F[k] += mean over the rows of k of the sum over all blocks of rowpart[b][i]; rowsum: [reward_slices(n_blocks)][R] scratch
int reward_slices(int n_blocks);
hipError_t reward_finish(hipStream_t st, const float* rowpart, int n_blocks, int R, const int32_t* row2cand, int K,
                         double* rowsum, float* F);
hipError_t reward_accumulate(hipStream_t st, int n_items, const void* const* Y, const int* d_out, const float* const* v,
                             int y_dtype, int R, const int32_t* row2cand, int K, float* rowdot /*[R] scratch*/, float* F);
}  // namespace essa_k
