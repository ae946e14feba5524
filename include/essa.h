/*
 * essa.h -- C ABI of the MI355X (gfx950) hot path of ESSA (arXiv 2507.04453):
 * the population-batched forward of SVD-parameterised LoRA attention projections on a shared
 * quantised base weight, the seed-to-candidate sampler and the rank-weighted CMA-ES update.
 *
 * Conventions
 *   - "DEVICE" pointers are HIP device memory on the context's GPU; "HOST" pointers are ordinary
 *     host memory.  Nothing here takes framework types.
 *   - All matrices are row-major and dense.  K = population size, r = LoRA rank, n = search
 *     dimension, R = rows (candidate-tokens) of one forward call, P = number of adapted matrices.
 *   - Ownership: the caller owns every buffer it passes, inputs and outputs alike; the library
 *     owns only what a *_create call returns (its own repacked copies and scratch).
 *   - Every hot-path call is asynchronous on the context's stream and allocates scratch only when
 *     a larger problem than any before is seen.  Argument errors are found on the host before any
 *     launch; no call aborts or throws.  On failure the return code is non-zero and
 *     essa_last_error() describes it.
 *   - One context per host thread.  Calls on one context are ordered by its stream.
 */
#ifndef ESSA_H
#define ESSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct essa_ctx essa_ctx;    /* device, stream, scratch                                      */
typedef struct essa_proj essa_proj;  /* one adapted projection: repacked W, V_A, V_B^T U_A, U_B, spectra */
typedef struct essa_cma essa_cma;    /* search distribution (n, t, sigma, m, p_sigma, p_c, C, B, D)   */

typedef enum {
    ESSA_OK = 0,
    ESSA_ERR_INVALID_ARG = 1, /* null pointer, negative size, bad enum, floor(alpha r) = 0 ...        */
    ESSA_ERR_SHAPE = 2,       /* sizes that do not fit each other or the format (d_in % 128 for int4) */
    ESSA_ERR_UNSUPPORTED = 3, /* a valid request this build has no kernel for                         */
    ESSA_ERR_OOM = 4,
    ESSA_ERR_HIP = 5,         /* a HIP runtime call failed; the message carries hipGetErrorString     */
    ESSA_ERR_STATE = 6        /* object used in the wrong state (blob of another n, ...)              */
} essa_status;

typedef enum { ESSA_F32 = 0, ESSA_BF16 = 1 } essa_dtype;

typedef enum {
    ESSA_QUANT_INT8_PERCH = 0, /* int8 symmetric, one fp32 scale per output channel                   */
    ESSA_QUANT_INT4_G128 = 1   /* 4-bit asymmetric, groups of 128 input columns, fp16 scale and zero  */
} essa_quant;

/* flags of the forward calls */
#define ESSA_COMPUTE_W8A8 0x1u /* int8 x int8 -> int32 MFMA on per-row quantised activations (int8 weights only) */
#define ESSA_LORA_ONLY 0x2u    /* test hook: Y = B_k A_k x only                                       */
#define ESSA_BASE_ONLY 0x4u    /* test hook: Y = W_deq x only                                         */
#define ESSA_COMPUTE_BF16 0x8u /* exact bf16 products on the bf16 MFMA instead of the default int8-limb path   */
#define ESSA_VALIDATE 0x10u    /* debug aid: copy every item's row2cand to the host first (one blocking copy per item)
                                  and fail with ESSA_ERR_INVALID_ARG, before any launch, if an entry is not in [0, K) */

/* ---------------------------------------------------------------------------------------------
 * Context
 * ------------------------------------------------------------------------------------------- */

/* Creates a context on GPU `device`.  `hip_stream` is a hipStream_t the caller owns (borrowed for
 * the context's lifetime); NULL means the default stream. */
essa_status essa_create(essa_ctx** out, int device, void* hip_stream);
void essa_destroy(essa_ctx* ctx);
/* Message of the last failing call on this host thread; valid until the next failing call. */
const char* essa_last_error(void);
const char* essa_version(void);
/* Blocks until everything queued on the context's stream has finished. */
essa_status essa_synchronize(essa_ctx* ctx);

/* ---------------------------------------------------------------------------------------------
 * Record and replay.  A generation is a fixed sequence of some dozens of short launches on fixed buffers; a
 * caller that repeats it can record the sequence once (a HIP graph of the context's stream) and replay it with
 * one call per generation.  Between essa_graph_begin and essa_graph_end every call on the context is recorded
 * instead of run (so is any other work the caller puts on that stream); nothing may allocate or wait meanwhile:
 * a call that would have to grow the scratch, upload constants or synchronise fails with ESSA_ERR_STATE, so run
 * the same sequence once, unrecorded, first.  The recorded launches keep their pointer arguments: the replay
 * reads and writes the same buffers, with whatever they hold then (new seeds, the updated search state).
 * The context must have been created on a stream of the caller's, not the default stream.
 * Lifetime: a graph's launches point into the context's scratch and into every object its calls used.  While a graph
 * of a context is alive, a call on that context that would have to grow the scratch (a larger problem than any before),
 * or an update with another population size than the state has seen last, fails with ESSA_ERR_STATE instead of moving
 * memory under the graph: destroy the graph first, or run the largest problem once before recording.  Projections and
 * search states used while recording must outlive the graph.  Destroying the context invalidates its graphs:
 * essa_graph_launch then fails with ESSA_ERR_STATE, essa_graph_destroy is still to be called.
 * ------------------------------------------------------------------------------------------- */
typedef struct essa_graph essa_graph;
essa_status essa_graph_begin(essa_ctx* ctx);
essa_status essa_graph_end(essa_ctx* ctx, essa_graph** out);
/* Queues one replay on the stream the graph was recorded on. */
essa_status essa_graph_launch(essa_graph* graph);
void essa_graph_destroy(essa_graph* graph);

/* Measurement aid: while enabled, every launch of the forward's GEMM kernel is bracketed by HIP
 * events on the context's stream (a call whose items split between the int8, the 4-bit and the generic kernels
 * launches one GEMM per kind, each with its own pair; the prep kernel in front of a GEMM is not timed).
 * essa_profile_read synchronises the stream, returns the summed kernel time in milliseconds and the number of
 * launches since the last read, and resets both. */
essa_status essa_profile_enable(essa_ctx* ctx, int on);
essa_status essa_profile_read(essa_ctx* ctx, double* total_ms, int* launches);

/* ---------------------------------------------------------------------------------------------
 * One adapted projection  (paper: Method, "LoRA + SVD parameterization"; Algorithm 1, SVD-init step)
 *
 * W0 (d_out x d_in) is the frozen quantised base weight and dW = B A its LoRA update with
 * B (d_out x r), A (r x d_in).  Creation is the one-time set-up step: on the host, in fp64, it takes
 * the thin SVDs A = U_A S_A V_A^T and B = U_B S_B V_B^T (singular values descending), forms the
 * r x r core V_B^T U_A, repacks the weight for the kernels and uploads everything.  All pointers in
 * the descriptor are HOST pointers and may be freed when the call returns.
 * ------------------------------------------------------------------------------------------- */
typedef struct essa_proj_desc {
    int32_t d_in, d_out, r;   /* 1 <= r <= 32, r <= min(d_in, d_out)                                  */
    int32_t quant;            /* essa_quant                                                           */
    const void* Wq;           /* INT8: int8 [d_out, d_in].  INT4: uint8 [d_out, d_in/2], column 2j in
                                 the low nibble and 2j+1 in the high nibble of byte j, values 0..15   */
    const void* scales;       /* INT8: float [d_out].  INT4: IEEE fp16 [d_out, d_in/128]              */
    const void* zeros;        /* INT8: NULL.  INT4: IEEE fp16 [d_out, d_in/128], in quantised units:
                                 W[o,j] = scale[o,g] * (q[o,j] - zero[o,g]), g = j / 128              */
    const float* lora_A;      /* float [r, d_in]                                                      */
    const float* lora_B;      /* float [d_out, r]                                                     */
} essa_proj_desc;

essa_status essa_proj_create(essa_ctx* ctx, const essa_proj_desc* desc, essa_proj** out);
void essa_proj_destroy(essa_proj* proj);
/* Copies the factors' own singular values S_A[r], S_B[r] (descending) to HOST arrays. */
essa_status essa_proj_spectrum(const essa_proj* proj, float* sA_host, float* sB_host);

/* ---------------------------------------------------------------------------------------------
 * Search distribution  (paper: Method, "Evolutionary optimization": N(m, sigma^2 C))
 *
 * C = B D^2 B^T with orthonormal columns in B and axis lengths D.  A new object has C = B = I,
 * D = 1, both evolution paths 0, t = 0.  The update moves C only; (B, D) change when the caller asks:
 * essa_cma_refresh_basis takes the eigendecomposition of the current C on the device, essa_cma_set_basis
 * installs a factorisation computed elsewhere.
 * ------------------------------------------------------------------------------------------- */
essa_status essa_cma_create(essa_ctx* ctx, int n, float sigma0, const float* m0_host /* [n] or NULL = 0 */,
                            essa_cma** out);
/* The other rank-based optimisers that run on the same seed sampler (paper: Experiments, "Alternative
 * gradient-free optimizers": plain isotropic (mu, lambda)-ES and ARS on the same search space and evaluation
 * budget; the paper names them and leaves the CMA-ES variant to a library's defaults, so each kind follows
 * its own publication).  essa_sample_candidates and essa_cmaes_update act according to the state's kind:
 *   ESSA_OPT_CMA         what essa_cma_create makes: (mu/mu_w, lambda)-CMA-ES, positive weights.
 *   ESSA_OPT_ACTIVE_CMA  the same with the negative weights of Hansen's tutorial (Table 1, Eqs. 46-58) in the
 *                        rank-mu term: all K candidates enter C, a negative one with w n / |z|^2.
 *   ESSA_OPT_SEP_CMA     Ros & Hansen 2008: only the diagonal of C exists (O(n) state, no B), both covariance
 *                        learning rates times (n + 2) / 3; theta = m + sigma sqrt(diag C) z, and the update
 *                        refreshes sqrt(diag C) itself, so the loop closes without an eigendecomposition.
 *   ESSA_OPT_ES          plain isotropic (mu/mu_I, lambda)-ES: theta = m + sigma z, the new mean is the average
 *                        of the floor(K / 2) best candidates, sigma stays at sigma0.
 *   ESSA_OPT_ARS         Mania, Guy & Recht 2018, Algorithm 1 (V1-t): K is even, seeds holds K / 2 words,
 *                        candidates 2j and 2j + 1 are m + sigma z_j and m - sigma z_j; the update keeps the
 *                        ars_top directions with the largest max(r+, r-) (ties: lower index; NaN = -inf) and
 *                        moves m by ars_alpha / (ars_top s_R) sum (r+ - r-) z, s_R the standard deviation
 *                        (divisor 2 ars_top) of the rewards used; s_R = 0 or a non-finite reward among them
 *                        leaves m alone.  order_out then holds the K / 2 directions, best first.
 * The last three kinds keep no n x n state: essa_cma_set_basis and essa_cma_refresh_basis refuse them with
 * ESSA_ERR_STATE, and their blob is header (reserved = kind) + float m[n], p_sigma[n], p_c[n], D[n], diagC[n]. */
typedef enum {
    ESSA_OPT_CMA = 0,
    ESSA_OPT_ACTIVE_CMA = 1,
    ESSA_OPT_SEP_CMA = 2,
    ESSA_OPT_ES = 3,
    ESSA_OPT_ARS = 4
} essa_optimizer;
typedef struct essa_opt_desc {
    int kind;         /* essa_optimizer */
    float ars_alpha;  /* ESSA_OPT_ARS: step size, > 0 */
    int ars_top;      /* ESSA_OPT_ARS: directions kept, >= 1; an update with fewer than that many pairs fails */
} essa_opt_desc;
essa_status essa_cma_create_opt(essa_ctx* ctx, int n, float sigma0, const float* m0_host, const essa_opt_desc* opt,
                                essa_cma** out);
int essa_cma_kind(const essa_cma* cma); /* essa_optimizer, or -1 for NULL */
void essa_cma_destroy(essa_cma* cma);
/* B: DEVICE float [n, n] (column j = j-th axis), D: DEVICE float [n].  Copied. */
essa_status essa_cma_set_basis(essa_cma* cma, const float* B_dev, const float* D_dev);
/* Flat HOST blob holding the whole state: header {u32 magic, u32 version, i32 n, i32 t, f32 sigma,
 * u32 reserved} then float m[n], p_sigma[n], p_c[n], D[n], C[n*n], B[n*n].  Export with blob = NULL
 * only reports the size.  Both calls synchronise the stream.  Import needs a blob of the same n. */
essa_status essa_cma_export(const essa_cma* cma, void* blob_host, size_t* bytes);
essa_status essa_cma_import(essa_cma* cma, const void* blob_host, size_t bytes);

/* ---------------------------------------------------------------------------------------------
 * Hot path 1: seeds -> candidates  (paper: Method, "Evolutionary optimization"; Algorithm 1, the
 * "sample candidate offsets from shared seeds" step; a seed is the 32-bit word workers exchange)
 *
 * For each of the K seeds: z = N(0,1)^n from Philox4x32-10 with key (seed, 0) and counter
 * (c, 0, 0, 0), block c giving z[4c..4c+3] by Box-Muller on 24-bit uniforms
 * (u = ((w >> 8) + 0.5) 2^-24; words (0,1) and (2,3) each give rho cos, rho sin); then
 * theta = m + sigma * B (D * z).
 *   seeds      DEVICE uint32 [K]
 *   theta_out  DEVICE float [K, n]
 *   z_out      DEVICE float [K, n] or NULL
 * The same seed gives the same bits on every call.  K >= 1.  States of another kind (essa_cma_create_opt)
 * sample their own distribution; z_out holds the N(0, I) vector each candidate was built from (ESSA_OPT_ARS:
 * with the candidate's sign, and seeds is [K / 2]).
 * ------------------------------------------------------------------------------------------- */
essa_status essa_sample_candidates(essa_ctx* ctx, const essa_cma* cma, const uint32_t* seeds, int K,
                                   float* theta_out, float* z_out);

/* Test hook: the raw Philox blocks 0..n_blocks-1 of every seed.  words_out DEVICE uint32 [K, n_blocks, 4]. */
essa_status essa_philox_words(essa_ctx* ctx, const uint32_t* seeds, int K, int n_blocks, uint32_t* words_out);

/* ---------------------------------------------------------------------------------------------
 * Hot path 2: theta -> singular values  (paper: Algorithm 1, reconstruction step, diag(sigma + delta);
 * Figure 1: one contiguous slice of theta per LoRA matrix)
 *
 * theta[k] holds, for projection p = 0..P-1 in order, n_top offsets for factor A then n_top offsets
 * for factor B (n = P * 2 * n_top, n_top = floor(alpha r) >= 1):
 *   sigmaA[k,p,j] = sft_A[p,j] + theta[k, p*2*n_top + j]          for j < n_top, sft_A[p,j] beyond
 *   sigmaB[k,p,j] = sft_B[p,j] + theta[k, p*2*n_top + n_top + j]  likewise
 * All pointers DEVICE float: sft_A, sft_B [P, r]; theta [K, n]; sigmaA, sigmaB [K, P, r].
 * ------------------------------------------------------------------------------------------- */
essa_status essa_theta_to_sigma(essa_ctx* ctx, int P, int r, int n_top, const float* sft_A, const float* sft_B,
                                const float* theta, int K, float* sigmaA, float* sigmaB);

/* ---------------------------------------------------------------------------------------------
 * Hot path 3: population-batched forward  (paper: Algorithm 1, reconstruction step
 * W' = W + B' A' with A' = U_A diag(sigma_A) V_A^T, B' = U_B diag(sigma_B) V_B^T, and the inference
 * pass that follows it)
 *
 * For every row i:  Y[i,:] = W_deq x_i + U_B ( sB_c * ( (V_B^T U_A) ( sA_c * (V_A^T x_i) ) ) ),
 * c = row2cand[i] -- the candidate's dense W' is never formed.
 *   X          DEVICE [R, d_in], x_dtype (bf16 = upper half of an fp32)
 *   row2cand   DEVICE int32 [R], values in [0, K) (trusted: an entry outside reads sigma out of bounds; the flag
 *              ESSA_VALIDATE checks them on the host first)
 *   sigmaA/B   DEVICE float, candidate k's r values at sigmaX + k * sigma_stride (absolute singular
 *              values, not offsets)
 *   Y          DEVICE [R, d_out], y_dtype, written in full
 * Arithmetic: fp32 X -> fp32 throughout.  bf16 X with int8 weights (default): each row of x is put in
 * 16-bit fixed point relative to its largest entry (x ~ delta_i (256 hi + lo), two signed int8 limbs, delta_i =
 * amax_i / 32639, error at most delta_i / 2 per entry) and the base term runs on the int8 MFMA with exact int32
 * accumulation, one pass per limb (4-bit weights likewise, their nibbles unpacked in registers, each group of 128 rescaled in fp32 and the
 * zero-point term added as a low-rank product); ESSA_COMPUTE_BF16 selects exact bf16 products on the bf16 MFMA
 * (fp32 accumulation) instead.  With ESSA_COMPUTE_W8A8 the base term uses x quantised per row to one int8
 * (amax/127, round to nearest even).  The LoRA term always sees the unquantised x.
 * A row of X that holds an Inf or a NaN gives a row of NaN (W_deq x + B_k A_k x is then non-finite in every element: NaN,
 * or an infinity of either sign).  A row whose largest magnitude is at most 2^-100 counts as zero in the base term.
 * R = 0 is a no-op.
 * ------------------------------------------------------------------------------------------- */
essa_status essa_svdlora_forward(essa_ctx* ctx, const essa_proj* proj, const void* X, int x_dtype, int R,
                                 const int32_t* row2cand, const float* sigmaA, const float* sigmaB,
                                 int64_t sigma_stride, int K, void* Y, int y_dtype, uint32_t flags);

/* The same call for callers that cannot allocate device memory (code under HIP graph capture by the caller, tight
 * serving loops, harnesses that forbid hipMalloc): it never calls hipMalloc, hipFree or any other allocating routine.
 * Where essa_svdlora_forward takes its scratch (activation limbs, rank-space vectors) from the context's buffer and
 * grows that on demand, this one lays the same scratch out in a fixed array of ESSA_NOALLOC_SCRATCH_BYTES (8 MiB) that
 * the library holds in device memory on every GPU it runs on until the process ends.  A problem that needs more fails
 * with ESSA_ERR_SHAPE and a message naming both sizes; as a guide, the bytes needed are about
 * 2 * ceil(R / 256) * 256 * ceil(d_in / 512) * 512 + R * (300 * rp + 4 * d_in / 128), i.e. R = 256 rows fit for d_in up
 * to 8192.  ESSA_VALIDATE and profiling (essa_profile_enable) are refused, since they allocate.  Results are bit for
 * bit those of essa_svdlora_forward.  All calls on one GPU share the array, which keeps the last call's contents
 * (nothing in it has to start at zero: every byte a kernel reads is written by the prep launch of the same call):
 * calls that overlap in time on one GPU -- two streams, two contexts -- race; calls on one stream are ordered. */
#define ESSA_NOALLOC_SCRATCH_BYTES (8u << 20)
essa_status essa_svdlora_forward_noalloc(essa_ctx* ctx, const essa_proj* proj, const void* X, int x_dtype, int R,
                                         const int32_t* row2cand, const float* sigmaA, const float* sigmaB,
                                         int64_t sigma_stride, int K, void* Y, int y_dtype, uint32_t flags);

/* The same for several projections in one launch sequence (q, k, v of a layer share X; o has its own). */
typedef struct essa_fwd_item {
    const essa_proj* proj;
    const void* X;
    const int32_t* row2cand;
    const float* sigmaA;
    const float* sigmaB;
    void* Y;
    int64_t sigma_stride;
    int32_t R;
    int32_t K;
} essa_fwd_item;
#define ESSA_MAX_GROUP 8
essa_status essa_svdlora_forward_group(essa_ctx* ctx, const essa_fwd_item* items /* HOST */, int n_items,
                                       int x_dtype, int y_dtype, uint32_t flags);

/* Test hook of the W8A8 mode: per-row quantised activations and the raw int32 accumulators.
 * xq_out DEVICE int8 [R, d_in], xscale_out DEVICE float [R], acc_out DEVICE int32 [R, d_out]. */
essa_status essa_w8a8_accumulators(essa_ctx* ctx, const essa_proj* proj, const void* X, int x_dtype, int R,
                                   int8_t* xq_out, float* xscale_out, int32_t* acc_out);

/* ---------------------------------------------------------------------------------------------
 * Hot path 4: synthetic reward  (stands in for Algorithm 1's "compute reward F" step, which needs a
 * model and data):  F[k] += < mean of the rows of Y owned by candidate k , v >.
 * A candidate without rows gets NaN.  Y DEVICE [R, d_out] y_dtype; v DEVICE float [d_out];
 * F DEVICE float [K], accumulated into (zero it before the first call of a generation).
 * ------------------------------------------------------------------------------------------- */
essa_status essa_reward_accumulate(essa_ctx* ctx, const void* Y, int y_dtype, int R, int d_out, const float* v,
                                   const int32_t* row2cand, int K, float* F);
/* The same over several outputs that share the rows (the projections of one layer) in one launch sequence:
 * F[k] += mean over the rows of k of  sum_g < Y_g[i,:], v_g >.  Y, d_out, v are HOST arrays of n_items entries
 * (1..ESSA_MAX_GROUP) holding DEVICE pointers / widths. */
essa_status essa_reward_accumulate_group(essa_ctx* ctx, int n_items, const void* const* Y, const int* d_out,
                                         const float* const* v, int y_dtype, int R, const int32_t* row2cand, int K,
                                         float* F);

/* The reward fused into the forward (same definition, no second pass over Y): forward of the group as
 * essa_svdlora_forward_group, and for every item g, every block b of ESSA_REWARD_BLOCK consecutive output channels
 * and every row i
 *     rowpart[block, i] = sum over o in the block of Y_g[i,o] v_g[o]     (Y as written, i.e. after rounding to y_dtype)
 * with the blocks of the call numbered block0, block0 + 1, ... item after item (item g has
 * ceil(d_out_g / ESSA_REWARD_BLOCK) of them).  Nothing is accumulated: successive calls of a generation (its layers)
 * take successive block ranges of one buffer, and essa_reward_finish adds them up in ascending order, so the reward
 * is bit-identical from run to run.  All items share R.
 *   v        HOST array of n_items DEVICE float pointers, v[g] of length d_out_g
 *   rowpart  DEVICE float [block_capacity, R]
 * essa_reward_finish: F[k] += mean over candidate k's rows of sum_{b < n_blocks} rowpart[b, i] (sums in fp64, one
 * rounding); a candidate without rows gets NaN. */
#define ESSA_REWARD_BLOCK 128
essa_status essa_svdlora_forward_reward_group(essa_ctx* ctx, const essa_fwd_item* items /* HOST */, int n_items,
                                              int x_dtype, int y_dtype, uint32_t flags, const float* const* v,
                                              float* rowpart, int64_t block_capacity, int64_t block0);
essa_status essa_reward_finish(essa_ctx* ctx, const float* rowpart, int64_t n_blocks, int R, const int32_t* row2cand,
                               int K, float* F);

/* ---------------------------------------------------------------------------------------------
 * Hot path 5: rank-weighted update  (paper: Algorithm 1, "each worker reconstructs the same
 * population and performs one CMA-ES update of (m, sigma, C)"; a reward is the 32-bit scalar workers
 * exchange)
 *
 * (mu/mu_w, lambda)-CMA-ES with lambda = K, mu = K/2, positive log weights and the default constants
 * of Hansen's tutorial.  Candidates are ordered by reward, larger first; equal rewards keep ascending
 * index; NaN counts as -infinity.  z_k is regenerated from seeds[k]; y_k = B (D * z_k).  Updates
 * m, p_sigma, p_c, C, sigma and t in place on the device; (B, D) are left alone.  The result is
 * bit-identical from run to run (fixed reduction order, no atomics).
 *   seeds    DEVICE uint32 [K]     rewards  DEVICE float [K]     order_out  DEVICE int32 [K] or NULL
 * K >= 2.  States of another kind (essa_cma_create_opt) run their own update from the same two arrays.
 * ------------------------------------------------------------------------------------------- */
essa_status essa_cmaes_update(essa_ctx* ctx, essa_cma* cma, const uint32_t* seeds, const float* rewards, int K,
                              int32_t* order_out);

/* Eigendecomposition of the covariance on the device, C = B diag(D^2) B^T (decomposition step of the CMA-ES of
 * Hansen's tutorial, Sec. B.2; the paper's Algorithm 1 samples candidates through this factorisation of the C it
 * updates).  Replaces the state's (B, D): columns of B are orthonormal eigenvectors (order and signs unspecified),
 * D the square roots of the eigenvalues (negative round-off clamped to zero).  C itself is left alone (it is read as
 * (C + C^T) / 2).  One-sided block Jacobi in fp64; sweeps until the largest |a_i . a_j| / (|a_i| |a_j|) over all
 * pairs of columns of C V met during a sweep is <= tol, at most max_sweeps (1..64) times; pairs already below tol / 100
 * are left alone, so a C that has not moved since the last refresh costs one pass over it.  The state keeps the basis of
 * its last refresh in fp64 and the next refresh starts from it (a few sweeps when C has moved little); after
 * essa_cma_set_basis or essa_cma_import the next refresh starts from the identity.  Off the per-generation
 * path: the tutorial refreshes the basis every 1 / (10 n (c_1 + c_mu)) generations.  The call waits for the device
 * after every sweep; it cannot be recorded into a graph.
 *   sweeps_out, off_out   HOST, optional: sweeps done and the last measure
 * ESSA_ERR_STATE if the measure is still above tol after max_sweeps (B, D then hold the last iterate). */
essa_status essa_cma_refresh_basis(essa_ctx* ctx, essa_cma* cma, int max_sweeps, float tol, int* sweeps_out,
                                   float* off_out);

/* The ranking alone.  rewards DEVICE float [K] -> order DEVICE int32 [K]; 1 <= K <= 1024. */
essa_status essa_rank_rewards(essa_ctx* ctx, const float* rewards, int K, int32_t* order);

#ifdef __cplusplus
}
#endif
#endif /* ESSA_H */
