// Fast path of the population-batched forward for int8 base weights and bf16 activations
// (paper: Algorithm 1, reconstruction step + inference pass; see kernels_forward.hip for the algebra).
//
// Idea: the int8 weights never leave the integer domain.  Each activation row is re-expressed in
// 16-bit signed fixed point relative to its own largest entry, x ~ delta_i * (256 * hi + lo) with two signed
// int8 limbs, and the base product runs on the int8 MFMA (exact int32 accumulation, one pass per limb):
//     W_deq x_i = delta_i * s_o * (256 * <hi_i, q_o> + <lo_i, q_o>).
// There is no weight conversion at all; every weight byte is loaded from HBM straight into the MFMA
// operand registers of the one wave that owns its 32 output channels (pre-tiled layout, 1 KB
// contiguous per load instruction, k-chunk major), while the activation limbs of all the rows of the tile are staged
// through LDS and shared by the four waves.  With one limb (ESSA_COMPUTE_W8A8) the same kernel is the
// plain W8A8 mode.  The rank-r term is added by bf16 head+tail MFMA steps in the epilogue.
#include "essa_internal.h"
#include <hip/hip_ext.h>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(16))) int i32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

// Phase stamps of wave 0 of every workgroup (shader-clock and 100 MHz counters), read back by a test harness: compiled in
// only with -DESSA_DEBUG_STAMPS, never in the shipped library.
#ifdef ESSA_DEBUG_STAMPS
__device__ unsigned long long essa_dbg[8 * 1024];
extern "C" void essa_dbg_read(unsigned long long* out) { (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(essa_dbg), sizeof(essa_dbg)); }
#define TSTAMP(i) if (lane == 0 && wave == 0 && blockIdx.x < 1024) { essa_dbg[blockIdx.x * 8 + (i)] = __builtin_amdgcn_s_memtime(); if ((i) == 1) essa_dbg[blockIdx.x * 8 + 6] = __builtin_amdgcn_s_memrealtime(); if ((i) == 2) essa_dbg[blockIdx.x * 8 + 7] = __builtin_amdgcn_s_memrealtime(); }
__device__ unsigned long long essa_dbg2[8 * 1024];
extern "C" void essa_dbg2_read(unsigned long long* out) { (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(essa_dbg2), sizeof(essa_dbg2)); }
#define QSTAMP(i) if ((threadIdx.x & 63) == 0 && (threadIdx.x >> 6) == 0 && blockIdx.x < 1024) essa_dbg2[blockIdx.x * 8 + (i)] = __builtin_amdgcn_s_memtime();
__device__ unsigned long long essa_dbg_prep[8 * 1024];
extern "C" void essa_dbg_prep_read(unsigned long long* out) { (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(essa_dbg_prep), sizeof(essa_dbg_prep)); }
#define PSTAMP(i) if (threadIdx.x == 0 && blockIdx.x < 1024) essa_dbg_prep[blockIdx.x * 8 + (i)] = (i) == 7 ? (unsigned long long)role_ : __builtin_amdgcn_s_memtime();
#else
#define TSTAMP(i)
#define QSTAMP(i)
#define PSTAMP(i)
#endif

namespace {

using essa_k::fwd_item;

struct stream_args {
    fwd_item it[ESSA_MAX_GROUP];
    int tile_start[ESSA_MAX_GROUP + 1];    // GEMM tiles per item (prefix sums)
    int quant_start[ESSA_MAX_GROUP + 1];   // prep kernel: rows to quantise per item (0 for items sharing an X)
    int lora_start[ESSA_MAX_GROUP + 1];    // prep kernel: 32-row blocks per item
    int n_items;
    unsigned flags;
    int limbs;
    // prep kernel, interleaved order (every item has the same row count and K slices; 0 in per_rb = off): the workgroups
    // of one block of 32 rows sit side by side in the grid -- per distinct X those that quantise its rows (4 of eight
    // rows each, or 16 of two rows each), then per K slice one per item -- so that a row is fetched from memory once and
    // found in the caches by the others
    int inter_per_rb, inter_nown, inter_slices;
    int inter_owner[ESSA_MAX_GROUP];       // the items that quantise
    // 64 x 256 kernel for 4-bit weights: rows below q4_big_rows go in 64-row tiles (tile_start), the rows from there on in
    // 32-row tiles (q4_small_start), which come last in the grid
    int q4_big_rows;
    int q4_small_start[ESSA_MAX_GROUP + 1];
    // prep kernel, interleaved order only: one workgroup per item and block of 32 rows walks all K slices and leaves the
    // finished u_i = sB_c * (M (sA_c * V_A^T x_i)) in U16 (bf16 head and tail) instead of the slices' shares in Tpart;
    // the 128 x 256 kernel then copies its tile of u instead of adding the shares up once per column tile
    int u_ready;
    // the limbs leave the prep kernel in MFMA-operand tiles, [block of 32 rows][K chunk of 32][half][row][16 bytes]
    // (one contiguous kilobyte per wave load), for the kernel that streams them straight into registers
    int limb_tiled;
};

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
    // round to nearest even in one instruction (v_cvt_pk_bf16_f32)
    return __builtin_bit_cast(uint16_t, (__bf16)f);
}

// The descriptor of one item, fetched from the kernel arguments in one batch of scalar loads: left to itself the
// compiler loads every field where it is first used, and each of those loads is a separate wait on the way to the
// first tile.
__device__ __forceinline__ fwd_item fetch_item(const fwd_item& src) {
    constexpr int NW = sizeof(fwd_item) / 4;
    static_assert(sizeof(fwd_item) % 4 == 0, "descriptor is a whole number of words");
    int raw[NW];
    const int* p = reinterpret_cast<const int*>(&src);
#pragma unroll
    for (int i = 0; i < NW; ++i) raw[i] = p[i];
#pragma unroll
    for (int i = 0; i < NW; ++i) asm volatile("" : "+s"(raw[i]));      // all words are in scalar registers from here on
    fwd_item it;
    __builtin_memcpy(&it, raw, sizeof(fwd_item));
    return it;
}

// Pointers that come out of a descriptor are generic; memory instructions through them would be flat ones, which
// count against both the vector-memory and the LDS counter and force full waits.  These name the global address space.
template <class T> using gptr = __attribute__((address_space(1))) T*;
template <class T> __device__ __forceinline__ gptr<const T> as_global(const T* p) { return (gptr<const T>)p; }
template <class T> __device__ __forceinline__ gptr<T> as_global_w(T* p) { return (gptr<T>)p; }

// A workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every outstanding access to
// global memory (one counter serves loads and stores), which would put loads that are meant to fly across the
// barrier back on the critical path.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// N consecutive words of the kernel arguments in one batch of scalar loads.
template <int N>
__device__ __forceinline__ void fetch_words(const int* p, int (&out)[N]) {
#pragma unroll
    for (int i = 0; i < N; ++i) out[i] = p[i];
#pragma unroll
    for (int i = 0; i < N; ++i) asm volatile("" : "+s"(out[i]));
}

// ------------------------------------------------------------------------------------------------
// prep kernel (512 threads): two kinds of workgroups in one launch.
//  (a) quantise two activation rows into limbs, one row per 256 threads (once per distinct X of the group); at row
//      counts in the thousands and rows up to 4096 wide, eight rows, one per wave;
//  (b) for one item, 32 rows and one K slice: the partial t = V_A^T x by bf16 MFMA against the head+tail copy of
//      V_A; each of the 8 waves takes 64 columns per 512 of the slice and the 8 partial tiles are summed through
//      LDS in a fixed order.  The GEMM kernel adds the slices up and turns t into u = sB_c * (M (sA_c * t)).
// A slice is 512 columns (1024 beyond d_in = 4096, so that there are never more than 8): the workgroups of this
// role are bound by what one CU can load, and twice as many of them with half the columns each halve that time.
// ------------------------------------------------------------------------------------------------
constexpr int PREP_NT = 512;
constexpr int UTP = 36;            // LDS pitch (floats) of the two small matrices (rank-space vectors t, core M)
using essa_k::prep_slice_cols;

// The two limbs of the default path: x ~ unit * (256 hi + lo) with hi and lo both signed int8, i.e. 16-bit fixed point
// relative to the row's largest entry.  LIMB_TOP = 127 * 256 + 127 is the largest magnitude whose high limb still fits.
constexpr float LIMB_TOP = 32639.0f;
// A row whose largest magnitude is at most this (2^-100) counts as a row of zeros in the base term: LIMB_TOP / amax
// would overflow long before amax reaches the smallest fp32.
constexpr float LIMB_TINY = 0x1p-100f;

// Largest magnitude of a row from the bit patterns of its bf16 entries (two per 32-bit word).  With the sign bit gone
// the patterns of finite values order like the values, and those of Inf and NaN lie above all of them: the integer
// maximum is the row's amax when the row is finite and says so when it is not (fmaxf would drop a NaN).  The low
// halves are compared shifted left by 17 (sign shifted out), the high halves masked: two operations per entry, as
// many as shift + fmaxf(|.|).
__device__ __forceinline__ void amax_accumulate(uint32_t& mlo, uint32_t& mhi, uint32_t two_bf16) {
    mlo = max(mlo, two_bf16 << 17);
    mhi = max(mhi, two_bf16 & 0x7fff0000u);
}
__device__ __forceinline__ uint32_t amax_join(uint32_t mlo, uint32_t mhi) { return max(mlo >> 1, mhi); }   // bits of amax as an fp32

// Row quantisation at row counts in the thousands: one wave per row, the whole row in the wave's registers (NK
// 16-byte chunks per lane, all asked for at once), the row maximum by shuffles alone.  No barrier and no LDS, so a
// workgroup keeps eight rows in flight instead of two; the arithmetic per element is that of the two-row form.  It pays
// for rows up to 4096 wide; beyond, with more arithmetic per wave between its loads and its stores, the two-row form is
// the faster one.
template <int NK>
__device__ __forceinline__ void quantise_row_wave(const fwd_item& it, int i, int lane, int a_limbs) {
    typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
    const int din = it.d_in, dpad = it.d_in_pad;
    const int nch = din / 8, kd = dpad / 512;             // 16-byte chunks of the row; trips of 64 chunks up to the padded width
    const gptr<const u32x4> xrow = as_global(reinterpret_cast<const u32x4*>((const uint16_t*)it.X + (size_t)i * din));
    u32x4 xr[NK];
#pragma unroll
    for (int k = 0; k < NK; ++k) xr[k] = xrow[min(64 * k + lane, nch - 1)];     // clamped: no branch between the loads
    __builtin_amdgcn_sched_barrier(0);
    uint32_t mlo = 0, mhi = 0;                             // see amax_accumulate
#pragma unroll
    for (int k = 0; k < NK; ++k) {
        if (64 * k + lane >= nch) xr[k] = (u32x4){0, 0, 0, 0};
#pragma unroll
        for (int e = 0; e < 4; ++e) amax_accumulate(mlo, mhi, xr[k][e]);
    }
    uint32_t mi = amax_join(mlo, mhi);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mi = max(mi, (uint32_t)__shfl_xor((int)mi, off, 64));
    const bool finite = mi < 0x7f800000u;                  // an Inf or NaN anywhere in the row: the whole output row is NaN
    const float amax = __uint_as_float(mi);
    const float top = a_limbs == 2 ? LIMB_TOP : 127.0f;
    const bool usable = finite && amax > (a_limbs == 2 ? LIMB_TINY : 0.f);
    const float inv = usable ? top / amax : 0.f;
    const float unit = !finite ? __builtin_nanf("") : (usable ? amax / top : 0.f);
    const gptr<u32x2> hrow = as_global_w(reinterpret_cast<u32x2*>(it.Xh + (size_t)i * dpad));
    const gptr<u32x2> lrow = as_global_w(reinterpret_cast<u32x2*>(it.Xl + (size_t)i * dpad));
    const gptr<uint16_t> xs16 = as_global_w(it.XS16);
#pragma unroll
    for (int k = 0; k < NK; ++k) {
        if (k >= kd) break;                                // wave-uniform: chunks up to the padded width quantise zeros
        const int c = 64 * k + lane;
        uint32_t hi[2] = {0, 0}, lo[2] = {0, 0};
        int qsum = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float x = (e & 1) ? __uint_as_float(xr[k][e >> 1] & 0xffff0000u) : __uint_as_float(xr[k][e >> 1] << 16);
            float q = rintf(x * inv);
            q = fminf(fmaxf(q, -top), top);
            const int qi = (int)q;
            qsum += qi;
            if (a_limbs == 2) {
                const int qh = (qi + 128) >> 8;            // see the two-row form below
                hi[e >> 2] |= (uint32_t)(qh & 0xff) << (8 * (e & 3));
                lo[e >> 2] |= (uint32_t)((qi - (qh << 8)) & 0xff) << (8 * (e & 3));
            } else {
                hi[e >> 2] |= (uint32_t)(qi & 0xff) << (8 * (e & 3));
            }
        }
        __builtin_nontemporal_store((u32x2){hi[0], hi[1]}, hrow + c);        // streaming stores, as in the two-row form
        if (a_limbs == 2) __builtin_nontemporal_store((u32x2){lo[0], lo[1]}, lrow + c);
        if (it.quant == ESSA_QUANT_INT4_G128) {
            int gs = qsum;                                 // a group of 128 columns is 16 consecutive lanes of one trip
#pragma unroll
            for (int off = 8; off > 0; off >>= 1) gs += __shfl_xor(gs, off, 64);
            const int grp16 = c >> 4;
            if ((lane & 15) == 0 && grp16 < it.Gp) {
                const float xs = unit * (float)gs;
                const uint16_t xh = f32_to_bf16_bits(xs);
                xs16[(size_t)i * 2 * it.Gp + grp16] = xh;
                xs16[(size_t)i * 2 * it.Gp + it.Gp + grp16] = f32_to_bf16_bits(xs - bf16_bits_to_f32(xh));
            }
        }
    }
    if (it.quant == ESSA_QUANT_INT4_G128)
        for (int gq = dpad / 128 + lane; gq < it.Gp; gq += 64) {
            xs16[(size_t)i * 2 * it.Gp + gq] = 0;
            xs16[(size_t)i * 2 * it.Gp + it.Gp + gq] = 0;
        }
    if (lane == 0) as_global_w(it.xdelta)[i] = unit;
}

// FULLK: the form for row counts in the thousands on their way to the 128 x 256 kernel (role (b) walks all K slices and
// finishes u); a separate instantiation, capped at 128 registers for two workgroups per CU, so that the decode form
// keeps its own register allocation.
template <bool FULLK>
__global__ __launch_bounds__(PREP_NT, FULLK ? 4 : 1) void prep_kernel(stream_args a) {
    __shared__ __attribute__((aligned(16))) float part[8][2][16][64];   // lora role: partial tiles of the 8 waves (64 KB)
    __shared__ uint32_t wred[8];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.x;
    // Two dependent fetches from the kernel arguments stand between the start of the kernel and its first load from
    // memory, each a batch of scalar loads: both work tables (entries past the last item repeat the totals), then the
    // descriptor of the item they point to.
    constexpr int NG = ESSA_MAX_GROUP + 1;
    static_assert(offsetof(stream_args, lora_start) == offsetof(stream_args, quant_start) + NG * sizeof(int) &&
                  offsetof(stream_args, flags) == offsetof(stream_args, quant_start) + (2 * NG + 1) * sizeof(int) &&
                  offsetof(stream_args, limbs) == offsetof(stream_args, flags) + sizeof(int), "tables and scalars are adjacent");
    static_assert(offsetof(stream_args, inter_per_rb) == offsetof(stream_args, limbs) + sizeof(int) &&
                  offsetof(stream_args, inter_owner) == offsetof(stream_args, limbs) + 4 * sizeof(int), "order fields follow");
    int tab[2 * NG + 3 + 3 + ESSA_MAX_GROUP];
    fetch_words(a.quant_start, tab);
    const int a_nitems = tab[2 * NG];
    const unsigned a_flags = (unsigned)tab[2 * NG + 1];
    const int a_limbs = tab[2 * NG + 2];
    const int per_rb = tab[2 * NG + 3], nown = tab[2 * NG + 4], islices = tab[2 * NG + 5];
    const int qw = per_rb > 0 ? (per_rb - a_nitems * islices) / nown : 0;    // quantising workgroups per owner and block of 32 rows
    bool quant_role;
    int g = 0, first = 0, lb = 0;
    int rel = 0;          // quant role: index of the row pair inside the item; other role: (row block) * slices + slice
    if (per_rb > 0) {
        const int rb = b / per_rb, rem = b % per_rb;
        quant_role = rem < qw * nown;
        if (quant_role) {
            const int oi = rem / qw;
#pragma unroll
            for (int i = 0; i < ESSA_MAX_GROUP; ++i) g = i == oi ? tab[2 * NG + 6 + i] : g;
            rel = rb * qw + rem % qw;                       // 4: eight rows each, one per wave; 16: two rows each
        } else {
            const int e = rem - qw * nown;
            g = e % a_nitems;
            rel = rb * islices + e / a_nitems;
        }
    } else {
        const int n_qblocks = tab[NG - 1];
        quant_role = b < n_qblocks;
        lb = b - n_qblocks;
#pragma unroll
        for (int i = 1; i < ESSA_MAX_GROUP; ++i) {
            const int start = quant_role ? tab[i] : tab[NG + i];
            const bool past = (quant_role ? b : lb) >= start;
            g += past ? 1 : 0;
            first = past ? start : first;
        }
        rel = (quant_role ? b : lb) - first;
    }
    const fwd_item it = fetch_item(a.it[g]);
    if (quant_role && qw == 4) {
        const int i = rel * 8 + wave;
        if (i < it.R) quantise_row_wave<8>(it, i, lane, a_limbs);
        return;
    }
    if (quant_role) {
        const int role_ = 1; (void)role_;
        PSTAMP(0) PSTAMP(7)
        // ---- (a) row quantisation: this 256-thread group takes row 2*b' + grp of its item ---------------
        const int grp = tid >> 8, t256 = tid & 255;
        const int i = rel * 2 + grp;
        const bool live = i < it.R;
        const int din = it.d_in, dpad = it.d_in_pad;
        const gptr<const u32x4> xrow = as_global(reinterpret_cast<const u32x4*>((const uint16_t*)it.X + (size_t)(live ? i : 0) * din));
        const int nch = din / 8;                          // 16-byte chunks of 8 bf16
        // the row is read once: the first four chunks of every thread (rows up to 8192 wide) wait in registers
        // between the two passes
        u32x4 xr[4];
        uint32_t mlo = 0, mhi = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int c = t256 + 256 * k;
            xr[k] = c < nch ? xrow[c] : (u32x4){0, 0, 0, 0};
#pragma unroll
            for (int e = 0; e < 4; ++e) amax_accumulate(mlo, mhi, xr[k][e]);
        }
        for (int c = t256 + 1024; c < nch; c += 256) {
            const u32x4 v = xrow[c];
#pragma unroll
            for (int e = 0; e < 4; ++e) amax_accumulate(mlo, mhi, v[e]);
        }
        uint32_t mi = amax_join(mlo, mhi);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) mi = max(mi, (uint32_t)__shfl_xor((int)mi, off, 64));
        if (lane == 0) wred[wave] = mi;
        __syncthreads();
        mi = max(max(wred[4 * grp], wred[4 * grp + 1]), max(wred[4 * grp + 2], wred[4 * grp + 3]));
        const bool finite = mi < 0x7f800000u;             // an Inf or NaN anywhere in the row: the whole output row is NaN
        const float amax = __uint_as_float(mi);
        const float top = a_limbs == 2 ? LIMB_TOP : 127.0f;
        const bool usable = finite && amax > (a_limbs == 2 ? LIMB_TINY : 0.f);
        const float inv = usable ? top / amax : 0.f;
        const float unit = !finite ? __builtin_nanf("") : (usable ? amax / top : 0.f);
        PSTAMP(1)
        if (!live) return;
        typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
        const gptr<u32x2> hrow = as_global_w(reinterpret_cast<u32x2*>(it.Xh));
        const gptr<u32x2> lrow = as_global_w(reinterpret_cast<u32x2*>(it.Xl));
        const gptr<uint16_t> xs16 = as_global_w(it.XS16);
        const int tiled = a.limb_tiled;
        // where chunk c (columns 8c .. 8c+7) of row i goes, in units of 8 bytes: row-major, or operand tiles
        auto limb_slot = [&](int c) -> size_t {
            if (!tiled) return ((size_t)i * dpad >> 3) + c;
            const size_t blk = (size_t)(i >> 5) * (dpad >> 5) + (c >> 2);                  // (row block, K chunk)
            return ((blk * 2 + ((c >> 1) & 1)) * 512 + (size_t)(i & 31) * 16 + (c & 1) * 8) >> 3;
        };
        auto quantise_chunk = [&](int c, const u32x4& v) {
            uint32_t hi[2] = {0, 0}, lo[2] = {0, 0};
            int qsum = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float x = (e & 1) ? __uint_as_float(v[e >> 1] & 0xffff0000u) : __uint_as_float(v[e >> 1] << 16);
                float q = rintf(x * inv);
                q = fminf(fmaxf(q, -top), top);
                const int qi = (int)q;
                qsum += qi;
                if (a_limbs == 2) {
                    const int qh = (qi + 128) >> 8;                                // arithmetic shift: hi in [-127,127]
                    hi[e >> 2] |= (uint32_t)(qh & 0xff) << (8 * (e & 3));
                    lo[e >> 2] |= (uint32_t)((qi - (qh << 8)) & 0xff) << (8 * (e & 3));   // lo in [-128,127]
                } else {
                    hi[e >> 2] |= (uint32_t)(qi & 0xff) << (8 * (e & 3));
                }
            }
            // streaming stores: the limbs are read by the next launch, from behind other L2s than this one
            const size_t slot = limb_slot(c);
            __builtin_nontemporal_store((u32x2){hi[0], hi[1]}, hrow + slot);
            if (a_limbs == 2) __builtin_nontemporal_store((u32x2){lo[0], lo[1]}, lrow + slot);
            if (it.quant == ESSA_QUANT_INT4_G128) {
                // sum of the row's fixed-point activations over each group of 128 columns (16 consecutive lanes),
                // times delta: what the zero-points of the 4-bit format multiply.  Kept as bf16 head + tail.
                int gs = qsum;
#pragma unroll
                for (int off = 8; off > 0; off >>= 1) gs += __shfl_xor(gs, off, 64);
                const int grp16 = c >> 4;
                if ((lane & 15) == 0 && grp16 < it.Gp) {
                    const float xs = unit * (float)gs;
                    const uint16_t xh = f32_to_bf16_bits(xs);
                    xs16[(size_t)i * 2 * it.Gp + grp16] = xh;
                    xs16[(size_t)i * 2 * it.Gp + it.Gp + grp16] = f32_to_bf16_bits(xs - bf16_bits_to_f32(xh));
                }
            }
        };
        // chunks past d_in (the zero padding up to d_in_pad) quantise zeros; whole waves enter or skip a chunk together
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (t256 + 256 * k < dpad / 8) quantise_chunk(t256 + 256 * k, xr[k]);
        for (int c = t256 + 1024; c < dpad / 8; c += 256) quantise_chunk(c, c < nch ? xrow[c] : (u32x4){0, 0, 0, 0});
        if (it.quant == ESSA_QUANT_INT4_G128)
            for (int gq = dpad / 128 + t256; gq < it.Gp; gq += 256) {
                xs16[(size_t)i * 2 * it.Gp + gq] = 0;
                xs16[(size_t)i * 2 * it.Gp + it.Gp + gq] = 0;
            }
        if (t256 == 0) as_global_w(it.xdelta)[i] = unit;
        PSTAMP(2)
        return;
    }
    // ---- (b) partial t = V_A^T x for 32 rows of one item over one K slice --------------------------------
    const int role_ = 2; (void)role_;
    PSTAMP(0) PSTAMP(7)
    constexpr int full_k = FULLK ? 1 : 0;                   // this workgroup walks all K slices and finishes u
    const int S = it.tslices;
    const int r0 = full_k ? rel * 32 : (rel / S) * 32;
    const int slice_begin = full_k ? 0 : rel % S, slice_end = full_k ? S : slice_begin + 1;
    const int l32 = lane & 31, h = lane >> 5;
    const int din = it.d_in, rp = it.rp, nbv = rp / 16, R = it.R;
    const int ksteps = din / 16;
    const int scols = prep_slice_cols(din);
    // The candidate's singular values for the (row, j) elements this thread finishes at the end (one for rank 16, two
    // for rank 32) are a chain of two dependent loads: the row's candidate is asked for right behind the tile loads
    // (loads come back in order, so it does not hold them up), the singular values once the MFMAs are issued, and
    // they arrive during the reduction.  Every thread asks, with clamped indices: a branch around a load would make
    // the compiler wait for the value where the branch ends.
    const int rsh = rp == 16 ? 4 : 5;                       // rp is 16 or 32
    int e_row[2], e_j[2], my_c[2];
    float my_sa[2], my_sb[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int e = tid + PREP_NT * i;                   // element e < 32 * rp is real
        e_row[i] = (e >> rsh) & 31;
        e_j[i] = e & (rp - 1);
    }
    auto ask_candidates = [&]() {
#pragma unroll
        for (int i = 0; i < 2; ++i) my_c[i] = as_global(it.row2cand)[min(r0 + e_row[i], R - 1)];
    };
    float tsum[2] = {0.f, 0.f};                             // full_k: this thread's elements of sA_c * (V_A^T x), slices added in ascending order
    for (int slice = slice_begin; slice < slice_end; ++slice) {
    f32x16 acc0 = {0}, acc1 = {0};
    if (a_flags & ESSA_BASE_ONLY) {
        if (slice == slice_begin) ask_candidates();
    } else {
        // wave w takes, of every 512 columns of the slice, the four consecutive steps 4w + u, i.e. 64 columns = 128 bytes
        // of each of the 32 rows.  x: four coalesced loads (instruction i: rows 8i..8i+7, whole 128-byte lines), turned
        // into operand order through a wave-private, XOR-swizzled 4 KB patch of LDS; V_A: operand tiles straight from memory.
        unsigned char* xs = reinterpret_cast<unsigned char*>(&part[0][0][0][0]) + wave * 4096;
        const int ch = lane & 7;
        const gptr<const u32x4> vt = as_global(reinterpret_cast<const u32x4*>(it.VAp)) + lane;
        for (int c0 = 0; c0 < scols; c0 += 512) {
            const int kbase = slice * scols + c0 + wave * 64;
            const int ks0 = kbase / 16;
            u32x4 xg[4], xa[4], v0[4], v1[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                // every lane loads (a column past the row reads the row's first chunk instead and is zeroed): no branch
                // stands between the loads
                const int row = 8 * i + (lane >> 3), col = kbase + ch * 8;
                xg[i] = *as_global(reinterpret_cast<const u32x4*>((const uint16_t*)it.X + (size_t)min(r0 + row, R - 1) * din + (col < din ? col : 0)));
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                v0[u] = vt[((size_t)(ks0 + u < ksteps ? ks0 + u : 0) * nbv) * 64];
                v1[u] = (u32x4){0, 0, 0, 0};
            }
            if (nbv == 2) {
#pragma unroll
                for (int u = 0; u < 4; ++u) v1[u] = vt[((size_t)(ks0 + u < ksteps ? ks0 + u : 0) * 2 + 1) * 64];
            }
            __builtin_amdgcn_sched_barrier(0);
            if (c0 == 0 && slice == slice_begin) ask_candidates();
            __builtin_amdgcn_sched_barrier(0);              // all loads are out before anything waits for one of them
            if (kbase + ch * 8 >= din) {
#pragma unroll
                for (int i = 0; i < 4; ++i) xg[i] = (u32x4){0, 0, 0, 0};
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (ks0 + u >= ksteps) v0[u] = v1[u] = (u32x4){0, 0, 0, 0};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = 8 * i + (lane >> 3);
                *reinterpret_cast<u32x4*>(xs + row * 128 + ((ch ^ ((row >> 1) & 7)) * 16)) = xg[i];
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int u = 0; u < 4; ++u) xa[u] = *reinterpret_cast<const u32x4*>(xs + l32 * 128 + (((2 * u + h) ^ ((l32 >> 1) & 7)) * 16));
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, xa[u]), __builtin_bit_cast(bf16x8, v0[u]), acc0, 0, 0, 0);
                if (nbv == 2)
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, xa[u]), __builtin_bit_cast(bf16x8, v1[u]), acc1, 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            // the patch is read again only by this wave, after its own next stores: wave-level ordering is enough
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    }
    if (slice == slice_begin) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const size_t at = (size_t)my_c[i] * it.sigma_stride + min(e_j[i], it.r - 1);
            my_sa[i] = as_global(it.sigmaA)[at];
            my_sb[i] = as_global(it.sigmaB)[at];
        }
    }
    lds_barrier();            // the staging patches become the reduction buffer
    PSTAMP(1)
    // the 8 partial tiles, added up below always in the same order (the second column block exists for rank 32 only)
#pragma unroll
    for (int q = 0; q < 16; ++q) part[wave][0][q][lane] = acc0[q];
    if (nbv == 2) {
#pragma unroll
        for (int q = 0; q < 16; ++q) part[wave][1][q][lane] = acc1[q];
    }
    lds_barrier();
    PSTAMP(2)
    // element (row, j): head and tail columns of V_A's column j meet here, and the candidate's sigma_A scales the
    // slice's share of t_j = <V_A[:, j], x>; the slice-0 workgroup also passes on the row's sigma_B
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        if (tid + PREP_NT * i < 32 * rp) {               // rank 16: the first element only (the same for the whole workgroup)
            const int row = e_row[i], j = e_j[i];
            const int q = 4 * (row >> 3) + (row & 3), lnr = 32 * ((row >> 2) & 1);
            float th[2];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int v = e * rp + j, nb = v >> 5, ln = lnr + (v & 31);
                th[e] = ((part[0][nb][q][ln] + part[1][nb][q][ln]) + (part[2][nb][q][ln] + part[3][nb][q][ln])) +
                        ((part[4][nb][q][ln] + part[5][nb][q][ln]) + (part[6][nb][q][ln] + part[7][nb][q][ln]));
            }
            // the eight slice slots of an element sit side by side (two 16-byte loads for the GEMM kernel); the slice-0
            // workgroup clears the slots no slice fills
            const float share = (j < it.r ? my_sa[i] : 0.f) * (th[0] + th[1]);
            if (full_k) {
                tsum[i] = slice == 0 ? share : tsum[i] + share;
            } else {
                const gptr<float> slot = as_global_w(it.Tpart) + ((size_t)(r0 + row) * rp + j) * 8;
                slot[slice] = share;
                if (slice == 0) {
                    for (int sl = S; sl < 8; ++sl) slot[sl] = 0.f;
                    if (r0 + row < R) as_global_w(it.SBrow)[(size_t)(r0 + row) * rp + j] = j < it.r ? my_sb[i] : 0.f;
                }
            }
        }
    }
    if (full_k) lds_barrier();     // the partial tiles are read: the memory goes back to the staging patches, or to the finish below
    }
    PSTAMP(3)
    if (!full_k) return;
    // ---- u_i = sB_c * (M t_i) for the 32 rows, with the operations (and their order) of the GEMM kernels' own prologue
    float* tvec = &part[0][0][0][0];                        // [32][UTP]
    float* Ms = tvec + 32 * UTP;                            // [rp][UTP]
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int e = tid + PREP_NT * i;
        if (e < rp * rp) Ms[(e >> rsh) * UTP + (e & (rp - 1))] = as_global(it.M)[e];
        if (e < 32 * rp) tvec[e_row[i] * UTP + e_j[i]] = tsum[i];
    }
    lds_barrier();
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        if (tid + PREP_NT * i < 32 * rp) {
            const int row = e_row[i], j = e_j[i];
            float u = 0.f;
            if (!(a_flags & ESSA_BASE_ONLY)) {
                for (int l0 = 0; l0 < rp; l0 += 16) {
                    f32x4 mv[4], tv[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        mv[q] = *reinterpret_cast<const f32x4*>(Ms + j * UTP + l0 + 4 * q);
                        tv[q] = *reinterpret_cast<const f32x4*>(tvec + row * UTP + l0 + 4 * q);
                    }
#pragma unroll
                    for (int q = 0; q < 16; ++q) u = fmaf(mv[q >> 2][q & 3], tv[q >> 2][q & 3], u);
                }
                u *= j < it.r ? my_sb[i] : 0.f;
            }
            if (r0 + row < R) {
                const uint16_t hi = f32_to_bf16_bits(u);
                const gptr<uint16_t> urow = as_global_w(it.U16) + (size_t)(r0 + row) * 2 * rp;
                urow[j] = hi;
                urow[rp + j] = f32_to_bf16_bits(u - bf16_bits_to_f32(hi));
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// int8-MFMA GEMM.  512 threads = 8 waves; tile = (32*MB rows) x 128 channels.  Wave (n, kh): n = 0..3
// owns channels 32n..32n+31 of the tile for all its rows, kh = 0..1 takes the even / odd pair of 32-wide
// K chunks of every K tile (two waves per SIMD hide each other's LDS and memory latency; int32 partial
// sums are exact, so the split costs nothing numerically).  K advances in tiles of 128:
//   weights      global -> registers, two 16-byte loads per lane and tile, PD tiles ahead;
//   activations  global -> registers -> LDS (two stages), issued three tiles ahead.
// Epilogue: the two K halves swap half of their accumulators through LDS, scale, add the rank-r term
// (operands fetched before the main loop), and the tile leaves through an LDS transpose as full rows.
// ------------------------------------------------------------------------------------------------
constexpr int KT = 128;            // K per tile (bytes per limb row)
constexpr int LROW = KT + 16;      // padded LDS row of an activation tile
constexpr int PD = 4;              // weight prefetch distance in K tiles; d_in_pad is a multiple of KT * PD
constexpr int NT = 512;            // threads per workgroup
constexpr int UROW = 144;          // LDS row of the u tile: 2 * rp bf16 (at most 128 B) + pad

// Loads of the main loop are buffer loads: (wave-uniform base in a resource descriptor) + (scalar offset that moves
// with the K tile) + (32-bit lane offset, fixed for the whole loop).  All address arithmetic is scalar, and the vector
// ALU, which the MFMAs also issue through, stays free.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base_uniform) {
    // raw buffer (stride 0), 32-bit data format; 2 GB window: offsets used here are far below it
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base_uniform), 0, 0x7fffffff, 0x00020000);
}
__device__ __forceinline__ u32x4 load16(rsrc_t r, uint32_t lane_off, uint32_t scalar_off) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, lane_off, scalar_off, 0);
}

// lane offsets of the activation-tile loads: vector e of thread tid is 16-byte part `part` of row `row` of limb e's tile
template <int LIMBS, int BM, int XV>
__device__ __forceinline__ void x_lane_offsets(uint32_t (&xoff)[XV], int dpad, int tid) {
#pragma unroll
    for (int e = 0; e < XV; ++e) {
        const int idx = tid + NT * e, rem = idx % (BM * 8), row = rem >> 3, part = rem & 7;
        xoff[e] = (uint32_t)row * (uint32_t)dpad + part * 16;
    }
}

// xbase[e]: start of the tile's rows in the limb that vector e of this wave belongs to (wave-uniform)
template <int LIMBS, int BM, int XV>
__device__ __forceinline__ void load_x(u32x4 (&xr)[XV], const rsrc_t (&xbase)[XV], const uint32_t (&xoff)[XV], int kt, int tid) {
#pragma unroll
    for (int e = 0; e < XV; ++e) {
        const int idx = tid + NT * e;
        if ((LIMBS * BM * 8) % NT != 0 && idx >= LIMBS * BM * 8) continue;
        xr[e] = load16(xbase[e], xoff[e], (uint32_t)kt * KT);
    }
}

template <int LIMBS, int BM, int XV>
__device__ __forceinline__ void store_x(const u32x4 (&xr)[XV], unsigned char* smem, int stage, int tid) {
#pragma unroll
    for (int e = 0; e < XV; ++e) {
        const int idx = tid + NT * e;
        if ((LIMBS * BM * 8) % NT != 0 && idx >= LIMBS * BM * 8) continue;
        const int limb = idx / (BM * 8), rem = idx % (BM * 8), row = rem >> 3, part = rem & 7;
        *reinterpret_cast<u32x4*>(smem + ((size_t)((stage * LIMBS + limb) * BM + row)) * LROW + part * 16) = xr[e];
    }
}

template <int LIMBS, int BM>
__device__ __forceinline__ void store_x_vec(const u32x4& v, unsigned char* smem, int stage, int tid, int e) {
    const int idx = tid + NT * e;
    if ((LIMBS * BM * 8) % NT != 0 && idx >= LIMBS * BM * 8) return;
    const int limb = idx / (BM * 8), rem = idx % (BM * 8), row = rem >> 3, part = rem & 7;
    *reinterpret_cast<u32x4*>(smem + ((size_t)((stage * LIMBS + limb) * BM + row)) * LROW + part * 16) = v;
}

// fragment of (K chunk cc of the wave, limb l, row block mb) of the tile in `stage`
template <int LIMBS, int BM>
__device__ __forceinline__ i32x4 read_frag(const unsigned char* smem, int stage, int cc, int l, int mb, int kh, int l32, int h) {
    return *reinterpret_cast<const i32x4*>(smem + ((size_t)((stage * LIMBS + l) * BM + mb * 32 + l32)) * LROW + (2 * kh + cc) * 32 + 16 * h);
}

// the wave's two K chunks of one tile
template <int LIMBS, int MB>
__device__ __forceinline__ void compute_tile(i32x16 (&acc)[LIMBS][MB], const u32x4 (&w)[2], const unsigned char* smem, int stage, int kh,
                                             int l32, int h) {
    constexpr int BM = 32 * MB;
    i32x4 fr[2][LIMBS][MB];
#pragma unroll
    for (int cc = 0; cc < 2; ++cc)
#pragma unroll
        for (int l = 0; l < LIMBS; ++l)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
                fr[cc][l][mb] = *reinterpret_cast<const i32x4*>(smem + ((size_t)((stage * LIMBS + l) * BM + mb * 32 + l32)) * LROW +
                                                                (2 * kh + cc) * 32 + 16 * h);
#pragma unroll
    for (int cc = 0; cc < 2; ++cc) {
        const i32x4 wv = (i32x4)w[cc];
#pragma unroll
        for (int l = 0; l < LIMBS; ++l)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) acc[l][mb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fr[cc][l][mb], wv, acc[l][mb], 0, 0, 0);
    }
}

// The same in two halves, with the fragments of a tile read one tile ahead of their use (int8 weights).
template <int LIMBS, int MB>
__device__ __forceinline__ void read_frags(i32x4 (&fr)[2][LIMBS][MB], const unsigned char* smem, int stage, int kh, int l32, int h) {
    constexpr int BM = 32 * MB;
#pragma unroll
    for (int cc = 0; cc < 2; ++cc)
#pragma unroll
        for (int l = 0; l < LIMBS; ++l)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
                fr[cc][l][mb] = *reinterpret_cast<const i32x4*>(smem + ((size_t)((stage * LIMBS + l) * BM + mb * 32 + l32)) * LROW +
                                                                (2 * kh + cc) * 32 + 16 * h);
}
template <int CC, int LIMBS, int MB>
__device__ __forceinline__ void mfma_chunk(i32x16 (&acc)[LIMBS][MB], const i32x4 (&fr)[2][LIMBS][MB], const u32x4 (&w)[2]) {
    const i32x4 wv = (i32x4)w[CC];
#pragma unroll
    for (int l = 0; l < LIMBS; ++l)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) acc[l][mb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fr[CC][l][mb], wv, acc[l][mb], 0, 0, 0);
}

// 4-bit weights: a 16-byte load holds two K chunks of the tile (low / high nibbles), two loads the whole tile.  The
// tile's integer sums are complete for the group (a K tile is one group of 128), so they are scaled and added to the
// fp32 totals right away: tot += s_g * (128 * <hi, q> + <lo, q>).
// 4-bit weights: wave (n, mh) owns channels 32n.. for the rows 32mh.. of the tile over the WHOLE K tile (no K split
// between waves; in the 32-row tile only waves 0..3 multiply).  The group's integer sums are scaled into fp32 on the
// vector ALU, three operations per output; a K split would have both waves of a pair scale a partial sum for every
// output of the pair, twice the vector-ALU work, which is what bounds this format -- and with the whole group summed
// in integers before it is scaled, a row's result does not depend on the tile height.
template <int LIMBS, int BM>
__device__ __forceinline__ void compute_tile_q4_rows(f32x16& tot, const u32x4 (&w)[2], float sg, const unsigned char* smem, int stage, int mh,
                                                     int l32, int h) {
    i32x4 fr[4][LIMBS];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int l = 0; l < LIMBS; ++l)
            fr[c][l] = *reinterpret_cast<const i32x4*>(smem + ((size_t)((stage * LIMBS + l) * BM + mh * 32 + l32)) * LROW + c * 32 + 16 * h);
    const u32x4 m4 = {0x0f0f0f0fu, 0x0f0f0f0fu, 0x0f0f0f0fu, 0x0f0f0f0fu};
    const i32x4 wq[4] = {(i32x4)(w[0] & m4), (i32x4)((w[0] >> 4) & m4), (i32x4)(w[1] & m4), (i32x4)((w[1] >> 4) & m4)};
    const i32x16 zero = {0};
    i32x16 t[LIMBS];
#pragma unroll
    for (int l = 0; l < LIMBS; ++l) {
        t[l] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fr[0][l], wq[0], zero, 0, 0, 0);
#pragma unroll
        for (int c = 1; c < 4; ++c) t[l] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fr[c][l], wq[c], t[l], 0, 0, 0);
    }
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int comb = LIMBS == 2 ? (t[0][q] << 8) + t[LIMBS - 1][q] : t[0][q];   // |t| < 2^18 per tile: no overflow
        tot[q] = fmaf(sg, (float)comb, tot[q]);
    }
}

__device__ __forceinline__ void load_w(u32x4 (&w)[2], rsrc_t wbase, uint32_t wstride_b, uint32_t lane16, int kt, int kh) {
#pragma unroll
    for (int cc = 0; cc < 2; ++cc) w[cc] = load16(wbase, lane16, (uint32_t)(kt * 4 + 2 * kh + cc) * wstride_b);
}

// LDS stages of the activation tiles: four for int8 weights (the tile of K step j sits in stage j % 4 and can be
// written before the step's barrier), two for 4-bit weights
template <int MB, bool Q4 = false>
constexpr int gemm_stages() { return (MB <= 2 && !Q4) ? 4 : 2; }     // the 4-bit loop alternates between two stages

template <int MB, int LIMBS, bool YBF16, bool Q4 = false>
constexpr size_t gemm_smem_bytes() {
    constexpr size_t BM = 32 * MB;
    constexpr size_t stages = gemm_stages<MB, Q4>() * LIMBS * BM * LROW;
    constexpr size_t exch = (size_t)4 * 2 * LIMBS * (MB >= 2 ? MB / 2 : 1) * 4096;   // sized for the accumulator dump, which exchanges every limb
    constexpr size_t ctile = BM * (128 * (YBF16 ? 2 : 4) + 16);
    constexpr size_t pre = stages + BM * 36 * 4 + 32 * 36 * 4;   // + sA*t, core matrix (before the main loop)
    constexpr size_t m1 = pre > exch ? pre : exch;
    constexpr size_t big = m1 > ctile ? m1 : ctile;
    return big + BM * 4 + BM * UROW;
}

// The tile of rank-space vectors u_i = sB_c * (M t_i), t_i = sum over the K slices (ascending) of the prep kernel's
// sA_c * (V_A^T x_i) shares, kept in LDS as bf16 head+tail rows of UROW bytes.  Two parts, so that a caller can put
// other loads between them: the global loads, then the arithmetic (which contains one workgroup barrier).
template <int BM, int EU>
__device__ __forceinline__ void u_tile_loads(const fwd_item& it, int m0, int tid, f32x4 (&tp)[EU][2], float (&sb)[EU], float (&mreg)[2]) {
    const int R = it.R, rp = it.rp, rpad = (R + 31) / 32 * 32;
    const int rsh = rp == 16 ? 4 : 5;                     // rp is 16 or 32: divisions become shifts
    const gptr<const f32x4> tpart = as_global(reinterpret_cast<const f32x4*>(it.Tpart));
#pragma unroll
    for (int i = 0; i < EU; ++i) {
        // loads are skipped only on a condition that holds for the whole workgroup (rank 16 fills half of the
        // entries): a scalar branch, no per-lane masking between the loads
        const int e = min(tid + NT * i, BM * rp - 1), row = e >> rsh, j = e & (rp - 1);
        const size_t at = ((size_t)min(m0 + row, rpad - 1) * rp + j) * 2;
        tp[i][0] = tp[i][1] = (f32x4){0.f, 0.f, 0.f, 0.f};
        sb[i] = 0.f;
        if (NT * i < BM * rp) {
            tp[i][0] = tpart[at];
            tp[i][1] = tpart[at + 1];
            sb[i] = as_global(it.SBrow)[(size_t)min(m0 + row, R - 1) * rp + j];
        }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) mreg[i] = as_global(it.M)[min(tid + NT * i, rp * rp - 1)];
}

template <int BM, int EU, bool LDS_ONLY = false>
__device__ __forceinline__ void u_tile_finish(const fwd_item& it, unsigned flags, int tid, const f32x4 (&tp)[EU][2], const float (&sb)[EU],
                                              const float (&mreg)[2], float* tvec, float* Ms, unsigned char* utile) {
    const int rp = it.rp, rsh = rp == 16 ? 4 : 5;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int e = tid + NT * i;
        if (e < rp * rp) Ms[(e >> rsh) * UTP + (e & (rp - 1))] = mreg[i];
    }
#pragma unroll
    for (int i = 0; i < EU; ++i) {
        const int e = tid + NT * i;
        if (e < BM * rp) {
            float t = tp[i][0][0];
#pragma unroll
            for (int sl = 1; sl < 8; ++sl) t += tp[i][sl >> 2][sl & 3];       // slices in ascending order; unused slots hold zeros
            tvec[(e >> rsh) * UTP + (e & (rp - 1))] = t;
        }
    }
    if (LDS_ONLY) lds_barrier();          // loads already in flight keep flying across it
    else __syncthreads();
#pragma unroll
    for (int i = 0; i < EU; ++i) {
        const int e = tid + NT * i;
        if (e < BM * rp) {
            const int row = e >> rsh, j = e & (rp - 1);
            float u = 0.f;
            if (!(flags & ESSA_BASE_ONLY)) {
                // columns past r hold zeros in both operands; 16-byte LDS reads, sixteen terms per trip
                for (int l0 = 0; l0 < rp; l0 += 16) {
                    f32x4 mv[4], tv[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        mv[q] = *reinterpret_cast<const f32x4*>(Ms + j * UTP + l0 + 4 * q);
                        tv[q] = *reinterpret_cast<const f32x4*>(tvec + row * UTP + l0 + 4 * q);
                    }
#pragma unroll
                    for (int q = 0; q < 16; ++q) u = fmaf(mv[q >> 2][q & 3], tv[q >> 2][q & 3], u);
                }
                u *= sb[i];
            }
            const uint16_t hi = f32_to_bf16_bits(u);
            uint16_t* urow = reinterpret_cast<uint16_t*>(utile + (size_t)row * UROW);
            urow[j] = hi;
            urow[rp + j] = f32_to_bf16_bits(u - bf16_bits_to_f32(hi));
        }
    }
}

// An output tile of BM rows x 128 channels, staged in LDS as rows of CROW bytes, leaves as full rows (16 bytes per
// thread where the output allows it).  With a reward vector, the tile's share <Y[i, block], v[block]> of every row
// goes to rowpart[blk][i]: one partial per (128-channel block, row); the blocks are added in a fixed order later.
// The reward-vector entries that this thread's 16-byte piece of an output row meets.  The piece is the same for every
// row a thread stores (NT is a multiple of the pieces per row), so they are fetched once, before the epilogue's
// arithmetic, instead of behind it.  Entries past the last channel, and all of them without a reward vector, are 0.
template <bool YBF16>
struct rv_piece { float v[YBF16 ? 8 : 4]; };
template <bool YBF16>
__device__ __forceinline__ rv_piece<YBF16> load_rv_piece(const fwd_item& it, int n0, int tid) {
    constexpr int EPV = YBF16 ? 8 : 4, PPR = 128 / EPV;
    static_assert(NT % PPR == 0, "a thread keeps its piece from row to row");
    rv_piece<YBF16> r;
#pragma unroll
    for (int e = 0; e < EPV; ++e) r.v[e] = 0.f;
    if (it.rv) {
        const int o = n0 + (tid % PPR) * EPV, dout = it.d_out;
        const gptr<const float> rv = as_global(it.rv);
        if ((reinterpret_cast<uintptr_t>(it.rv) & 15) == 0 && o + EPV <= dout) {
#pragma unroll
            for (int e4 = 0; e4 < EPV / 4; ++e4) {
                const f32x4 r4 = *reinterpret_cast<gptr<const f32x4>>(rv + o + 4 * e4);
#pragma unroll
                for (int e = 0; e < 4; ++e) r.v[4 * e4 + e] = r4[e];
            }
        } else {
#pragma unroll
            for (int e = 0; e < EPV; ++e)
                if (o + e < dout) r.v[e] = rv[o + e];
        }
    }
    return r;
}

template <bool YBF16, int BM>
__device__ __forceinline__ void store_ctile(const unsigned char* ctile, const fwd_item& it, int m0, int n0, int blk, int tid,
                                            const rv_piece<YBF16>& rvp) {
    constexpr int ESZ = YBF16 ? 2 : 4, EPV = 16 / ESZ, PPR = 128 / EPV;     // elements per vector, vectors per row
    constexpr int CROW = 128 * ESZ + 16;
    const int R = it.R, dout = it.d_out;
    const gptr<unsigned char> Yb = as_global_w(reinterpret_cast<unsigned char*>(it.Y));
    const bool vec_ok = (dout % EPV == 0) && ((reinterpret_cast<uintptr_t>(it.Y) & 15) == 0);
    const bool with_reward = it.rv != nullptr;
#pragma unroll
    for (int p0 = 0; p0 < BM * PPR; p0 += NT) {           // BM * PPR is a multiple of NT: every lane takes part in the shuffles
        const int p = p0 + tid;
        const int row = p / PPR, piece = p % PPR;
        const int i = m0 + row, o = n0 + piece * EPV;
        const bool valid = i < R && o < dout;
        const unsigned char* src = ctile + (size_t)row * CROW + piece * 16;
        const u32x4 val = *reinterpret_cast<const u32x4*>(src);
        if (valid) {
            if (vec_ok && o + EPV <= dout) {
                // streaming store: the output is not read again by this launch, and lines left dirty in the L2 are written
                // back when the kernel ends, before the next one may start
                __builtin_nontemporal_store(val, reinterpret_cast<gptr<u32x4>>(Yb + ((size_t)i * dout + o) * ESZ));
            } else {
                for (int e = 0; e < EPV && o + e < dout; ++e) {
                    if (YBF16) reinterpret_cast<gptr<uint16_t>>(Yb)[(size_t)i * dout + o + e] = reinterpret_cast<const uint16_t*>(src)[e];
                    else reinterpret_cast<gptr<float>>(Yb)[(size_t)i * dout + o + e] = reinterpret_cast<const float*>(src)[e];
                }
            }
        }
        if (with_reward) {
            float s = 0.f;
            if (valid) {
#pragma unroll
                for (int e = 0; e < EPV; ++e) {
                    const float y = YBF16 ? __uint_as_float((e & 1) ? (val[e >> 1] & 0xffff0000u) : (val[e >> 1] << 16)) : __uint_as_float(val[e]);
                    s = fmaf(o + e < dout ? y : 0.f, rvp.v[e], s);     // what lies past the last channel in the LDS tile is not data
                }
            }
#pragma unroll
            for (int off = PPR / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
            if (piece == 0 && i < R && n0 < dout) as_global_w(it.rowpart)[(size_t)blk * R + i] = s;   // a half tile past the last channel has no block
        }
    }
}

// 4-bit weights, 64-row tile: registers capped at 128 so that two workgroups share a CU (what spills is the epilogue's
// operands, across the main loop)
template <int MB, int LIMBS, bool YBF16, bool DUMP, bool Q4>
__global__ __launch_bounds__(NT, (Q4 && MB == 2) ? 4 : 1) void gemm_i8_kernel(stream_args a, int32_t* __restrict__ acc_out) {
    constexpr int BM = 32 * MB;
    constexpr int XTOT = LIMBS * BM * 8;               // 16-byte vectors of X per K tile
    constexpr int XV = (XTOT + NT - 1) / NT;
    constexpr int MBO = MB >= 2 ? MB / 2 : 1;          // row blocks a wave finishes in the epilogue
    constexpr size_t BIG = gemm_smem_bytes<MB, LIMBS, YBF16, Q4>() - BM * 4 - BM * UROW;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float* xd = reinterpret_cast<float*>(smem + BIG);                  // [BM] value of one fixed-point unit per row
    unsigned char* utile = smem + BIG + BM * 4;                        // [BM][UROW] bf16 head+tail of u_i

    QSTAMP(0)
    // Blocks go round-robin over the 8 XCDs, each with an L2 of its own.  XCD x takes the contiguous range
    // [x T/8, (x+1) T/8) of the group's T tiles (row tile fastest, then column tile, then item): the row tiles that share a
    // weight tile sit behind one L2 and start together, no weight tile is read behind two L2s, and an XCD whose range lies
    // inside the items that read one X (q, k, v) never touches the limbs of the other (o).
    const int total = a.tile_start[ESSA_MAX_GROUP];
    int b = blockIdx.x;
    const bool by_group = (total & 7) == 0;
    if (by_group) b = (b & 7) * (total >> 3) + (b >> 3);
    // which item this tile belongs to: the whole table comes in with one scalar load, the count is branch-free
    int g = 0;
#pragma unroll
    for (int i = 1; i < ESSA_MAX_GROUP; ++i) g += (i < a.n_items && b >= a.tile_start[i]) ? 1 : 0;
    const fwd_item it = fetch_item(a.it[g]);
    const int ntile = a.tile_start[g + 1] - a.tile_start[g];
    int tile = b - a.tile_start[g];
    if (!by_group && (ntile & 7) == 0 && (a.tile_start[g] & 7) == 0) tile = (tile & 7) * (ntile >> 3) + (tile >> 3);   // per item, where that works
    const int tiles_m = (it.R + BM - 1) / BM;
    const int m0 = (tile % tiles_m) * BM, nb0 = (tile / tiles_m) * 4;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // in a scalar register: what depends on it alone stays scalar
    const int nw = wave & 3, kh = wave >> 2;
    const int l32 = lane & 31, h = lane >> 5;
    const int R = it.R, dout = it.d_out, dpad = it.d_in_pad, rp = it.rp;
    const int nk = dpad / KT;                              // a multiple of PD
    const int nbw = min(nb0 + nw, it.n_blocks - 1);        // a wave past the last n-block repeats it; nothing of it is stored
    // weights are stored k-chunk major, [kc][n-block][1 KB]: at any moment the waves of the whole grid read one
    // contiguous stretch of memory, which spreads over all HBM channels
    const uint32_t wstride_b = (uint32_t)it.n_blocks * 1024;   // bytes per k chunk; a projection's weights stay below 2 GB
    const rsrc_t wbase = make_rsrc(reinterpret_cast<const unsigned char*>(it.Wt) + (size_t)nbw * 1024);
    const uint32_t lane16 = lane * 16, lane4 = l32 * 4;
    // activation tiles: per-thread offsets fixed for the whole loop, wave-uniform bases (the limb of vector e)
    uint32_t xoff[XV];
    x_lane_offsets<LIMBS, BM, XV>(xoff, dpad, tid);
    rsrc_t xbase[XV];
#pragma unroll
    for (int e = 0; e < XV; ++e) {
        const int limb = (wave * 64 + NT * e) / (BM * 8);     // BM * 8 is a multiple of 64: one limb per wave and vector
        xbase[e] = make_rsrc((limb == 0 ? it.Xh : it.Xl) + (size_t)m0 * dpad);
    }

    TSTAMP(0)
    QSTAMP(1)
    // 4-bit: the group scale of this lane's channel, [group][channel]
    const rsrc_t sbase = make_rsrc(Q4 ? it.St + (size_t)nbw * 32 : nullptr);
    const uint32_t sstride_b = (uint32_t)it.n_blocks * 32 * 4;
    auto fetch_w = [&](u32x4 (&w)[2], int kt) { load_w(w, wbase, wstride_b, lane16, kt, kh); };
    // u tile, part 1: the loads, issued ahead of the weight and activation tiles so that they come back first (loads
    // return in order) and the arithmetic of part 2 runs while those tiles are still on their way
    constexpr size_t STG = (size_t)gemm_stages<MB, Q4>() * LIMBS * BM * LROW;
    float* tvec = reinterpret_cast<float*>(smem + STG);                        // [BM][UTP]
    float* Ms = tvec + BM * UTP;                                               // [rp][UTP]
    constexpr int EU = (BM * 32 + NT - 1) / NT;           // (row, j) entries of u per thread at the widest rank
    f32x4 tp[EU][2];
    float sb[EU], mreg[2];
    float xdreg = 0.f;                                     // the row's fixed-point unit; parked in LDS on the way into the loop
    if (!DUMP) {
        u_tile_loads<BM, EU>(it, m0, tid, tp, sb, mreg);
        xdreg = as_global(it.xdelta)[min(m0 + min(tid, BM - 1), R - 1)];
    }
    __builtin_amdgcn_sched_barrier(0);

    u32x4 w0[2], w1[2], w2[2], w3[2];
    constexpr bool ROWSPLIT = Q4;                         // 4-bit: waves split the rows of the tile, not K (kh names the row half)
    static_assert(!Q4 || MB <= 2, "one row block per wave");
    const bool q4_works = MB == 2 || kh == 0;             // 32-row tile: waves 4..7 only move activation tiles
    float sg0 = 0.f, sg1 = 0.f, sg2 = 0.f, sg3 = 0.f;     // ROWSPLIT: the group scales travel beside the two nibble vectors
    auto fetch_q = [&](u32x4 (&w)[2], float& sg, int kt) {
        w[0] = load16(wbase, lane16, (uint32_t)(kt * 2) * wstride_b);
        w[1] = load16(wbase, lane16, (uint32_t)(kt * 2 + 1) * wstride_b);
        sg = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(sbase, lane4, (uint32_t)kt * sstride_b, 0));
    };
    if constexpr (ROWSPLIT) {
        if (q4_works) {
            fetch_q(w0, sg0, 0);
            fetch_q(w1, sg1, 1);
            fetch_q(w2, sg2, 2);
            fetch_q(w3, sg3, 3);
        }
    } else {
        fetch_w(w0, 0);
        fetch_w(w1, 1);
    }
    u32x4 xa[XV], xb[XV];
    load_x<LIMBS, BM, XV>(xa, xbase, xoff, 0, tid);
    if constexpr (!Q4) load_x<LIMBS, BM, XV>(xb, xbase, xoff, min(1, nk - 1), tid);

    // epilogue operands, fetched now so that their latency hides behind the main loop
    const int oc = min(nbw * 32 + l32, dout - 1);
    float wscale = 0.f;
    u32x4 ubf[2][2];                                       // [ks][head, tail] fragments of U_B for this lane's channel
    if (!DUMP) {
        if (!Q4) wscale = as_global(it.scale)[oc];
        const uint16_t* bp = it.UB16 + (size_t)oc * 2 * rp + 8 * h;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            ubf[ks][0] = ubf[ks][1] = (u32x4){0, 0, 0, 0};
            if (ks * 16 < rp) {
                ubf[ks][0] = *as_global(reinterpret_cast<const u32x4*>(bp + ks * 16));
                ubf[ks][1] = *as_global(reinterpret_cast<const u32x4*>(bp + rp + ks * 16));
            }
        }
    }
    if (!DUMP) u_tile_finish<BM, EU>(it, a.flags, tid, tp, sb, mreg, tvec, Ms, utile);   // part 2 (one barrier inside)

    i32x16 acc[LIMBS][MB];
    f32x16 tot[MB];                                          // 4-bit only: group-scaled running totals
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
        for (int l = 0; l < LIMBS; ++l)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[l][mb][q] = 0;
#pragma unroll
        for (int q = 0; q < 16; ++q) tot[mb][q] = 0.f;
    }

    if constexpr (Q4) {
    if (!DUMP && tid < BM) xd[tid] = xdreg;
    store_x<LIMBS, BM, XV>(xa, smem, 0, tid);
    load_x<LIMBS, BM, XV>(xa, xbase, xoff, 1, tid);
    load_x<LIMBS, BM, XV>(xb, xbase, xoff, min(2, nk - 1), tid);
    __syncthreads();
    TSTAMP(1)
    // One step: multiply K tile kt (weights in W), refill W with tile kt+PD, move activation tile kt+1 (in XS)
    // into the other LDS stage and refill XS with tile kt+3.  Tile indices past the end are clamped: that data
    // is fetched again and never used.
    f32x16 trow = {0};                                    // ROWSPLIT: the wave's own row block (kh names the row half there)
#define ESSA_STEP(W, SG, XS, KTI)                                                    \
    {                                                                                \
        const int kt_ = (KTI);                                                       \
        if (q4_works) {                                                              \
            compute_tile_q4_rows<LIMBS, BM>(trow, W, SG, smem, kt_ & 1, MB == 2 ? kh : 0, l32, h); \
            fetch_q(W, SG, min(kt_ + PD, nk - 1));                                   \
        }                                                                            \
        store_x<LIMBS, BM, XV>(XS, smem, (kt_ + 1) & 1, tid);                        \
        __syncthreads();                                                             \
        load_x<LIMBS, BM, XV>(XS, xbase, xoff, min(kt_ + 3, nk - 1), tid);      \
    }
    for (int kt0 = 0; kt0 < nk; kt0 += PD) {
        ESSA_STEP(w0, sg0, xa, kt0)
        ESSA_STEP(w1, sg1, xb, kt0 + 1)
        ESSA_STEP(w2, sg2, xa, kt0 + 2)
        ESSA_STEP(w3, sg3, xb, kt0 + 3)
    }
#undef ESSA_STEP
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) tot[mb] = trow;        // the epilogue reads the block this wave finishes
    } else {
    // int8 weights.  The MFMAs of a K step run from fragments that were read during the previous step, and the one
    // barrier of a step sits between its two halves.  With four LDS stages (tile j in stage j % 4):
    //   first half (K chunk 0 of step kt): MFMAs interleaved with the LDS writes of tile kt+2 (loaded two steps ago)
    //   barrier: tile kt+1 is complete in LDS, and nobody reads tile kt-1's stage any more
    //   second half (K chunk 1): MFMAs interleaved with the fragment reads of tile kt+1; then the loads of weight
    //   tile kt+PD and activation tile kt+4
    // so no LDS or memory latency sits between two MFMAs of a wave.  (With only two stages tile kt+2 would be
    // written after the barrier instead, into the stage tile kt was read from; both tile heights have four.)
    // Tile indices past the end are clamped: that data is fetched again and never used.
    constexpr int NS = gemm_stages<MB, Q4>();
    constexpr bool EARLY = NS == 4;
    constexpr int NF = LIMBS * MB;                      // MFMAs per K chunk
    static_assert(!EARLY || NF >= XV, "one LDS write per MFMA slot");
    QSTAMP(4)
    if (!DUMP && tid < BM) xd[tid] = xdreg;
    store_x<LIMBS, BM, XV>(xa, smem, 0, tid);
    store_x<LIMBS, BM, XV>(xb, smem, 1, tid);
    QSTAMP(5)
    // the last loads before the loop, in the order the loop's own steps issue them (the compiler sizes the loop's
    // waits for the tighter of the two ways into it): activations before weights, so that waiting for an activation
    // tile (needed two steps after its load) never waits for the weight tile loaded in the same step (needed four
    // steps later) -- loads complete in order
    __builtin_amdgcn_sched_barrier(0);
    load_x<LIMBS, BM, XV>(xa, xbase, xoff, min(2, nk - 1), tid);
    __builtin_amdgcn_sched_barrier(0);
    fetch_w(w2, 2);
    __builtin_amdgcn_sched_barrier(0);
    load_x<LIMBS, BM, XV>(xb, xbase, xoff, min(3, nk - 1), tid);
    __builtin_amdgcn_sched_barrier(0);
    fetch_w(w3, 3);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    i32x4 fA[2][LIMBS][MB], fB[2][LIMBS][MB];
    read_frags<LIMBS, MB>(fA, smem, 0, kh, l32, h);
    TSTAMP(1)
#define ESSA_STEP(W, XS, KTI, SI, FC, FN)                                                                        \
    {                                                                                                            \
        const int kt_ = (KTI);                                                                                   \
        _Pragma("unroll") for (int i_ = 0; i_ < NF; ++i_) {                                                      \
            acc[i_ / MB][i_ % MB] = __builtin_amdgcn_mfma_i32_32x32x32_i8(FC[0][i_ / MB][i_ % MB], (i32x4)W[0],  \
                                                                          acc[i_ / MB][i_ % MB], 0, 0, 0);       \
            if (EARLY && i_ < XV) store_x_vec<LIMBS, BM>(XS[i_], smem, ((SI) + 2) % NS, tid, i_);   \
            __builtin_amdgcn_sched_barrier(0);                                                                   \
        }                                                                                                        \
        __syncthreads();                                                                                         \
        __builtin_amdgcn_sched_barrier(0);                                                                       \
        _Pragma("unroll") for (int i_ = 0; i_ < NF; ++i_) {                                                      \
            acc[i_ / MB][i_ % MB] = __builtin_amdgcn_mfma_i32_32x32x32_i8(FC[1][i_ / MB][i_ % MB], (i32x4)W[1],  \
                                                                          acc[i_ / MB][i_ % MB], 0, 0, 0);       \
            FN[0][i_ / MB][i_ % MB] = read_frag<LIMBS, BM>(smem, ((SI) + 1) % NS, 0, i_ / MB, i_ % MB, kh, l32, h); \
            FN[1][i_ / MB][i_ % MB] = read_frag<LIMBS, BM>(smem, ((SI) + 1) % NS, 1, i_ / MB, i_ % MB, kh, l32, h); \
            __builtin_amdgcn_sched_barrier(0);                                                                   \
        }                                                                                                        \
        if (!EARLY) store_x<LIMBS, BM, XV>(XS, smem, (SI) % NS, tid);                               \
        load_x<LIMBS, BM, XV>(XS, xbase, xoff, min(kt_ + 4, nk - 1), tid);                             \
        __builtin_amdgcn_sched_barrier(0);                                                                       \
        fetch_w(W, min(kt_ + PD, nk - 1));                                                             \
        __builtin_amdgcn_sched_barrier(0);                                                                       \
    }
    for (int kt0 = 0; kt0 < nk; kt0 += PD) {
        ESSA_STEP(w0, xa, kt0, 0, fA, fB)
        ESSA_STEP(w1, xb, kt0 + 1, 1, fB, fA)
        ESSA_STEP(w2, xa, kt0 + 2, 2, fA, fB)
        ESSA_STEP(w3, xb, kt0 + 3, 3, fB, fA)
    }
#undef ESSA_STEP
    __syncthreads();          // the stages become the exchange area
    }
    TSTAMP(2)

    // ---- epilogue 1: the two K halves exchange accumulators.  Half kh keeps row blocks with (mb & 1) == kh
    // (all of them when there is only one) and hands the others to its partner.  With two limbs each half first
    // folds them into one fp32 value, 256 hi + lo, so that half as many bytes cross the LDS (one more rounding of
    // 2^-24; the accumulator dump keeps its integers).
    // exchange slot (n, writer kh, limb, j): 16 x 64 ints, written as [q/4][lane] 16-byte vectors
    constexpr bool FSUM = Q4 || (LIMBS == 2 && !DUMP);       // one fp32 value per element travels instead of the limbs
    auto slot = [&](int n_, int kh_, int l_, int j_) { return smem + ((size_t)((n_ * 2 + kh_) * LIMBS + l_) * MBO + j_) * 4096; };
    if constexpr (!ROWSPLIT) {
    if (FSUM) {   // the values travel as bit patterns in the accumulator of limb 0
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                if (!Q4) tot[mb][q] = fmaf(256.0f, (float)acc[0][mb][q], (float)acc[LIMBS - 1][mb][q]);
                acc[0][mb][q] = (int)__float_as_uint(tot[mb][q]);
            }
    }
#pragma unroll
    for (int l = 0; l < (FSUM ? 1 : LIMBS); ++l)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const bool mine = MB >= 2 ? ((mb & 1) == kh) : (kh == 0);
            if (!mine) {
                unsigned char* dst = slot(nw, kh, l, MB >= 2 ? mb / 2 : 0);
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
                    *reinterpret_cast<i32x4*>(dst + (q4 * 64 + lane) * 16) =
                        (i32x4){acc[l][mb][4 * q4], acc[l][mb][4 * q4 + 1], acc[l][mb][4 * q4 + 2], acc[l][mb][4 * q4 + 3]};
            }
        }
    }
    __syncthreads();
    if constexpr (!ROWSPLIT) {
#pragma unroll
    for (int l = 0; l < (FSUM ? 1 : LIMBS); ++l)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const bool mine = MB >= 2 ? ((mb & 1) == kh) : (kh == 0);
            if (mine) {
                const unsigned char* src = slot(nw, kh ^ 1, l, MB >= 2 ? mb / 2 : 0);
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const i32x4 o4 = *reinterpret_cast<const i32x4*>(src + (q4 * 64 + lane) * 16);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        // fp32 values: always (K half 0) + (K half 1)
                        if (FSUM) tot[mb][4 * q4 + e] = kh == 0 ? tot[mb][4 * q4 + e] + __uint_as_float((uint32_t)o4[e])
                                                              : __uint_as_float((uint32_t)o4[e]) + tot[mb][4 * q4 + e];
                        else acc[l][mb][4 * q4 + e] += o4[e];
                    }
                }
            }
        }
    }
    if (DUMP) {
        const int o = (nb0 + nw) * 32 + l32;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const bool mine = MB >= 2 ? ((mb & 1) == kh) : (kh == 0);
            if (!mine) continue;
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int i = m0 + mb * 32 + 8 * (q >> 2) + 4 * h + (q & 3);
                if (i < R && o < dout) acc_out[(size_t)i * dout + o] = acc[0][mb][q];
            }
        }
        return;
    }
    const rv_piece<YBF16> rvp = load_rv_piece<YBF16>(it, nb0 * 32, tid);      // used by the very last step: on its way from here
    __syncthreads();   // exchange slots are read; the same memory now becomes the output tile
    TSTAMP(3)

    // ---- epilogue 2: scale, rank-r term, into the LDS output tile [BM][128 channels]
    constexpr int CROW = 128 * (YBF16 ? 2 : 4) + 16;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const bool mine = MB >= 2 ? ((mb & 1) == kh) : (kh == 0);
        if (!mine) continue;
        // fragments of u for the rank-r term: read now, used after the scaling arithmetic
        bf16x8 ua[2][2];
        {
            const unsigned char* up = utile + (size_t)(mb * 32 + l32) * UROW + 16 * h;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const int kso = ks * 16 < rp ? ks : 0;      // rank 16: the first fragments again, unused
                ua[ks][0] = *reinterpret_cast<const bf16x8*>(up + kso * 32);
                ua[ks][1] = *reinterpret_cast<const bf16x8*>(up + 2 * rp + kso * 32);
            }
        }
        f32x16 v;
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const int rl = mb * 32 + 8 * (q >> 2) + 4 * h + (q & 3);
            const float sc = xd[rl] * wscale;
            if (Q4) v[q] = tot[mb][q] * xd[rl];
            else if (FSUM) v[q] = tot[mb][q] * sc;
            else v[q] = (float)acc[0][mb][q] * sc;
            if (a.flags & ESSA_LORA_ONLY) v[q] = 0.f;
        }
        if (Q4 && !(a.flags & ESSA_LORA_ONLY)) {
            // zero-point term of the asymmetric format, - sum_g (s z)[o,g] * (delta_i * sum_{k in g} x^[i,k]): one more
            // low-rank product over the groups, bf16 head+tail operands straight from memory
            const int Gp = it.Gp;
            const uint16_t* xs = it.XS16 + (size_t)min(m0 + mb * 32 + l32, R - 1) * 2 * Gp + 8 * h;
            const uint16_t* sz = it.SZ16 + (size_t)(nbw * 32 + l32) * 2 * Gp + 8 * h;
            for (int ks = 0; ks < Gp / 16; ++ks) {
                const bf16x8 xa_hi = *as_global(reinterpret_cast<const bf16x8*>(xs + ks * 16));
                const bf16x8 xa_lo = *as_global(reinterpret_cast<const bf16x8*>(xs + Gp + ks * 16));
                const bf16x8 zb_hi = *as_global(reinterpret_cast<const bf16x8*>(sz + ks * 16));
                const bf16x8 zb_lo = *as_global(reinterpret_cast<const bf16x8*>(sz + Gp + ks * 16));
                v = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa_lo, zb_hi, v, 0, 0, 0);
                v = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa_hi, zb_lo, v, 0, 0, 0);
                v = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa_hi, zb_hi, v, 0, 0, 0);
            }
        }
        if (!(a.flags & ESSA_BASE_ONLY)) {
            // rank-r term U_B u_i: bf16 head+tail operands, lo*hi + hi*lo + hi*hi per 16 rank columns
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                if (ks * 16 < rp) {
                    const bf16x8 ub_hi = __builtin_bit_cast(bf16x8, ubf[ks][0]);
                    const bf16x8 ub_lo = __builtin_bit_cast(bf16x8, ubf[ks][1]);
                    v = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ua[ks][1], ub_hi, v, 0, 0, 0);
                    v = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ua[ks][0], ub_lo, v, 0, 0, 0);
                    v = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ua[ks][0], ub_hi, v, 0, 0, 0);
                }
            }
        }
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const int rl = mb * 32 + 8 * (q >> 2) + 4 * h + (q & 3);
            unsigned char* dst = smem + (size_t)rl * CROW + (nw * 32 + l32) * (YBF16 ? 2 : 4);
            if (YBF16) *reinterpret_cast<uint16_t*>(dst) = f32_to_bf16_bits(v[q]);
            else *reinterpret_cast<float*>(dst) = v[q];
        }
    }
    __syncthreads();
    TSTAMP(4)

    // ---- epilogue 3: the tile leaves as full rows, 16 bytes per thread where the output allows it
    store_ctile<YBF16, BM>(smem, it, m0, nb0 * 32, nb0 >> 2, tid, rvp);
    TSTAMP(5)
}

// ------------------------------------------------------------------------------------------------
// int8 weights at row counts up to 32 (the decode sizes bound by the weight stream): every CU streams weights.
// One workgroup per block of 32 output channels, all the rows (MB blocks of 32), the whole K; its 8 waves
// split K, wave w taking the chunks of 32 columns kc = w, w + 8, ...  There is no LDS and no barrier in the loop: a
// wave loads the weight block of its chunk (one kilobyte, operand order) and the activation limbs of the same chunk
// (operand tiles written by the prep kernel, one kilobyte per limb and row block) straight into MFMA operand
// registers, D chunks ahead.  What bounds a decode launch is the bytes its busiest CU takes in; here that is
// K x (32 + 2 R) instead of K x (128 + 2 x 32) on a quarter of the CUs (at 32 rows), and all 256 CUs pull on HBM.
// Loads past the wave's last chunk and the limb rows past R are sent out of the buffer's range: they return zeros
// without touching memory.
// After the loop the partial sums meet in LDS.  The integer sums of the chunks with kc % 4 in {0, 1} and in {2, 3} are
// each folded into one fp32 value (256 hi + lo) and the two are added in that order: exactly what the two K halves of
// the 32- and 64-row tiles of gemm_i8_kernel compute, so a row's result does not depend on which of them took it.
// Wave mb then finishes row block mb like the other kernels do (scale, rank-r term by bf16 head+tail MFMA steps).
// The reward partials, one per 128 channels, span four workgroups here: the launcher takes them in a pass of its own.
// ------------------------------------------------------------------------------------------------
template <int MB, int LIMBS>
constexpr size_t stream_smem_bytes() { return (size_t)8 * LIMBS * MB * 4096 + (size_t)MB * 4096 + (size_t)32 * MB * 4 + (size_t)32 * MB * UROW; }

template <int MB, int LIMBS, bool YBF16>
__global__ __launch_bounds__(NT, 1) void gemm_i8_stream_kernel(stream_args a) {
    constexpr int BM = 32 * MB;
    // A wave asks for the weights of NW of its chunks at once and then lets the activation limbs of those chunks stream past,
    // DX chunks ahead of their MFMAs.  A CU's loads complete in order: weights come from HBM, limbs out of the L2, and limb
    // loads issued between weight loads would each wait for the weight load in front of them.
    constexpr int NW = 16;                                 // 16 chunks per wave = 4096 columns: one bunch at the 7B and 8B shapes
    constexpr int DX = 4;
    constexpr size_t RED = (size_t)8 * LIMBS * MB * 4096;  // the 8 waves' partial sums; before the loop: t vectors and the core matrix
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    int* red = reinterpret_cast<int*>(smem);               // [wave][limb][row block][q][lane]
    float* totb = reinterpret_cast<float*>(smem + RED);    // [row block][q][lane] folded base sums
    float* xd = reinterpret_cast<float*>(smem + RED + (size_t)MB * 4096);
    unsigned char* utile = smem + RED + (size_t)MB * 4096 + BM * 4;
    float* tvec = reinterpret_cast<float*>(smem);
    float* Ms = tvec + BM * UTP;
    static_assert((size_t)(BM + 32) * UTP * 4 <= RED, "the prologue's matrices fit where the partial sums go later");

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, h = lane >> 5;
    TSTAMP(0)
    int g = 0;
#pragma unroll
    for (int i = 1; i < ESSA_MAX_GROUP; ++i) g += (i < a.n_items && (int)blockIdx.x >= a.tile_start[i]) ? 1 : 0;
    const fwd_item it = fetch_item(a.it[g]);
    const int nb = blockIdx.x - a.tile_start[g];           // this workgroup's block of 32 channels
    const int R = it.R, dout = it.d_out, dpad = it.d_in_pad, rp = it.rp;
    const int nkc = dpad >> 5;                             // chunks of 32 columns; a multiple of 16
    const int n = nkc >> 3;                                // chunks of this wave
    const uint32_t wstride_b = (uint32_t)it.n_blocks * 1024;
    const rsrc_t wbase = make_rsrc(reinterpret_cast<const unsigned char*>(it.Wt) + (size_t)nb * 1024);
    rsrc_t xbase[LIMBS];
#pragma unroll
    for (int l = 0; l < LIMBS; ++l) xbase[l] = make_rsrc(l == 0 ? it.Xh : it.Xl);
    constexpr uint32_t OUT_OF_RANGE = 0x80000000u;         // beyond the descriptor's 2 GB: the load returns zeros, no memory access
    const uint32_t lane16 = lane * 16;
    uint32_t xoff[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) xoff[mb] = (mb * 32 + l32 < R) ? (uint32_t)(mb * nkc) * 1024u + lane16 : OUT_OF_RANGE;

    // the small loads first (loads return in order): rank-space vectors, row units, this lane's channel scale and U_B
    constexpr int EU = (BM * 32 + NT - 1) / NT;
    f32x4 tp[EU][2];
    float sb[EU], mreg[2];
    u_tile_loads<BM, EU>(it, 0, tid, tp, sb, mreg);
    const float xdreg = as_global(it.xdelta)[min(min(tid, BM - 1), R - 1)];
    const int oc = min(nb * 32 + l32, dout - 1);
    const float wscale = as_global(it.scale)[oc];
    u32x4 ubf[2][2];
    {
        const uint16_t* bp = it.UB16 + (size_t)oc * 2 * rp + 8 * h;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            ubf[ks][0] = ubf[ks][1] = (u32x4){0, 0, 0, 0};
            if (ks * 16 < rp) {
                ubf[ks][0] = *as_global(reinterpret_cast<const u32x4*>(bp + ks * 16));
                ubf[ks][1] = *as_global(reinterpret_cast<const u32x4*>(bp + rp + ks * 16));
            }
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    TSTAMP(1)

    // chunk j of this wave is K chunk kc = wave + 8 j; a chunk past the last one is asked for outside the descriptor (zeros,
    // no memory access), and its products add nothing
    u32x4 wr[NW], xr[DX][LIMBS][MB];
    auto issue_w = [&](int j, int slot) {
        const uint32_t gone = j < n ? 0u : OUT_OF_RANGE;   // wave-uniform
        wr[slot] = load16(wbase, lane16 | gone, (uint32_t)(wave + 8 * j) * wstride_b);
    };
    auto issue_x = [&](int j, int slot) {
        const uint32_t gone = j < n ? 0u : OUT_OF_RANGE;
#pragma unroll
        for (int l = 0; l < LIMBS; ++l)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) xr[slot][l][mb] = load16(xbase[l], xoff[mb] | gone, (uint32_t)(wave + 8 * j) * 1024u);
    };
#pragma unroll
    for (int s = 0; s < NW; ++s) issue_w(s, s);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int s = 0; s < DX; ++s) issue_x(s, s);
    __builtin_amdgcn_sched_barrier(0);
    TSTAMP(2)

    u_tile_finish<BM, EU, true>(it, a.flags, tid, tp, sb, mreg, tvec, Ms, utile);
    if (tid < BM) xd[tid] = xdreg;
    TSTAMP(3)

    i32x16 acc[LIMBS][MB];
#pragma unroll
    for (int l = 0; l < LIMBS; ++l)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[l][mb][q] = 0;
    for (int j0 = 0; j0 < n; j0 += NW) {
        if (j0 > 0) {                                      // rows wider than 4096: the next bunch of weights, then its first limbs
#pragma unroll
            for (int s = 0; s < NW; ++s) issue_w(j0 + s, s);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int s = 0; s < DX; ++s) issue_x(j0 + s, s);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int s = 0; s < NW; ++s) {
#pragma unroll
            for (int l = 0; l < LIMBS; ++l)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
                    acc[l][mb] = __builtin_amdgcn_mfma_i32_32x32x32_i8((i32x4)xr[s % DX][l][mb], (i32x4)wr[s], acc[l][mb], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (s + DX < NW) issue_x(j0 + s + DX, s % DX);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    TSTAMP(4)
    lds_barrier();            // the prologue's matrices have been read by everyone: the area becomes the reduction slots
#pragma unroll
    for (int l = 0; l < LIMBS; ++l)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int q = 0; q < 16; ++q) red[(((wave * LIMBS + l) * MB + mb) * 16 + q) * 64 + lane] = acc[l][mb][q];
    lds_barrier();
    // element (row block, q, lane): the integer sums of the two K halves, folded and added as the other decode tiles do
#pragma unroll
    for (int i = 0; i < 2 * MB; ++i) {
        const int e = tid + NT * i, mb = e >> 10, ql = e & 1023;
        int sum[2][LIMBS];                                 // [K half][limb]
#pragma unroll
        for (int kh = 0; kh < 2; ++kh)
#pragma unroll
            for (int l = 0; l < LIMBS; ++l) {
                int t = 0;
#pragma unroll
                for (int wi = 0; wi < 4; ++wi) {
                    const int w = 2 * kh + (wi & 1) + 4 * (wi >> 1);       // K half 0: waves 0, 1, 4, 5 (kc % 4 in {0, 1}); half 1: 2, 3, 6, 7
                    t += red[((w * LIMBS + l) * MB + mb) * 1024 + ql];
                }
                sum[kh][l] = t;
            }
        float tot;
        if (LIMBS == 2) tot = fmaf(256.0f, (float)sum[0][0], (float)sum[0][1]) + fmaf(256.0f, (float)sum[1][0], (float)sum[1][1]);
        else tot = (float)(sum[0][0] + sum[1][0]);
        totb[e] = tot;
    }
    lds_barrier();
    if (wave >= MB) return;
    const int mb = wave;
    bf16x8 ua[2][2];
    {
        const unsigned char* up = utile + (size_t)(mb * 32 + l32) * UROW + 16 * h;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const int kso = ks * 16 < rp ? ks : 0;
            ua[ks][0] = *reinterpret_cast<const bf16x8*>(up + kso * 32);
            ua[ks][1] = *reinterpret_cast<const bf16x8*>(up + 2 * rp + kso * 32);
        }
    }
    f32x16 v;
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int rl = mb * 32 + 8 * (q >> 2) + 4 * h + (q & 3);
        const float sc = xd[rl] * wscale;
        v[q] = totb[(mb * 16 + q) * 64 + lane] * sc;
        if (a.flags & ESSA_LORA_ONLY) v[q] = 0.f;
    }
    if (!(a.flags & ESSA_BASE_ONLY)) {
        // rank-r term U_B u_i: bf16 head+tail operands, lo*hi + hi*lo + hi*hi per 16 rank columns
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            if (ks * 16 < rp) {
                const bf16x8 ub_hi = __builtin_bit_cast(bf16x8, ubf[ks][0]);
                const bf16x8 ub_lo = __builtin_bit_cast(bf16x8, ubf[ks][1]);
                v = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ua[ks][1], ub_hi, v, 0, 0, 0);
                v = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ua[ks][0], ub_lo, v, 0, 0, 0);
                v = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ua[ks][0], ub_hi, v, 0, 0, 0);
            }
        }
    }
    // 32 consecutive channels of a row sit in 32 consecutive lanes: 64 or 128 contiguous bytes per store instruction
    const int o = nb * 32 + l32;
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int i = mb * 32 + 8 * (q >> 2) + 4 * h + (q & 3);
        if (i < R && o < dout) {
            if (YBF16) __builtin_nontemporal_store(f32_to_bf16_bits(v[q]), as_global_w(reinterpret_cast<uint16_t*>(it.Y)) + (size_t)i * dout + o);
            else __builtin_nontemporal_store(v[q], as_global_w(reinterpret_cast<float*>(it.Y)) + (size_t)i * dout + o);
        }
    }
    TSTAMP(5)
}

// ------------------------------------------------------------------------------------------------
// 4-bit weights, once the group fills the chip with tiles of 64 rows x 256 channels.  What bounds this format next to
// the vector-ALU scaling is the number of 128-byte requests a workgroup sends to the L2 per K tile; with 256 channels
// per tile the activation limbs (as many bytes per K tile as the nibbles of 256 channels) are asked for half as often
// as with 128.  Wave n owns channels 32n.. of the tile for both blocks of 32 rows, over the whole K tile: per row
// block the hi-limb MFMAs, a shift by 8 of their sums, the lo-limb MFMAs on top of them, then one conversion and one
// FMA with the group's scale per output -- the same integer sum and the same fp32 operations as the narrower tiles,
// so a row's result does not depend on which kernel took it.  Registers are capped at 128: two workgroups share a CU
// and overlap each other's MFMA, scaling and LDS phases (the loop itself runs them one after the other).
// ------------------------------------------------------------------------------------------------
constexpr int QW_NB = 8;           // 32-channel blocks per tile

template <int LIMBS, bool YBF16, int RB>
constexpr size_t q4w_smem_bytes() {
    constexpr int QW_BM = 32 * RB;
    constexpr size_t stages = (size_t)2 * LIMBS * QW_BM * LROW;
    constexpr size_t pre = stages + (size_t)QW_BM * UTP * 4 + 32 * UTP * 4;
    constexpr size_t ctile = (size_t)QW_BM * (128 * (YBF16 ? 2 : 4) + 16);
    constexpr size_t big = pre > ctile ? pre : ctile;
    return big + QW_BM * 4 + (size_t)QW_BM * UROW;
}

template <int LIMBS, bool YBF16, int RB>
__device__ __forceinline__ void q4w_tile(const stream_args& a, const fwd_item& it, const int m0, const int nb0) {
    constexpr int BM = 32 * RB;
    constexpr int XV = (LIMBS * BM * 8 + NT - 1) / NT;
    constexpr size_t BIG = q4w_smem_bytes<LIMBS, YBF16, RB>() - BM * 4 - (size_t)BM * UROW;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float* xd = reinterpret_cast<float*>(smem + BIG);
    unsigned char* utile = smem + BIG + BM * 4;

    const int R = it.R, dout = it.d_out, dpad = it.d_in_pad, rp = it.rp;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, h = lane >> 5;
    const int nk = dpad / KT;
    const int nbw = min(nb0 + wave, it.n_blocks - 1);      // a wave past the last block repeats it; nothing of it is stored
    const uint32_t wstride_b = (uint32_t)it.n_blocks * 1024;
    const rsrc_t wbase = make_rsrc(reinterpret_cast<const unsigned char*>(it.Wt) + (size_t)nbw * 1024);
    const rsrc_t sbase = make_rsrc(it.St + (size_t)nbw * 32);
    const uint32_t sstride_b = (uint32_t)it.n_blocks * 32 * 4;
    const uint32_t lane16 = lane * 16, lane4 = l32 * 4;
    uint32_t xoff[XV];
    x_lane_offsets<LIMBS, BM, XV>(xoff, dpad, tid);
    rsrc_t xbase[XV];
#pragma unroll
    for (int e = 0; e < XV; ++e) {
        const int limb = (wave * 64 + NT * e) / (BM * 8);
        xbase[e] = make_rsrc((limb == 0 ? it.Xh : it.Xl) + (size_t)m0 * dpad);
    }
    auto fetch_q = [&](u32x4 (&w)[2], float& sg, int kt) {
        w[0] = load16(wbase, lane16, (uint32_t)(kt * 2) * wstride_b);
        w[1] = load16(wbase, lane16, (uint32_t)(kt * 2 + 1) * wstride_b);
        sg = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(sbase, lane4, (uint32_t)kt * sstride_b, 0));
    };

    // rank-space vectors of the tile's rows and the rows' fixed-point units, then the first tiles
    constexpr size_t STG = (size_t)2 * LIMBS * BM * LROW;
    float* tvec = reinterpret_cast<float*>(smem + STG);
    float* Ms = tvec + BM * UTP;
    constexpr int EU = (BM * 32 + NT - 1) / NT;
    u32x4 w0[2], w1[2], xa[XV], xb[XV];
    float sg0, sg1;
    {
        f32x4 tp[EU][2];
        float sbv[EU], mreg[2];
        u_tile_loads<BM, EU>(it, m0, tid, tp, sbv, mreg);
        const float xdreg = as_global(it.xdelta)[min(m0 + min(tid, BM - 1), R - 1)];
        fetch_q(w0, sg0, 0);
        fetch_q(w1, sg1, min(1, nk - 1));
        load_x<LIMBS, BM, XV>(xa, xbase, xoff, 0, tid);
        u_tile_finish<BM, EU>(it, a.flags, tid, tp, sbv, mreg, tvec, Ms, utile);
        if (tid < BM) xd[tid] = xdreg;
    }
    store_x<LIMBS, BM, XV>(xa, smem, 0, tid);
    load_x<LIMBS, BM, XV>(xa, xbase, xoff, min(1, nk - 1), tid);
    load_x<LIMBS, BM, XV>(xb, xbase, xoff, min(2, nk - 1), tid);
    __syncthreads();

    f32x16 tot[RB];
#pragma unroll
    for (int mb = 0; mb < RB; ++mb)
#pragma unroll
        for (int q = 0; q < 16; ++q) tot[mb][q] = 0.f;
    const u32x4 m4 = {0x0f0f0f0fu, 0x0f0f0f0fu, 0x0f0f0f0fu, 0x0f0f0f0fu};
    constexpr int FD = 3;                                 // fragments in flight ahead of their MFMA
    const i32x16 zero = {0};
    // One step: multiply K tile kt (weights in W), refill W with tile kt+2, move activation tile kt+1 (in XS) into the
    // other LDS stage and refill XS with tile kt+3.  Tile indices past the end are clamped: fetched again, never used.
#define Q4W_STEP(W, SG, XS, KTI)                                                                                   \
    {                                                                                                              \
        const int kt_ = (KTI);                                                                                     \
        const i32x4 wq_[4] = {(i32x4)(W[0] & m4), (i32x4)((W[0] >> 4) & m4), (i32x4)(W[1] & m4), (i32x4)((W[1] >> 4) & m4)}; \
        const unsigned char* st_ = smem + (size_t)((kt_ & 1) * LIMBS) * BM * LROW + (size_t)l32 * LROW + 16 * h;    \
        /* the step's fragments in the order of their MFMAs (row block, limb, chunk), read FD ahead of their use */ \
        constexpr int NFR_ = RB * LIMBS * 4;                                                                       \
        i32x4 fr_[FD];                                                                                             \
        _Pragma("unroll") for (int i_ = 0; i_ < FD; ++i_)                                                          \
            fr_[i_] = *reinterpret_cast<const i32x4*>(st_ + (size_t)(((i_ >> 2) % LIMBS) * BM + (i_ / (4 * LIMBS)) * 32) * LROW + (i_ & 3) * 32); \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        i32x16 t_ = zero;                                                                                          \
        _Pragma("unroll") for (int i_ = 0; i_ < NFR_; ++i_) {                                                      \
            const int mb_ = i_ / (4 * LIMBS), l_ = (i_ >> 2) % LIMBS, c_ = i_ & 3;                                 \
            if (c_ == 0 && l_ == 0) t_ = zero;                                                                     \
            if (c_ == 0 && l_ == 1) { _Pragma("unroll") for (int q = 0; q < 16; ++q) t_[q] <<= 8; }                \
            t_ = __builtin_amdgcn_mfma_i32_32x32x32_i8(fr_[i_ % FD], wq_[c_], t_, 0, 0, 0);                        \
            if (i_ + FD < NFR_) {                                                                                  \
                const int n_ = i_ + FD;                                                                            \
                fr_[i_ % FD] = *reinterpret_cast<const i32x4*>(st_ + (size_t)(((n_ >> 2) % LIMBS) * BM + (n_ / (4 * LIMBS)) * 32) * LROW + (n_ & 3) * 32); \
            }                                                                                                      \
            __builtin_amdgcn_sched_barrier(0);                                                                     \
            if (c_ == 3 && l_ == LIMBS - 1) {                                                                      \
                _Pragma("unroll") for (int q = 0; q < 16; ++q) tot[mb_][q] = fmaf(SG, (float)t_[q], tot[mb_][q]);  \
                __builtin_amdgcn_sched_barrier(0);                                                                 \
            }                                                                                                      \
        }                                                                                                          \
        fetch_q(W, SG, min(kt_ + 2, nk - 1));                                                                      \
        store_x<LIMBS, BM, XV>(XS, smem, (kt_ + 1) & 1, tid);                                                      \
        __syncthreads();                                                                                           \
        load_x<LIMBS, BM, XV>(XS, xbase, xoff, min(kt_ + 3, nk - 1), tid);                                         \
    }
    for (int kt0 = 0; kt0 < nk; kt0 += 2) {                // d_in_pad is a multiple of 512: nk is even
        Q4W_STEP(w0, sg0, xa, kt0)
        Q4W_STEP(w1, sg1, xb, kt0 + 1)
    }
#undef Q4W_STEP

    // ---- epilogue, one half of the tile (128 channels, four waves) at a time
    constexpr int CROW = 128 * (YBF16 ? 2 : 4) + 16;
    const int oc = min(nbw * 32 + l32, dout - 1);
    u32x4 ubf[2][2];
    {
        const uint16_t* bp = it.UB16 + (size_t)oc * 2 * rp + 8 * h;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            ubf[ks][0] = ubf[ks][1] = (u32x4){0, 0, 0, 0};
            if (ks * 16 < rp) {
                ubf[ks][0] = *as_global(reinterpret_cast<const u32x4*>(bp + ks * 16));
                ubf[ks][1] = *as_global(reinterpret_cast<const u32x4*>(bp + rp + ks * 16));
            }
        }
    }
#pragma unroll 1
    for (int half = 0; half < 2; ++half) {
        const rv_piece<YBF16> rvp = load_rv_piece<YBF16>(it, nb0 * 32 + half * 128, tid);
        if ((wave >> 2) == half) {
#pragma unroll
            for (int mb = 0; mb < RB; ++mb) {
                f32x16 v;
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int rl = mb * 32 + 8 * (q >> 2) + 4 * h + (q & 3);
                    v[q] = (a.flags & ESSA_LORA_ONLY) ? 0.f : tot[mb][q] * xd[rl];
                }
                if (!(a.flags & ESSA_LORA_ONLY)) {
                    // zero-point term of the asymmetric format, - sum_g (s z)[o,g] * (delta_i * sum_{k in g} x^[i,k]): one more
                    // low-rank product over the groups, bf16 head+tail operands straight from memory
                    const int Gp = it.Gp;
                    const uint16_t* xs = it.XS16 + (size_t)min(m0 + mb * 32 + l32, R - 1) * 2 * Gp + 8 * h;
                    const uint16_t* sz = it.SZ16 + (size_t)(nbw * 32 + l32) * 2 * Gp + 8 * h;
                    for (int ks = 0; ks < Gp / 16; ++ks) {
                        const bf16x8 xa_hi = *as_global(reinterpret_cast<const bf16x8*>(xs + ks * 16));
                        const bf16x8 xa_lo = *as_global(reinterpret_cast<const bf16x8*>(xs + Gp + ks * 16));
                        const bf16x8 zb_hi = *as_global(reinterpret_cast<const bf16x8*>(sz + ks * 16));
                        const bf16x8 zb_lo = *as_global(reinterpret_cast<const bf16x8*>(sz + Gp + ks * 16));
                        v = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa_lo, zb_hi, v, 0, 0, 0);
                        v = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa_hi, zb_lo, v, 0, 0, 0);
                        v = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa_hi, zb_hi, v, 0, 0, 0);
                    }
                }
                if (!(a.flags & ESSA_BASE_ONLY)) {
                    // rank-r term U_B u_i: bf16 head+tail operands, lo*hi + hi*lo + hi*hi per 16 rank columns
                    const unsigned char* up = utile + (size_t)(mb * 32 + l32) * UROW + 16 * h;
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) {
                        if (ks * 16 < rp) {
                            const bf16x8 ua_hi = *reinterpret_cast<const bf16x8*>(up + ks * 32);
                            const bf16x8 ua_lo = *reinterpret_cast<const bf16x8*>(up + 2 * rp + ks * 32);
                            const bf16x8 ub_hi = __builtin_bit_cast(bf16x8, ubf[ks][0]);
                            const bf16x8 ub_lo = __builtin_bit_cast(bf16x8, ubf[ks][1]);
                            v = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ua_lo, ub_hi, v, 0, 0, 0);
                            v = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ua_hi, ub_lo, v, 0, 0, 0);
                            v = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ua_hi, ub_hi, v, 0, 0, 0);
                        }
                    }
                }
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int rl = mb * 32 + 8 * (q >> 2) + 4 * h + (q & 3);
                    unsigned char* dst = smem + (size_t)rl * CROW + ((wave & 3) * 32 + l32) * (YBF16 ? 2 : 4);
                    if (YBF16) *reinterpret_cast<uint16_t*>(dst) = f32_to_bf16_bits(v[q]);
                    else *reinterpret_cast<float*>(dst) = v[q];
                }
            }
        }
        __syncthreads();
        store_ctile<YBF16, BM>(smem, it, m0, nb0 * 32 + half * 128, (nb0 >> 2) + half, tid, rvp);
        __syncthreads();
    }
}

// The grid: the 64-row tiles of all items, then the 32-row tiles of all items.  The launcher gives the rows of a last,
// sparsely filled round of 64-row tiles to 32-row tiles instead: a round in which one workgroup sits alone on a CU has
// nobody to overlap its phases with, and twice as many workgroups of half the height finish it in about half the time.
// A row's result does not depend on the height of its tile.
template <int LIMBS, bool YBF16>
__global__ __launch_bounds__(NT, 4) void gemm_q4_wide_kernel(stream_args a) {
    const int nbig = a.tile_start[a.n_items];
    const bool small = (int)blockIdx.x >= nbig;
    const int bb = small ? (int)blockIdx.x - nbig : (int)blockIdx.x;
    int g = 0;
#pragma unroll
    for (int i = 1; i < ESSA_MAX_GROUP; ++i) g += (i < a.n_items && bb >= (small ? a.q4_small_start[i] : a.tile_start[i])) ? 1 : 0;
    const fwd_item it = fetch_item(a.it[g]);
    const int start = small ? a.q4_small_start[g] : a.tile_start[g];
    const int ntile = (small ? a.q4_small_start[g + 1] : a.tile_start[g + 1]) - start;
    int tile = bb - start;
    if ((ntile & 7) == 0 && ((start + (small ? nbig : 0)) & 7) == 0) tile = (tile & 7) * (ntile >> 3) + (tile >> 3);   // an XCD takes a contiguous range of tiles
    const int big_rows = min(a.q4_big_rows, (it.R + 63) / 64 * 64);
    if (!small) {
        const int tiles_m = big_rows / 64;
        q4w_tile<LIMBS, YBF16, 2>(a, it, (tile % tiles_m) * 64, (tile / tiles_m) * QW_NB);
    } else {
        const int tiles_m = (it.R - big_rows + 31) / 32;
        q4w_tile<LIMBS, YBF16, 1>(a, it, big_rows + (tile % tiles_m) * 32, (tile / tiles_m) * QW_NB);
    }
}

// ------------------------------------------------------------------------------------------------
// The same product for prefill-sized row counts.  Tile = 128 rows x 256 channels; the 8 waves form a 2 (rows) x 4
// (channels) grid and each owns a 64 x 64 patch, i.e. 2 x 2 MFMA blocks per limb with no K split: every activation
// fragment meets two weight fragments and every weight fragment four activation fragments (both limbs), so a K
// chunk costs 6 LDS fragment reads for 8 MFMAs.  Both operands go through LDS here (a weight block is needed by two
// waves): per K step of 64 a workgroup brings in 16 KB of limbs and 16 KB of weights for 1024 MFMA cycles per SIMD,
// half the load per MFMA of the decode tile.  Weight blocks keep their pre-tiled operand order in LDS (1 KB each,
// read back as one contiguous kilobyte per wave); activation rows are 64 bytes with their four 16-byte parts
// XOR-swizzled by the row, so that both the row-wise writes and the fragment reads are free of bank conflicts.
// One step: fragments of chunk 0 <- LDS; MFMAs of chunk 0 interleaved with the fragment reads of chunk 1; tile kt+1
// (in registers since two steps ago) -> the other LDS stage; loads of tile kt+3 into those registers; MFMAs of
// chunk 1; barrier.
// ------------------------------------------------------------------------------------------------
// events of the launch being timed (set by forward_stream around its GEMM launch, null otherwise)
thread_local hipEvent_t tl_ev_start = nullptr, tl_ev_stop = nullptr;

constexpr int BK = 64;             // K per step
constexpr int BXROW = BK;          // LDS pitch of an activation row: no padding, the four 16-byte parts of row r sit at part ^ ((r >> 2) & 3)
constexpr int BIG_BM = 128;        // rows per tile
constexpr int BIG_NB = 8;          // 32-channel blocks per tile (256 channels)

template <int LIMBS>
constexpr size_t big_stage_bytes() { return (size_t)LIMBS * BIG_BM * BXROW + 2 * BIG_NB * 1024; }

template <int LIMBS, bool YBF16>
constexpr size_t big_smem_bytes() {
    constexpr size_t stages = 3 * big_stage_bytes<LIMBS>();
    constexpr size_t ctile = (size_t)BIG_BM * (128 * (YBF16 ? 2 : 4) + 16);
    constexpr size_t pre = stages + (size_t)BIG_BM * UTP * 4 + 32 * UTP * 4;
    constexpr size_t big = pre > ctile ? pre : ctile;
    return big + BIG_BM * 4 + (size_t)BIG_BM * UROW;
}

template <int LIMBS, bool YBF16, bool DUMP = false>
__global__ __launch_bounds__(NT) void gemm_i8_big_kernel(stream_args a, int32_t* __restrict__ acc_out) {
    constexpr int BM = BIG_BM;
    constexpr size_t STAGE = big_stage_bytes<LIMBS>();
    constexpr size_t WOFF = (size_t)LIMBS * BM * BXROW;                // weight blocks inside a stage
    constexpr size_t BIG = big_smem_bytes<LIMBS, YBF16>() - BM * 4 - (size_t)BM * UROW;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float* xd = reinterpret_cast<float*>(smem + BIG);                  // [BM] value of one fixed-point unit per row
    unsigned char* utile = smem + BIG + BM * 4;                        // [BM][UROW] bf16 head+tail of u_i

    int g = 0;
#pragma unroll
    for (int i = 1; i < ESSA_MAX_GROUP; ++i) g += (i < a.n_items && (int)blockIdx.x >= a.tile_start[i]) ? 1 : 0;
    const fwd_item it = fetch_item(a.it[g]);
    const int R = it.R, dout = it.d_out, dpad = it.d_in_pad, rp = it.rp;
    const int tiles_m = (R + BM - 1) / BM, tiles_n = (it.n_blocks + BIG_NB - 1) / BIG_NB;
    // blocks go round-robin over the 8 XCDs: give each XCD a contiguous range of tiles, and inside it walk patches of
    // 4 row tiles x all column tiles, column tile fastest, so that the 32 workgroups an XCD runs at a time share a
    // few activation and weight tiles behind its L2
    const int ntile = a.tile_start[g + 1] - a.tile_start[g];
    int tile = blockIdx.x - a.tile_start[g];
    if ((ntile & 7) == 0 && (a.tile_start[g] & 7) == 0) tile = (tile & 7) * (ntile >> 3) + (tile >> 3);
    int tm, tn;
    {
        const int per_group = 4 * tiles_n, grp = tile / per_group, rem = tile % per_group;
        const int rows_in_group = min(4, tiles_m - 4 * grp);               // the last group may hold fewer row tiles
        tn = rem / rows_in_group;
        tm = 4 * grp + rem % rows_in_group;
    }
    const int m0 = tm * BM, nb0 = tn * BIG_NB;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave >> 2, wc = wave & 3;
    const int l32 = lane & 31, h = lane >> 5;
    const int nk = dpad / BK;                                          // even: d_in_pad is a multiple of 512
    TSTAMP(0)

    // global -> LDS staging.  Activations: vector e of thread tid is 16-byte part (tid & 3) of row (tid >> 2) of limb e.
    // Weights: vector e of wave w is K chunk e of the step, 32-channel block w of the tile (one kilobyte per wave).
    rsrc_t xres[LIMBS];
#pragma unroll
    for (int e = 0; e < LIMBS; ++e) xres[e] = make_rsrc((e == 0 ? it.Xh : it.Xl) + (size_t)m0 * dpad);
    const uint32_t xoff = (uint32_t)(tid >> 2) * (uint32_t)dpad + (tid & 3) * 16;
    const uint32_t xdst = (uint32_t)(tid >> 2) * BXROW + (((tid & 3) ^ ((tid >> 4) & 3)) * 16);
    const uint32_t wstride_b = (uint32_t)it.n_blocks * 1024;
    const rsrc_t wres = make_rsrc(reinterpret_cast<const unsigned char*>(it.Wt) + (size_t)min(nb0 + wave, it.n_blocks - 1) * 1024);
    const uint32_t lane16 = lane * 16;
    const uint32_t wdst = (uint32_t)WOFF + wave * 1024 + lane16;

    // two register sets: tile kt+1 waits in one (loaded two steps ago) while tile kt+2 is on its way into the other
    u32x4 xs0[LIMBS], ws0[2], xs1[LIMBS], ws1[2];
    auto load_tile = [&](u32x4 (&xs)[LIMBS], u32x4 (&ws)[2], int kt) {
#pragma unroll
        for (int e = 0; e < LIMBS; ++e) xs[e] = load16(xres[e], xoff, (uint32_t)kt * BK);
#pragma unroll
        for (int e = 0; e < 2; ++e) ws[e] = load16(wres, lane16, (uint32_t)(kt * 2 + e) * wstride_b);
    };
    auto store_tile = [&](const u32x4 (&xs)[LIMBS], const u32x4 (&ws)[2], uint32_t stage_off) {
        unsigned char* sb_ = smem + stage_off;
#pragma unroll
        for (int e = 0; e < LIMBS; ++e) *reinterpret_cast<u32x4*>(sb_ + (size_t)e * BM * BXROW + xdst) = xs[e];
#pragma unroll
        for (int e = 0; e < 2; ++e) *reinterpret_cast<u32x4*>(sb_ + wdst + (size_t)e * BIG_NB * 1024) = ws[e];
    };

    // rank-space vectors of the tile's rows, and the rows' fixed-point units
    float* tvec = reinterpret_cast<float*>(smem + 3 * STAGE);
    float* Ms = tvec + BM * UTP;
    constexpr int EU = (BM * 32 + NT - 1) / NT;
    if constexpr (DUMP) {
        load_tile(xs0, ws0, 0);                             // accumulator dump: no rank-space work, no scales
    } else if (a.u_ready) {
        // the prep kernel has left the finished rows of u (bf16 head, then tail: 4 rp bytes per row): a plain copy
        const int ppr = rp / 4;                                      // 16-byte pieces per row
        u32x4 up[2];
        const gptr<const u32x4> usrc = as_global(reinterpret_cast<const u32x4*>(it.U16));
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int p_ = min(tid + NT * i, BM * ppr - 1), row = p_ / ppr, pc = p_ % ppr;
            up[i] = usrc[(size_t)min(m0 + row, R - 1) * ppr + pc];
        }
        const float xdreg = as_global(it.xdelta)[min(m0 + min(tid, BM - 1), R - 1)];
        load_tile(xs0, ws0, 0);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int p_ = tid + NT * i;
            if (p_ < BM * ppr) *reinterpret_cast<u32x4*>(utile + (size_t)(p_ / ppr) * UROW + (p_ % ppr) * 16) = up[i];
        }
        if (tid < BM) xd[tid] = xdreg;
    } else {
        f32x4 tp[EU][2];
        float sbv[EU], mreg[2];
        u_tile_loads<BM, EU>(it, m0, tid, tp, sbv, mreg);
        const float xdreg = as_global(it.xdelta)[min(m0 + min(tid, BM - 1), R - 1)];
        load_tile(xs0, ws0, 0);
        u_tile_finish<BM, EU>(it, a.flags, tid, tp, sbv, mreg, tvec, Ms, utile);
        if (tid < BM) xd[tid] = xdreg;
    }
    // tiles 0 and 1 go to stages 0 and 1; tiles 2 and 3 wait in the two register sets
    load_tile(xs1, ws1, min(1, nk - 1));
    store_tile(xs0, ws0, 0);
    store_tile(xs1, ws1, (uint32_t)STAGE);
    __builtin_amdgcn_sched_barrier(0);
    load_tile(xs0, ws0, min(2, nk - 1));          // in the order the loop's steps issue them (even tile, then odd tile)
    __builtin_amdgcn_sched_barrier(0);
    load_tile(xs1, ws1, min(3, nk - 1));
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();

    i32x16 acc[LIMBS][2][2];
#pragma unroll
    for (int l = 0; l < LIMBS; ++l)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int q = 0; q < 16; ++q) acc[l][mb][nb][q] = 0;

    // fragment addresses of this lane inside a stage
    const uint32_t afrag = (uint32_t)(wr * 64 + l32) * BXROW;                          // + (l * BM + mb * 32) * BXROW + swizzled part
    const uint32_t asw = (l32 >> 2) & 3;                                               // rows 32 apart share the swizzle
    const uint32_t bfrag = (uint32_t)WOFF + (uint32_t)(wc * 2) * 1024 + lane16;       // + (c * BIG_NB + nb) * 1024
    constexpr int NA = LIMBS * 2;                       // activation fragments per chunk
    i32x4 fa0[NA], fb0[2], fa1[NA], fb1[2];
#define BIG_READ_A(F, SOFF, C, I) F[I] = *reinterpret_cast<const i32x4*>(smem + (SOFF) + afrag + (size_t)(((I) >> 1) * BM + ((I) & 1) * 32) * BXROW + ((((C) * 2 + h) ^ asw) * 16))
#define BIG_READ_B(F, SOFF, C, I) F[I] = *reinterpret_cast<const i32x4*>(smem + (SOFF) + bfrag + (size_t)((C) * BIG_NB + (I)) * 1024)
    // tile j lives in stage j % 3.  One step (tile kt): MFMAs of chunk 0 (fragments read during the previous step)
    // interleaved with the fragment reads of chunk 1; tile kt+2 (in registers since two steps ago) -> the stage tile
    // kt-1 has left; loads of tile kt+4; MFMAs of chunk 1 interleaved with the reads of chunk 0 of tile kt+1 (complete
    // in LDS since the last barrier); barrier.  No LDS or memory latency sits between the barrier and the next MFMA.
    uint32_t s_cur = 0, s_nxt = (uint32_t)STAGE, s_wr = 2 * (uint32_t)STAGE;
    _Pragma("unroll") for (int i_ = 0; i_ < NA; ++i_) BIG_READ_A(fa0, s_cur, 0, i_);
    _Pragma("unroll") for (int i_ = 0; i_ < 2; ++i_) BIG_READ_B(fb0, s_cur, 0, i_);
#define BIG_STEP(KTI, XS, WS)                                                                                  \
    {                                                                                                          \
        const int kt_ = (KTI);                                                                                 \
        _Pragma("unroll") for (int i_ = 0; i_ < NA * 2; ++i_) {                                                \
            acc[i_ >> 2][(i_ >> 1) & 1][i_ & 1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(                       \
                fa0[i_ >> 1], fb0[i_ & 1], acc[i_ >> 2][(i_ >> 1) & 1][i_ & 1], 0, 0, 0);                      \
            if (i_ < NA) BIG_READ_A(fa1, s_cur, 1, i_);                                                        \
            else if (i_ < NA + 2) BIG_READ_B(fb1, s_cur, 1, i_ - NA);                                          \
            __builtin_amdgcn_sched_barrier(0);                                                                 \
        }                                                                                                      \
        store_tile(XS, WS, s_wr);                                                                              \
        __builtin_amdgcn_sched_barrier(0);                                                                     \
        load_tile(XS, WS, min(kt_ + 4, nk - 1));                                                               \
        __builtin_amdgcn_sched_barrier(0);                                                                     \
        _Pragma("unroll") for (int i_ = 0; i_ < NA * 2; ++i_) {                                                \
            acc[i_ >> 2][(i_ >> 1) & 1][i_ & 1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(                       \
                fa1[i_ >> 1], fb1[i_ & 1], acc[i_ >> 2][(i_ >> 1) & 1][i_ & 1], 0, 0, 0);                      \
            if (i_ < NA) BIG_READ_A(fa0, s_nxt, 0, i_);                                                        \
            else if (i_ < NA + 2) BIG_READ_B(fb0, s_nxt, 0, i_ - NA);                                          \
            __builtin_amdgcn_sched_barrier(0);                                                                 \
        }                                                                                                      \
        __syncthreads();                                                                                       \
        __builtin_amdgcn_sched_barrier(0);                                                                     \
        { const uint32_t t_ = s_cur; s_cur = s_nxt; s_nxt = s_wr; s_wr = t_; }                                 \
    }
    TSTAMP(1)
    for (int kt0 = 0; kt0 < nk; kt0 += 2) {
        BIG_STEP(kt0, xs0, ws0)
        BIG_STEP(kt0 + 1, xs1, ws1)
    }
    TSTAMP(2)
#undef BIG_STEP
#undef BIG_READ_A
#undef BIG_READ_B

    if constexpr (DUMP) {
        // test hook: the raw int32 sums of the (single) limb, element (row, channel) of this lane's accumulators
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                const int o = (nb0 + wc * 2 + nb) * 32 + l32;
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int i = m0 + wr * 64 + mb * 32 + 8 * (q >> 2) + 4 * h + (q & 3);
                    if (i < R && o < dout) acc_out[(size_t)i * dout + o] = acc[0][mb][nb][q];
                }
            }
        return;
    }
    // ---- epilogue, one half of the tile (128 channels) at a time: scale, rank-r term, LDS output tile, store
    constexpr int CROW = 128 * (YBF16 ? 2 : 4) + 16;
#pragma unroll 1
    for (int half = 0; half < 2; ++half) {
        const rv_piece<YBF16> rvp = load_rv_piece<YBF16>(it, nb0 * 32 + half * 128, tid);
        if ((wc >> 1) == half) {
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                const int oc = min((nb0 + wc * 2 + nb) * 32 + l32, dout - 1);
                const float wscale = as_global(it.scale)[oc];
                u32x4 ubf[2][2];
                const uint16_t* bp = it.UB16 + (size_t)oc * 2 * rp + 8 * h;
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    ubf[ks][0] = ubf[ks][1] = (u32x4){0, 0, 0, 0};
                    if (ks * 16 < rp) {
                        ubf[ks][0] = *as_global(reinterpret_cast<const u32x4*>(bp + ks * 16));
                        ubf[ks][1] = *as_global(reinterpret_cast<const u32x4*>(bp + rp + ks * 16));
                    }
                }
#pragma unroll
                for (int mb = 0; mb < 2; ++mb) {
                    f32x16 v;
#pragma unroll
                    for (int q = 0; q < 16; ++q) {
                        const int rl = wr * 64 + mb * 32 + 8 * (q >> 2) + 4 * h + (q & 3);
                        const float sc = xd[rl] * wscale;
                        if (LIMBS == 2) v[q] = fmaf(256.0f, (float)acc[0][mb][nb][q], (float)acc[LIMBS - 1][mb][nb][q]) * sc;
                        else v[q] = (float)acc[0][mb][nb][q] * sc;
                        if (a.flags & ESSA_LORA_ONLY) v[q] = 0.f;
                    }
                    if (!(a.flags & ESSA_BASE_ONLY)) {
                        // rank-r term U_B u_i: bf16 head+tail operands, lo*hi + hi*lo + hi*hi per 16 rank columns
                        const unsigned char* up = utile + (size_t)(wr * 64 + mb * 32 + l32) * UROW + 16 * h;
#pragma unroll
                        for (int ks = 0; ks < 2; ++ks) {
                            if (ks * 16 < rp) {
                                const bf16x8 ua_hi = *reinterpret_cast<const bf16x8*>(up + ks * 32);
                                const bf16x8 ua_lo = *reinterpret_cast<const bf16x8*>(up + 2 * rp + ks * 32);
                                const bf16x8 ub_hi = __builtin_bit_cast(bf16x8, ubf[ks][0]);
                                const bf16x8 ub_lo = __builtin_bit_cast(bf16x8, ubf[ks][1]);
                                v = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ua_lo, ub_hi, v, 0, 0, 0);
                                v = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ua_hi, ub_lo, v, 0, 0, 0);
                                v = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ua_hi, ub_hi, v, 0, 0, 0);
                            }
                        }
                    }
#pragma unroll
                    for (int q = 0; q < 16; ++q) {
                        const int rl = wr * 64 + mb * 32 + 8 * (q >> 2) + 4 * h + (q & 3);
                        unsigned char* dst = smem + (size_t)rl * CROW + ((wc & 1) * 64 + nb * 32 + l32) * (YBF16 ? 2 : 4);
                        if (YBF16) *reinterpret_cast<uint16_t*>(dst) = f32_to_bf16_bits(v[q]);
                        else *reinterpret_cast<float*>(dst) = v[q];
                    }
                }
            }
        }
        __syncthreads();
        store_ctile<YBF16, BM>(smem, it, m0, nb0 * 32 + half * 128, (nb0 >> 2) + half, tid, rvp);
        __syncthreads();
    }
}

template <int LIMBS, bool YBF16>
hipError_t launch_gemm_q4_wide(hipStream_t st, stream_args& a) {
    // column tiles of the group, and whether all items have the same rows (the split below is one row index for all)
    int ct = 0;
    bool same = true;
    for (int g = 0; g < a.n_items; ++g) {
        ct += (a.it[g].n_blocks + QW_NB - 1) / QW_NB;
        same = same && a.it[g].R == a.it[0].R;
    }
    const int R0 = a.it[0].R, nrt = (R0 + 63) / 64;
    // two workgroups per CU: 512 at a time.  When the 64-row tiles end in a round that is at most a quarter full, the
    // last row tiles of every column are cut into 32-row tiles, so that the 64-row tiles fill whole rounds only.
    constexpr int SLOTS = 512;
    int small_rt = 0;                                   // 64-row tiles per column that are cut in two
    const long long all = (long long)nrt * ct;
    if (same && all > SLOTS && all % SLOTS != 0 && all % SLOTS <= SLOTS / 4) {
        small_rt = (int)((all % SLOTS + ct - 1) / ct);
        if (small_rt >= nrt) small_rt = 0;
    }
    a.q4_big_rows = same ? (nrt - small_rt) * 64 : 0x7fffffc0;
    int total = 0, total_s = 0;
    for (int g = 0; g < a.n_items; ++g) {
        const int cols = (a.it[g].n_blocks + QW_NB - 1) / QW_NB;
        const int big_rows = std::min(a.q4_big_rows, (a.it[g].R + 63) / 64 * 64);
        a.tile_start[g] = total;
        a.q4_small_start[g] = total_s;
        total += (big_rows / 64) * cols;
        total_s += ((a.it[g].R - std::min(a.it[g].R, big_rows) + 31) / 32) * cols;
    }
    for (int g = a.n_items; g <= ESSA_MAX_GROUP; ++g) {
        a.tile_start[g] = total;
        a.q4_small_start[g] = total_s;
    }
    constexpr size_t smem = q4w_smem_bytes<LIMBS, YBF16, 2>();
    static_assert(2 * smem <= 160 * 1024, "two workgroups share the LDS of a CU");
    auto kern = gemm_q4_wide_kernel<LIMBS, YBF16>;
    static bool attr_done = false;   // one flag per instantiation
    if (!attr_done && smem > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    if (tl_ev_start) hipExtLaunchKernelGGL(kern, dim3(total + total_s), dim3(NT), (uint32_t)smem, st, tl_ev_start, tl_ev_stop, 0, a);
    else hipLaunchKernelGGL(kern, dim3(total + total_s), dim3(NT), smem, st, a);
    return hipGetLastError();
}

template <int LIMBS, bool YBF16, bool DUMP = false>
hipError_t launch_gemm_big(hipStream_t st, stream_args& a, int32_t* acc_out = nullptr) {
    int total = 0;
    for (int g = 0; g < a.n_items; ++g) {
        a.tile_start[g] = total;
        total += ((a.it[g].R + BIG_BM - 1) / BIG_BM) * ((a.it[g].n_blocks + BIG_NB - 1) / BIG_NB);
    }
    a.tile_start[a.n_items] = total;
    constexpr size_t smem = big_smem_bytes<LIMBS, YBF16>();
    static_assert(smem <= 160 * 1024, "tile does not fit the LDS of a CU");
    auto kern = gemm_i8_big_kernel<LIMBS, YBF16, DUMP>;
    static bool attr_done = false;   // one flag per instantiation
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    if (tl_ev_start) hipExtLaunchKernelGGL(kern, dim3(total), dim3(NT), (uint32_t)smem, st, tl_ev_start, tl_ev_stop, 0, a, acc_out);
    else hipLaunchKernelGGL(kern, dim3(total), dim3(NT), smem, st, a, acc_out);
    return hipGetLastError();
}

template <int MB, int LIMBS, bool YBF16, bool DUMP, bool Q4 = false>
hipError_t launch_gemm(hipStream_t st, stream_args& a, int32_t* acc_out) {
    int total = 0;
    for (int g = 0; g < a.n_items; ++g) {
        a.tile_start[g] = total;
        total += ((a.it[g].R + 32 * MB - 1) / (32 * MB)) * ((a.it[g].n_blocks + 3) / 4);
    }
    for (int g = a.n_items; g <= ESSA_MAX_GROUP; ++g) a.tile_start[g] = total;   // the last entry is the grid size
    constexpr size_t smem = gemm_smem_bytes<MB, LIMBS, YBF16, Q4>();
    static_assert(smem <= 160 * 1024, "tile does not fit the LDS of a CU");
    auto kern = gemm_i8_kernel<MB, LIMBS, YBF16, DUMP, Q4>;
    static bool attr_done = false;   // one flag per instantiation
    if (!attr_done && smem > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    // with a pair of events the launch itself stamps them at the kernel's first and last cycle (what a profiler reports
    // as the kernel's duration); events recorded around the launch would add the dispatch latency
    if (tl_ev_start) hipExtLaunchKernelGGL(kern, dim3(total), dim3(NT), (uint32_t)smem, st, tl_ev_start, tl_ev_stop, 0, a, acc_out);
    else hipLaunchKernelGGL(kern, dim3(total), dim3(NT), smem, st, a, acc_out);
    return hipGetLastError();
}

template <int MB, int LIMBS, bool YBF16>
hipError_t launch_gemm_stream(hipStream_t st, stream_args& a) {
    int total = 0;
    for (int g = 0; g < a.n_items; ++g) {
        a.tile_start[g] = total;
        total += a.it[g].n_blocks;
    }
    for (int g = a.n_items; g <= ESSA_MAX_GROUP; ++g) a.tile_start[g] = total;
    constexpr size_t smem = stream_smem_bytes<MB, LIMBS>();
    static_assert(smem <= 160 * 1024, "does not fit the LDS of a CU");
    auto kern = gemm_i8_stream_kernel<MB, LIMBS, YBF16>;
    static bool attr_done = false;   // one flag per instantiation
    if (!attr_done && smem > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    if (tl_ev_start) hipExtLaunchKernelGGL(kern, dim3(total), dim3(NT), (uint32_t)smem, st, tl_ev_start, tl_ev_stop, 0, a);
    else hipLaunchKernelGGL(kern, dim3(total), dim3(NT), smem, st, a);
    return hipGetLastError();
}

// Row counts up to this take the kernel that streams weights on every CU (int8 weights), with one block of 32 rows per
// workgroup or two.  At the 7B shapes two row blocks take 17.3 us per launch at 64 rows against 18.7 for the 32-row tiles of
// gemm_i8_kernel; the activation limbs, which every workgroup loads for all its rows, are then four fifths of the bytes a
// CU takes in, and four row blocks (128 rows) would need more registers than a wave has.
constexpr int STREAM_MAX_ROWS = 64;
bool takes_stream_kernel(const stream_args& a) {
    for (int g = 0; g < a.n_items; ++g)
        if (a.it[g].quant != ESSA_QUANT_INT8_PERCH || a.it[g].R > STREAM_MAX_ROWS) return false;
    return a.n_items > 0;
}
int stream_row_blocks(const stream_args& a) {
    int r = 0;
    for (int g = 0; g < a.n_items; ++g) r = std::max(r, a.it[g].R);
    return r > 32 ? 2 : 1;
}

template <int LIMBS, bool YBF16, bool Q4>
hipError_t launch_gemm_mb(hipStream_t st, stream_args& a, int mb) {
    switch (mb) {
        case 1: return launch_gemm<1, LIMBS, YBF16, false, Q4>(st, a, nullptr);
        case 2: return launch_gemm<2, LIMBS, YBF16, false, Q4>(st, a, nullptr);
        default:
            // no taller tile: with int8 weights its double-buffered fragments do not fit the register file (row counts
            // that large take the 128 x 256 kernel anyway), and with 4-bit weights, whose loop runs its MFMA, scaling
            // and LDS phases one after the other, two 64-row workgroups per CU overlap each other's phases and beat
            // one 128-row workgroup (c4: 290 -> 240 us per launch)
            return launch_gemm<2, LIMBS, YBF16, false, Q4>(st, a, nullptr);
    }
}

// rows per tile: the largest of 128/64 that still leaves every CU a tile, else 32
int pick_mb(const stream_args& a) {
    int maxR = 0;
    for (int g = 0; g < a.n_items; ++g) maxR = a.it[g].R > maxR ? a.it[g].R : maxR;
    for (int mb : {2}) {
        if (maxR <= 16 * mb) continue;     // tile would be more than half empty
        long long tiles = 0;
        for (int g = 0; g < a.n_items; ++g) tiles += (long long)((a.it[g].R + 32 * mb - 1) / (32 * mb)) * ((a.it[g].n_blocks + 3) / 4);
        if (tiles >= 256) return mb;
    }
    return 1;     // fewer tiles than CUs either way: the 32-row tile gives twice as many workgroups and loads less per K tile
}

// 4-bit weights: rows per 256-channel tile, 0 = the group is too small for these tiles.  (32-row tiles of the same
// width throughout fill the last round of workgroups better on the 72B shapes and run no faster, 214 us either way:
// only the rows of a sparsely filled last round get them, see launch_gemm_q4_wide.)
int pick_q4_wide(const stream_args& a) {
    long long tiles = 0;
    for (int g = 0; g < a.n_items; ++g) tiles += (long long)((a.it[g].R + 63) / 64) * ((a.it[g].n_blocks + QW_NB - 1) / QW_NB);
    return tiles >= 256 ? 64 : 0;
}

// the 128 x 256 tile pays off once it fills the chip a few times over
bool takes_big(const stream_args& a) {
    long long tiles = 0;
    for (int g = 0; g < a.n_items; ++g)
        tiles += (long long)((a.it[g].R + BIG_BM - 1) / BIG_BM) * ((a.it[g].n_blocks + BIG_NB - 1) / BIG_NB);
    return tiles >= 512;
}

// returns the grid size of the prep kernel
int fill_prep_tables(stream_args& a, bool finish_u) {
    // interleaved order when every item has the same rows and slices and the rows do not fit the caches as a whole
    // (at decode sizes the order makes no difference to the traffic, and the plain one is a little faster)
    bool same = a.n_items > 0 && a.it[0].R >= 2048;
    int nown = 0;
    for (int g = 0; g < a.n_items; ++g) {
        same = same && a.it[g].R == a.it[0].R && a.it[g].tslices == a.it[0].tslices;
        if (a.it[g].x_owner) a.inter_owner[nown++] = g;
    }
    a.inter_per_rb = 0;
    a.u_ready = 0;
    if (same && a.n_items > 0) {
        a.u_ready = finish_u ? 1 : 0;                   // one workgroup per item and row block for all K slices
        a.inter_nown = nown;
        a.inter_slices = finish_u ? 1 : a.it[0].tslices;
        // rows up to 4096 wide are quantised eight to a workgroup, one wave each (at 3584 columns the prep launch of
        // 32768 rows takes 388 us instead of 440); wider rows two to a workgroup (5120 columns: 640 us against 855)
        bool narrow = true;
        for (int g = 0; g < a.n_items; ++g) narrow = narrow && a.it[g].d_in <= 4096;
        a.inter_per_rb = (narrow ? 4 : 16) * nown + a.n_items * a.inter_slices;
    }
    int q = 0, l = 0;
    for (int g = 0; g < a.n_items; ++g) {
        a.quant_start[g] = q;
        a.lora_start[g] = l;
        if (a.it[g].x_owner) q += (a.it[g].R + 1) / 2;
        l += ((a.it[g].R + 31) / 32) * a.it[g].tslices;
    }
    for (int g = a.n_items; g <= ESSA_MAX_GROUP; ++g) {     // the kernel reads the totals from the last entry
        a.quant_start[g] = q;
        a.lora_start[g] = l;
    }
    return a.inter_per_rb > 0 ? ((a.it[0].R + 31) / 32) * a.inter_per_rb : q + l;
}

}  // namespace

namespace essa_k {

hipError_t forward_stream(hipStream_t st, const fwd_item* items, int n_items, int y_dtype, unsigned flags,
                          hipEvent_t ev_start, hipEvent_t ev_stop) {
    stream_args a{};
    for (int g = 0; g < n_items; ++g) a.it[g] = items[g];
    a.n_items = n_items;
    a.flags = flags;
    a.limbs = (flags & ESSA_COMPUTE_W8A8) ? 1 : 2;
    // rows in the thousands on their way to the 128 x 256 kernel: the prep kernel finishes u itself
    const bool to_big = items[0].quant != ESSA_QUANT_INT4_G128 && takes_big(a);
    const bool to_stream = takes_stream_kernel(a);
    a.limb_tiled = to_stream ? 1 : 0;
    const int prep_blocks = fill_prep_tables(a, to_big);
    if (a.u_ready) hipLaunchKernelGGL(prep_kernel<true>, dim3(prep_blocks), dim3(PREP_NT), 0, st, a);
    else hipLaunchKernelGGL(prep_kernel<false>, dim3(prep_blocks), dim3(PREP_NT), 0, st, a);
    const int mb = pick_mb(a);
    tl_ev_start = ev_start;
    tl_ev_stop = ev_stop;
    hipError_t e;
    const int q4_rows = items[0].quant == ESSA_QUANT_INT4_G128 ? pick_q4_wide(a) : 0;   // all items of a call share the weight format
    if (to_stream) {
        const bool yb = y_dtype == ESSA_BF16;
        if (stream_row_blocks(a) == 2) {
            if (a.limbs == 2) e = yb ? launch_gemm_stream<2, 2, true>(st, a) : launch_gemm_stream<2, 2, false>(st, a);
            else e = yb ? launch_gemm_stream<2, 1, true>(st, a) : launch_gemm_stream<2, 1, false>(st, a);
        } else if (a.limbs == 2) e = yb ? launch_gemm_stream<1, 2, true>(st, a) : launch_gemm_stream<1, 2, false>(st, a);
        else e = yb ? launch_gemm_stream<1, 1, true>(st, a) : launch_gemm_stream<1, 1, false>(st, a);
        tl_ev_start = tl_ev_stop = nullptr;
        if (e != hipSuccess) return e;
        // the reward partials (one per 128 channels and row) span four of this kernel's workgroups: a pass of their own
        return essa_k::rowdot_blocks(st, items, n_items, y_dtype);
    } else if (to_big) {
        if (a.limbs == 2) e = y_dtype == ESSA_BF16 ? launch_gemm_big<2, true>(st, a) : launch_gemm_big<2, false>(st, a);
        else e = y_dtype == ESSA_BF16 ? launch_gemm_big<1, true>(st, a) : launch_gemm_big<1, false>(st, a);
    } else if (q4_rows == 64)
        e = y_dtype == ESSA_BF16 ? launch_gemm_q4_wide<2, true>(st, a) : launch_gemm_q4_wide<2, false>(st, a);
    else if (items[0].quant == ESSA_QUANT_INT4_G128)
        e = y_dtype == ESSA_BF16 ? launch_gemm_mb<2, true, true>(st, a, mb) : launch_gemm_mb<2, false, true>(st, a, mb);
    else if (a.limbs == 2) e = y_dtype == ESSA_BF16 ? launch_gemm_mb<2, true, false>(st, a, mb) : launch_gemm_mb<2, false, false>(st, a, mb);
    else e = y_dtype == ESSA_BF16 ? launch_gemm_mb<1, true, false>(st, a, mb) : launch_gemm_mb<1, false, false>(st, a, mb);
    tl_ev_start = tl_ev_stop = nullptr;
    return e != hipSuccess ? e : hipGetLastError();
}

hipError_t w8a8_accumulators_stream(hipStream_t st, const fwd_item& it, int32_t* acc_out) {
    stream_args a{};
    a.it[0] = it;
    a.it[0].x_owner = 1;
    a.n_items = 1;
    a.flags = ESSA_BASE_ONLY | ESSA_COMPUTE_W8A8;
    a.limbs = 1;
    for (int g = 1; g <= ESSA_MAX_GROUP; ++g) a.quant_start[g] = (it.R + 1) / 2;      // quantise only: no rank-space work (lora_start stays zero)
    hipLaunchKernelGGL(prep_kernel<false>, dim3(a.quant_start[1]), dim3(PREP_NT), 0, st, a);
    // the kernel the forward itself would take at this size dumps its sums: the 128 x 256 tile once it fills the chip
    if (takes_big(a)) return launch_gemm_big<1, false, true>(st, a, acc_out);
    return launch_gemm<2, 1, false, true>(st, a, acc_out);
}

}  // namespace essa_k
