// Host glue of libessa: argument checks, set-up (SVD, repacking, upload), scratch planning and
// the launch sequences behind every extern "C" entry point declared in essa.h.
#include <cmath>
#include <cstring>
#include <memory>

#include "essa_internal.h"

static thread_local std::string g_err;

essa_status essa_fail(essa_status code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

extern "C" const char* essa_last_error(void) { return g_err.c_str(); }
extern "C" const char* essa_version(void) { return "essa-mi355x 0.1 (gfx950)"; }

// ---------------------------------------------------------------------------------------------
// context
// ---------------------------------------------------------------------------------------------
extern "C" essa_status essa_create(essa_ctx** out, int device, void* hip_stream) {
    if (!out) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_create: out is NULL");
    *out = nullptr;
    int count = 0;
    ESSA_HIP(hipGetDeviceCount(&count));
    if (device < 0 || device >= count)
        return essa_fail(ESSA_ERR_INVALID_ARG, "essa_create: device %d out of range (%d visible)", device, count);
    ESSA_HIP(hipSetDevice(device));
    hipDeviceProp_t prop;
    ESSA_HIP(hipGetDeviceProperties(&prop, device));
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0)
        return essa_fail(ESSA_ERR_UNSUPPORTED, "essa_create: kernels are built for gfx950, device is %s",
                         prop.gcnArchName);
    auto* c = new essa_ctx();
    c->device = device;
    c->stream = (hipStream_t)hip_stream;
    *out = c;
    return ESSA_OK;
}

extern "C" void essa_destroy(essa_ctx* ctx) {
    if (!ctx) return;
    (void)hipSetDevice(ctx->device);
    (void)hipStreamSynchronize(ctx->stream);
    // graphs recorded on this context hold pointers into its scratch: they die with it (launching one afterwards fails)
    for (essa_graph* g : ctx->graphs) {
        if (g->exec) (void)hipGraphExecDestroy(g->exec);
        if (g->graph) (void)hipGraphDestroy(g->graph);
        g->exec = nullptr;
        g->graph = nullptr;
        g->ctx = nullptr;
    }
    if (ctx->ws) (void)hipFree(ctx->ws);
    for (hipEvent_t e : ctx->ev) (void)hipEventDestroy(e);
    delete ctx;
}

extern "C" essa_status essa_synchronize(essa_ctx* ctx) {
    if (!ctx) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_synchronize: ctx is NULL");
    if (ctx->capturing) return essa_fail(ESSA_ERR_STATE, "essa_synchronize: not while a graph is being recorded");
    ESSA_HIP(hipStreamSynchronize(ctx->stream));
    return ESSA_OK;
}

// ---------------------------------------------------------------------------------------------
// record and replay
// ---------------------------------------------------------------------------------------------
extern "C" essa_status essa_graph_begin(essa_ctx* ctx) {
    if (!ctx) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_graph_begin: ctx is NULL");
    if (ctx->capturing) return essa_fail(ESSA_ERR_STATE, "essa_graph_begin: already recording");
    if (!ctx->stream) return essa_fail(ESSA_ERR_STATE, "essa_graph_begin: the context runs on the default stream, which cannot be recorded");
    ESSA_HIP(hipSetDevice(ctx->device));
    ESSA_HIP(hipStreamBeginCapture(ctx->stream, hipStreamCaptureModeThreadLocal));
    ctx->capturing = true;
    return ESSA_OK;
}

extern "C" essa_status essa_graph_end(essa_ctx* ctx, essa_graph** out) {
    if (!ctx || !out) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_graph_end: NULL argument");
    *out = nullptr;
    if (!ctx->capturing) return essa_fail(ESSA_ERR_STATE, "essa_graph_end: not recording");
    ctx->capturing = false;
    ESSA_HIP(hipSetDevice(ctx->device));
    hipGraph_t graph = nullptr;
    ESSA_HIP(hipStreamEndCapture(ctx->stream, &graph));
    if (!graph) return essa_fail(ESSA_ERR_HIP, "essa_graph_end: the recording was invalidated by a call that cannot be recorded");
    hipGraphExec_t exec = nullptr;
    hipError_t e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    if (e != hipSuccess) {
        (void)hipGraphDestroy(graph);
        return essa_fail(ESSA_ERR_HIP, "hipGraphInstantiate failed: %s", hipGetErrorString(e));
    }
    auto* g = new essa_graph();
    g->ctx = ctx;
    ctx->graphs.push_back(g);
    g->device = ctx->device;
    g->stream = ctx->stream;
    g->graph = graph;
    g->exec = exec;
    *out = g;
    return ESSA_OK;
}

extern "C" essa_status essa_graph_launch(essa_graph* g) {
    if (!g) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_graph_launch: graph is NULL");
    if (!g->ctx || !g->exec) return essa_fail(ESSA_ERR_STATE, "essa_graph_launch: the context this graph was recorded on has been destroyed");
    ESSA_HIP(hipSetDevice(g->device));
    ESSA_HIP(hipGraphLaunch(g->exec, g->stream));
    return ESSA_OK;
}

extern "C" void essa_graph_destroy(essa_graph* g) {
    if (!g) return;
    (void)hipSetDevice(g->device);
    if (g->ctx) {
        (void)hipStreamSynchronize(g->stream);
        auto& v = g->ctx->graphs;
        for (size_t i = 0; i < v.size(); ++i)
            if (v[i] == g) { v.erase(v.begin() + i); break; }
    }
    if (g->exec) (void)hipGraphExecDestroy(g->exec);
    if (g->graph) (void)hipGraphDestroy(g->graph);
    delete g;
}

extern "C" essa_status essa_profile_enable(essa_ctx* ctx, int on) {
    if (!ctx) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_profile_enable: ctx is NULL");
    if (ctx->capturing) return essa_fail(ESSA_ERR_STATE, "essa_profile_enable: not while a graph is being recorded");
    ESSA_HIP(hipSetDevice(ctx->device));
    ESSA_HIP(hipStreamSynchronize(ctx->stream));
    ctx->profiling = on != 0;
    ctx->ev_used = 0;
    return ESSA_OK;
}

extern "C" essa_status essa_profile_read(essa_ctx* ctx, double* total_ms, int* launches) {
    if (!ctx || !total_ms || !launches) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_profile_read: NULL argument");
    ESSA_HIP(hipSetDevice(ctx->device));
    ESSA_HIP(hipStreamSynchronize(ctx->stream));
    double sum = 0;
    for (size_t i = 0; i + 1 < ctx->ev_used; i += 2) {
        float ms = 0.f;
        ESSA_HIP(hipEventElapsedTime(&ms, ctx->ev[i], ctx->ev[i + 1]));
        sum += ms;
    }
    *total_ms = sum;
    *launches = (int)(ctx->ev_used / 2);
    ctx->ev_used = 0;
    return ESSA_OK;
}

// next (start, stop) event pair while profiling, else (null, null)
static essa_status next_events(essa_ctx* ctx, hipEvent_t* a, hipEvent_t* b) {
    *a = *b = nullptr;
    if (!ctx->profiling || ctx->capturing) return ESSA_OK;
    while (ctx->ev.size() < ctx->ev_used + 2) {
        hipEvent_t e;
        ESSA_HIP(hipEventCreate(&e));
        ctx->ev.push_back(e);
    }
    *a = ctx->ev[ctx->ev_used];
    *b = ctx->ev[ctx->ev_used + 1];
    ctx->ev_used += 2;
    return ESSA_OK;
}

essa_status essa_ws_reserve(essa_ctx* ctx, size_t bytes) {
    if (bytes <= ctx->ws_bytes) return ESSA_OK;
    if (ctx->capturing)
        return essa_fail(ESSA_ERR_STATE, "scratch would have to grow to %zu bytes while a graph is being recorded: run the same calls once before essa_graph_begin", bytes);
    if (!ctx->graphs.empty())
        return essa_fail(ESSA_ERR_STATE, "scratch would have to grow to %zu bytes, but %zu recorded graph(s) of this context still point into the current one: destroy them first (or run the largest problem once before recording)", bytes, ctx->graphs.size());
    ESSA_HIP(hipStreamSynchronize(ctx->stream));
    if (ctx->ws) ESSA_HIP(hipFree(ctx->ws));
    ctx->ws = nullptr;
    ctx->ws_bytes = 0;
    size_t want = bytes + bytes / 4 + (1u << 20);
    hipError_t e = hipMalloc(&ctx->ws, want);
    if (e != hipSuccess) return essa_fail(ESSA_ERR_OOM, "scratch of %zu bytes: %s", want, hipGetErrorString(e));
    ctx->ws_bytes = want;
    return ESSA_OK;
}

template <class T>
static essa_status upload(T** dst, const T* src, size_t count) {
    *dst = nullptr;
    hipError_t e = hipMalloc((void**)dst, count * sizeof(T) + 256);   // slack: kernels may over-read a vector
    if (e != hipSuccess) return essa_fail(ESSA_ERR_OOM, "hipMalloc of %zu bytes: %s", count * sizeof(T), hipGetErrorString(e));
    ESSA_HIP(hipMemset(*dst, 0, count * sizeof(T) + 256));
    ESSA_HIP(hipMemcpy(*dst, src, count * sizeof(T), hipMemcpyHostToDevice));
    return ESSA_OK;
}

static uint16_t f32_to_bf16_rne(float f) {
    uint32_t u;
    std::memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

static float f16_to_f32(uint16_t h) {
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16, exp = (h >> 10) & 0x1f, man = h & 0x3ffu, u;
    if (exp == 0) {
        if (man == 0) u = sign;
        else {
            int e = -1;
            do { man <<= 1; ++e; } while (!(man & 0x400u));
            u = sign | ((uint32_t)(127 - 15 - e) << 23) | ((man & 0x3ffu) << 13);
        }
    } else if (exp == 31) u = sign | 0x7f800000u | (man << 13);
    else u = sign | ((exp + 112) << 23) | (man << 13);
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}

// ---------------------------------------------------------------------------------------------
// projection set-up
// ---------------------------------------------------------------------------------------------
extern "C" void essa_proj_destroy(essa_proj* p) {
    if (!p) return;
    (void)hipSetDevice(p->device);
    (void)hipDeviceSynchronize();
    void* ptrs[] = {p->Wq, p->scale, p->zero, p->VA32, p->VA16, p->UB32, p->UB16, p->M, p->Wt, p->VAp, p->St, p->SZ16};
    for (void* q : ptrs)
        if (q) (void)hipFree(q);
    delete p;
}

extern "C" essa_status essa_proj_create(essa_ctx* ctx, const essa_proj_desc* d, essa_proj** out) {
    if (!ctx || !d || !out) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_proj_create: NULL argument");
    *out = nullptr;
    if (!d->Wq || !d->scales || !d->lora_A || !d->lora_B)
        return essa_fail(ESSA_ERR_INVALID_ARG, "essa_proj_create: NULL tensor in descriptor");
    if (d->d_in <= 0 || d->d_out <= 0) return essa_fail(ESSA_ERR_SHAPE, "essa_proj_create: d_in=%d d_out=%d", d->d_in, d->d_out);
    if (d->r < 1 || d->r > 32 || d->r > d->d_in || d->r > d->d_out)
        return essa_fail(ESSA_ERR_SHAPE, "essa_proj_create: rank %d not in [1, min(32, d_in, d_out)]", d->r);
    if (d->quant != ESSA_QUANT_INT8_PERCH && d->quant != ESSA_QUANT_INT4_G128)
        return essa_fail(ESSA_ERR_INVALID_ARG, "essa_proj_create: unknown quant %d", d->quant);
    if (d->quant == ESSA_QUANT_INT4_G128) {
        if (d->d_in % 128 != 0) return essa_fail(ESSA_ERR_SHAPE, "essa_proj_create: int4 needs d_in %% 128 == 0, got %d", d->d_in);
        if (!d->zeros) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_proj_create: int4 needs zeros");
    }
    ESSA_HIP(hipSetDevice(ctx->device));
    std::unique_ptr<essa_proj, void (*)(essa_proj*)> p(new essa_proj(), essa_proj_destroy);
    p->ctx = ctx;
    p->device = ctx->device;
    p->stream = ctx->stream;
    p->d_in = d->d_in;
    p->d_out = d->d_out;
    p->r = d->r;
    p->rp = d->r <= 16 ? 16 : 32;
    p->quant = d->quant;
    const int r = d->r, rp = p->rp, din = d->d_in, dout = d->d_out;

    // thin SVDs in fp64.  A is r x d_in: decompose A^T (d_in x r) = V_A S U_A^T.
    std::vector<double> At((size_t)din * r), VA((size_t)din * r), sA(r), UA((size_t)r * r);
    for (int j = 0; j < r; ++j)
        for (int i = 0; i < din; ++i) At[(size_t)i * r + j] = d->lora_A[(size_t)j * din + i];
    essa_host_thin_svd(At.data(), din, r, VA.data(), sA.data(), UA.data());
    std::vector<double> Bd((size_t)dout * r), UB((size_t)dout * r), sB(r), VB((size_t)r * r);
    for (size_t i = 0; i < Bd.size(); ++i) Bd[i] = d->lora_B[i];
    essa_host_thin_svd(Bd.data(), dout, r, UB.data(), sB.data(), VB.data());
    p->sA.assign(sA.begin(), sA.end());
    p->sB.assign(sB.begin(), sB.end());

    std::vector<float> M((size_t)rp * rp, 0.f), VA32((size_t)din * rp, 0.f), UB32((size_t)dout * rp, 0.f);
    std::vector<uint16_t> VA16((size_t)rp * din, 0), UB16((size_t)dout * 2 * rp, 0);
    for (int b = 0; b < r; ++b)
        for (int a = 0; a < r; ++a) {
            double acc = 0;
            for (int t = 0; t < r; ++t) acc += VB[(size_t)t * r + b] * UA[(size_t)t * r + a];
            M[(size_t)b * rp + a] = (float)acc;
        }
    for (int i = 0; i < din; ++i)
        for (int j = 0; j < r; ++j) {
            float v = (float)VA[(size_t)i * r + j];
            VA32[(size_t)i * rp + j] = v;
            VA16[(size_t)j * din + i] = f32_to_bf16_rne(v);
        }
    for (int o = 0; o < dout; ++o)
        for (int j = 0; j < r; ++j) {
            float v = (float)UB[(size_t)o * r + j];
            UB32[(size_t)o * rp + j] = v;
            const uint16_t hi = f32_to_bf16_rne(v);   // bf16 head and tail, v = hi + lo
            uint32_t hb = (uint32_t)hi << 16;
            float hf;
            std::memcpy(&hf, &hb, 4);
            UB16[(size_t)o * 2 * rp + j] = hi;
            UB16[(size_t)o * 2 * rp + rp + j] = f32_to_bf16_rne(v - hf);
        }
    ESSA_TRY(upload(&p->M, M.data(), M.size()));
    ESSA_TRY(upload(&p->VA32, VA32.data(), VA32.size()));
    ESSA_TRY(upload(&p->VA16, VA16.data(), VA16.size()));
    ESSA_TRY(upload(&p->UB32, UB32.data(), UB32.size()));
    ESSA_TRY(upload(&p->UB16, UB16.data(), UB16.size()));

    {   // V_A^T as bf16 heads and tails, tiled for the MFMA down-projection: [k step of 16][block of 32 rows][lane][8],
        // lane (h, l32) of a block holding row 32 b + l32 (rows 0..rp-1 heads of V_A's columns, rp..2rp-1 their
        // tails), columns 16 ks + 8 h .. + 7 -- one contiguous kilobyte per wave load
        const int ksteps = (din + 15) / 16, nbv = 2 * rp / 32;
        std::vector<uint16_t> VAp((size_t)ksteps * nbv * 64 * 8, 0);
        for (int i = 0; i < din; ++i)
            for (int j = 0; j < r; ++j) {
                const float v = (float)VA[(size_t)i * r + j];
                const uint16_t hi = f32_to_bf16_rne(v);
                uint32_t hb = (uint32_t)hi << 16;
                float hf;
                std::memcpy(&hf, &hb, 4);
                const uint16_t parts[2] = {hi, f32_to_bf16_rne(v - hf)};
                for (int e = 0; e < 2; ++e) {
                    const int row = e * rp + j, ks = i / 16, h = (i % 16) / 8;
                    VAp[((((size_t)ks * nbv + row / 32) * 2 + h) * 32 + row % 32) * 8 + i % 8] = parts[e];
                }
            }
        ESSA_TRY(upload(&p->VAp, VAp.data(), VAp.size()));
    }
    if (d->quant == ESSA_QUANT_INT8_PERCH) {
        int8_t* w = nullptr;
        ESSA_TRY(upload(&w, (const int8_t*)d->Wq, (size_t)dout * din));
        p->Wq = w;
        ESSA_TRY(upload(&p->scale, (const float*)d->scales, (size_t)dout));
        // tiled copy: 1 KB blocks of 32 channels x 32 k, laid out as the int8 MFMA wants its operand
        p->d_in_pad = (din + 511) / 512 * 512;   // four K tiles of 128: the GEMM's unrolled pipeline
        p->n_blocks = (dout + 31) / 32;
        const int kch = p->d_in_pad / 32;
        std::vector<int8_t> Wt((size_t)p->n_blocks * kch * 1024, 0);
        const int8_t* src = (const int8_t*)d->Wq;
        for (int nb = 0; nb < p->n_blocks; ++nb)
            for (int n = 0; n < 32; ++n) {
                const int o = nb * 32 + n;
                if (o >= dout) continue;
                for (int k = 0; k < din; ++k) {
                    const int kc = k >> 5, hh = (k >> 4) & 1, j = k & 15;
                    Wt[((size_t)kc * p->n_blocks + nb) * 1024 + (size_t)(hh * 32 + n) * 16 + j] = src[(size_t)o * din + k];
                }
            }
        ESSA_TRY(upload(&p->Wt, Wt.data(), Wt.size()));
    } else {
        p->groups = din / 128;
        uint8_t* w = nullptr;
        ESSA_TRY(upload(&w, (const uint8_t*)d->Wq, (size_t)dout * din / 2));
        p->Wq = w;
        size_t ng = (size_t)dout * p->groups;
        std::vector<float> s(ng), z(ng);
        const uint16_t* sh = (const uint16_t*)d->scales;
        const uint16_t* zh = (const uint16_t*)d->zeros;
        for (size_t i = 0; i < ng; ++i) { s[i] = f16_to_f32(sh[i]); z[i] = f16_to_f32(zh[i]); }
        ESSA_TRY(upload(&p->scale, s.data(), ng));
        ESSA_TRY(upload(&p->zero, z.data(), ng));
        // fast-path copies: nibbles tiled for the int8 MFMA operand, scales group major, -scale*zero as bf16 head+tail
        p->d_in_pad = (din + 511) / 512 * 512;
        p->n_blocks = (dout + 31) / 32;
        p->Gp = (p->groups + 15) / 16 * 16;
        const int pairs = p->d_in_pad / 64, nbs = p->n_blocks;
        const uint8_t* src = (const uint8_t*)d->Wq;
        auto nib = [&](int o, int k) -> uint8_t {
            if (o >= dout || k >= din) return 0;
            const uint8_t b = src[((size_t)o * din + k) >> 1];
            return (k & 1) ? (uint8_t)(b >> 4) : (uint8_t)(b & 15);
        };
        std::vector<int8_t> Wt((size_t)pairs * nbs * 1024, 0);
        for (int pr = 0; pr < pairs; ++pr)
            for (int nb = 0; nb < nbs; ++nb)
                for (int hh = 0; hh < 2; ++hh)
                    for (int n = 0; n < 32; ++n)
                        for (int j = 0; j < 16; ++j) {
                            const int o = nb * 32 + n, k0 = pr * 64 + 16 * hh + j;
                            Wt[((size_t)pr * nbs + nb) * 1024 + (size_t)(hh * 32 + n) * 16 + j] = (int8_t)(nib(o, k0) | (nib(o, k0 + 32) << 4));
                        }
        ESSA_TRY(upload(&p->Wt, Wt.data(), Wt.size()));
        const int gpad = p->d_in_pad / 128;
        std::vector<float> St((size_t)gpad * nbs * 32, 0.f);
        std::vector<uint16_t> SZ((size_t)nbs * 32 * 2 * p->Gp, 0);
        for (int o = 0; o < dout; ++o)
            for (int g = 0; g < p->groups; ++g) {
                const float sv = s[(size_t)o * p->groups + g], zv = z[(size_t)o * p->groups + g];
                St[(size_t)g * nbs * 32 + o] = sv;
                const float m = -(sv * zv);
                const uint16_t hi = f32_to_bf16_rne(m);
                uint32_t hb = (uint32_t)hi << 16;
                float hf;
                std::memcpy(&hf, &hb, 4);
                SZ[((size_t)o * 2 + 0) * p->Gp + g] = hi;
                SZ[((size_t)o * 2 + 1) * p->Gp + g] = f32_to_bf16_rne(m - hf);
            }
        ESSA_TRY(upload(&p->St, St.data(), St.size()));
        ESSA_TRY(upload(&p->SZ16, SZ.data(), SZ.size()));
    }
    *out = p.release();
    return ESSA_OK;
}

extern "C" essa_status essa_proj_spectrum(const essa_proj* p, float* sA_host, float* sB_host) {
    if (!p || !sA_host || !sB_host) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_proj_spectrum: NULL argument");
    std::memcpy(sA_host, p->sA.data(), p->r * sizeof(float));
    std::memcpy(sB_host, p->sB.data(), p->r * sizeof(float));
    return ESSA_OK;
}

// ---------------------------------------------------------------------------------------------
// search distribution
// ---------------------------------------------------------------------------------------------
struct cma_blob_header {
    uint32_t magic, version;
    int32_t n, t;
    float sigma;
    uint32_t reserved;
};
static const uint32_t kCmaMagic = 0x41535345u;  // "ESSA"

extern "C" void essa_cma_destroy(essa_cma* c) {
    if (!c) return;
    (void)hipSetDevice(c->device);
    (void)hipDeviceSynchronize();
    void* ptrs[] = {c->m, c->p_sigma, c->p_c, c->D, c->C, c->B, c->Cdiag, c->sc, c->weights, c->eigV};
    for (void* q : ptrs)
        if (q) (void)hipFree(q);
    delete c;
}

static bool has_matrix(const essa_cma* c) { return c->kind == ESSA_OPT_CMA || c->kind == ESSA_OPT_ACTIVE_CMA; }

extern "C" essa_status essa_cma_create_opt(essa_ctx* ctx, int n, float sigma0, const float* m0_host, const essa_opt_desc* opt,
                                           essa_cma** out) {
    if (!ctx || !out) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_cma_create: NULL argument");
    *out = nullptr;
    const int kind = opt ? opt->kind : (int)ESSA_OPT_CMA;
    if (kind < ESSA_OPT_CMA || kind > ESSA_OPT_ARS) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_cma_create: unknown optimiser kind %d", kind);
    if (n < 1 || n > (kind >= ESSA_OPT_SEP_CMA ? (1 << 24) : 16384))
        return essa_fail(ESSA_ERR_SHAPE, "essa_cma_create: n=%d not in [1, %d]", n, kind >= ESSA_OPT_SEP_CMA ? (1 << 24) : 16384);
    if (!(sigma0 > 0.f) || !std::isfinite(sigma0)) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_cma_create: sigma0 must be positive and finite");
    if (kind == ESSA_OPT_ARS && (!(opt->ars_alpha > 0.f) || !std::isfinite(opt->ars_alpha) || opt->ars_top < 1 || opt->ars_top > 1024))
        return essa_fail(ESSA_ERR_INVALID_ARG, "essa_cma_create: ARS needs ars_alpha > 0 and 1 <= ars_top <= 1024 (got %g, %d)",
                         (double)opt->ars_alpha, opt->ars_top);
    ESSA_HIP(hipSetDevice(ctx->device));
    std::unique_ptr<essa_cma, void (*)(essa_cma*)> c(new essa_cma(), essa_cma_destroy);
    c->ctx = ctx;
    c->device = ctx->device;
    c->stream = ctx->stream;
    c->n = n;
    c->kind = kind;
    if (kind == ESSA_OPT_ARS) { c->ars_alpha = opt->ars_alpha; c->ars_top = opt->ars_top; }
    std::vector<float> zeros((size_t)n, 0.f), ones((size_t)n, 1.f);
    ESSA_TRY(upload(&c->m, m0_host ? m0_host : zeros.data(), (size_t)n));
    ESSA_TRY(upload(&c->p_sigma, zeros.data(), (size_t)n));
    ESSA_TRY(upload(&c->p_c, zeros.data(), (size_t)n));
    ESSA_TRY(upload(&c->D, ones.data(), (size_t)n));
    if (has_matrix(c.get())) {
        std::vector<float> eye((size_t)n * n, 0.f);
        for (int i = 0; i < n; ++i) eye[(size_t)i * n + i] = 1.f;
        ESSA_TRY(upload(&c->C, eye.data(), eye.size()));
        ESSA_TRY(upload(&c->B, eye.data(), eye.size()));
    } else {
        ESSA_TRY(upload(&c->Cdiag, ones.data(), (size_t)n));
    }
    essa_cma_scalars sc{sigma0, 0, 1.f, 0.f};
    ESSA_TRY(upload(&c->sc, &sc, 1));
    *out = c.release();
    return ESSA_OK;
}

extern "C" essa_status essa_cma_create(essa_ctx* ctx, int n, float sigma0, const float* m0_host, essa_cma** out) {
    return essa_cma_create_opt(ctx, n, sigma0, m0_host, nullptr, out);
}

extern "C" int essa_cma_kind(const essa_cma* c) { return c ? c->kind : -1; }

extern "C" essa_status essa_cma_set_basis(essa_cma* c, const float* B_dev, const float* D_dev) {
    if (!c || !B_dev || !D_dev) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_cma_set_basis: NULL argument");
    if (!has_matrix(c)) return essa_fail(ESSA_ERR_STATE, "essa_cma_set_basis: an optimiser of kind %d keeps no basis", c->kind);
    ESSA_HIP(hipSetDevice(c->device));
    ESSA_HIP(hipMemcpyAsync(c->B, B_dev, (size_t)c->n * c->n * sizeof(float), hipMemcpyDeviceToDevice, c->stream));
    ESSA_HIP(hipMemcpyAsync(c->D, D_dev, (size_t)c->n * sizeof(float), hipMemcpyDeviceToDevice, c->stream));
    c->eigV_valid = false;
    return ESSA_OK;
}

static size_t blob_bytes(const essa_cma* c) {
    const size_t n = c->n;
    return sizeof(cma_blob_header) + (has_matrix(c) ? 4 * n + 2 * n * n : 5 * n) * sizeof(float);
}

extern "C" essa_status essa_cma_export(const essa_cma* c, void* blob, size_t* bytes) {
    if (!c || !bytes) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_cma_export: NULL argument");
    const size_t n = c->n, need = blob_bytes(c);
    if (!blob) { *bytes = need; return ESSA_OK; }
    if (*bytes < need) { *bytes = need; return essa_fail(ESSA_ERR_SHAPE, "essa_cma_export: blob too small, need %zu bytes", need); }
    ESSA_HIP(hipSetDevice(c->device));
    ESSA_HIP(hipStreamSynchronize(c->stream));
    essa_cma_scalars sc;
    ESSA_HIP(hipMemcpy(&sc, c->sc, sizeof sc, hipMemcpyDeviceToHost));
    cma_blob_header h{kCmaMagic, 1u, (int32_t)n, sc.t, sc.sigma, (uint32_t)c->kind};
    char* dst = (char*)blob;
    std::memcpy(dst, &h, sizeof h);
    dst += sizeof h;
    const float* vecs[] = {c->m, c->p_sigma, c->p_c, c->D};
    for (const float* v : vecs) { ESSA_HIP(hipMemcpy(dst, v, n * sizeof(float), hipMemcpyDeviceToHost)); dst += n * sizeof(float); }
    if (has_matrix(c)) {
        ESSA_HIP(hipMemcpy(dst, c->C, n * n * sizeof(float), hipMemcpyDeviceToHost));
        dst += n * n * sizeof(float);
        ESSA_HIP(hipMemcpy(dst, c->B, n * n * sizeof(float), hipMemcpyDeviceToHost));
    } else {
        ESSA_HIP(hipMemcpy(dst, c->Cdiag, n * sizeof(float), hipMemcpyDeviceToHost));
    }
    *bytes = need;
    return ESSA_OK;
}

extern "C" essa_status essa_cma_import(essa_cma* c, const void* blob, size_t bytes) {
    if (!c || !blob) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_cma_import: NULL argument");
    const size_t n = c->n, need = blob_bytes(c);
    if (bytes < sizeof(cma_blob_header)) return essa_fail(ESSA_ERR_SHAPE, "essa_cma_import: blob shorter than its header");
    cma_blob_header h;
    std::memcpy(&h, blob, sizeof h);
    if (h.magic != kCmaMagic || h.version != 1u) return essa_fail(ESSA_ERR_STATE, "essa_cma_import: not a state blob of this library");
    if (h.reserved != (uint32_t)c->kind) return essa_fail(ESSA_ERR_STATE, "essa_cma_import: blob of optimiser kind %u, object of kind %d", h.reserved, c->kind);
    if ((size_t)h.n != n || bytes != need) return essa_fail(ESSA_ERR_STATE, "essa_cma_import: blob holds n=%d (%zu bytes), object has n=%zu (%zu bytes)", h.n, bytes, n, need);
    if (!(h.sigma > 0.f) || h.t < 0) return essa_fail(ESSA_ERR_STATE, "essa_cma_import: sigma=%g t=%d", h.sigma, h.t);
    ESSA_HIP(hipSetDevice(c->device));
    ESSA_HIP(hipStreamSynchronize(c->stream));
    essa_cma_scalars sc{h.sigma, h.t, 1.f, 0.f};
    ESSA_HIP(hipMemcpy(c->sc, &sc, sizeof sc, hipMemcpyHostToDevice));
    const char* src = (const char*)blob + sizeof h;
    float* vecs[] = {c->m, c->p_sigma, c->p_c, c->D};
    for (float* v : vecs) { ESSA_HIP(hipMemcpy(v, src, n * sizeof(float), hipMemcpyHostToDevice)); src += n * sizeof(float); }
    if (has_matrix(c)) {
        ESSA_HIP(hipMemcpy(c->C, src, n * n * sizeof(float), hipMemcpyHostToDevice));
        src += n * n * sizeof(float);
        ESSA_HIP(hipMemcpy(c->B, src, n * n * sizeof(float), hipMemcpyHostToDevice));
    } else {
        ESSA_HIP(hipMemcpy(c->Cdiag, src, n * sizeof(float), hipMemcpyHostToDevice));
    }
    c->eigV_valid = false;
    return ESSA_OK;
}

// ---------------------------------------------------------------------------------------------
// hot path: sampling and theta -> sigma
// ---------------------------------------------------------------------------------------------
static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

extern "C" essa_status essa_philox_words(essa_ctx* ctx, const uint32_t* seeds, int K, int n_blocks, uint32_t* words_out) {
    if (!ctx || !seeds || !words_out) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_philox_words: NULL argument");
    if (K < 1 || n_blocks < 1) return essa_fail(ESSA_ERR_SHAPE, "essa_philox_words: K=%d n_blocks=%d", K, n_blocks);
    ESSA_HIP(hipSetDevice(ctx->device));
    ESSA_HIP(essa_k::philox_words(ctx->stream, seeds, K, n_blocks, words_out));
    return ESSA_OK;
}

extern "C" essa_status essa_sample_candidates(essa_ctx* ctx, const essa_cma* cma, const uint32_t* seeds, int K,
                                              float* theta_out, float* z_out) {
    if (!ctx || !cma || !seeds || !theta_out) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_sample_candidates: NULL argument");
    if (K < 1 || K > 65536) return essa_fail(ESSA_ERR_SHAPE, "essa_sample_candidates: K=%d not in [1, 65536]", K);
    if (cma->ctx != ctx) return essa_fail(ESSA_ERR_STATE, "essa_sample_candidates: state belongs to another context");
    ESSA_HIP(hipSetDevice(ctx->device));
    const int n = cma->n;
    if (!has_matrix(cma)) {
        const int pairs = cma->kind == ESSA_OPT_ARS;
        if (pairs && (K & 1)) return essa_fail(ESSA_ERR_SHAPE, "essa_sample_candidates: ARS draws candidates in pairs, K=%d is odd", K);
        ESSA_HIP(essa_k::sample_diag(ctx->stream, seeds, K, n, cma->m, cma->kind == ESSA_OPT_SEP_CMA ? cma->D : nullptr, cma->sc, pairs,
                                     theta_out, z_out));
        return ESSA_OK;
    }
    ESSA_TRY(essa_ws_reserve(ctx, align256((size_t)K * n * sizeof(float))));
    float* S = (float*)ctx->ws;
    ESSA_HIP(essa_k::normals_scaled(ctx->stream, seeds, nullptr, K, n, cma->D, S, z_out));
    ESSA_HIP(essa_k::skinny_gemm_nt(ctx->stream, S, K, cma->B, n, cma->m, cma->sc, 1, theta_out));
    return ESSA_OK;
}

extern "C" essa_status essa_theta_to_sigma(essa_ctx* ctx, int P, int r, int n_top, const float* sft_A, const float* sft_B,
                                           const float* theta, int K, float* sigmaA, float* sigmaB) {
    if (!ctx || !sft_A || !sft_B || !theta || !sigmaA || !sigmaB) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_theta_to_sigma: NULL argument");
    if (n_top < 1) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_theta_to_sigma: floor(alpha r) = %d leaves no trainable singular value", n_top);
    if (P < 1 || r < 1 || n_top > r || K < 1) return essa_fail(ESSA_ERR_SHAPE, "essa_theta_to_sigma: P=%d r=%d n_top=%d K=%d", P, r, n_top, K);
    ESSA_HIP(hipSetDevice(ctx->device));
    ESSA_HIP(essa_k::theta_to_sigma(ctx->stream, P, r, n_top, sft_A, sft_B, theta, K, sigmaA, sigmaB));
    return ESSA_OK;
}

// ---------------------------------------------------------------------------------------------
// hot path: forward
// ---------------------------------------------------------------------------------------------
// The items of one call, planned: fixed-size, so that planning itself allocates nothing.
struct item_list {
    essa_k::fwd_item it[ESSA_MAX_GROUP];
    int n = 0;
    void push(const essa_k::fwd_item& k) { it[n++] = k; }
};

// With ESSA_VALIDATE: every entry of the item's row -> candidate map is checked on the host (one blocking copy).
static essa_status validate_row2cand(essa_ctx* ctx, const essa_fwd_item& it, int index, const char* who) {
    if (ctx->capturing) return essa_fail(ESSA_ERR_STATE, "%s: ESSA_VALIDATE copies the map to the host and cannot be recorded", who);
    std::vector<int32_t> host((size_t)it.R);
    ESSA_HIP(hipStreamSynchronize(ctx->stream));
    ESSA_HIP(hipMemcpy(host.data(), it.row2cand, (size_t)it.R * sizeof(int32_t), hipMemcpyDeviceToHost));
    for (int i = 0; i < it.R; ++i)
        if (host[i] < 0 || host[i] >= it.K)
            return essa_fail(ESSA_ERR_INVALID_ARG, "%s: item %d, row2cand[%d] = %d is not in [0, %d)", who, index, i, host[i], it.K);
    return ESSA_OK;
}

// Checks the items and lays their scratch out.  scratch == nullptr: the context's own buffer, grown when it has to be;
// otherwise the caller's buffer of scratch_bytes, which is never exceeded (ESSA_ERR_SHAPE says how much was needed).
static essa_status plan_items(essa_ctx* ctx, const essa_fwd_item* items, int n_items, int x_dtype, int y_dtype,
                              unsigned flags, item_list& out, const char* who,
                              const float* const* rv = nullptr, float* rowpart = nullptr, void* scratch = nullptr, size_t scratch_bytes = 0) {
    if (x_dtype != ESSA_F32 && x_dtype != ESSA_BF16) return essa_fail(ESSA_ERR_INVALID_ARG, "%s: x_dtype %d", who, x_dtype);
    if (y_dtype != ESSA_F32 && y_dtype != ESSA_BF16) return essa_fail(ESSA_ERR_INVALID_ARG, "%s: y_dtype %d", who, y_dtype);
    if (flags & ~(ESSA_COMPUTE_W8A8 | ESSA_LORA_ONLY | ESSA_BASE_ONLY | ESSA_COMPUTE_BF16 | ESSA_VALIDATE)) return essa_fail(ESSA_ERR_INVALID_ARG, "%s: unknown flag bits 0x%x", who, flags);
    if ((flags & ESSA_LORA_ONLY) && (flags & ESSA_BASE_ONLY)) return essa_fail(ESSA_ERR_INVALID_ARG, "%s: LORA_ONLY and BASE_ONLY exclude each other", who);
    size_t total = 0;
    size_t block0 = 0;       // fused reward: first 128-channel block of the item within the call's range
    out.n = 0;
    for (int i = 0; i < n_items; ++i) {
        const essa_fwd_item& it = items[i];
        if (!it.proj) return essa_fail(ESSA_ERR_INVALID_ARG, "%s: item %d has no projection", who, i);
        if (it.proj->ctx != ctx) return essa_fail(ESSA_ERR_STATE, "%s: item %d belongs to another context", who, i);
        if (it.R < 0 || it.K < 1) return essa_fail(ESSA_ERR_SHAPE, "%s: item %d has R=%d K=%d", who, i, it.R, it.K);
        if (it.R > 0 && (!it.X || !it.row2cand || !it.sigmaA || !it.sigmaB || !it.Y))
            return essa_fail(ESSA_ERR_INVALID_ARG, "%s: item %d has a NULL tensor", who, i);
        if (it.sigma_stride < it.proj->r && it.K > 1)
            return essa_fail(ESSA_ERR_SHAPE, "%s: item %d sigma_stride %lld < r", who, i, (long long)it.sigma_stride);
        const essa_proj* p = it.proj;
        if ((flags & ESSA_COMPUTE_W8A8) && p->quant != ESSA_QUANT_INT8_PERCH)
            return essa_fail(ESSA_ERR_UNSUPPORTED, "%s: W8A8 needs int8 weights (item %d)", who, i);
        if ((flags & ESSA_COMPUTE_W8A8) && x_dtype != ESSA_BF16)
            return essa_fail(ESSA_ERR_UNSUPPORTED, "%s: W8A8 takes bf16 activations", who);
        if (it.R == 0) continue;
        if (flags & ESSA_VALIDATE) ESSA_TRY(validate_row2cand(ctx, it, i, who));
        essa_k::fwd_item k{};
        k.X = it.X; k.row2cand = it.row2cand; k.sigmaA = it.sigmaA; k.sigmaB = it.sigmaB; k.Y = it.Y;
        k.sigma_stride = it.sigma_stride; k.R = it.R; k.K = it.K;
        k.d_in = p->d_in; k.d_out = p->d_out; k.r = p->r; k.rp = p->rp; k.quant = p->quant; k.groups = p->groups;
        k.Wq = p->Wq; k.scale = p->scale; k.zero = p->zero; k.VA32 = p->VA32; k.VA16 = p->VA16;
        k.UB32 = p->UB32; k.UB16 = p->UB16; k.M = p->M;
        k.Wt = p->Wt; k.VAp = p->VAp; k.d_in_pad = p->d_in_pad; k.n_blocks = p->n_blocks;
        k.St = p->St; k.SZ16 = p->SZ16; k.Gp = p->Gp;
        if (rv) {
            k.rv = rv[i];
            k.rowpart = rowpart + block0 * (size_t)it.R;
            block0 += (size_t)(p->d_out + ESSA_REWARD_BLOCK - 1) / ESSA_REWARD_BLOCK;
        }
        out.push(k);
        const size_t R = it.R;
        total += align256(R * p->rp * 4) + align256(R * p->rp * 4) + align256(R * (p->groups > 0 ? p->groups : 1) * 4);
        if (flags & ESSA_COMPUTE_W8A8) total += align256(R * (size_t)p->d_in) + align256(R * 4);
        if (p->Wt) total += 2 * align256((R + 255) / 256 * 256 * (size_t)p->d_in_pad) + align256(R * 4) + align256(R * 2 * (size_t)(p->Gp + 16) * 2) +
                            align256((size_t)((R + 31) / 32 * 32) * p->rp * 8 * 4);
    }
    char* w;
    if (scratch) {
        if (total > scratch_bytes)
            return essa_fail(ESSA_ERR_SHAPE, "%s: this problem needs %zu bytes of scratch, the fixed buffer holds %zu", who, total, scratch_bytes);
        w = (char*)scratch;
    } else {
        ESSA_TRY(essa_ws_reserve(ctx, total));
        w = (char*)ctx->ws;
    }
    for (int ki = 0; ki < out.n; ++ki) {
        essa_k::fwd_item& k = out.it[ki];
        const size_t R = k.R;
        k.U32 = (float*)w; w += align256(R * k.rp * 4);
        k.SBrow = k.U32;                      // the int8-limb path keeps the gathered sigma_B where the generic path keeps u
        k.U16 = (uint16_t*)w; w += align256(R * k.rp * 4);
        k.xsum = (float*)w; w += align256(R * (k.groups > 0 ? k.groups : 1) * 4);
        if (flags & ESSA_COMPUTE_W8A8) {
            k.Xq = (int8_t*)w; w += align256(R * (size_t)k.d_in);
            k.xscale = (float*)w; w += align256(R * 4);
        }
        if (k.Wt) {
            k.tslices = essa_k::prep_slices(k.d_in);
            k.Tpart = (float*)w; w += align256((size_t)((R + 31) / 32 * 32) * k.rp * 8 * 4);
            // items reading the same X share one set of limbs; the first of them quantises
            const essa_k::fwd_item* first = nullptr;
            for (int oi = 0; oi < ki; ++oi) {
                const essa_k::fwd_item& o = out.it[oi];
                if (o.Wt && o.X == k.X && o.R == k.R && o.d_in == k.d_in && o.quant == k.quant) { first = &o; break; }
            }
            if (first) {
                k.Xh = first->Xh; k.Xl = first->Xl; k.xdelta = first->xdelta; k.XS16 = first->XS16; k.x_owner = 0;
            } else {
                const size_t limb = align256((R + 255) / 256 * 256 * (size_t)k.d_in_pad);
                k.Xh = (int8_t*)w; w += limb;
                k.Xl = (int8_t*)w; w += limb;
                k.xdelta = (float*)w; w += align256(R * 4);
                k.XS16 = (uint16_t*)w; w += align256(R * 2 * (size_t)(k.Gp + 16) * 2);
                k.x_owner = 1;
            }
        }
    }
    return ESSA_OK;
}

// int8 weights, bf16 activations, 16-byte rows: the int8-limb kernels take the item
static bool takes_stream(const essa_k::fwd_item& k, int x_dtype, unsigned flags) {
    // at most 8 K slices in the rank-space partial sums: 512 columns each up to d_in 4096, 1024 beyond
    return k.Wt && x_dtype == ESSA_BF16 && k.d_in % 16 == 0 && k.d_in <= 8192 && !(flags & ESSA_COMPUTE_BF16) && ((uintptr_t)k.X & 15) == 0 &&
           !(k.quant == ESSA_QUANT_INT4_G128 && (flags & ESSA_COMPUTE_W8A8));
}

static essa_status run_items(essa_ctx* ctx, item_list& ks, int x_dtype, int y_dtype, unsigned flags) {
    // three launch groups: int8 and 4-bit items on the int8-limb kernels (different instantiations of the GEMM), and the
    // rest on the generic kernels
    item_list f8, f4, rest;
    for (int i = 0; i < ks.n; ++i) {
        const essa_k::fwd_item& k = ks.it[i];
        if (!takes_stream(k, x_dtype, flags)) rest.push(k);
        else (k.quant == ESSA_QUANT_INT8_PERCH ? f8 : f4).push(k);
    }
    const unsigned kflags = flags & ~(ESSA_COMPUTE_BF16 | ESSA_VALIDATE);
    // while profiling, every GEMM launch of the call gets its own pair of events
    for (item_list* grp : {&f8, &f4}) {
        if (grp->n == 0) continue;
        for (int i = 0; i < grp->n; ++i) {                  // every set of limbs needs exactly one producer in its launch
            bool found = false;
            for (int j = 0; j < i; ++j) found = found || (grp->it[j].x_owner && grp->it[j].Xh == grp->it[i].Xh);
            grp->it[i].x_owner = found ? 0 : 1;
        }
        hipEvent_t e0, e1;
        ESSA_TRY(next_events(ctx, &e0, &e1));
        ESSA_HIP(essa_k::forward_stream(ctx->stream, grp->it, grp->n, y_dtype, kflags, e0, e1));
    }
    if (rest.n > 0) {
        hipEvent_t e0, e1;
        ESSA_TRY(next_events(ctx, &e0, &e1));
        ESSA_HIP(essa_k::forward_group(ctx->stream, rest.it, rest.n, x_dtype, y_dtype, kflags, e0, e1));
        ESSA_HIP(essa_k::rowdot_blocks(ctx->stream, rest.it, rest.n, y_dtype));   // no-op without reward vectors
    }
    return ESSA_OK;
}

essa_status essa_forward_on_scratch(essa_ctx* ctx, const essa_fwd_item* item, int x_dtype, int y_dtype, unsigned flags, void* scratch,
                                    size_t scratch_bytes, const char* who) {
    if (flags & ESSA_VALIDATE) return essa_fail(ESSA_ERR_INVALID_ARG, "%s: ESSA_VALIDATE allocates and waits; use the ordinary entry point for it", who);
    if (ctx->profiling && !ctx->capturing) return essa_fail(ESSA_ERR_STATE, "%s: profiling creates events; switch it off for this entry point", who);
    item_list ks;
    ESSA_TRY(plan_items(ctx, item, 1, x_dtype, y_dtype, flags, ks, who, nullptr, nullptr, scratch, scratch_bytes));
    if (ks.n == 0) return ESSA_OK;
    return run_items(ctx, ks, x_dtype, y_dtype, flags);
}

extern "C" essa_status essa_svdlora_forward_group(essa_ctx* ctx, const essa_fwd_item* items, int n_items, int x_dtype,
                                                  int y_dtype, uint32_t flags) {
    if (!ctx || !items) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_svdlora_forward_group: NULL argument");
    if (n_items < 1 || n_items > ESSA_MAX_GROUP) return essa_fail(ESSA_ERR_SHAPE, "essa_svdlora_forward_group: %d items, at most %d", n_items, ESSA_MAX_GROUP);
    ESSA_HIP(hipSetDevice(ctx->device));
    item_list ks;
    ESSA_TRY(plan_items(ctx, items, n_items, x_dtype, y_dtype, flags, ks, "essa_svdlora_forward_group"));
    if (ks.n == 0) return ESSA_OK;
    return run_items(ctx, ks, x_dtype, y_dtype, flags);
}

extern "C" essa_status essa_svdlora_forward_reward_group(essa_ctx* ctx, const essa_fwd_item* items, int n_items, int x_dtype,
                                                         int y_dtype, uint32_t flags, const float* const* v, float* rowpart,
                                                         int64_t block_capacity, int64_t block0) {
    const char* who = "essa_svdlora_forward_reward_group";
    if (!ctx || !items || !v || !rowpart) return essa_fail(ESSA_ERR_INVALID_ARG, "%s: NULL argument", who);
    if (n_items < 1 || n_items > ESSA_MAX_GROUP) return essa_fail(ESSA_ERR_SHAPE, "%s: %d items, at most %d", who, n_items, ESSA_MAX_GROUP);
    int64_t blocks = 0;
    for (int g = 0; g < n_items; ++g) {
        if (!v[g] || !items[g].proj) return essa_fail(ESSA_ERR_INVALID_ARG, "%s: item %d has no reward vector or no projection", who, g);
        if (items[g].R != items[0].R) return essa_fail(ESSA_ERR_SHAPE, "%s: item %d has R=%d, item 0 has R=%d", who, g, items[g].R, items[0].R);
        blocks += (items[g].proj->d_out + ESSA_REWARD_BLOCK - 1) / ESSA_REWARD_BLOCK;
    }
    if (block0 < 0 || block0 + blocks > block_capacity)
        return essa_fail(ESSA_ERR_SHAPE, "%s: blocks %lld..%lld do not fit a buffer of %lld", who, (long long)block0, (long long)(block0 + blocks), (long long)block_capacity);
    ESSA_HIP(hipSetDevice(ctx->device));
    item_list ks;
    ESSA_TRY(plan_items(ctx, items, n_items, x_dtype, y_dtype, flags, ks, who, v, rowpart + (size_t)block0 * (size_t)items[0].R));
    if (ks.n == 0) return ESSA_OK;
    return run_items(ctx, ks, x_dtype, y_dtype, flags);
}

extern "C" essa_status essa_reward_finish(essa_ctx* ctx, const float* rowpart, int64_t n_blocks, int R, const int32_t* row2cand, int K,
                                          float* F) {
    if (!ctx || !rowpart || !row2cand || !F) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_reward_finish: NULL argument");
    if (R < 1 || K < 1 || n_blocks < 1 || n_blocks > INT32_MAX) return essa_fail(ESSA_ERR_SHAPE, "essa_reward_finish: R=%d K=%d blocks=%lld", R, K, (long long)n_blocks);
    ESSA_HIP(hipSetDevice(ctx->device));
    ESSA_TRY(essa_ws_reserve(ctx, (size_t)essa_k::reward_slices((int)n_blocks) * R * sizeof(double)));
    ESSA_HIP(essa_k::reward_finish(ctx->stream, rowpart, (int)n_blocks, R, row2cand, K, (double*)ctx->ws, F));
    return ESSA_OK;
}

extern "C" essa_status essa_svdlora_forward(essa_ctx* ctx, const essa_proj* proj, const void* X, int x_dtype, int R,
                                            const int32_t* row2cand, const float* sigmaA, const float* sigmaB,
                                            int64_t sigma_stride, int K, void* Y, int y_dtype, uint32_t flags) {
    if (!ctx) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_svdlora_forward: ctx is NULL");
    essa_fwd_item it{proj, X, row2cand, sigmaA, sigmaB, Y, sigma_stride, R, K};
    item_list ks;
    ESSA_HIP(hipSetDevice(ctx->device));
    ESSA_TRY(plan_items(ctx, &it, 1, x_dtype, y_dtype, flags, ks, "essa_svdlora_forward"));
    if (ks.n == 0) return ESSA_OK;
    return run_items(ctx, ks, x_dtype, y_dtype, flags);
}

extern "C" essa_status essa_w8a8_accumulators(essa_ctx* ctx, const essa_proj* proj, const void* X, int x_dtype, int R,
                                              int8_t* xq_out, float* xscale_out, int32_t* acc_out) {
    if (!ctx || !proj || !X || !xq_out || !xscale_out || !acc_out) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_w8a8_accumulators: NULL argument");
    if (proj->quant != ESSA_QUANT_INT8_PERCH) return essa_fail(ESSA_ERR_UNSUPPORTED, "essa_w8a8_accumulators: int8 weights only");
    if (x_dtype != ESSA_BF16) return essa_fail(ESSA_ERR_UNSUPPORTED, "essa_w8a8_accumulators: bf16 activations only");
    if (R < 1) return essa_fail(ESSA_ERR_SHAPE, "essa_w8a8_accumulators: R=%d", R);
    ESSA_HIP(hipSetDevice(ctx->device));
    essa_k::fwd_item k{};
    k.X = X; k.R = R; k.K = 1;
    k.d_in = proj->d_in; k.d_out = proj->d_out; k.r = proj->r; k.rp = proj->rp; k.quant = proj->quant;
    k.Wq = proj->Wq; k.scale = proj->scale;
    if (proj->d_in % 16 == 0 && ((uintptr_t)X & 15) == 0) {
        // the production int8 kernel, one limb, dumping its accumulators
        k.Wt = proj->Wt; k.d_in_pad = proj->d_in_pad; k.n_blocks = proj->n_blocks;
        const size_t limb = align256((size_t)(R + 255) / 256 * 256 * (size_t)k.d_in_pad);
        ESSA_TRY(essa_ws_reserve(ctx, 2 * limb));
        k.Xh = (int8_t*)ctx->ws;
        k.Xl = k.Xh + limb;
        k.xdelta = xscale_out;
        ESSA_HIP(essa_k::w8a8_accumulators_stream(ctx->stream, k, acc_out));
        ESSA_HIP(hipMemcpy2DAsync(xq_out, (size_t)k.d_in, k.Xh, (size_t)k.d_in_pad, (size_t)k.d_in, (size_t)R,
                                  hipMemcpyDeviceToDevice, ctx->stream));
        return ESSA_OK;
    }
    k.Xq = xq_out; k.xscale = xscale_out;
    ESSA_HIP(essa_k::w8a8_accumulators(ctx->stream, k, x_dtype, acc_out));
    return ESSA_OK;
}

extern "C" essa_status essa_reward_accumulate_group(essa_ctx* ctx, int n_items, const void* const* Y, const int* d_out,
                                                    const float* const* v, int y_dtype, int R, const int32_t* row2cand, int K,
                                                    float* F) {
    if (!ctx || !Y || !d_out || !v || !row2cand || !F) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_reward_accumulate_group: NULL argument");
    if (n_items < 1 || n_items > ESSA_MAX_GROUP) return essa_fail(ESSA_ERR_SHAPE, "essa_reward_accumulate_group: %d items, at most %d", n_items, ESSA_MAX_GROUP);
    if (y_dtype != ESSA_F32 && y_dtype != ESSA_BF16) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_reward_accumulate_group: y_dtype %d", y_dtype);
    if (R < 1 || K < 1) return essa_fail(ESSA_ERR_SHAPE, "essa_reward_accumulate_group: R=%d K=%d", R, K);
    for (int g = 0; g < n_items; ++g) {
        if (!Y[g] || !v[g]) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_reward_accumulate_group: item %d has a NULL tensor", g);
        if (d_out[g] < 1) return essa_fail(ESSA_ERR_SHAPE, "essa_reward_accumulate_group: item %d has d_out=%d", g, d_out[g]);
    }
    ESSA_HIP(hipSetDevice(ctx->device));
    ESSA_TRY(essa_ws_reserve(ctx, align256((size_t)R * 4)));
    ESSA_HIP(essa_k::reward_accumulate(ctx->stream, n_items, Y, d_out, v, y_dtype, R, row2cand, K, (float*)ctx->ws, F));
    return ESSA_OK;
}

extern "C" essa_status essa_reward_accumulate(essa_ctx* ctx, const void* Y, int y_dtype, int R, int d_out, const float* v,
                                              const int32_t* row2cand, int K, float* F) {
    return essa_reward_accumulate_group(ctx, 1, &Y, &d_out, &v, y_dtype, R, row2cand, K, F);
}

// ---------------------------------------------------------------------------------------------
// hot path: ranking and update
// ---------------------------------------------------------------------------------------------
extern "C" essa_status essa_rank_rewards(essa_ctx* ctx, const float* rewards, int K, int32_t* order) {
    if (!ctx || !rewards || !order) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_rank_rewards: NULL argument");
    if (K < 1 || K > 1024) return essa_fail(ESSA_ERR_SHAPE, "essa_rank_rewards: K=%d not in [1, 1024]", K);
    ESSA_HIP(hipSetDevice(ctx->device));
    ESSA_HIP(essa_k::rank_rewards(ctx->stream, rewards, K, order));
    return ESSA_OK;
}

static essa_k::cma_consts make_consts(int n, int K, int kind, std::vector<float>& w) {
    // default strategy parameters of Hansen's tutorial, evaluated in fp64 on the host
    essa_k::cma_consts c{};
    c.n = n; c.K = K; c.mu = K / 2;
    std::vector<double> wd(K);
    double sum = 0, sum2 = 0;
    for (int i = 0; i < K; ++i) wd[i] = std::log((K + 1) / 2.0) - std::log(i + 1.0);
    for (int i = 0; i < c.mu; ++i) sum += wd[i];
    for (int i = 0; i < c.mu; ++i) { wd[i] /= sum; sum2 += wd[i] * wd[i]; }
    const double mu_eff = 1.0 / sum2, nn = n;
    const double c_sigma = (mu_eff + 2.0) / (nn + mu_eff + 5.0);
    const double d_sigma = 1.0 + 2.0 * std::fmax(0.0, std::sqrt((mu_eff - 1.0) / (nn + 1.0)) - 1.0) + c_sigma;
    const double c_c = (4.0 + mu_eff / nn) / (nn + 4.0 + 2.0 * mu_eff / nn);
    double c_1 = 2.0 / ((nn + 1.3) * (nn + 1.3) + mu_eff);
    double c_mu = std::fmin(1.0 - c_1, 2.0 * (mu_eff - 2.0 + 1.0 / mu_eff) / ((nn + 2.0) * (nn + 2.0) + mu_eff));
    const double chi_n = std::sqrt(nn) * (1.0 - 1.0 / (4.0 * nn) + 1.0 / (21.0 * nn * nn));
    c.ny = c.mu;
    double w_sum = 1.0;
    if (kind == ESSA_OPT_ACTIVE_CMA) {
        // tutorial, Eqs. (50)-(53), (58): the rank-mu rate with its extra 1/4, negative weights scaled to the smallest of three bounds
        c_mu = std::fmin(1.0 - c_1, 2.0 * (0.25 + mu_eff + 1.0 / mu_eff - 2.0) / ((nn + 2.0) * (nn + 2.0) + mu_eff));
        double nsum = 0, nsum2 = 0;
        for (int i = c.mu; i < K; ++i) { nsum += wd[i]; nsum2 += wd[i] * wd[i]; }
        const double mu_eff_neg = nsum2 > 0 ? nsum * nsum / nsum2 : 0.0;
        const double a_mu = 1.0 + c_1 / c_mu, a_mueff = 1.0 + 2.0 * mu_eff_neg / (mu_eff + 2.0), a_pd = (1.0 - c_1 - c_mu) / (nn * c_mu);
        const double a = std::fmin(a_mu, std::fmin(a_mueff, a_pd));
        for (int i = c.mu; i < K; ++i) { wd[i] = nsum < 0 ? a * wd[i] / -nsum : 0.0; w_sum += wd[i]; }
        c.ny = K;
    } else if (kind == ESSA_OPT_SEP_CMA) {
        // Ros & Hansen 2008: both learning rates of the (now diagonal) covariance times (n + 2) / 3
        const double f = (nn + 2.0) / 3.0;
        c_1 = std::fmin(1.0, c_1 * f);
        c_mu = std::fmin(1.0 - c_1, c_mu * f);
    }
    c.mu_eff = (float)mu_eff; c.c_sigma = (float)c_sigma; c.d_sigma = (float)d_sigma; c.c_c = (float)c_c;
    c.c_1 = (float)c_1; c.c_mu = (float)c_mu; c.chi_n = (float)chi_n; c.w_sum = (float)w_sum;
    w.resize(c.ny);
    for (int i = 0; i < c.ny; ++i) w[i] = (float)wd[i];
    return c;
}

extern "C" essa_status essa_cma_refresh_basis(essa_ctx* ctx, essa_cma* cma, int max_sweeps, float tol, int* sweeps_out, float* off_out) {
    if (!ctx || !cma) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_cma_refresh_basis: NULL argument");
    if (cma->ctx != ctx) return essa_fail(ESSA_ERR_STATE, "essa_cma_refresh_basis: state belongs to another context");
    if (!has_matrix(cma)) return essa_fail(ESSA_ERR_STATE, "essa_cma_refresh_basis: an optimiser of kind %d keeps no covariance matrix", cma->kind);
    if (ctx->capturing) return essa_fail(ESSA_ERR_STATE, "essa_cma_refresh_basis: waits for the device after every sweep and cannot be recorded");
    if (max_sweeps < 1 || max_sweeps > 64 || !(tol >= 0.f)) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_cma_refresh_basis: max_sweeps=%d tol=%g", max_sweeps, (double)tol);
    ESSA_HIP(hipSetDevice(ctx->device));
    ESSA_TRY(essa_ws_reserve(ctx, essa_k::eig_workspace_bytes(cma->n)));
    if (!cma->eigV) {
        hipError_t e = hipMalloc((void**)&cma->eigV, essa_k::eig_basis_bytes(cma->n));
        if (e != hipSuccess) return essa_fail(ESSA_ERR_OOM, "fp64 basis of %zu bytes: %s", essa_k::eig_basis_bytes(cma->n), hipGetErrorString(e));
        cma->eigV_valid = false;
    }
    int sweeps = 0;
    float off = 0.f;
    ESSA_HIP(essa_k::eig_refresh(ctx->stream, cma->C, cma->n, ctx->ws, cma->eigV, cma->eigV_valid ? 1 : 0, max_sweeps, tol, cma->B, cma->D,
                                 &sweeps, &off));
    cma->eigV_valid = true;
    if (sweeps_out) *sweeps_out = sweeps;
    if (off_out) *off_out = off;
    if (off > tol) return essa_fail(ESSA_ERR_STATE, "essa_cma_refresh_basis: not converged after %d sweeps (largest relative off-diagonal %g > %g); B and D hold the last iterate", sweeps, (double)off, (double)tol);
    return ESSA_OK;
}

extern "C" essa_status essa_cmaes_update(essa_ctx* ctx, essa_cma* cma, const uint32_t* seeds, const float* rewards, int K,
                                         int32_t* order_out) {
    if (!ctx || !cma || !seeds || !rewards) return essa_fail(ESSA_ERR_INVALID_ARG, "essa_cmaes_update: NULL argument");
    if (cma->ctx != ctx) return essa_fail(ESSA_ERR_STATE, "essa_cmaes_update: state belongs to another context");
    if (K < 2 || K > 1024) return essa_fail(ESSA_ERR_SHAPE, "essa_cmaes_update: K=%d not in [2, 1024]", K);
    ESSA_HIP(hipSetDevice(ctx->device));
    const int n = cma->n;

    if (cma->kind == ESSA_OPT_ARS) {
        // Mania, Guy & Recht 2018, Algorithm 1: scratch order[N] | coef[b] | Z[b, n]
        const int N = K / 2, b = cma->ars_top;
        if (K & 1) return essa_fail(ESSA_ERR_SHAPE, "essa_cmaes_update: ARS evaluates candidates in pairs, K=%d is odd", K);
        if (b > N) return essa_fail(ESSA_ERR_SHAPE, "essa_cmaes_update: ARS keeps %d directions, only %d were evaluated", b, N);
        const size_t off_coef = align256((size_t)N * 4), off_Z = off_coef + align256((size_t)b * 4);
        ESSA_TRY(essa_ws_reserve(ctx, off_Z + align256((size_t)b * n * 4)));
        int32_t* order = (int32_t*)ctx->ws;
        float* coef = (float*)((char*)ctx->ws + off_coef);
        float* Z = (float*)((char*)ctx->ws + off_Z);
        ESSA_HIP(essa_k::ars_prepare(ctx->stream, rewards, N, b, cma->ars_alpha, order, coef));
        if (order_out) ESSA_HIP(hipMemcpyAsync(order_out, order, (size_t)N * 4, hipMemcpyDeviceToDevice, ctx->stream));
        ESSA_HIP(essa_k::normals_scaled(ctx->stream, seeds, order, b, n, nullptr, Z, nullptr));
        ESSA_HIP(essa_k::mean_step(ctx->stream, Z, coef, 0.0, b, n, cma->sc, 0, cma->m));
        return ESSA_OK;
    }
    if (cma->kind == ESSA_OPT_ES) {
        // plain (mu/mu_I, lambda)-ES: scratch order[K] | Z[mu, n]
        const int mu = K / 2;
        const size_t off_Z = align256((size_t)K * 4);
        ESSA_TRY(essa_ws_reserve(ctx, off_Z + align256((size_t)mu * n * 4)));
        int32_t* order = (int32_t*)ctx->ws;
        float* Z = (float*)((char*)ctx->ws + off_Z);
        if (K <= essa_k::kRankInKernelMax) {
            ESSA_HIP(essa_k::normals_scaled(ctx->stream, seeds, nullptr, mu, n, nullptr, Z, nullptr, rewards, K, order));
        } else {
            ESSA_HIP(essa_k::rank_rewards(ctx->stream, rewards, K, order));
            ESSA_HIP(essa_k::normals_scaled(ctx->stream, seeds, order, mu, n, nullptr, Z, nullptr));
        }
        if (order_out) ESSA_HIP(hipMemcpyAsync(order_out, order, (size_t)K * 4, hipMemcpyDeviceToDevice, ctx->stream));
        ESSA_HIP(essa_k::mean_step(ctx->stream, Z, nullptr, 1.0 / mu, mu, n, cma->sc, 1, cma->m));
        return ESSA_OK;
    }

    std::vector<float> w;
    essa_k::cma_consts c = make_consts(n, K, cma->kind, w);
    if (cma->weights_K != K) {
        if (ctx->capturing)
            return essa_fail(ESSA_ERR_STATE, "essa_cmaes_update: the weights for K=%d are not on the device yet: run the update once before essa_graph_begin", K);
        if (!ctx->graphs.empty() && cma->weights)
            return essa_fail(ESSA_ERR_STATE, "essa_cmaes_update: K changed from %d to %d while %zu recorded graph(s) of this context may still read the old weights: destroy them first", cma->weights_K, K, ctx->graphs.size());
        ESSA_HIP(hipStreamSynchronize(ctx->stream));
        if (cma->weights) ESSA_HIP(hipFree(cma->weights));
        cma->weights = nullptr;
        cma->weights_K = 0;
        ESSA_TRY(upload(&cma->weights, w.data(), w.size()));
        cma->weights_K = K;
    }
    // scratch: order[K] | zn2[ny] | S[(ny+2), n] | BY[(ny+2), n] | Z[ny, n];  S rows: D*z_i (i < ny), z_w, D*z_w
    const size_t rows = (size_t)c.ny + 2;
    const size_t off_zn = align256((size_t)K * 4), off_S = off_zn + align256((size_t)c.ny * 4), off_BY = off_S + align256(rows * n * 4);
    const size_t off_Z = off_BY + align256(rows * n * 4);
    ESSA_TRY(essa_ws_reserve(ctx, off_Z + align256(rows * n * 4)));
    int32_t* order = (int32_t*)ctx->ws;
    float* zn2 = (float*)((char*)ctx->ws + off_zn);
    float* S = (float*)((char*)ctx->ws + off_S);
    float* BY = (float*)((char*)ctx->ws + off_BY);
    float* Z = (float*)((char*)ctx->ws + off_Z);
    // the ranking: inside the kernel that regenerates the normals when the population is small, else a launch of its own
    const bool rank_inside = K <= essa_k::kRankInKernelMax;
    if (!rank_inside) ESSA_HIP(essa_k::rank_rewards(ctx->stream, rewards, K, order));
    ESSA_HIP(essa_k::cma_build_rhs(ctx->stream, seeds, order, rank_inside ? rewards : nullptr, cma->weights, c, cma->D, S, Z));
    if (order_out) ESSA_HIP(hipMemcpyAsync(order_out, order, (size_t)K * 4, hipMemcpyDeviceToDevice, ctx->stream));
    if (cma->kind == ESSA_OPT_SEP_CMA) {
        // B = I: the rows of S are the y_i, z_w and y_w themselves
        ESSA_HIP(essa_k::cma_vectors(ctx->stream, c, cma->weights, S, cma->m, cma->p_sigma, cma->p_c, cma->sc));
        ESSA_HIP(essa_k::sep_covariance(ctx->stream, c, cma->weights, S, cma->p_c, cma->sc, cma->Cdiag, cma->D));
        return ESSA_OK;
    }
    if (cma->kind == ESSA_OPT_ACTIVE_CMA) ESSA_HIP(essa_k::row_norms2(ctx->stream, Z, c.ny, n, zn2));
    ESSA_HIP(essa_k::skinny_gemm_nt(ctx->stream, S, (int)rows, cma->B, n, nullptr, nullptr, 0, BY));
    ESSA_HIP(essa_k::cma_vectors(ctx->stream, c, cma->weights, BY, cma->m, cma->p_sigma, cma->p_c, cma->sc));
    ESSA_HIP(essa_k::cma_covariance(ctx->stream, c, cma->weights, BY, cma->p_c, cma->sc, cma->kind == ESSA_OPT_ACTIVE_CMA ? zn2 : nullptr, cma->C));
    return ESSA_OK;
}
