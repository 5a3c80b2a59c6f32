// C ABI of libspotlight: argument checks (host only, before any HIP call), the context and its
// workspace, stage timing, and the three calls of the decode step.
#include <new>
#include <string.h>

#include "internal.h"

namespace spotlight {

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

int make_plan(const spotlight_config* c, Plan* p)
{
    if (!c) return SPOTLIGHT_ERR_INVALID_ARG;
    if (c->batch < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1) return SPOTLIGHT_ERR_INVALID_ARG;
    if (c->n_q_heads % c->n_kv_heads != 0) return SPOTLIGHT_ERR_INVALID_ARG;
    if (c->code_bits < 32 || c->code_bits > 1024 || c->code_bits % 32 != 0) return SPOTLIGHT_ERR_INVALID_ARG;
    if (c->hidden < 0 || c->hidden > 4096) return SPOTLIGHT_ERR_INVALID_ARG;
    if (c->max_tokens < 1 || c->max_tokens > 0x7fffffffLL) return SPOTLIGHT_ERR_INVALID_ARG;
    if (c->max_topk < 1 || c->max_topk > c->max_tokens) return SPOTLIGHT_ERR_INVALID_ARG;
    if ((c->kv_dtype != SPOTLIGHT_F32 && c->kv_dtype != SPOTLIGHT_BF16) ||
        (c->weight_dtype != SPOTLIGHT_F32 && c->weight_dtype != SPOTLIGHT_BF16))
        return SPOTLIGHT_ERR_INVALID_ARG;
    if (c->head_dim != kHeadDim) return SPOTLIGHT_ERR_UNSUPPORTED;
    const int G = c->n_q_heads / c->n_kv_heads;
    if (G > kMaxGroup) return SPOTLIGHT_ERR_UNSUPPORTED;
    // code lengths: every multiple of 32 up to 512 bits, and 1024 bits with at most two query heads per kv head
    if (c->code_bits > 512 && (c->code_bits != 1024 || G > 2)) return SPOTLIGHT_ERR_UNSUPPORTED;
    if (c->hidden % 8 != 0) return SPOTLIGHT_ERR_UNSUPPORTED;
    if (static_cast<int64_t>(c->batch) * c->n_q_heads > 65535) return SPOTLIGHT_ERR_UNSUPPORTED;

    p->B = c->batch;
    p->Hq = c->n_q_heads;
    p->Hkv = c->n_kv_heads;
    p->G = G;
    p->L = c->code_bits;
    p->W = c->code_bits / 32;
    p->hidden = c->hidden;
    p->Nmax = c->max_tokens;
    p->max_topk = c->max_topk;
    p->kv_dtype = c->kv_dtype;
    p->w_dtype = c->weight_dtype;

    p->max_blocks = static_cast<int>((p->Nmax + kTokensPerBlock - 1) / kTokensPerBlock);
    p->max_splits = (p->max_topk + kAttendMinRows - 1) / kAttendMinRows;

    const size_t BH = static_cast<size_t>(p->B) * p->Hq;
    const size_t bins = static_cast<size_t>(p->L) + 2;   // one bin for forced tokens, L + 1 for distances 0 .. L
    size_t off = 0;
    p->off_qcode = off;     off = align_up(off + BH * p->W * 4, 256);
    p->off_gcum = off;      off = align_up(off + BH * bins * 4, 256);
    p->off_blockcum = off;  off = align_up(off + BH * p->max_blocks * bins * 4, 256);
    p->off_blockmeta = off; off = align_up(off + BH * p->max_blocks * 8, 256);
    p->off_cand = off;      off = align_up(off + BH * p->max_blocks * static_cast<size_t>(kCandCap) * 4, 256);
    p->off_part_ml = off;   off = align_up(off + BH * p->max_splits * 8, 256);
    p->off_part_acc = off;  off = align_up(off + BH * p->max_splits * static_cast<size_t>(kHeadDim) * 4, 256);
    p->off_wnorm = off;     off = align_up(off + static_cast<size_t>(p->Hkv) * p->L * 4, 256);
    pack_sizes(p->hidden, p->L, &p->pack_w1_elems, &p->pack_out_elems);
    const size_t welem = p->w_dtype == SPOTLIGHT_BF16 ? 2 : 4;
    p->off_pack_w1 = off;   off = align_up(off + static_cast<size_t>(p->Hkv) * p->pack_w1_elems * welem, 256);
    p->off_pack_out = off;  off = align_up(off + static_cast<size_t>(p->Hkv) * p->pack_out_elems * welem, 256);
    p->off_audit = off;     off = align_up(off + sizeof(AuditRec), 256);
    p->total_bytes = off;
    return SPOTLIGHT_OK;
}

StageTimer::StageTimer(spotlight_ctx* c, int stage) : ctx(c), rec(nullptr)
{
    if (!c->profiling || c->n_rec >= kMaxProfile) return;
    ProfileRec* r = &c->recs[c->n_rec];
    if (c->n_rec >= c->n_events) {
        if (hipEventCreate(&r->start) != hipSuccess) return;
        if (hipEventCreate(&r->stop) != hipSuccess) { (void)hipEventDestroy(r->start); return; }
        c->n_events = c->n_rec + 1;
    }
    r->stage = stage;
    rec = r;
}

int allow_dynamic_lds(spotlight_ctx* ctx, const void* kernel, size_t bytes)
{
    if (bytes <= 48 * 1024) return SPOTLIGHT_OK;
    for (int i = 0; i < ctx->n_big_lds_kernels; ++i)
        if (ctx->big_lds_kernels[i] == kernel) return SPOTLIGHT_OK;
    // the limit is raised to all the LDS a workgroup may have, so that one call serves every later size
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, ctx->max_lds) != hipSuccess)
        return SPOTLIGHT_ERR_HIP;
    const int cap = static_cast<int>(sizeof(ctx->big_lds_kernels) / sizeof(ctx->big_lds_kernels[0]));
    if (ctx->n_big_lds_kernels < cap) ctx->big_lds_kernels[ctx->n_big_lds_kernels++] = kernel;
    return SPOTLIGHT_OK;
}

static bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

static int check_weights(const spotlight_ctx* ctx, const spotlight_hash_weights* w)
{
    if (!w || !w->w1) return SPOTLIGHT_ERR_INVALID_ARG;
    if (ctx->plan.hidden > 0 && (!w->b1 || !w->w2)) return SPOTLIGHT_ERR_INVALID_ARG;
    if (misaligned(w->w1) || (ctx->plan.hidden > 0 && misaligned(w->w2))) return SPOTLIGHT_ERR_INVALID_ARG;
    return SPOTLIGHT_OK;
}

}  // namespace spotlight

using namespace spotlight;

extern "C" {

int spotlight_validate_config(const spotlight_config* cfg)
{
    Plan p;
    return make_plan(cfg, &p);
}

size_t spotlight_workspace_bytes(const spotlight_config* cfg)
{
    Plan p;
    if (make_plan(cfg, &p) != SPOTLIGHT_OK) return 0;
    return p.total_bytes;
}

const char* spotlight_strerror(int rc)
{
    switch (rc) {
    case SPOTLIGHT_OK: return "ok";
    case SPOTLIGHT_ERR_INVALID_ARG: return "invalid argument";
    case SPOTLIGHT_ERR_UNSUPPORTED: return "unsupported configuration";
    case SPOTLIGHT_ERR_WORKSPACE: return "workspace allocation failed";
    case SPOTLIGHT_ERR_HIP: return "HIP runtime error";
    case SPOTLIGHT_ERR_TOO_LARGE: return "problem too large for the static scratch buffer";
    default: return "unknown error";
    }
}

int spotlight_create(spotlight_ctx** out, const spotlight_config* cfg)
{
    if (!out) return SPOTLIGHT_ERR_INVALID_ARG;
    Plan plan;
    const int rc = make_plan(cfg, &plan);
    if (rc != SPOTLIGHT_OK) return rc;
    spotlight_ctx* ctx = new (std::nothrow) spotlight_ctx;
    if (!ctx) return SPOTLIGHT_ERR_WORKSPACE;
    memset(ctx, 0, sizeof(*ctx));
    ctx->cfg = *cfg;
    ctx->plan = plan;
    ctx->stream = static_cast<hipStream_t>(cfg->stream);
    ctx->recs = new (std::nothrow) ProfileRec[kMaxProfile];
    if (!ctx->recs) { delete ctx; return SPOTLIGHT_ERR_WORKSPACE; }
    int dev = 0, lds = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) {
        delete[] ctx->recs;
        delete ctx;
        return SPOTLIGHT_ERR_HIP;
    }
    ctx->max_lds = lds;
    ctx->n_cus = cus;
    ctx->opt[SPOTLIGHT_OPT_BULK_HASH_MATRIX_CORES] = 1;
    void* ws = nullptr;
    if (hipMalloc(&ws, plan.total_bytes) != hipSuccess) {
        (void)hipGetLastError();
        delete[] ctx->recs;
        delete ctx;
        return SPOTLIGHT_ERR_WORKSPACE;
    }
    ctx->workspace = static_cast<char*>(ws);
    if (hipMemsetAsync(ctx->workspace + plan.off_audit, 0, sizeof(AuditRec), ctx->stream) != hipSuccess) {
        (void)hipFree(ws);
        delete[] ctx->recs;
        delete ctx;
        return SPOTLIGHT_ERR_HIP;
    }
    *out = ctx;
    return SPOTLIGHT_OK;
}

int spotlight_destroy(spotlight_ctx* ctx)
{
    if (!ctx) return SPOTLIGHT_OK;
    int rc = hip_rc(hipStreamSynchronize(ctx->stream));
    for (int i = 0; i < ctx->n_events; ++i) {
        (void)hipEventDestroy(ctx->recs[i].start);
        (void)hipEventDestroy(ctx->recs[i].stop);
    }
    if (ctx->workspace && hipFree(ctx->workspace) != hipSuccess) rc = SPOTLIGHT_ERR_HIP;
    delete[] ctx->recs;
    delete ctx;
    return rc;
}

#ifndef SPOTLIGHT_BUILD_ID_STRING
#define SPOTLIGHT_BUILD_ID_STRING "SPOTLIGHT_BUILD_ID=unknown"
#endif
const char* spotlight_build_id(void) { return SPOTLIGHT_BUILD_ID_STRING; }

int spotlight_set_option(spotlight_ctx* ctx, int option, int value)
{
    if (!ctx || option < 0 || option >= SPOTLIGHT_OPT_COUNT || (value != 0 && value != 1)) return SPOTLIGHT_ERR_INVALID_ARG;
    ctx->opt[option] = value;
    return SPOTLIGHT_OK;
}

int spotlight_bulk_hash_audit_read(spotlight_ctx* ctx, int64_t* outputs, int64_t* listed, int64_t* wrong,
                                   double* max_ratio, double* eps)
{
    if (!ctx) return SPOTLIGHT_ERR_INVALID_ARG;
    AuditRec rec;
    char* dev = ctx->workspace + ctx->plan.off_audit;
    if (hipMemcpyAsync(&rec, dev, sizeof(rec), hipMemcpyDeviceToHost, ctx->stream) != hipSuccess ||
        hipMemsetAsync(dev, 0, sizeof(rec), ctx->stream) != hipSuccess ||
        hipStreamSynchronize(ctx->stream) != hipSuccess)
        return SPOTLIGHT_ERR_HIP;
    if (outputs) *outputs = static_cast<int64_t>(rec.outputs);
    if (listed) *listed = static_cast<int64_t>(rec.listed);
    if (wrong) *wrong = static_cast<int64_t>(rec.wrong);
    if (max_ratio) {
        float f;
        memcpy(&f, &rec.max_ratio_bits, sizeof(f));
        *max_ratio = f;
    }
    if (eps) *eps = bulk_hash_eps(ctx->plan.hidden);
    return SPOTLIGHT_OK;
}

int spotlight_set_stream(spotlight_ctx* ctx, void* stream)
{
    if (!ctx) return SPOTLIGHT_ERR_INVALID_ARG;
    ctx->stream = static_cast<hipStream_t>(stream);
    return SPOTLIGHT_OK;
}

// The packed copy of the weights serves a job only if it was made from exactly these arrays.
static void attach_packed(const spotlight_ctx* ctx, const spotlight_hash_weights* w, HashLaunch* h)
{
    const Plan& p = ctx->plan;
    const bool match = ctx->packed_w1 && ctx->packed_w1 == w->w1 && ctx->packed_b1 == w->b1 && ctx->packed_w2 == w->w2;
    h->pack_w1 = match && p.pack_w1_elems ? ctx->workspace + p.off_pack_w1 : nullptr;
    h->pack_out = match && p.pack_out_elems ? ctx->workspace + p.off_pack_out : nullptr;
}

// The hash job of n_new key rows of every (batch, kv head), written into the code cache.
static HashLaunch key_job(const spotlight_ctx* ctx, const void* K, const spotlight_hash_weights* w, int64_t t0,
                          int64_t n_new, uint32_t* codes)
{
    const Plan& p = ctx->plan;
    HashLaunch h;
    h.x = K;
    h.x_dtype = p.kv_dtype;
    h.x_head_stride = p.Nmax * kHeadDim;
    h.x_row0 = t0;
    h.n_rows = n_new;
    h.n_xheads = p.B * p.Hkv;
    h.heads_per_batch = p.Hkv;
    h.group = 1;
    h.w1 = w->w1;
    h.b1 = w->b1;
    h.w2 = w->w2;
    h.w_dtype = p.w_dtype;
    h.hidden = p.hidden;
    h.L = p.L;
    h.codes = codes;
    h.code_head_stride = p.Nmax * p.W;
    h.code_row0 = t0;
    h.zero = nullptr;
    h.zero_words = 0;
    h.wnorm = ctx->opt[SPOTLIGHT_OPT_BULK_HASH_MATRIX_CORES] ? reinterpret_cast<float*>(ctx->workspace + p.off_wnorm) : nullptr;
    h.audit = ctx->opt[SPOTLIGHT_OPT_BULK_HASH_AUDIT] ? reinterpret_cast<AuditRec*>(ctx->workspace + p.off_audit) : nullptr;
    attach_packed(ctx, w, &h);
    return h;
}

// The hash job of the queries, written into the workspace; it also clears the heads' cumulative
// histograms, which the score kernel adds into.
static HashLaunch query_job(const spotlight_ctx* ctx, const void* q, const spotlight_hash_weights* w)
{
    const Plan& p = ctx->plan;
    HashLaunch h;
    h.x = q;
    h.x_dtype = p.kv_dtype;
    h.x_head_stride = kHeadDim;
    h.x_row0 = 0;
    h.n_rows = 1;
    h.n_xheads = p.B * p.Hq;
    h.heads_per_batch = p.Hq;
    h.group = p.G;
    h.w1 = w->w1;
    h.b1 = w->b1;
    h.w2 = w->w2;
    h.w_dtype = p.w_dtype;
    h.hidden = p.hidden;
    h.L = p.L;
    h.codes = reinterpret_cast<uint32_t*>(ctx->workspace + p.off_qcode);
    h.code_head_stride = p.W;
    h.code_row0 = 0;
    h.zero = reinterpret_cast<uint32_t*>(ctx->workspace + p.off_gcum);
    h.zero_words = p.L + 2;
    h.wnorm = nullptr;
    h.audit = nullptr;
    attach_packed(ctx, w, &h);
    return h;
}

int spotlight_prepack_weights(spotlight_ctx* ctx, const spotlight_hash_weights* w)
{
    if (!ctx) return SPOTLIGHT_ERR_INVALID_ARG;
    ctx->packed_w1 = ctx->packed_b1 = ctx->packed_w2 = nullptr;
    if (!w) return SPOTLIGHT_OK;   // the copy is dropped
    const Plan& p = ctx->plan;
    const int rc = check_weights(ctx, w);
    if (rc != SPOTLIGHT_OK) return rc;
    if (p.pack_out_elems == 0) return SPOTLIGHT_OK;   // no kernel would read a copy for this hash shape
    const int rc2 = launch_pack_weights(ctx, w->w1, w->w2, p.w_dtype, ctx->workspace + p.off_pack_w1,
                                        ctx->workspace + p.off_pack_out);
    if (rc2 != SPOTLIGHT_OK) return rc2;
    ctx->packed_w1 = w->w1;
    ctx->packed_b1 = w->b1;
    ctx->packed_w2 = w->w2;
    return SPOTLIGHT_OK;
}

int spotlight_hash_keys(spotlight_ctx* ctx, const void* K, const spotlight_hash_weights* w, int64_t t0,
                        int64_t n_new, uint32_t* codes)
{
    if (!ctx || !K || !codes) return SPOTLIGHT_ERR_INVALID_ARG;
    const Plan& p = ctx->plan;
    int rc = check_weights(ctx, w);
    if (rc != SPOTLIGHT_OK) return rc;
    if (t0 < 0 || n_new < 0 || t0 > p.Nmax || n_new > p.Nmax - t0) return SPOTLIGHT_ERR_INVALID_ARG;
    if (misaligned(K) || misaligned(codes)) return SPOTLIGHT_ERR_INVALID_ARG;
    if (n_new == 0) return SPOTLIGHT_OK;
    return launch_hash(ctx, key_job(ctx, K, w, t0, n_new, codes), SPOTLIGHT_STAGE_HASH_KEYS);
}

int spotlight_retrieve_topk(spotlight_ctx* ctx, const void* q, const spotlight_hash_weights* w,
                            const uint32_t* codes, int64_t n_tokens, int32_t k, int32_t* out_idx,
                            uint32_t* out_qcode, uint16_t* out_dist)
{
    if (!ctx || !q || !codes || !out_idx) return SPOTLIGHT_ERR_INVALID_ARG;
    const Plan& p = ctx->plan;
    int rc = check_weights(ctx, w);
    if (rc != SPOTLIGHT_OK) return rc;
    if (n_tokens < 1 || n_tokens > p.Nmax) return SPOTLIGHT_ERR_INVALID_ARG;
    if (k < 1 || k > n_tokens || k > p.max_topk) return SPOTLIGHT_ERR_INVALID_ARG;
    if (misaligned(q) || misaligned(codes)) return SPOTLIGHT_ERR_INVALID_ARG;

    rc = launch_hash(ctx, query_job(ctx, q, w), SPOTLIGHT_STAGE_HASH_QUERY);
    if (rc != SPOTLIGHT_OK) return rc;
    if (out_qcode) {
        if (hipMemcpyAsync(out_qcode, ctx->workspace + p.off_qcode, static_cast<size_t>(p.B) * p.Hq * p.W * 4,
                           hipMemcpyDeviceToDevice, ctx->stream) != hipSuccess)
            return SPOTLIGHT_ERR_HIP;
    }
    return launch_retrieve(ctx, codes, n_tokens, k, 0, 0, out_idx, out_dist);
}

}  // extern "C"

namespace spotlight {

// Host-only argument checks of the decode step.
int check_step_args(const spotlight_ctx* ctx, const void* q, const void* K, const void* V, const spotlight_hash_weights* w,
                    const uint32_t* codes, int64_t n_tokens, int32_t k, int32_t n_sink, int32_t n_local,
                    const int32_t* out_idx, const float* out)
{
    if (!ctx || !q || !K || !V || !codes || !out_idx || !out) return SPOTLIGHT_ERR_INVALID_ARG;
    const Plan& p = ctx->plan;
    const int rc = check_weights(ctx, w);
    if (rc != SPOTLIGHT_OK) return rc;
    if (n_tokens < 1 || n_tokens > p.Nmax) return SPOTLIGHT_ERR_INVALID_ARG;
    if (k < 1 || k > n_tokens || k > p.max_topk) return SPOTLIGHT_ERR_INVALID_ARG;
    if (n_sink < 0 || n_local < 0) return SPOTLIGHT_ERR_INVALID_ARG;
    const int64_t n_forced = static_cast<int64_t>(n_sink) + n_local >= n_tokens ? n_tokens : static_cast<int64_t>(n_sink) + n_local;
    if (n_forced > k) return SPOTLIGHT_ERR_INVALID_ARG;
    if (misaligned(q) || misaligned(K) || misaligned(V) || misaligned(codes)) return SPOTLIGHT_ERR_INVALID_ARG;
    return SPOTLIGHT_OK;
}

// The decode step of spotlight_decode_step and spotlight_decode_step_noalloc: argument checks, then five launches.
int decode_step(spotlight_ctx* ctx, const void* q, const void* K, const void* V, const spotlight_hash_weights* w,
                uint32_t* codes, int64_t n_tokens, int32_t k, int32_t n_sink, int32_t n_local, float scale,
                int32_t* out_idx, float* out)
{
    int rc = check_step_args(ctx, q, K, V, w, codes, n_tokens, k, n_sink, n_local, out_idx, out);
    if (rc != SPOTLIGHT_OK) return rc;
    if (step_small_applies(ctx, n_tokens))   // a short context: the whole step is one kernel
        return launch_step_small(ctx, query_job(ctx, q, w), key_job(ctx, K, w, n_tokens - 1, 1, codes), q, K, V, codes,
                                 n_tokens, k, n_sink, n_local, scale, out_idx, out);
    // queries first: their workgroups also clear the histograms
    rc = launch_hash_pair(ctx, query_job(ctx, q, w), key_job(ctx, K, w, n_tokens - 1, 1, codes), SPOTLIGHT_STAGE_HASH_QUERY);
    if (rc != SPOTLIGHT_OK) return rc;
    rc = launch_retrieve(ctx, codes, n_tokens, k, n_sink, n_local, out_idx, nullptr);
    if (rc != SPOTLIGHT_OK) return rc;
    return launch_attend(ctx, q, K, V, out_idx, k, scale, out);
}

}  // namespace spotlight

extern "C" {

int spotlight_decode_step(spotlight_ctx* ctx, const void* q, const void* K, const void* V,
                          const spotlight_hash_weights* w, uint32_t* codes, int64_t n_tokens, int32_t k,
                          int32_t n_sink, int32_t n_local, float scale, int32_t* out_idx, float* out)
{
    return decode_step(ctx, q, K, V, w, codes, n_tokens, k, n_sink, n_local, scale, out_idx, out);
}

int spotlight_sparse_decode(spotlight_ctx* ctx, const void* q, const void* K, const void* V, const int32_t* idx,
                            int32_t k, float scale, float* out)
{
    if (!ctx || !q || !K || !V || !idx || !out) return SPOTLIGHT_ERR_INVALID_ARG;
    const Plan& p = ctx->plan;
    if (k < 1 || k > p.max_topk) return SPOTLIGHT_ERR_INVALID_ARG;
    if (misaligned(q) || misaligned(K) || misaligned(V)) return SPOTLIGHT_ERR_INVALID_ARG;
    return launch_attend(ctx, q, K, V, idx, k, scale, out);
}

int spotlight_profile_enable(spotlight_ctx* ctx, int on)
{
    if (!ctx) return SPOTLIGHT_ERR_INVALID_ARG;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SPOTLIGHT_ERR_HIP;
    ctx->profiling = on ? 1 : 0;
    ctx->n_rec = 0;
    for (int s = 0; s < SPOTLIGHT_STAGE_COUNT; ++s) { ctx->stage_ms[s] = 0.0; ctx->stage_launches[s] = 0; }
    return SPOTLIGHT_OK;
}

int spotlight_profile_read(spotlight_ctx* ctx, int stage, double* total_ms, int64_t* launches)
{
    if (!ctx || stage < 0 || stage >= SPOTLIGHT_STAGE_COUNT) return SPOTLIGHT_ERR_INVALID_ARG;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SPOTLIGHT_ERR_HIP;
    int rc = SPOTLIGHT_OK;
    for (int i = 0; i < ctx->n_rec; ++i) {
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, ctx->recs[i].start, ctx->recs[i].stop) != hipSuccess) { rc = SPOTLIGHT_ERR_HIP; continue; }
        ctx->stage_ms[ctx->recs[i].stage] += ms;
        ctx->stage_launches[ctx->recs[i].stage] += 1;
    }
    ctx->n_rec = 0;
    if (total_ms) *total_ms = ctx->stage_ms[stage];
    if (launches) *launches = ctx->stage_launches[stage];
    return rc;
}

}  // extern "C"
