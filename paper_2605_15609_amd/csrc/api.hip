// C ABI of libpsd: argument checks, handle management and the Alg. 1 block loop.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <new>

#include "psd_internal.h"

static thread_local char g_err[512] = "";

void psd_set_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

namespace {

// A sequence enters a block: the number of masks in it, and which positions they are (a 64-bit set in the
// sequence's counters).  only != NULL: just the sequences b with only[b] != 0.
__global__ void count_masks_kernel(const int32_t *__restrict__ tokens, int N, BlockStart bs, int L, int32_t mask_id,
                                   int32_t *__restrict__ n_left, int32_t *__restrict__ devstats,
                                   const int32_t *__restrict__ only) {
    const int b = blockIdx.x, j = threadIdx.x;
    if (only && only[b] == 0) return;
    const bool live = j < L && tokens[(int64_t)b * N + bs.of_row(b) + j] == mask_id;
    const uint64_t set = __ballot(live);
    if (j == 0) {
        n_left[b] = __popcll(set);
        devstats[(int64_t)b * PSD_DEVSTAT_WORDS + PSD_DEVSTAT_ENTRY] = (int32_t)(uint32_t)set;
        devstats[(int64_t)b * PSD_DEVSTAT_WORDS + PSD_DEVSTAT_ENTRY + 1] = (int32_t)(uint32_t)(set >> 32);
        devstats[(int64_t)b * PSD_DEVSTAT_WORDS + PSD_DEVSTAT_EOS] = 0;
    }
}

__global__ void fill_i32_kernel(int32_t *p, int64_t n, int32_t v) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

int32_t check_cfg(const psd_model_config *c) {
    if (!c) PSD_FAIL(PSD_ERR_INVALID_ARG, "config is NULL");
    if (c->n_layers < 1 || c->d_model < 1 || c->n_heads < 1 || c->n_kv_heads < 1 || c->d_head < 2 || c->d_ffn < 1 ||
        c->vocab < 2 || c->max_seq < 1)
        PSD_FAIL(PSD_ERR_SHAPE, "non-positive model dimension");
    if (c->n_heads % c->n_kv_heads) PSD_FAIL(PSD_ERR_SHAPE, "n_heads must be a multiple of n_kv_heads");
    if (c->d_head % 2) PSD_FAIL(PSD_ERR_SHAPE, "d_head must be even (rotary pairs)");
    if (c->mask_id < 0 || c->mask_id >= c->vocab) PSD_FAIL(PSD_ERR_SHAPE, "mask_id outside the embedding table");
    if (c->dtype != PSD_DTYPE_FP32 && c->dtype != PSD_DTYPE_BF16) PSD_FAIL(PSD_ERR_UNSUPPORTED, "dtype %d", c->dtype);
    if (c->attention != PSD_ATTN_BIDIRECTIONAL && c->attention != PSD_ATTN_BLOCK_CAUSAL)
        PSD_FAIL(PSD_ERR_UNSUPPORTED, "attention mode %d", c->attention);
    if (c->dtype == PSD_DTYPE_BF16) {
        if (c->d_head != 64 && c->d_head != 128) PSD_FAIL(PSD_ERR_UNSUPPORTED, "bf16 path needs d_head 64 or 128");
        if (c->d_model % 64 || c->d_ffn % 64) PSD_FAIL(PSD_ERR_UNSUPPORTED, "bf16 path needs d_model, d_ffn multiples of 64");
    }
    return PSD_OK;
}

int32_t check_block(const psd_handle *h, int B, int N, int block_start, int L) {
    if (!h) PSD_FAIL(PSD_ERR_INVALID_ARG, "handle is NULL");
    if (B < 1) PSD_FAIL(PSD_ERR_SHAPE, "batch %d", B);
    if (N < 1 || N > h->cfg.max_seq) PSD_FAIL(PSD_ERR_SHAPE, "sequence length %d outside 1..max_seq=%d", N, h->cfg.max_seq);
    if (L < 1 || L > PSD_MAX_BLOCK) PSD_FAIL(PSD_ERR_SHAPE, "block length %d outside 1..%d", L, PSD_MAX_BLOCK);
    if (block_start < 0 || block_start + L > N) PSD_FAIL(PSD_ERR_SHAPE, "block [%d, %d) outside the sequence of %d", block_start,
                                                         block_start + L, N);
    return PSD_OK;
}

int32_t check_graph(const psd_graph *g, GraphArg *out) {
    if (!g) PSD_FAIL(PSD_ERR_INVALID_ARG, "graph is NULL");
    if (g->K < 1 || g->K > PSD_MAX_NODES) PSD_FAIL(PSD_ERR_SHAPE, "graph with %d nodes (1..%d)", g->K, PSD_MAX_NODES);
    if (g->rank_set[0] != 0) PSD_FAIL(PSD_ERR_INVALID_ARG, "node 0 must be the root (empty rank set)");
    out->K = g->K;
    for (int k = 0; k < PSD_MAX_NODES; ++k) out->rank_set[k] = k < g->K ? g->rank_set[k] : 0;
    return PSD_OK;
}

int32_t check_policy(const psd_policy *p) {
    if (!p) PSD_FAIL(PSD_ERR_INVALID_ARG, "policy is NULL");
    if (p->k_min < 0 || p->k_max < 0) PSD_FAIL(PSD_ERR_INVALID_ARG, "negative k_min / k_max");
    if (p->tau != p->tau) PSD_FAIL(PSD_ERR_INVALID_ARG, "tau is NaN");
    return PSD_OK;
}

#define CHECK(expr)                  \
    do {                             \
        int32_t rc_ = (expr);        \
        if (rc_ != PSD_OK) return rc_; \
    } while (0)

struct DecodeScratch {
    int64_t top1, conf, sigma, m, n_left, drafts, v_top1, v_conf, k_star, accepted, devstats, rows, starts, flags, total;
};

DecodeScratch plan_decode(int64_t B, int64_t N, int64_t L, int64_t K) {
    DecodeScratch s;
    int64_t off = 0;
    auto take = [&](int64_t bytes) {
        const int64_t o = off;
        off += align_up(bytes, 256);
        return o;
    };
    s.top1 = take(B * L * 4);
    s.conf = take(B * L * 4);
    s.sigma = take(B * L * 4);
    s.m = take(B * 4);
    s.n_left = take(B * 4);
    s.drafts = take(B * K * N * 4);
    s.v_top1 = take(B * K * L * 4);
    s.v_conf = take(B * K * L * 4);
    s.k_star = take(B * 4);
    s.accepted = take(B * K);
    s.devstats = take(B * PSD_DEVSTAT_WORDS * 4);
    s.rows = take(B * K * 4);
    s.starts = take(B * 4);
    s.flags = take(B * 4);
    s.total = off;
    return s;
}

}   // namespace

static std::atomic<int> g_kernel_choice_epoch{0};
int kernel_choice_epoch() { return g_kernel_choice_epoch.load(); }
void bump_kernel_choice_epoch() { g_kernel_choice_epoch.fetch_add(1); }

extern "C" {

const char *psd_status_string(int32_t status) {
    switch (status) {
        case PSD_OK: return "ok";
        case PSD_ERR_INVALID_ARG: return "invalid argument";
        case PSD_ERR_SHAPE: return "shape out of range";
        case PSD_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case PSD_ERR_DEVICE: return "HIP device error";
        case PSD_ERR_UNSUPPORTED: return "unsupported configuration";
        default: return "unknown status";
    }
}

const char *psd_last_error(void) { return g_err; }

int32_t psd_create(const psd_model_config *cfg, const psd_weights *w, psd_handle **out) {
    if (!out) PSD_FAIL(PSD_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    CHECK(check_cfg(cfg));
    if (!w) PSD_FAIL(PSD_ERR_INVALID_ARG, "weights is NULL");
    if (!w->tok_emb || !w->final_norm || !w->lm_head || !w->rope_cos || !w->rope_sin || !w->attn_norm || !w->wq || !w->wk ||
        !w->wv || !w->wo || !w->ffn_norm || !w->w_gate || !w->w_up || !w->w_down)
        PSD_FAIL(PSD_ERR_INVALID_ARG, "a weight pointer is NULL");
    if (cfg->qkv_bias && (!w->bq || !w->bk || !w->bv)) PSD_FAIL(PSD_ERR_INVALID_ARG, "qkv_bias set but a bias array is NULL");
    if (w->w_down_stride != 0 && (w->w_down_stride < cfg->d_ffn || w->w_down_stride % 8 || w->w_down_stride > (1 << 20)))
        PSD_FAIL(PSD_ERR_SHAPE, "w_down_stride %d: 0 or a multiple of 8 in [d_ffn, 2^20]", w->w_down_stride);
    int dev = 0;
    PSD_HIP(hipGetDevice(&dev));
    hipDeviceProp_t prop;
    PSD_HIP(hipGetDeviceProperties(&prop, dev));
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
        PSD_FAIL(PSD_ERR_DEVICE, "device %d is %s; this library is built for gfx950 only", dev, prop.gcnArchName);
    psd_handle *h = new (std::nothrow) psd_handle();
    if (!h) PSD_FAIL(PSD_ERR_DEVICE, "out of host memory");
    h->cfg = *cfg;
    h->tok_emb = w->tok_emb;
    h->lm_head = w->lm_head;
    h->final_norm = w->final_norm;
    h->rope_cos = w->rope_cos;
    h->rope_sin = w->rope_sin;
    h->w_down_stride = w->w_down_stride ? w->w_down_stride : cfg->d_ffn;
    h->device = dev;
    h->plain_mask = 0;
    h->layers.resize(cfg->n_layers);
    for (int l = 0; l < cfg->n_layers; ++l) {
        psd_handle::Layer &L = h->layers[l];
        L.attn_norm = w->attn_norm[l];
        L.ffn_norm = w->ffn_norm[l];
        L.wq = w->wq[l];
        L.wk = w->wk[l];
        L.wv = w->wv[l];
        L.wo = w->wo[l];
        L.w_gate = w->w_gate[l];
        L.w_up = w->w_up[l];
        L.w_down = w->w_down[l];
        L.bq = cfg->qkv_bias ? w->bq[l] : nullptr;
        L.bk = cfg->qkv_bias ? w->bk[l] : nullptr;
        L.bv = cfg->qkv_bias ? w->bv[l] : nullptr;
        if (!L.attn_norm || !L.ffn_norm || !L.wq || !L.wk || !L.wv || !L.wo || !L.w_gate || !L.w_up || !L.w_down ||
            (cfg->qkv_bias && (!L.bq || !L.bk || !L.bv))) {
            delete h;
            PSD_FAIL(PSD_ERR_INVALID_ARG, "layer %d has a NULL weight pointer", l);
        }
    }
    h->lm_head_packed = nullptr;
    if (cfg->dtype == PSD_DTYPE_BF16) {
        // second copy of the LM-head in MFMA-fragment order for the streaming confidence pass
        hipError_t pe = hipMalloc(&h->lm_head_packed, packed_rows_bytes(cfg->vocab, cfg->d_model));
        if (pe != hipSuccess) {
            delete h;
            PSD_FAIL(PSD_ERR_DEVICE, "hipMalloc of the packed LM-head: %s", hipGetErrorString(pe));
        }
        launch_pack_rows((const bf16_t *)w->lm_head, cfg->vocab, cfg->d_model, (bf16_t *)h->lm_head_packed, nullptr);
        pe = hipDeviceSynchronize();
        if (pe != hipSuccess) {
            (void)hipFree(h->lm_head_packed);
            delete h;
            PSD_FAIL(PSD_ERR_DEVICE, "packing the LM-head: %s", hipGetErrorString(pe));
        }
    }
    h->host_counts_cap = 1 << 16;
    hipError_t e = hipHostMalloc((void **)&h->host_counts, sizeof(int32_t) * h->host_counts_cap, hipHostMallocDefault);
    if (e != hipSuccess) {
        if (h->lm_head_packed) (void)hipFree(h->lm_head_packed);
        delete h;
        PSD_FAIL(PSD_ERR_DEVICE, "hipHostMalloc: %s", hipGetErrorString(e));
    }
    *out = h;
    return PSD_OK;
}

int32_t psd_destroy(psd_handle *h) {
    if (!h) return PSD_OK;
    if (h->host_counts) (void)hipHostFree(h->host_counts);
    if (h->lm_head_packed) (void)hipFree(h->lm_head_packed);
    for (hipEvent_t e : h->probe.ev) (void)hipEventDestroy(e);
    for (hipEvent_t e : h->probe_head.ev) (void)hipEventDestroy(e);
    for (hipEvent_t e : h->probe_call.ev) (void)hipEventDestroy(e);
    for (psd_handle::GraphEntry &g : h->graphs)
        if (g.exec) (void)hipGraphExecDestroy(g.exec);
    if (h->capture_stream) (void)hipStreamDestroy(h->capture_stream);
    delete h;
    return PSD_OK;
}

int32_t psd_debug_set_plain(psd_handle *h, int32_t mask) {
    if (!h) PSD_FAIL(PSD_ERR_INVALID_ARG, "handle is NULL");
    h->plain_mask = mask;
    bump_kernel_choice_epoch();
    return PSD_OK;
}

int32_t psd_debug_force_gemm_tile(int32_t tile) {
    gemm_bf16_force_tile(tile);
    bump_kernel_choice_epoch();
    return PSD_OK;
}

int32_t psd_debug_set_graphs(psd_handle *h, int32_t enabled, int64_t *replays) {
    if (!h) PSD_FAIL(PSD_ERR_INVALID_ARG, "handle is NULL");
    if (replays) *replays = (int64_t)h->graph_replays;
    if (enabled >= 0) h->graphs_enabled = enabled != 0;
    return PSD_OK;
}

namespace {
psd_handle::Probe &probe_of(psd_handle *h, int32_t kind) { return kind == 4 ? h->probe_head : kind == 5 ? h->probe_call : h->probe; }
}   // namespace

int32_t psd_probe_begin(psd_handle *h, int32_t epilogue, int32_t tile, int32_t max_launches) {
    if (!h) PSD_FAIL(PSD_ERR_INVALID_ARG, "handle is NULL");
    if (epilogue < 0 || epilogue > 5 || tile < 0 || tile >= gemm_bf16_tile_count() || max_launches < 1 || max_launches > (1 << 20))
        PSD_FAIL(PSD_ERR_INVALID_ARG, "bad probe arguments");
    psd_handle::Probe &pr = probe_of(h, epilogue);
    while (pr.ev.size() < (size_t)max_launches * 2) {
        hipEvent_t e;
        PSD_HIP(hipEventCreate(&e));
        pr.ev.push_back(e);
    }
    pr.enabled = 1;
    pr.epi = epilogue;
    pr.tile = tile;
    pr.used = 0;
    pr.flops = 0.0;
    pr.a.clear();
    pr.b.clear();
    return PSD_OK;
}

int32_t psd_probe_end(psd_handle *h, int32_t epilogue, double *total_ms, int64_t *launches, double *flops) {
    if (!h || !total_ms || !launches || !flops) PSD_FAIL(PSD_ERR_INVALID_ARG, "NULL argument");
    if (epilogue < 0 || epilogue > 5) PSD_FAIL(PSD_ERR_INVALID_ARG, "probe kind %d", epilogue);
    psd_handle::Probe &pr = probe_of(h, epilogue);
    pr.enabled = 0;
    double ms = 0.0;
    for (size_t i = 0; i + 1 < pr.used; i += 2) {
        PSD_HIP(hipEventSynchronize(pr.ev[i + 1]));
        float t = 0.f;
        PSD_HIP(hipEventElapsedTime(&t, pr.ev[i], pr.ev[i + 1]));
        ms += t;
    }
    *total_ms = ms;
    *launches = (int64_t)(pr.used / 2);
    *flops = pr.flops;
    return PSD_OK;
}

int32_t psd_probe_read(psd_handle *h, int32_t epilogue, int32_t max_n, float *ms, int64_t *a, int64_t *b) {
    if (!h || !ms || !a || !b || max_n < 0) PSD_FAIL(PSD_ERR_INVALID_ARG, "bad arguments");
    if (epilogue < 0 || epilogue > 5) PSD_FAIL(PSD_ERR_INVALID_ARG, "probe kind %d", epilogue);
    psd_handle::Probe &pr = probe_of(h, epilogue);
    if (pr.enabled) PSD_FAIL(PSD_ERR_INVALID_ARG, "the probe is still running: call psd_probe_end first");
    const size_t n = std::min<size_t>(pr.used / 2, (size_t)max_n);
    for (size_t i = 0; i < n; ++i) {
        float t = 0.f;
        PSD_HIP(hipEventElapsedTime(&t, pr.ev[2 * i], pr.ev[2 * i + 1]));
        ms[i] = t;
        a[i] = i < pr.a.size() ? pr.a[i] : 0;
        b[i] = i < pr.b.size() ? pr.b[i] : 0;
    }
    return (int32_t)n;
}

int64_t psd_workspace_bytes(const psd_model_config *cfg, int32_t max_seqs, int32_t N, int32_t L) {
    int32_t rc = check_cfg(cfg);
    if (rc != PSD_OK) return rc;
    if (max_seqs < 1 || N < 1 || L < 1 || L > PSD_MAX_BLOCK || L > N) {
        psd_set_error("psd_workspace_bytes: bad max_seqs/N/L %d/%d/%d", max_seqs, N, L);
        return PSD_ERR_SHAPE;
    }
    return plan_forward(*cfg, max_seqs, N, L).total;
}

int64_t psd_decode_scratch_bytes(int32_t B, int32_t N, int32_t L, int32_t K) {
    if (B < 1 || N < 1 || L < 1 || K < 1) {
        psd_set_error("psd_decode_scratch_bytes: bad B/N/L/K");
        return PSD_ERR_SHAPE;
    }
    return plan_decode(B, N, L, K).total;
}

int32_t psd_struct_sizes(int32_t *out, int32_t n) {
    const int32_t sizes[] = {(int32_t)sizeof(psd_model_config), (int32_t)sizeof(psd_weights), (int32_t)sizeof(psd_policy),
                             (int32_t)sizeof(psd_graph),        (int32_t)sizeof(psd_stats),   (int32_t)sizeof(psd_work),
                             (int32_t)sizeof(psd_graph_score), (int32_t)sizeof(psd_debug_layout)};
    const int32_t count = (int32_t)(sizeof(sizes) / sizeof(sizes[0]));
    for (int32_t i = 0; out && i < n && i < count; ++i) out[i] = sizes[i];
    return count;
}

int32_t psd_graph_chain(int32_t K, int32_t width, psd_graph *out) {
    if (!out) PSD_FAIL(PSD_ERR_INVALID_ARG, "out is NULL");
    if (K < 1 || K > PSD_MAX_NODES || width < 1) PSD_FAIL(PSD_ERR_SHAPE, "chain with K=%d width=%d", K, width);
    if ((int64_t)(K - 1) * width > 64) PSD_FAIL(PSD_ERR_SHAPE, "chain deeper than 64 ranks");
    memset(out, 0, sizeof(*out));
    out->K = K;
    for (int k = 0; k < K; ++k) {
        const int n = k * width;
        out->rank_set[k] = n >= 64 ? ~0ull : ((1ull << n) - 1ull);
    }
    return PSD_OK;
}

int32_t psd_graph_lattice(int32_t depth, psd_graph *out) {
    if (!out) PSD_FAIL(PSD_ERR_INVALID_ARG, "out is NULL");
    if (depth < 0 || (1 << depth) > PSD_MAX_NODES) PSD_FAIL(PSD_ERR_SHAPE, "lattice over %d ranks (0..5)", depth);
    memset(out, 0, sizeof(*out));
    out->K = 1 << depth;
    int k = 0;
    for (int size = 0; size <= depth; ++size)            // by subset size, then by value: the root comes first
        for (uint64_t set = 0; set < (1ull << depth); ++set)
            if (__builtin_popcountll(set) == size) out->rank_set[k++] = set;
    return PSD_OK;
}

int32_t psd_forward_confidence(psd_handle *h, const int32_t *tokens, int32_t S, int32_t N, int32_t block_start, int32_t L,
                               int32_t *top1, float *conf, void *ws, int64_t ws_bytes, void *stream) {
    CHECK(check_block(h, S, N, block_start, L));
    if (!tokens || !top1 || !conf) PSD_FAIL(PSD_ERR_INVALID_ARG, "NULL tokens/top1/conf");
    hipStream_t st = (hipStream_t)stream;
    CHECK(run_forward_hidden(h, tokens, nullptr, S, N, block_start, L, ws, ws_bytes, st));
    return run_head_confidence(h, tokens, nullptr, S, N, block_start, L, top1, conf, nullptr, ws, st);
}

int32_t psd_forward_logits(psd_handle *h, const int32_t *tokens, int32_t S, int32_t N, int32_t block_start, int32_t L,
                           float *logits, void *ws, int64_t ws_bytes, void *stream) {
    CHECK(check_block(h, S, N, block_start, L));
    if (!tokens || !logits) PSD_FAIL(PSD_ERR_INVALID_ARG, "NULL tokens/logits");
    hipStream_t st = (hipStream_t)stream;
    CHECK(run_forward_hidden(h, tokens, nullptr, S, N, block_start, L, ws, ws_bytes, st));
    return run_head_logits(h, S, N, L, logits, ws, st);
}

int32_t psd_debug_workspace_layout(const psd_model_config *cfg, int32_t S, int32_t N, int32_t L, psd_debug_layout *out) {
    CHECK(check_cfg(cfg));
    if (!out || S < 1 || N < 1 || L < 1 || L > PSD_MAX_BLOCK || L > N) PSD_FAIL(PSD_ERR_INVALID_ARG, "bad arguments");
    const ForwardPlan p = plan_forward(*cfg, S, N, L);
    out->off_a = p.off_a;
    out->off_qkv = p.off_qkv;
    out->off_vt = p.off_vt;
    out->off_o = p.off_o;
    out->off_act = p.off_act;
    out->ld_qkv = (int32_t)qkv_row_stride((int64_t)(cfg->n_heads + 2 * cfg->n_kv_heads) * cfg->d_head);
    out->ld_act = (int32_t)act_row_stride(*cfg);
    out->ld_vt = (int32_t)vt_row_stride(N);
    return PSD_OK;
}

int32_t psd_debug_layer(psd_handle *h, int32_t layer, float *hidden, int32_t S, int32_t N, int32_t L, int32_t stop_after, void *ws,
                        int64_t ws_bytes, void *stream) {
    CHECK(check_block(h, S, N, 0, L));
    if (!hidden) PSD_FAIL(PSD_ERR_INVALID_ARG, "hidden is NULL");
    if (layer < 0 || layer >= h->cfg.n_layers) PSD_FAIL(PSD_ERR_SHAPE, "layer %d outside 0..%d", layer, h->cfg.n_layers - 1);
    if (stop_after != 0 && stop_after != 1) PSD_FAIL(PSD_ERR_INVALID_ARG, "stop_after %d", stop_after);
    return run_debug_layer(h, layer, hidden, S, N, L, stop_after, ws, ws_bytes, (hipStream_t)stream);
}

int32_t psd_select_unmask(psd_handle *h, int32_t *tokens, int32_t B, int32_t N, int32_t block_start, int32_t L,
                          const int32_t *top1, const float *conf, const psd_policy *policy, uint8_t *transfer_mask,
                          int32_t *n_selected, void *stream) {
    CHECK(check_block(h, B, N, block_start, L));
    CHECK(check_policy(policy));
    if (!tokens || !top1 || !conf) PSD_FAIL(PSD_ERR_INVALID_ARG, "NULL tokens/top1/conf");
    launch_select_unmask(tokens, B, N, block_start, L, top1, conf, *policy, h->cfg.mask_id, transfer_mask, n_selected,
                         nullptr, nullptr, nullptr, (hipStream_t)stream);
    PSD_HIP(hipGetLastError());
    return PSD_OK;
}

int32_t psd_build_drafts(psd_handle *h, const int32_t *tokens, int32_t B, int32_t N, int32_t block_start, int32_t L,
                         const int32_t *top1, const float *conf, const psd_graph *graph, int32_t *sigma, int32_t *m,
                         int32_t *drafts, void *stream) {
    CHECK(check_block(h, B, N, block_start, L));
    GraphArg g;
    CHECK(check_graph(graph, &g));
    if (!tokens || !top1 || !conf || !sigma || !m || !drafts) PSD_FAIL(PSD_ERR_INVALID_ARG, "NULL argument");
    launch_build_drafts(tokens, B, N, block_start, L, top1, conf, g, h->cfg.mask_id, sigma, m, drafts, (hipStream_t)stream);
    PSD_HIP(hipGetLastError());
    return PSD_OK;
}

int32_t psd_accept(psd_handle *h, int32_t *tokens, const int32_t *drafts, int32_t B, int32_t N, int32_t block_start,
                   int32_t L, const int32_t *sigma, const int32_t *m, const psd_graph *graph, const psd_policy *policy,
                   const int32_t *v_top1, const float *v_conf, int32_t *k_star, uint8_t *accepted, void *stream) {
    CHECK(check_block(h, B, N, block_start, L));
    GraphArg g;
    CHECK(check_graph(graph, &g));
    CHECK(check_policy(policy));
    if (!tokens || !drafts || !sigma || !m || !v_top1 || !v_conf) PSD_FAIL(PSD_ERR_INVALID_ARG, "NULL argument");
    launch_accept(tokens, drafts, B, N, block_start, L, sigma, m, g, *policy, h->cfg.mask_id, v_top1, v_conf, k_star,
                  accepted, nullptr, nullptr, nullptr, nullptr, (hipStream_t)stream);
    PSD_HIP(hipGetLastError());
    return PSD_OK;
}

int32_t psd_verify_accept(psd_handle *h, int32_t *tokens, const int32_t *drafts, int32_t B, int32_t N, int32_t block_start,
                          int32_t L, const int32_t *sigma, const int32_t *m, const psd_graph *graph,
                          const psd_policy *policy, int32_t *k_star, uint8_t *accepted, int32_t *v_top1, float *v_conf,
                          void *ws, int64_t ws_bytes, void *stream) {
    CHECK(check_block(h, B, N, block_start, L));
    GraphArg g;
    CHECK(check_graph(graph, &g));
    CHECK(check_policy(policy));
    if (!tokens || !drafts || !sigma || !m || !v_top1 || !v_conf) PSD_FAIL(PSD_ERR_INVALID_ARG, "NULL argument");
    hipStream_t st = (hipStream_t)stream;
    const int S = B * g.K;
    CHECK(run_forward_hidden(h, drafts, nullptr, S, N, block_start, L, ws, ws_bytes, st));
    CHECK(run_head_confidence(h, drafts, nullptr, S, N, block_start, L, v_top1, v_conf, nullptr, ws, st));
    launch_accept(tokens, drafts, B, N, block_start, L, sigma, m, g, *policy, h->cfg.mask_id, v_top1, v_conf, k_star,
                  accepted, nullptr, nullptr, nullptr, nullptr, st);
    PSD_HIP(hipGetLastError());
    return PSD_OK;
}

namespace {

// Alg. 1 over B sequences, each on its own block (Alg. 1; App. B.1 for the outer loop over blocks and EOS stopping).
// starts [B] (host, in/out): first position of every sequence's current block.  advance = false: every sequence
// decodes that one block and is done; advance = true: a sequence whose block is resolved moves on to the next one
// (start + L) in the following iteration, until the end of the sequence -- the semi-autoregressive outer loop.  An
// iteration is one stage-1 call over all running sequences plus one batched verification call over those that still
// have masks after the stage-1 commit.  policy->single_forward: a sequence that went through a verification in this
// call and is still inside its block has no stage-1 call in the next iteration -- the accept kernel left the verifier
// output of its accepted draft in (top1, conf), its post-verification commit was the stage-1 commit, and the drafts
// are built from those tables.  max_iterations > 0 ends the call after that many iterations (starts then says
// where every sequence stands).  kv != NULL: model calls on the block rows against the sequences' KV caches; all
// sequences must then share one block and advance must be false.
int32_t decode_impl(psd_handle *h, int32_t *tokens, int32_t B, int32_t N, int32_t *starts, int32_t L, const psd_policy *policy,
                    const psd_graph *graph, psd_stats *stats, bool advance, int32_t max_iterations, int32_t *iterations_done,
                    void *ws, int64_t ws_bytes, void *stream, const KvCacheArg *kv) {
    if (!h) PSD_FAIL(PSD_ERR_INVALID_ARG, "handle is NULL");
    if (!starts) PSD_FAIL(PSD_ERR_INVALID_ARG, "block starts are NULL");
    if (B < 1) PSD_FAIL(PSD_ERR_SHAPE, "batch %d", B);
    for (int b = 0; b < B; ++b) {
        if (advance && starts[b] >= N) continue;          // a sequence that is already at its end
        CHECK(check_block(h, 1, N, starts[b], L));
        if (kv && starts[b] != starts[0]) PSD_FAIL(PSD_ERR_UNSUPPORTED, "cached model calls need one block start for the whole batch");
    }
    if (kv && advance) PSD_FAIL(PSD_ERR_UNSUPPORTED, "cached model calls decode one block per call");
    GraphArg g;
    CHECK(check_graph(graph, &g));
    CHECK(check_policy(policy));
    const bool eos_stop = policy->eos_stop != 0;
    const bool single_forward = policy->single_forward != 0;
    if (single_forward && kv && kv->dual)
        PSD_FAIL(PSD_ERR_UNSUPPORTED, "the single-forward loop is not built for the approximate cache");
    if (eos_stop && (policy->eos_id < 0 || policy->eos_id >= h->cfg.vocab || policy->eos_id == h->cfg.mask_id))
        PSD_FAIL(PSD_ERR_INVALID_ARG, "eos_id %d: a token id below the vocabulary size %d other than the mask token",
                 policy->eos_id, h->cfg.vocab);
    if (!tokens || !stats) PSD_FAIL(PSD_ERR_INVALID_ARG, "NULL tokens/stats");
    if (max_iterations < 0) PSD_FAIL(PSD_ERR_INVALID_ARG, "max_iterations %d", max_iterations);
    const int K = g.K;
    const bool dual = kv && kv->dual;  // approximate cache: the first model call runs over whole sequences and fills it
    const int plan_N = kv ? L : N;     // rows per sequence that a model call runs over
    int64_t fwd_bytes = plan_forward(h->cfg, (int64_t)B * K, plan_N, L).total;
    if (dual) fwd_bytes = std::max(fwd_bytes, plan_forward(h->cfg, B, N, L).total);
    const DecodeScratch sc = plan_decode(B, N, L, K);
    if (!ws || ws_bytes < fwd_bytes + sc.total)
        PSD_FAIL(PSD_ERR_WORKSPACE, "workspace of %lld bytes, decoding needs %lld", (long long)ws_bytes,
                 (long long)(fwd_bytes + sc.total));
    if ((reinterpret_cast<uintptr_t>(ws) & 255) != 0) PSD_FAIL(PSD_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    if ((int64_t)B * (K + 4 + PSD_DEVSTAT_WORDS) > h->host_counts_cap) PSD_FAIL(PSD_ERR_SHAPE, "batch too large for the control buffer");
    hipStream_t st = (hipStream_t)stream;
    char *base = (char *)ws + fwd_bytes;
    int32_t *top1 = (int32_t *)(base + sc.top1), *sigma = (int32_t *)(base + sc.sigma), *m = (int32_t *)(base + sc.m);
    int32_t *n_left = (int32_t *)(base + sc.n_left), *drafts = (int32_t *)(base + sc.drafts);
    int32_t *v_top1 = (int32_t *)(base + sc.v_top1), *k_star = (int32_t *)(base + sc.k_star);
    int32_t *devstats = (int32_t *)(base + sc.devstats), *rows = (int32_t *)(base + sc.rows);
    int32_t *d_starts = (int32_t *)(base + sc.starts), *d_flags = (int32_t *)(base + sc.flags);
    float *conf = (float *)(base + sc.conf), *v_conf = (float *)(base + sc.v_conf);
    uint8_t *accepted = (uint8_t *)(base + sc.accepted);
    // pinned staging: [0, B) counts read back; [B, B + B*K) row lists; then block starts, flags, final counters
    int32_t *hc = h->host_counts;
    int32_t *hrows = hc + B, *hstarts = hrows + (int64_t)B * K, *hflags = hstarts + B, *hstats = hflags + B;
    const int32_t mask_id = h->cfg.mask_id;
    // whole-sequence model calls take the block start of every sequence from the device array; the cached calls use the
    // common one (their KV lengths and rotary positions are per call)
    const BlockStart bs_seq = kv ? BlockStart(starts[0]) : BlockStart(d_starts, 1);
    const BlockStart bs_draft = kv ? BlockStart(starts[0]) : BlockStart(d_starts, K);

    // one model call: forward + top-1 confidence of the sequences listed in `rows` (device) out of src [*, N]
    bool refreshed = false;
    auto model_call_eager = [&](const int32_t *src, const int32_t *rows_dev, int S, int seqs_per_cache, const BlockStart &bs,
                                int32_t *t1, float *cf, hipStream_t st_) -> int32_t {
        if (dual && !refreshed) {   // the stage-1 call that enters the block: exact, and it freezes the context
            refreshed = true;
            CHECK(run_forward_hidden(h, src, rows_dev, S, N, bs, L, ws, fwd_bytes, st_, kv));
            return run_head_confidence(h, src, rows_dev, S, N, bs, L, t1, cf, rows_dev, ws, st_, N);
        }
        if (kv) {
            KvCacheArg a = *kv;
            a.seqs_per_cache = seqs_per_cache;
            a.append = false;
            CHECK(run_forward_cached(h, src, rows_dev, S, N, bs.common, L, a, ws, fwd_bytes, st_));
        } else {
            CHECK(run_forward_hidden(h, src, rows_dev, S, N, bs, L, ws, fwd_bytes, st_));
        }
        return run_head_confidence(h, src, rows_dev, S, N, bs, L, t1, cf, rows_dev, ws, st_, plan_N);
    };
    // Whole-sequence calls go through the handle's graph cache: what changes between two calls of one key (the tokens,
    // the row list, the block starts) lives in device memory the kernels read, not in their arguments.
    auto model_call_untimed = [&](const int32_t *src, const int32_t *rows_dev, int S, int seqs_per_cache, const BlockStart &bs,
                                  int32_t *t1, float *cf, hipStream_t st_) -> int32_t {
        const bool probing = h->probe.enabled || h->probe_head.enabled || h->probe_call.enabled;
        if (kv || !h->graphs_enabled || probing) return model_call_eager(src, rows_dev, S, seqs_per_cache, bs, t1, cf, st_);
        const psd_handle::GraphKey key = {src, rows_dev, t1, cf, ws, bs.per_seq, fwd_bytes, S, N, L, bs.common, bs.rows_per_seq,
                                          kernel_choice_epoch()};
        psd_handle::GraphEntry *e = nullptr;
        for (psd_handle::GraphEntry &g : h->graphs)
            if (g.key == key) e = &g;
        if (!e) {   // first sight: eager, and remember the key
            if (h->graphs.size() < psd_handle::kMaxGraphs) {
                h->graphs.emplace_back();
                e = &h->graphs.back();
            } else {
                e = &h->graphs[0];
                for (psd_handle::GraphEntry &g : h->graphs)
                    if (g.last_use < e->last_use) e = &g;
                if (e->exec) (void)hipGraphExecDestroy(e->exec);
                *e = psd_handle::GraphEntry();
            }
            e->key = key;
            e->last_use = ++h->graph_clock;
            return model_call_eager(src, rows_dev, S, seqs_per_cache, bs, t1, cf, st_);
        }
        e->last_use = ++h->graph_clock;
        if (!e->exec && !e->failed) {   // second sight: capture on the handle's own stream (the caller's may be the null stream)
            if (!h->capture_stream && hipStreamCreateWithFlags(&h->capture_stream, hipStreamNonBlocking) != hipSuccess) {
                h->capture_stream = nullptr;
                e->failed = true;
            }
            if (!e->failed) {
                hipGraph_t graph = nullptr;
                int32_t rc = PSD_OK;
                if (hipStreamBeginCapture(h->capture_stream, hipStreamCaptureModeThreadLocal) != hipSuccess) {
                    e->failed = true;
                } else {
                    rc = model_call_eager(src, rows_dev, S, seqs_per_cache, bs, t1, cf, h->capture_stream);
                    const hipError_t end = hipStreamEndCapture(h->capture_stream, &graph);
                    if (rc != PSD_OK || end != hipSuccess || !graph ||
                        hipGraphInstantiate(&e->exec, graph, nullptr, nullptr, 0) != hipSuccess) {
                        e->exec = nullptr;
                        e->failed = true;
                    }
                    if (graph) (void)hipGraphDestroy(graph);
                }
                (void)hipGetLastError();   // a refused capture must not be reported by the next call
            }
        }
        if (!e->exec) return model_call_eager(src, rows_dev, S, seqs_per_cache, bs, t1, cf, st_);
        PSD_HIP(hipGraphLaunch(e->exec, st_));
        ++h->graph_replays;
        return PSD_OK;
    };
    // the same between two HIP events when model calls are being timed (psd_probe_begin kind 5)
    auto model_call = [&](const int32_t *src, const int32_t *rows_dev, int S, int seqs_per_cache, const BlockStart &bs, int32_t *t1,
                          float *cf, hipStream_t st_) -> int32_t {
        psd_handle::Probe &pr = h->probe_call;
        const bool timed = pr.enabled && pr.used + 2 <= pr.ev.size();
        if (timed) (void)hipEventRecord(pr.ev[pr.used], st_);
        const int32_t rc = model_call_untimed(src, rows_dev, S, seqs_per_cache, bs, t1, cf, st_);
        if (timed) {
            (void)hipEventRecord(pr.ev[pr.used + 1], st_);
            pr.used += 2;
            pr.note(S, seqs_per_cache);
        }
        return rc;
    };

    {
        const int64_t n = (int64_t)B * PSD_DEVSTAT_WORDS;
        hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, devstats, n, 0);
    }
    enum { ENTER, RUN, DONE };
    std::vector<int> state(B, ENTER);
    std::vector<int64_t> invocations(B, 0);
    std::vector<int32_t> eos_pos(B, -1);
    std::vector<char> stopped(B, 0);
    std::vector<char> have_tables(B, 0);   // single-forward loop: (top1, conf)[b] hold the accepted draft's verifier output
    for (int b = 0; b < B; ++b)
        if (advance && starts[b] >= N) state[b] = DONE;
    auto upload_starts = [&]() -> int32_t {
        for (int b = 0; b < B; ++b) hstarts[b] = std::min(starts[b], N - L);    // a finished sequence keeps its last block
        PSD_HIP(hipMemcpyAsync(d_starts, hstarts, sizeof(int32_t) * B, hipMemcpyHostToDevice, st));
        return PSD_OK;
    };
    auto upload_flags = [&](auto pred) -> int32_t {
        for (int b = 0; b < B; ++b) hflags[b] = pred(b) ? 1 : 0;
        PSD_HIP(hipMemcpyAsync(d_flags, hflags, sizeof(int32_t) * B, hipMemcpyHostToDevice, st));
        return PSD_OK;
    };
    // the sequences that leave their block: close its token count, then move on (or finish)
    auto leave_blocks = [&](const std::vector<int> &who, std::vector<char> &stopped) -> int32_t {
        if (who.empty()) return PSD_OK;
        std::vector<char> mark(B, 0);
        for (int b : who) mark[b] = 1;
        CHECK(upload_flags([&](int b) { return mark[b] != 0; }));
        launch_finish_counts(tokens, B, N, bs_seq, L, mask_id, policy->eos_stop, policy->eos_id, devstats, d_flags, st);
        if (eos_stop) PSD_HIP(hipMemcpyAsync(hstats, devstats, sizeof(int32_t) * B * PSD_DEVSTAT_WORDS, hipMemcpyDeviceToHost, st));
        // (the staging buffer may be rewritten by the next upload: the copy of the flags must have been consumed)
        PSD_HIP(hipStreamSynchronize(st));
        for (int b : who) {
            // an EOS token in the block it leaves ends the sequence (App. B.1), whatever is still masked in it
            const int32_t eos = eos_stop ? hstats[(int64_t)b * PSD_DEVSTAT_WORDS + PSD_DEVSTAT_EOS] : 0;
            if (eos > 0) {
                stopped[b] = 1;
                eos_pos[b] = std::min(starts[b], N - L) + eos - 1;
            }
            if (stopped[b] || !advance) {
                state[b] = DONE;
                if (advance && !stopped[b]) starts[b] += L;
            } else {
                starts[b] += L;
                state[b] = starts[b] + L <= N ? ENTER : DONE;
            }
        }
        return PSD_OK;
    };

    CHECK(upload_starts());
    int iterations = 0, stalled = 0;
    while (true) {
        // sequences entering a block: count its masks; a block without masks is left at once
        bool entering = false;
        for (int b = 0; b < B; ++b) entering = entering || state[b] == ENTER;
        while (entering) {
            CHECK(upload_starts());
            CHECK(upload_flags([&](int b) { return state[b] == ENTER; }));
            hipLaunchKernelGGL(count_masks_kernel, dim3(B), dim3(64), 0, st, tokens, N, bs_seq, L, mask_id, n_left, devstats, d_flags);
            PSD_HIP(hipMemcpyAsync(hc, n_left, sizeof(int32_t) * B, hipMemcpyDeviceToHost, st));
            PSD_HIP(hipStreamSynchronize(st));
            std::vector<int> empty;
            for (int b = 0; b < B; ++b) {
                if (state[b] != ENTER) continue;
                have_tables[b] = 0;        // the call that enters a block is a stage-1 call
                if (hc[b] > 0) state[b] = RUN;
                else empty.push_back(b);
            }
            CHECK(leave_blocks(empty, stopped));
            entering = false;
            for (int b = 0; b < B; ++b) entering = entering || state[b] == ENTER;
        }
        std::vector<int> active;
        for (int b = 0; b < B; ++b)
            if (state[b] == RUN) active.push_back(b);
        if (active.empty()) break;
        if (max_iterations > 0 && iterations >= max_iterations) break;
        // every model call commits at least one token of every sequence it runs (k_min >= 1), so a block of L positions
        // is resolved after at most L iterations; a batch in which no sequence leaves a block for longer has a model
        // that returns no usable predictions
        if (++stalled > L + 1)
            PSD_FAIL(PSD_ERR_DEVICE, "no block resolved in %d iterations: the model calls make no progress (k_min = %d; non-finite "
                     "logits?)", L + 1, policy->k_min);
        ++iterations;
        // stage 1: one forward over the running sequences (those without tables of their own), policy commit, drafts
        std::vector<int> fresh;
        for (int b : active)
            if (!have_tables[b]) fresh.push_back(b);
        const int S1 = (int)fresh.size();
        if (S1 > 0) {
            for (int s = 0; s < S1; ++s) hrows[s] = fresh[s];
            PSD_HIP(hipMemcpyAsync(rows, hrows, sizeof(int32_t) * S1, hipMemcpyHostToDevice, st));
            CHECK(model_call(tokens, rows, S1, 1, bs_seq, top1, conf, st));
            for (int b : fresh) invocations[b] += 1;
            const int32_t *only = nullptr;
            if (single_forward) {   // the others committed already, by the policy on their accepted draft's output
                std::vector<char> mark(B, 0);
                for (int b : fresh) mark[b] = 1;
                CHECK(upload_flags([&](int b) { return mark[b] != 0; }));
                only = d_flags;
            }
            launch_select_unmask(tokens, B, N, bs_seq, L, top1, conf, *policy, mask_id, nullptr, nullptr, n_left, devstats, only, st);
        }
        launch_build_drafts(tokens, B, N, bs_seq, L, top1, conf, g, mask_id, sigma, m, drafts, st);
        if (eos_stop) launch_eos_stop(tokens, B, N, bs_seq, L, policy->eos_id, n_left, m, devstats, st);
        PSD_HIP(hipMemcpyAsync(hc, m, sizeof(int32_t) * B, hipMemcpyDeviceToHost, st));
        PSD_HIP(hipStreamSynchronize(st));
        std::vector<int> vset;
        for (int b : active)
            if (hc[b] > 0) vset.push_back(b);
        if (!vset.empty()) {
            // stage 3: one batched forward over the K drafts of every sequence that still has masks
            const int S3 = (int)vset.size() * K;
            for (size_t i = 0; i < vset.size(); ++i)
                for (int k = 0; k < K; ++k) hrows[i * K + k] = vset[i] * K + k;
            PSD_HIP(hipMemcpyAsync(rows, hrows, sizeof(int32_t) * S3, hipMemcpyHostToDevice, st));
            CHECK(model_call(drafts, rows, S3, K, bs_draft, v_top1, v_conf, st));
            for (int b : vset) invocations[b] += 1;
            launch_accept(tokens, drafts, B, N, bs_seq, L, sigma, m, g, *policy, mask_id, v_top1, v_conf, k_star, accepted,
                          n_left, devstats, single_forward ? top1 : nullptr, single_forward ? conf : nullptr, st);
            if (single_forward)
                for (int b : vset) have_tables[b] = 1;
            if (eos_stop) launch_eos_stop(tokens, B, N, bs_seq, L, policy->eos_id, n_left, nullptr, devstats, st);
        }
        // who is done with the block: no masks left, or stopped on an EOS token (its mask counts were zeroed)
        PSD_HIP(hipMemcpyAsync(hc, n_left, sizeof(int32_t) * B, hipMemcpyDeviceToHost, st));
        PSD_HIP(hipStreamSynchronize(st));
        std::vector<int> leaving;
        for (int b : active)
            if (hc[b] == 0) leaving.push_back(b);
        if (!leaving.empty()) stalled = 0;
        CHECK(leave_blocks(leaving, stopped));
    }
    // sequences still inside a block when the call ends (max_iterations): what they resolved so far counts for this call
    {
        std::vector<int> open;
        for (int b = 0; b < B; ++b)
            if (state[b] == RUN) open.push_back(b);
        if (!open.empty()) {
            std::vector<char> mark(B, 0);
            for (int b : open) mark[b] = 1;
            CHECK(upload_flags([&](int b) { return mark[b] != 0; }));
            launch_finish_counts(tokens, B, N, bs_seq, L, mask_id, policy->eos_stop, policy->eos_id, devstats, d_flags, st);
        }
    }
    PSD_HIP(hipMemcpyAsync(hstats, devstats, sizeof(int32_t) * B * PSD_DEVSTAT_WORDS, hipMemcpyDeviceToHost, st));
    PSD_HIP(hipStreamSynchronize(st));
    for (int b = 0; b < B; ++b) {
        const int32_t *ds = hstats + (int64_t)b * PSD_DEVSTAT_WORDS;
        stats[b].invocations += invocations[b];
        stats[b].tokens_policy += ds[PSD_DEVSTAT_POLICY];
        stats[b].tokens_draft += ds[PSD_DEVSTAT_DRAFT];
        stats[b].tokens_postverify += ds[PSD_DEVSTAT_POST];
        stats[b].tokens_counted += ds[PSD_DEVSTAT_COUNTED];
        if (stopped[b]) {
            stats[b].stopped = 1;
            stats[b].eos_pos = eos_pos[b];
        }
        for (int i = 0; i <= PSD_MAX_BLOCK; ++i) stats[b].depth_hist[i] += ds[PSD_DEVSTAT_HIST + i];
    }
    if (iterations_done) *iterations_done = iterations;
    if (kv && !dual) {   // the block is finished: its keys and values become context
        KvCacheArg a = *kv;
        a.seqs_per_cache = 1;
        a.append = true;
        CHECK(run_forward_cached(h, tokens, nullptr, B, N, starts[0], L, a, ws, fwd_bytes, st));
    }
    PSD_HIP(hipGetLastError());
    return PSD_OK;
}

// one block, the same for every sequence of the batch (the cached model calls)
int32_t decode_block_impl(psd_handle *h, int32_t *tokens, int32_t B, int32_t N, int32_t block_start, int32_t L,
                          const psd_policy *policy, const psd_graph *graph, psd_stats *stats, void *ws, int64_t ws_bytes,
                          void *stream, const KvCacheArg *kv) {
    if (B < 1) PSD_FAIL(PSD_ERR_SHAPE, "batch %d", B);
    std::vector<int32_t> starts(B, block_start);
    return decode_impl(h, tokens, B, N, starts.data(), L, policy, graph, stats, false, 0, nullptr, ws, ws_bytes, stream, kv);
}

int32_t check_kv(const psd_handle *h, const void *cache, int32_t capacity, int32_t block_start, int32_t L) {
    if (!h) PSD_FAIL(PSD_ERR_INVALID_ARG, "handle is NULL");
    if (h->cfg.attention != PSD_ATTN_BLOCK_CAUSAL)
        PSD_FAIL(PSD_ERR_UNSUPPORTED, "a KV cache is exact only for context-causal block attention (config.attention)");
    if (!cache) PSD_FAIL(PSD_ERR_INVALID_ARG, "cache is NULL");
    if ((reinterpret_cast<uintptr_t>(cache) & 255) != 0) PSD_FAIL(PSD_ERR_WORKSPACE, "cache must be 256-byte aligned");
    if (capacity < 1 || capacity > h->cfg.max_seq) PSD_FAIL(PSD_ERR_SHAPE, "cache capacity %d outside 1..max_seq", capacity);
    if (L < 1 || block_start % L) PSD_FAIL(PSD_ERR_SHAPE, "blocks are aligned to multiples of the block length %d", L);
    if (L % 16) PSD_FAIL(PSD_ERR_SHAPE, "a cached block length must be a multiple of 16 (value layout), not %d", L);
    if (block_start + L > capacity) PSD_FAIL(PSD_ERR_SHAPE, "block [%d, %d) exceeds the cache capacity %d", block_start,
                                             block_start + L, capacity);
    return PSD_OK;
}

// the approximate cache of a bidirectional model: room for the N - L positions outside a block
int32_t check_kv_approx(const psd_handle *h, const void *cache, int32_t capacity, int32_t N, int32_t L) {
    if (!h) PSD_FAIL(PSD_ERR_INVALID_ARG, "handle is NULL");
    if (h->cfg.attention != PSD_ATTN_BIDIRECTIONAL)
        PSD_FAIL(PSD_ERR_UNSUPPORTED, "the approximate cache is for bidirectional models; a block-causal model has an exact one");
    if (!cache) PSD_FAIL(PSD_ERR_INVALID_ARG, "cache is NULL");
    if ((reinterpret_cast<uintptr_t>(cache) & 255) != 0) PSD_FAIL(PSD_ERR_WORKSPACE, "cache must be 256-byte aligned");
    if (capacity < 1 || capacity > h->cfg.max_seq) PSD_FAIL(PSD_ERR_SHAPE, "cache capacity %d outside 1..max_seq", capacity);
    if (L < 1 || L % 16) PSD_FAIL(PSD_ERR_SHAPE, "a cached block length must be a multiple of 16 (value layout), not %d", L);
    if (N - L < 1 || N - L > capacity) PSD_FAIL(PSD_ERR_SHAPE, "the %d positions outside the block need a cache of that capacity, not %d",
                                                N - L, capacity);
    return PSD_OK;
}

}   // namespace

int32_t psd_decode_block(psd_handle *h, int32_t *tokens, int32_t B, int32_t N, const int32_t *block_start, int32_t L,
                         const psd_policy *policy, const psd_graph *graph, psd_stats *stats, void *ws, int64_t ws_bytes,
                         void *stream) {
    if (!block_start) PSD_FAIL(PSD_ERR_INVALID_ARG, "block_start is NULL");
    if (B < 1) PSD_FAIL(PSD_ERR_SHAPE, "batch %d", B);
    std::vector<int32_t> starts(block_start, block_start + B);
    return decode_impl(h, tokens, B, N, starts.data(), L, policy, graph, stats, false, 0, nullptr, ws, ws_bytes, stream, nullptr);
}

int32_t psd_decode(psd_handle *h, int32_t *tokens, int32_t B, int32_t N, int32_t *block_start, int32_t L, const psd_policy *policy,
                   const psd_graph *graph, psd_stats *stats, int32_t max_iterations, int32_t *iterations_done, void *ws,
                   int64_t ws_bytes, void *stream) {
    if (!block_start) PSD_FAIL(PSD_ERR_INVALID_ARG, "block_start is NULL");
    if (!h) PSD_FAIL(PSD_ERR_INVALID_ARG, "handle is NULL");
    for (int b = 0; b < B; ++b)
        if (block_start[b] < N && (N - block_start[b]) % L)
            PSD_FAIL(PSD_ERR_SHAPE, "sequence %d: the %d positions from its block start %d on are not whole blocks of %d", b,
                     N - block_start[b], block_start[b], L);
    return decode_impl(h, tokens, B, N, block_start, L, policy, graph, stats, true, max_iterations, iterations_done, ws, ws_bytes,
                       stream, nullptr);
}

// ---- context-causal block attention with an exact prefix KV cache ----

int64_t psd_kv_cache_bytes(const psd_model_config *cfg, int32_t capacity) {
    int32_t rc = check_cfg(cfg);
    if (rc != PSD_OK) return rc;
    if (capacity < 1 || capacity > cfg->max_seq) {
        psd_set_error("psd_kv_cache_bytes: capacity %d outside 1..max_seq", capacity);
        return PSD_ERR_SHAPE;
    }
    return align_up(kv_layout(*cfg, capacity).per_seq * (cfg->dtype == PSD_DTYPE_BF16 ? 2 : 4), 256);
}

int32_t psd_kv_reset(psd_handle *h, void *cache, int32_t n_seqs, int32_t capacity, void *stream) {
    if (!h || !cache) PSD_FAIL(PSD_ERR_INVALID_ARG, "NULL handle / cache");
    if ((reinterpret_cast<uintptr_t>(cache) & 255) != 0) PSD_FAIL(PSD_ERR_WORKSPACE, "cache must be 256-byte aligned");
    if (capacity < 1 || capacity > h->cfg.max_seq) PSD_FAIL(PSD_ERR_SHAPE, "cache capacity %d outside 1..max_seq", capacity);
    if (n_seqs < 1) PSD_FAIL(PSD_ERR_SHAPE, "n_seqs %d", n_seqs);
    const int64_t words = psd_kv_cache_bytes(&h->cfg, capacity) / 4 * n_seqs;
    hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, (hipStream_t)stream, (int32_t *)cache,
                       words, 0);
    PSD_HIP(hipGetLastError());
    return PSD_OK;
}

int32_t psd_kv_prefill(psd_handle *h, const int32_t *tokens, int32_t B, int32_t N, int32_t n_prompt, int32_t L, void *cache,
                       int32_t capacity, void *ws, int64_t ws_bytes, void *stream) {
    CHECK(check_block(h, B, N, 0, L));
    CHECK(check_kv(h, cache, capacity, 0, L));
    if (!tokens) PSD_FAIL(PSD_ERR_INVALID_ARG, "tokens is NULL");
    if (n_prompt < 0 || n_prompt % L || n_prompt > N || n_prompt > capacity)
        PSD_FAIL(PSD_ERR_SHAPE, "prompt length %d: a multiple of the block length within the sequence and the cache", n_prompt);
    KvCacheArg a;
    a.base = cache;
    a.capacity = capacity;
    a.seqs_per_cache = 1;
    a.append = true;
    for (int start = 0; start < n_prompt; start += L) {   // block by block: each sees the blocks before it
        a.len = start;
        CHECK(run_forward_cached(h, tokens, nullptr, B, N, start, L, a, ws, ws_bytes, (hipStream_t)stream));
    }
    return PSD_OK;
}

int32_t psd_forward_confidence_cached(psd_handle *h, const int32_t *tokens, int32_t S, int32_t N, int32_t block_start, int32_t L,
                                      int32_t seqs_per_cache, const void *cache, int32_t capacity, int32_t *top1, float *conf,
                                      float *logits, void *ws, int64_t ws_bytes, void *stream) {
    CHECK(check_block(h, S, N, block_start, L));
    CHECK(check_kv(h, cache, capacity, block_start, L));
    if (!tokens || (!logits && (!top1 || !conf))) PSD_FAIL(PSD_ERR_INVALID_ARG, "NULL tokens/top1/conf");
    if (seqs_per_cache < 1 || S % seqs_per_cache) PSD_FAIL(PSD_ERR_SHAPE, "S must be a multiple of seqs_per_cache");
    KvCacheArg a;
    a.base = const_cast<void *>(cache);
    a.capacity = capacity;
    a.len = block_start;
    a.seqs_per_cache = seqs_per_cache;
    hipStream_t st = (hipStream_t)stream;
    CHECK(run_forward_cached(h, tokens, nullptr, S, N, block_start, L, a, ws, ws_bytes, st));
    if (logits) CHECK(run_head_logits(h, S, L, L, logits, ws, st));
    if (top1 && conf) return run_head_confidence(h, tokens, nullptr, S, N, block_start, L, top1, conf, nullptr, ws, st, L);
    return PSD_OK;
}

int32_t psd_decode_block_cached(psd_handle *h, int32_t *tokens, int32_t B, int32_t N, int32_t block_start, int32_t L,
                                const psd_policy *policy, const psd_graph *graph, psd_stats *stats, void *cache,
                                int32_t capacity, void *ws, int64_t ws_bytes, void *stream) {
    CHECK(check_kv(h, cache, capacity, block_start, L));
    KvCacheArg a;
    a.base = cache;
    a.capacity = capacity;
    a.len = block_start;
    return decode_block_impl(h, tokens, B, N, block_start, L, policy, graph, stats, ws, ws_bytes, stream, &a);
}

// ---- approximate prefix + suffix KV cache for bidirectional models ----

int32_t psd_forward_confidence_approx(psd_handle *h, const int32_t *tokens, int32_t S, int32_t N, int32_t block_start, int32_t L,
                                      int32_t refresh, int32_t seqs_per_cache, void *cache, int32_t capacity, int32_t *top1,
                                      float *conf, float *logits, void *ws, int64_t ws_bytes, void *stream) {
    CHECK(check_block(h, S, N, block_start, L));
    CHECK(check_kv_approx(h, cache, capacity, N, L));
    if (!tokens || (!logits && (!top1 || !conf))) PSD_FAIL(PSD_ERR_INVALID_ARG, "NULL tokens/top1/conf");
    if (seqs_per_cache < 1 || S % seqs_per_cache) PSD_FAIL(PSD_ERR_SHAPE, "S must be a multiple of seqs_per_cache");
    if (refresh && seqs_per_cache != 1) PSD_FAIL(PSD_ERR_INVALID_ARG, "a refreshing call fills one cache per sequence");
    KvCacheArg a;
    a.base = cache;
    a.capacity = capacity;
    a.len = N - L;
    a.seqs_per_cache = seqs_per_cache;
    a.dual = true;
    hipStream_t st = (hipStream_t)stream;
    const int plan_N = refresh ? N : L;
    if (refresh)
        CHECK(run_forward_hidden(h, tokens, nullptr, S, N, block_start, L, ws, ws_bytes, st, &a));
    else
        CHECK(run_forward_cached(h, tokens, nullptr, S, N, block_start, L, a, ws, ws_bytes, st));
    if (logits) CHECK(run_head_logits(h, S, plan_N, L, logits, ws, st));
    if (top1 && conf) return run_head_confidence(h, tokens, nullptr, S, N, block_start, L, top1, conf, nullptr, ws, st, plan_N);
    return PSD_OK;
}

int32_t psd_decode_block_approx(psd_handle *h, int32_t *tokens, int32_t B, int32_t N, int32_t block_start, int32_t L,
                                const psd_policy *policy, const psd_graph *graph, psd_stats *stats, void *cache,
                                int32_t capacity, void *ws, int64_t ws_bytes, void *stream) {
    CHECK(check_kv_approx(h, cache, capacity, N, L));
    KvCacheArg a;
    a.base = cache;
    a.capacity = capacity;
    a.len = N - L;
    a.dual = true;
    return decode_block_impl(h, tokens, B, N, block_start, L, policy, graph, stats, ws, ws_bytes, stream, &a);
}

// ---- offline calibration of the draft graph ----

int32_t psd_calibrate_graph(psd_handle *h, const int32_t *tokens, int32_t *work_tokens, int32_t B, int32_t N, int32_t n_prompt,
                            int32_t L, const psd_policy *policy, const psd_graph *candidates, int32_t n_candidates,
                            psd_graph_score *scores, int32_t *best, void *cache, int32_t capacity, void *ws, int64_t ws_bytes,
                            void *stream) {
    CHECK(check_block(h, B, N, 0, L));
    CHECK(check_policy(policy));
    if (!tokens || !work_tokens || !candidates || !scores || !best) PSD_FAIL(PSD_ERR_INVALID_ARG, "NULL argument");
    if (n_candidates < 1) PSD_FAIL(PSD_ERR_INVALID_ARG, "no candidate graph");
    if (n_prompt < 0 || n_prompt >= N || (N - n_prompt) % L) PSD_FAIL(PSD_ERR_SHAPE, "the generated part must be whole blocks of %d", L);
    if (cache && n_prompt % L) PSD_FAIL(PSD_ERR_SHAPE, "cached decoding needs a prompt of whole blocks");
    GraphArg g;
    for (int c = 0; c < n_candidates; ++c) CHECK(check_graph(candidates + c, &g));   // all checked before anything runs
    psd_policy pol = *policy;
    pol.eos_stop = 0;
    hipStream_t st = (hipStream_t)stream;
    hipEvent_t e0, e1;
    PSD_HIP(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        PSD_FAIL(PSD_ERR_DEVICE, "hipEventCreate failed");
    }
    int32_t rc = PSD_OK;
    std::vector<psd_stats> stats(B);
    for (int c = 0; c < n_candidates && rc == PSD_OK; ++c) {
        memset(stats.data(), 0, sizeof(psd_stats) * B);
        if (hipMemcpyAsync(work_tokens, tokens, sizeof(int32_t) * (size_t)B * N, hipMemcpyDeviceToDevice, st) != hipSuccess) {
            rc = PSD_ERR_DEVICE;
            psd_set_error("psd_calibrate_graph: copy of the calibration batch failed");
            break;
        }
        if (cache) {
            rc = psd_kv_reset(h, cache, B, capacity, stream);
            if (rc == PSD_OK) rc = psd_kv_prefill(h, work_tokens, B, N, n_prompt, L, cache, capacity, ws, ws_bytes, stream);
            if (rc != PSD_OK) break;
        }
        (void)hipEventRecord(e0, st);
        for (int start = n_prompt; start < N && rc == PSD_OK; start += L)
            rc = cache ? psd_decode_block_cached(h, work_tokens, B, N, start, L, &pol, candidates + c, stats.data(), cache, capacity,
                                                 ws, ws_bytes, stream)
                       : decode_block_impl(h, work_tokens, B, N, start, L, &pol, candidates + c, stats.data(), ws, ws_bytes, stream,
                                           nullptr);
        if (rc != PSD_OK) break;
        (void)hipEventRecord(e1, st);
        float ms = 0.f;
        if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) {
            rc = PSD_ERR_DEVICE;
            psd_set_error("psd_calibrate_graph: timing failed");
            break;
        }
        psd_graph_score &sc = scores[c];
        sc.tokens = sc.invocations = 0;
        for (int b = 0; b < B; ++b) {
            sc.tokens += stats[b].tokens_policy + stats[b].tokens_draft + stats[b].tokens_postverify;
            sc.invocations += stats[b].invocations;
        }
        sc.seconds = ms * 1e-3;
        sc.tokens_per_s = sc.seconds > 0 ? sc.tokens / sc.seconds : 0.0;
        sc.tpf = sc.invocations > 0 ? (double)sc.tokens / (double)sc.invocations : 0.0;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != PSD_OK) return rc;
    *best = 0;
    for (int c = 1; c < n_candidates; ++c)
        if (scores[c].tokens_per_s > scores[*best].tokens_per_s) *best = c;
    return PSD_OK;
}

// ---- kernel-level hooks: the same launchers the forward uses, on caller-provided buffers ----

int32_t psd_kernel_gemm_bf16(const void *A, const void *W, const void *W2, int64_t M, int32_t Nout, int32_t Kin,
                             int32_t lda, int32_t ldw, int32_t epilogue, const float *bias, void *out, float *resid,
                             int32_t ldo, void *stream) {
    if (!A || !W || M < 1 || M > (1 << 30) || Nout < 1 || Kin < 1) PSD_FAIL(PSD_ERR_INVALID_ARG, "bad GEMM arguments");
    if (Kin % 64 || Nout % 64) PSD_FAIL(PSD_ERR_SHAPE, "Nout and Kin must be multiples of 64");
    if (lda < Kin || ldw < Kin || lda % 8 || ldw % 8 || lda > (1 << 20) || ldw > (1 << 20))
        PSD_FAIL(PSD_ERR_SHAPE, "row strides must be multiples of 8 in [Kin, 2^20]");
    if (epilogue < 0 || epilogue > 3) PSD_FAIL(PSD_ERR_INVALID_ARG, "epilogue %d", epilogue);
    if (epilogue == EPI_SWIGLU && !W2) PSD_FAIL(PSD_ERR_INVALID_ARG, "SwiGLU needs the second weight");
    if (epilogue == EPI_BIAS && !bias) PSD_FAIL(PSD_ERR_INVALID_ARG, "bias is NULL");
    if (epilogue == EPI_RESIDUAL ? !resid : !out) PSD_FAIL(PSD_ERR_INVALID_ARG, "output is NULL");
    if (ldo < Nout) PSD_FAIL(PSD_ERR_SHAPE, "ldo < Nout");
    launch_gemm_bf16((const bf16_t *)A, (const bf16_t *)W, (const bf16_t *)W2, M, Nout, Kin, lda, ldw, epilogue, bias, (bf16_t *)out,
                     resid, ldo, (hipStream_t)stream);
    PSD_HIP(hipGetLastError());
    return PSD_OK;
}

int32_t psd_kernel_gemm_residual_splitk(const void *A, const void *W, int64_t M, int32_t Nout, int32_t Kin, float *resid,
                                        float *partial, int64_t partial_bytes, int32_t k_splits, int32_t *used_splits,
                                        void *stream) {
    if (!A || !W || !resid || M < 1 || M > (1 << 30) || Nout < 1 || Kin < 1) PSD_FAIL(PSD_ERR_INVALID_ARG, "bad GEMM arguments");
    if (Kin % 64 || Nout % 64) PSD_FAIL(PSD_ERR_SHAPE, "Nout and Kin must be multiples of 64");
    if (k_splits < 0 || k_splits > 8) PSD_FAIL(PSD_ERR_INVALID_ARG, "k_splits %d", k_splits);
    const int splits = k_splits == 0 ? gemm_bf16_splits(M, Nout, Kin) : k_splits;
    if (Kin % (64 * splits)) PSD_FAIL(PSD_ERR_SHAPE, "Kin must be a multiple of 64 * k_splits");
    if (splits > 1 && (!partial || partial_bytes < (int64_t)(splits - 1) * M * Nout * 4))
        PSD_FAIL(PSD_ERR_WORKSPACE, "partial sums need %lld bytes", (long long)((int64_t)(splits - 1) * M * Nout * 4));
    launch_gemm_bf16_split((const bf16_t *)A, (const bf16_t *)W, M, Nout, Kin, Kin, Kin, resid, Nout, partial, splits,
                           (hipStream_t)stream);
    launch_fold_partials(resid, M, Nout, Nout, partial, splits - 1, (hipStream_t)stream);
    PSD_HIP(hipGetLastError());
    if (used_splits) *used_splits = splits;
    return PSD_OK;
}

int64_t psd_kernel_attention_scratch_bytes(int32_t S, int32_t N, int32_t n_kv_heads, int32_t d_head) {
    if (S < 1 || N < 1 || n_kv_heads < 1 || d_head < 1) return -1;
    return (int64_t)S * vt_row_stride(N) * n_kv_heads * d_head * 2;
}

int32_t psd_kernel_attention_bf16(const void *qkv, int32_t ld_qkv, int32_t S, int32_t N, int32_t n_heads, int32_t n_kv_heads,
                                  int32_t d_head, void *vT, void *out, void *stream) {
    if (!qkv || !vT || !out || S < 1 || N < 1) PSD_FAIL(PSD_ERR_INVALID_ARG, "bad attention arguments");
    if (n_heads < 1 || n_kv_heads < 1 || ld_qkv < (n_heads + 2 * n_kv_heads) * d_head || ld_qkv % 8)
        PSD_FAIL(PSD_ERR_SHAPE, "ld_qkv must be a multiple of 8 and at least the row width");
    if ((d_head != 64 && d_head != 128) || N % 8 || n_kv_heads < 1 || n_heads % n_kv_heads)
        PSD_FAIL(PSD_ERR_SHAPE, "attention needs d_head 64/128, N a multiple of 8, n_heads a multiple of n_kv_heads");
    launch_transpose_v((const bf16_t *)qkv, ld_qkv, S, N, n_heads, n_kv_heads, d_head, (bf16_t *)vT, (hipStream_t)stream);
    launch_attention_bf16((const bf16_t *)qkv, ld_qkv, (const bf16_t *)vT, S, N, n_heads, n_kv_heads, d_head, (bf16_t *)out,
                          KvPrefix(), (hipStream_t)stream);
    PSD_HIP(hipGetLastError());
    return PSD_OK;
}

int64_t psd_kernel_head_scratch_bytes(int32_t rows, int32_t vocab) {
    if (rows < 1 || vocab < 2) return PSD_ERR_SHAPE;
    return head_partial_bytes(rows, vocab);
}

int64_t psd_kernel_packed_bytes(int64_t R, int32_t K) {
    if (R < 1 || K < 16 || K % 16) return PSD_ERR_SHAPE;
    return packed_rows_bytes(R, K);
}

int32_t psd_kernel_pack_rows(const void *src, int64_t R, int32_t K, void *dst, void *stream) {
    if (!src || !dst || R < 1 || K < 64 || K % 64) PSD_FAIL(PSD_ERR_INVALID_ARG, "bad pack arguments");
    launch_pack_rows((const bf16_t *)src, R, K, (bf16_t *)dst, (hipStream_t)stream);
    PSD_HIP(hipGetLastError());
    return PSD_OK;
}

int32_t psd_kernel_head_stream_bf16(const void *y_packed, const void *W_packed, int32_t rows, int32_t vocab, int32_t d,
                                    float scale, int32_t mask_id, void *scratch, float *row_sum, int32_t *row_arg,
                                    void *stream) {
    if (!y_packed || !W_packed || !scratch || !row_sum || !row_arg || rows < 1 || vocab < 2)
        PSD_FAIL(PSD_ERR_INVALID_ARG, "bad arguments");
    if (!head_stream_supported(rows, d)) PSD_FAIL(PSD_ERR_SHAPE, "streaming head takes at most 192 rows and d a multiple of 64");
    launch_head_stream_bf16((const bf16_t *)y_packed, (const bf16_t *)W_packed, rows, vocab, d, scale, mask_id, scratch, row_sum,
                            row_arg, (hipStream_t)stream);
    PSD_HIP(hipGetLastError());
    return PSD_OK;
}

int32_t psd_kernel_head_confidence_bf16(const void *y, const void *W, int32_t rows, int32_t vocab, int32_t d, float scale,
                                        int32_t mask_id, void *scratch, float *row_sum, int32_t *row_arg, void *stream) {
    if (!y || !W || !scratch || !row_sum || !row_arg || rows < 1 || vocab < 2) PSD_FAIL(PSD_ERR_INVALID_ARG, "bad arguments");
    if (d % 64) PSD_FAIL(PSD_ERR_SHAPE, "d must be a multiple of 64");
    launch_head_confidence_bf16((const bf16_t *)y, (const bf16_t *)W, rows, vocab, d, scale, mask_id, scratch, row_sum,
                                row_arg, (hipStream_t)stream);
    PSD_HIP(hipGetLastError());
    return PSD_OK;
}

int32_t psd_kernel_mfma_rate(const void *operands, int64_t operand_bytes, int32_t iters, void *sink, int64_t sink_bytes,
                             double *flops, void *stream) {
    if (!operands || !sink || !flops || operand_bytes < 16 || iters < 1) PSD_FAIL(PSD_ERR_INVALID_ARG, "bad arguments");
    if (sink_bytes < (int64_t)256 * 256 * 64) PSD_FAIL(PSD_ERR_WORKSPACE, "sink needs 4 MiB");
    launch_mfma_rate(operands, (int)(operand_bytes / 16 > (1 << 20) ? (1 << 20) : operand_bytes / 16), iters, sink,
                     (hipStream_t)stream);
    PSD_HIP(hipGetLastError());
    *flops = 256.0 * 4.0 * iters * 16.0 * 32768.0;
    return PSD_OK;
}

int32_t psd_kernel_gemm_tile(int64_t M, int32_t Nout, int32_t epilogue) {
    if (M < 1 || Nout < 1 || epilogue < 0 || epilogue > 3) PSD_FAIL(PSD_ERR_INVALID_ARG, "bad arguments");
    return gemm_bf16_tile(M, Nout, epilogue);
}

int32_t psd_kernel_gemm_tile_count(void) { return gemm_bf16_tile_count(); }
const char *psd_kernel_gemm_tile_name(int32_t tile) { return gemm_bf16_tile_name(tile); }

int32_t psd_forward_work(const psd_model_config *c, int32_t S, int32_t N, int32_t L, psd_work *out) {
    CHECK(check_cfg(c));
    if (!out || S < 1 || N < 1 || L < 1) PSD_FAIL(PSD_ERR_INVALID_ARG, "bad arguments");
    const double esz = c->dtype == PSD_DTYPE_BF16 ? 2.0 : 4.0;
    const double d = c->d_model, hq = (double)c->n_heads * c->d_head, hkv = (double)c->n_kv_heads * c->d_head, f = c->d_ffn;
    const double layer_params = d * hq + 2.0 * d * hkv + hq * d + 3.0 * d * f;
    const double T = (double)S * N, rows = (double)S * L;
    out->gemm_flops = 2.0 * T * layer_params * c->n_layers;
    out->attn_flops = 4.0 * (double)N * N * hq * S * c->n_layers;
    out->head_flops = 2.0 * rows * c->vocab * d;
    out->head_bytes = (double)c->vocab * d * esz + rows * d * esz + rows * 8.0;
    out->weight_bytes = layer_params * esz * c->n_layers;
    return PSD_OK;
}

}   // extern "C"
