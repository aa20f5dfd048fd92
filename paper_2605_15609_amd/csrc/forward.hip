// The model call of the PSD step (Sec. 3.1): bidirectional transformer forward over S
// sequences of N tokens, then top-1 token and confidence on the L rows of the active block.
// This file only sequences kernels on one stream; every operation runs in the kernels of
// elementwise.hip, gemm_mfma.hip, attention_mfma.hip, lm_head.hip (plain_kernels.hip on the
// debug path).
#include "psd_internal.h"

// Row stride of the SwiGLU output [tokens, d_ffn]: 64 elements of padding.  With dense rows of 24 KB
// (d_ffn = 12288) the row tiles of the down projection's activation operand all start in the same
// cache channel and the fetches of a K-stage queue up behind each other (measured: 123 -> 93 us at
// 512 tokens); other widths do not care.
int64_t act_row_stride(const psd_model_config &cfg) { return padded_row_stride(cfg.d_ffn); }

ForwardPlan plan_forward(const psd_model_config &cfg, int64_t S, int64_t N, int64_t L) {
    const int64_t T = S * N, rows = S * L;
    const int64_t esz = cfg.dtype == PSD_DTYPE_BF16 ? 2 : 4;
    const int64_t qkv_w = (int64_t)(cfg.n_heads + 2 * cfg.n_kv_heads) * cfg.d_head;
    ForwardPlan p;
    int64_t off = 0;
    auto take = [&](int64_t bytes) {
        const int64_t o = off;
        off += align_up(bytes, 256);
        return o;
    };
    p.off_h = take(T * cfg.d_model * 4);
    p.off_a = take(T * cfg.d_model * esz);
    p.off_qkv = take(T * qkv_row_stride(qkv_w) * esz);
    p.off_vt = take(S * vt_row_stride(N) * (int64_t)cfg.n_kv_heads * cfg.d_head * esz);
    p.off_o = take(T * (int64_t)cfg.n_heads * cfg.d_head * esz);
    p.off_act = take(T * act_row_stride(cfg) * esz);
    p.off_ksplit = take(cfg.dtype == PSD_DTYPE_BF16 ? ksplit_bytes(cfg) : 0);
    p.off_oc = take(rows * (int64_t)cfg.n_heads * cfg.d_head * esz);   // last layer: attention output and residual
    p.off_hc = take(rows * cfg.d_model * 4);                           // stream of the block rows only
    p.off_y = take(rows * cfg.d_model * esz);
    p.off_ypack = take(cfg.dtype == PSD_DTYPE_BF16 ? packed_rows_bytes(rows, cfg.d_model) : 0);
    p.off_rowsum = take(rows * 4);
    p.off_rowarg = take(rows * 4);
    // LM-head scratch: per-slab partial (max, sum, argmax) triples on the fused path; the
    // debug path stores full logits here instead
    int64_t part = rows * (int64_t)cfg.vocab * 4;
    if (cfg.dtype == PSD_DTYPE_BF16) {
        const int64_t fused = head_partial_bytes((int)rows, cfg.vocab);
        if (fused > part) part = fused;
    }
    p.off_part = take(part);
    p.total = off;
    return p;
}

namespace {

template <typename T>
struct Dispatch;

template <>
struct Dispatch<float> {
    // A [M, Kin] with row stride lda; weights [Nout, Kin] with row stride ldw
    static PendingSums gemm(psd_handle *, const float *A, int lda, const void *W, const void *W2, int ldw, int64_t M, int Nout,
                            int Kin, int epi, const float *bias, float *out, float *resid, int ldo, float *, hipStream_t st) {
        launch_plain_gemm<float, float>(A, (const float *)W, (const float *)W2, M, Nout, Kin, lda, ldw, epi, bias, 1.0f, out,
                                        resid, ldo, st);
        return PendingSums();
    }
    static bool qkv_fused(psd_handle *, const float *, const void *, int64_t, int, int, int, int, int, const float *, float *, int,
                          float *, int, hipStream_t) {
        return false;
    }
    static void rope_attention(psd_handle *h, float *qkv, int ld_qkv, float *, int S, int N, int pos0, int H, int Hkv, int dh,
                               float *out, const KvPrefix &pre, int block_len, hipStream_t st, bool = false) {
        launch_rope<float>(qkv, ld_qkv, (int64_t)S * N, N, pos0, H, Hkv, dh, h->rope_cos, h->rope_sin, st);
        launch_plain_attention<float>(qkv, ld_qkv, S, N, H, Hkv, dh, out, pre, block_len, st);
    }
};

template <>
struct Dispatch<bf16_t> {
    // returns the K-split partial sums (left in `ksplit`) that the next reader of resid has to add
    static PendingSums gemm(psd_handle *h, const bf16_t *A, int lda, const void *W, const void *W2, int ldw, int64_t M, int Nout,
                            int Kin, int epi, const float *bias, bf16_t *out, float *resid, int ldo, float *ksplit,
                            hipStream_t st) {
        PendingSums pend;
        if (h->plain_mask & 1)
            launch_plain_gemm<bf16_t, bf16_t>(A, (const bf16_t *)W, (const bf16_t *)W2, M, Nout, Kin, lda, ldw, epi, bias, 1.0f, out,
                                              resid, ldo, st);
        else if (const int splits = (epi == EPI_RESIDUAL && ksplit && ldo == Nout) ? gemm_bf16_splits(M, Nout, Kin) : 1;
                 splits > 1 && (splits - 1) * M * Nout * 4 <= ksplit_bytes(h->cfg)) {
            launch_gemm_bf16_split(A, (const bf16_t *)W, M, Nout, Kin, lda, ldw, resid, ldo, ksplit, splits, st);
            pend.partial = ksplit;
            pend.n = splits - 1;
            pend.stride = M * Nout;
        } else {
            psd_handle::Probe &pr = h->probe;
            const bool timed = pr.enabled && epi == pr.epi && gemm_bf16_tile(M, Nout, epi, Kin) == pr.tile &&
                               pr.used + 2 <= pr.ev.size();
            if (timed) (void)hipEventRecord(pr.ev[pr.used], st);
            launch_gemm_bf16(A, (const bf16_t *)W, (const bf16_t *)W2, M, Nout, Kin, lda, ldw, epi, bias, out, resid, ldo, st);
            if (timed) {
                (void)hipEventRecord(pr.ev[pr.used + 1], st);
                pr.used += 2;
                pr.flops += 2.0 * (double)M * Nout * Kin * (epi == EPI_SWIGLU ? 2.0 : 1.0);
                pr.note(M, Nout);
            }
        }
        return pend;
    }
    // The QKV projection of [M = S * N, d] rows with wq | wk | wv as one matrix, rotary and the V transpose in its
    // epilogue; false (nothing launched) when the matrix-core attention will not run on its output, the shape has no
    // tile that holds whole heads, or a debug switch (plain_mask bit 3) asks for the two-pass form.
    static bool qkv_fused(psd_handle *h, const bf16_t *A, const void *W, int64_t M, int N, int pos0, int H, int Hkv, int dh,
                          const float *bias, bf16_t *qkv, int ld_qkv, bf16_t *vT, int block_len, hipStream_t st) {
        if ((h->plain_mask & (1 | 2 | 8)) || (N % 8) != 0 || (block_len > 0 && block_len < N)) return false;
        if (h->probe.enabled && (h->probe.epi == EPI_STORE || h->probe.epi == EPI_BIAS)) return false;   // that probe times the plain store
        const int d = h->cfg.d_model, qkv_w = (H + 2 * Hkv) * dh;
        const int tile = gemm_bf16_qkv_tile(M, qkv_w, dh, (H + Hkv) * dh, N);
        if (tile < 0) return false;
        launch_gemm_bf16_qkv(A, (const bf16_t *)W, M, qkv_w, d, d, d, bias, qkv, ld_qkv, dh, (H + Hkv) * dh, N, pos0, h->rope_cos,
                             h->rope_sin, vT, (int)vt_row_stride(N), tile, st);
        return true;
    }
    // Rotary on q and k (row i of a sequence sits at position pos0 + i), then attention.
    // pre: KV prefix that every own row sees; block_len > 0: context-causal blocks among the own rows (only the
    // plain kernel masks; the product path of that attention mode keeps finished blocks in the prefix instead).
    // rotated: qkv_fused produced qkv and vT, only the attention is left.
    static void rope_attention(psd_handle *h, bf16_t *qkv, int ld_qkv, bf16_t *vT, int S, int N, int pos0, int H, int Hkv, int dh,
                               bf16_t *out, const KvPrefix &pre, int block_len, hipStream_t st, bool rotated = false) {
        if (rotated) {
            launch_attention_bf16(qkv, ld_qkv, vT, S, N, H, Hkv, dh, out, pre, st);
        } else if ((h->plain_mask & 2) || (N % 8) != 0 || (block_len > 0 && block_len < N)) {
            launch_rope<bf16_t>(qkv, ld_qkv, (int64_t)S * N, N, pos0, H, Hkv, dh, h->rope_cos, h->rope_sin, st);
            launch_plain_attention<bf16_t>(qkv, ld_qkv, S, N, H, Hkv, dh, out, pre, block_len, st);
        } else {
            // the matrix-core kernel reads V transposed; rotary and that transpose share one launch
            launch_rope_transpose_v(qkv, ld_qkv, S, N, pos0, H, Hkv, dh, h->rope_cos, h->rope_sin, vT, st);
            launch_attention_bf16(qkv, ld_qkv, vT, S, N, H, Hkv, dh, out, pre, st);
        }
    }
};

template <typename T>
int32_t forward_hidden_impl(psd_handle *h, const int32_t *tokens, const int32_t *seq_rows, int S, int N, BlockStart block_start,
                            int L, char *ws, hipStream_t st, const KvCacheArg *store) {
    const psd_model_config &c = h->cfg;
    const ForwardPlan p = plan_forward(c, S, N, L);
    const int64_t ntok = (int64_t)S * N;
    const int d = c.d_model, H = c.n_heads, Hkv = c.n_kv_heads, dh = c.d_head, F = c.d_ffn;
    const int qkv_w = (H + 2 * Hkv) * dh;
    float *hbuf = (float *)(ws + p.off_h);
    T *a = (T *)(ws + p.off_a), *qkv = (T *)(ws + p.off_qkv), *vT = (T *)(ws + p.off_vt), *o = (T *)(ws + p.off_o);
    T *act = (T *)(ws + p.off_act), *y = (T *)(ws + p.off_y);
    const int ld_act = (int)act_row_stride(c), ld_qkv = (int)qkv_row_stride(qkv_w);

    float *final_in = hbuf;
    // No K-split on this path: the sums of a sequence's rows must not depend on how many sequences share the
    // call (whole-sequence results are bit-identical across batch sizes; only the block-row path trades that for
    // bandwidth at small row counts).
    float *ksplit = nullptr;
    PendingSums pend;   // stays empty here; the norms take it for the block-row path
    launch_embed<T>(tokens, seq_rows, S, N, (const T *)h->tok_emb, c.vocab, d, hbuf, st);
    for (size_t li = 0; li < h->layers.size(); ++li) {
        const psd_handle::Layer &lw = h->layers[li];
        launch_rmsnorm<T>(hbuf, ntok, d, lw.attn_norm, c.rms_eps, a, pend, st);
        const int epi_qkv = c.qkv_bias ? EPI_BIAS : EPI_STORE;
        // one launch when wq | wk | wv (and the biases) sit back to back in memory, as one [qkv_w, d] matrix
        const T *wq = (const T *)lw.wq, *wk = (const T *)lw.wk, *wv = (const T *)lw.wv;
        const bool fused = wk == wq + (int64_t)H * dh * d && wv == wk + (int64_t)Hkv * dh * d &&
                           (!c.qkv_bias || (lw.bk == lw.bq + H * dh && lw.bv == lw.bk + Hkv * dh));
        const int block_len = c.attention == PSD_ATTN_BLOCK_CAUSAL ? L : 0;
        bool rotated = false;
        if (fused) {
            // (the approximate-cache refresh reads V row-major out of qkv afterwards: two-pass form there)
            rotated = !store && ld_qkv == qkv_w &&
                      Dispatch<T>::qkv_fused(h, a, wq, ntok, N, 0, H, Hkv, dh, c.qkv_bias ? lw.bq : nullptr, qkv, ld_qkv, vT, block_len, st);
            if (!rotated) Dispatch<T>::gemm(h, a, d, wq, nullptr, d, ntok, qkv_w, d, epi_qkv, lw.bq, qkv, nullptr, ld_qkv, nullptr, st);
        } else {
            Dispatch<T>::gemm(h, a, d, wq, nullptr, d, ntok, H * dh, d, epi_qkv, lw.bq, qkv, nullptr, ld_qkv, nullptr, st);
            Dispatch<T>::gemm(h, a, d, wk, nullptr, d, ntok, Hkv * dh, d, epi_qkv, lw.bk, qkv + H * dh, nullptr, ld_qkv, nullptr, st);
            Dispatch<T>::gemm(h, a, d, wv, nullptr, d, ntok, Hkv * dh, d, epi_qkv, lw.bv, qkv + (H + Hkv) * dh, nullptr, ld_qkv, nullptr, st);
        }
        Dispatch<T>::rope_attention(h, qkv, ld_qkv, vT, S, N, 0, H, Hkv, dh, o, KvPrefix(), block_len, st, rotated);
        if (store) {
            // approximate cache: freeze this layer's keys / values of every position outside the block, prefix first
            const KvLayout lay = kv_layout(c, store->capacity);
            T *k_cache = (T *)store->base + (int64_t)li * (lay.k_elems + lay.vt_elems), *vt_cache = k_cache + lay.k_elems;
            KvPrefix at;
            at.ld_k = (int)lay.ld_k;
            at.ld_vt = (int)lay.ld_vt;
            at.stride_k = at.stride_vt = lay.per_seq;
            at.seq_rows = seq_rows;
            at.len = 0;
            const int b0 = block_start.common;     // (a common block start: checked by run_forward_hidden)
            launch_kv_store<T>(qkv, ld_qkv, S, N, 0, b0, H, Hkv, dh, k_cache, vt_cache, at, st);
            at.len = b0;
            launch_kv_store<T>(qkv, ld_qkv, S, N, b0 + L, N - b0 - L, H, Hkv, dh, k_cache, vt_cache, at, st);
        }
        // After the last attention only the block rows feed the LM-head: the rest of that layer (output
        // projection, FFN) and the final norm run on those S*L rows alone, gathered into a packed stream.
        float *hs = hbuf;
        T *os = o;
        int64_t nrow = ntok;
        if (li + 1 == h->layers.size() && L < N) {
            hs = (float *)(ws + p.off_hc);
            os = (T *)(ws + p.off_oc);
            nrow = (int64_t)S * L;
            launch_gather_block_rows<float>(hbuf, hs, d, seq_rows, S, N, block_start, L, st);
            launch_gather_block_rows<T>(o, os, H * dh, seq_rows, S, N, block_start, L, st);
            final_in = hs;
        }
        pend = Dispatch<T>::gemm(h, os, H * dh, lw.wo, nullptr, H * dh, nrow, d, H * dh, EPI_RESIDUAL, nullptr, nullptr, hs, d, ksplit, st);
        launch_rmsnorm<T>(hs, nrow, d, lw.ffn_norm, c.rms_eps, a, pend, st);
        Dispatch<T>::gemm(h, a, d, lw.w_gate, lw.w_up, d, nrow, F, d, EPI_SWIGLU, nullptr, act, nullptr, ld_act, nullptr, st);
        pend = Dispatch<T>::gemm(h, act, ld_act, lw.w_down, nullptr, h->w_down_stride, nrow, d, F, EPI_RESIDUAL, nullptr, nullptr, hs, d, ksplit, st);
    }
    T *ypack = (c.dtype == PSD_DTYPE_BF16 && h->lm_head_packed && head_stream_supported(S * L, d)) ? (T *)(ws + p.off_ypack) : nullptr;
    if (final_in != hbuf)   // already the packed block rows
        launch_rmsnorm_block<T>(final_in, nullptr, S, L, 0, L, d, h->final_norm, c.rms_eps, y, ypack, pend, st);
    else
        launch_rmsnorm_block<T>(hbuf, seq_rows, S, N, block_start, L, d, h->final_norm, c.rms_eps, y, ypack, pend, st);
    return PSD_OK;
}

// The same model call on the L block rows alone, for context-causal block attention: everything before the block
// is finished, its keys and values sit in the sequence's KV cache (kv.len = block_start positions), and nothing
// after the block is visible.  S sequences of L rows; with kv.append the rows' keys and values are stored
// behind the cache (the block is finished and becomes context).
template <typename T>
int32_t forward_cached_impl(psd_handle *h, const int32_t *tokens, const int32_t *seq_rows, int S, int N, int block_start,
                            int L, const KvCacheArg &kv, char *ws, hipStream_t st) {
    const psd_model_config &c = h->cfg;
    const ForwardPlan p = plan_forward(c, S, L, L);
    const int64_t nrow = (int64_t)S * L;
    const int d = c.d_model, H = c.n_heads, Hkv = c.n_kv_heads, dh = c.d_head, F = c.d_ffn;
    const int qkv_w = (H + 2 * Hkv) * dh;
    float *hbuf = (float *)(ws + p.off_h);
    T *a = (T *)(ws + p.off_a), *qkv = (T *)(ws + p.off_qkv), *vT = (T *)(ws + p.off_vt), *o = (T *)(ws + p.off_o);
    T *act = (T *)(ws + p.off_act), *y = (T *)(ws + p.off_y);
    const int ld_act = (int)act_row_stride(c), ld_qkv = (int)qkv_row_stride(qkv_w);
    const KvLayout lay = kv_layout(c, kv.capacity);
    KvPrefix pre;
    pre.len = kv.len;
    pre.ld_k = (int)lay.ld_k;
    pre.ld_vt = (int)lay.ld_vt;
    pre.stride_k = pre.stride_vt = lay.per_seq;
    pre.seq_rows = seq_rows;
    pre.seqs_per_cache = kv.seqs_per_cache;

    float *ksplit = c.dtype == PSD_DTYPE_BF16 ? (float *)(ws + p.off_ksplit) : nullptr;
    PendingSums pend;
    launch_embed_block<T>(tokens, seq_rows, S, N, block_start, L, (const T *)h->tok_emb, c.vocab, d, hbuf, st);
    for (size_t li = 0; li < h->layers.size(); ++li) {
        const psd_handle::Layer &lw = h->layers[li];
        T *k_cache = (T *)kv.base + (int64_t)li * (lay.k_elems + lay.vt_elems), *vt_cache = k_cache + lay.k_elems;
        pre.k = k_cache;
        pre.vt = vt_cache;
        launch_rmsnorm<T>(hbuf, nrow, d, lw.attn_norm, c.rms_eps, a, pend, st);
        const int epi_qkv = c.qkv_bias ? EPI_BIAS : EPI_STORE;
        const T *wq = (const T *)lw.wq, *wk = (const T *)lw.wk, *wv = (const T *)lw.wv;
        const bool fused = wk == wq + (int64_t)H * dh * d && wv == wk + (int64_t)Hkv * dh * d &&
                           (!c.qkv_bias || (lw.bk == lw.bq + H * dh && lw.bv == lw.bk + Hkv * dh));
        if (fused) {
            Dispatch<T>::gemm(h, a, d, wq, nullptr, d, nrow, qkv_w, d, epi_qkv, lw.bq, qkv, nullptr, ld_qkv, nullptr, st);
        } else {
            Dispatch<T>::gemm(h, a, d, wq, nullptr, d, nrow, H * dh, d, epi_qkv, lw.bq, qkv, nullptr, ld_qkv, nullptr, st);
            Dispatch<T>::gemm(h, a, d, wk, nullptr, d, nrow, Hkv * dh, d, epi_qkv, lw.bk, qkv + H * dh, nullptr, ld_qkv, nullptr, st);
            Dispatch<T>::gemm(h, a, d, wv, nullptr, d, nrow, Hkv * dh, d, epi_qkv, lw.bv, qkv + (H + Hkv) * dh, nullptr, ld_qkv, nullptr, st);
        }
        Dispatch<T>::rope_attention(h, qkv, ld_qkv, vT, S, L, block_start, H, Hkv, dh, o, pre, 0, st);
        if (kv.append) launch_kv_store<T>(qkv, ld_qkv, S, L, 0, L, H, Hkv, dh, k_cache, vt_cache, pre, st);
        pend = Dispatch<T>::gemm(h, o, H * dh, lw.wo, nullptr, H * dh, nrow, d, H * dh, EPI_RESIDUAL, nullptr, nullptr, hbuf, d, ksplit, st);
        launch_rmsnorm<T>(hbuf, nrow, d, lw.ffn_norm, c.rms_eps, a, pend, st);
        Dispatch<T>::gemm(h, a, d, lw.w_gate, lw.w_up, d, nrow, F, d, EPI_SWIGLU, nullptr, act, nullptr, ld_act, nullptr, st);
        pend = Dispatch<T>::gemm(h, act, ld_act, lw.w_down, nullptr, h->w_down_stride, nrow, d, F, EPI_RESIDUAL, nullptr, nullptr, hbuf, d, ksplit, st);
    }
    T *ypack = (c.dtype == PSD_DTYPE_BF16 && h->lm_head_packed && head_stream_supported(S * L, d)) ? (T *)(ws + p.off_ypack) : nullptr;
    launch_rmsnorm_block<T>(hbuf, nullptr, S, L, 0, L, d, h->final_norm, c.rms_eps, y, ypack, pend, st);
    return PSD_OK;
}

// One layer of the stack on a residual stream handed in by the caller (all S*N rows, no block-row shortcut), with
// the tile choices and kernels the forward makes for S*N rows.  stop_after = 1 returns once the attention output
// is in the workspace (the stream is then untouched, and `a` still holds the first norm's output).
template <typename T>
int32_t debug_layer_impl(psd_handle *h, int li, float *hbuf, int S, int N, int L, int stop_after, char *ws, hipStream_t st) {
    const psd_model_config &c = h->cfg;
    const ForwardPlan p = plan_forward(c, S, N, L);
    const int64_t ntok = (int64_t)S * N;
    const int d = c.d_model, H = c.n_heads, Hkv = c.n_kv_heads, dh = c.d_head, F = c.d_ffn;
    const int qkv_w = (H + 2 * Hkv) * dh;
    T *a = (T *)(ws + p.off_a), *qkv = (T *)(ws + p.off_qkv), *vT = (T *)(ws + p.off_vt), *o = (T *)(ws + p.off_o);
    T *act = (T *)(ws + p.off_act);
    const int ld_act = (int)act_row_stride(c), ld_qkv = (int)qkv_row_stride(qkv_w);
    const psd_handle::Layer &lw = h->layers[li];
    launch_rmsnorm<T>(hbuf, ntok, d, lw.attn_norm, c.rms_eps, a, PendingSums(), st);
    const int epi_qkv = c.qkv_bias ? EPI_BIAS : EPI_STORE;
    Dispatch<T>::gemm(h, a, d, lw.wq, nullptr, d, ntok, H * dh, d, epi_qkv, lw.bq, qkv, nullptr, ld_qkv, nullptr, st);
    Dispatch<T>::gemm(h, a, d, lw.wk, nullptr, d, ntok, Hkv * dh, d, epi_qkv, lw.bk, qkv + H * dh, nullptr, ld_qkv, nullptr, st);
    Dispatch<T>::gemm(h, a, d, lw.wv, nullptr, d, ntok, Hkv * dh, d, epi_qkv, lw.bv, qkv + (H + Hkv) * dh, nullptr, ld_qkv, nullptr, st);
    Dispatch<T>::rope_attention(h, qkv, ld_qkv, vT, S, N, 0, H, Hkv, dh, o, KvPrefix(), c.attention == PSD_ATTN_BLOCK_CAUSAL ? L : 0, st);
    if (stop_after == 1) return PSD_OK;
    Dispatch<T>::gemm(h, o, H * dh, lw.wo, nullptr, H * dh, ntok, d, H * dh, EPI_RESIDUAL, nullptr, nullptr, hbuf, d, nullptr, st);
    launch_rmsnorm<T>(hbuf, ntok, d, lw.ffn_norm, c.rms_eps, a, PendingSums(), st);
    Dispatch<T>::gemm(h, a, d, lw.w_gate, lw.w_up, d, ntok, F, d, EPI_SWIGLU, nullptr, act, nullptr, ld_act, nullptr, st);
    Dispatch<T>::gemm(h, act, ld_act, lw.w_down, nullptr, h->w_down_stride, ntok, d, F, EPI_RESIDUAL, nullptr, nullptr, hbuf, d, nullptr, st);
    return PSD_OK;
}

}   // namespace

int32_t run_debug_layer(psd_handle *h, int layer, float *hidden, int S, int N, int L, int stop_after, void *ws, int64_t ws_bytes,
                        hipStream_t st) {
    const ForwardPlan p = plan_forward(h->cfg, S, N, L);
    if (ws == nullptr || ws_bytes < p.total)
        PSD_FAIL(PSD_ERR_WORKSPACE, "workspace of %lld bytes, one layer over %d x %d tokens needs %lld", (long long)ws_bytes, S, N,
                 (long long)p.total);
    if ((reinterpret_cast<uintptr_t>(ws) & 255) != 0) PSD_FAIL(PSD_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    int32_t rc;
    if (h->cfg.dtype == PSD_DTYPE_BF16)
        rc = debug_layer_impl<bf16_t>(h, layer, hidden, S, N, L, stop_after, (char *)ws, st);
    else
        rc = debug_layer_impl<float>(h, layer, hidden, S, N, L, stop_after, (char *)ws, st);
    if (rc != PSD_OK) return rc;
    PSD_HIP(hipGetLastError());
    return PSD_OK;
}

int32_t run_forward_cached(psd_handle *h, const int32_t *tokens, const int32_t *seq_rows, int S, int N, int block_start, int L,
                           const KvCacheArg &kv, void *ws, int64_t ws_bytes, hipStream_t st) {
    const ForwardPlan p = plan_forward(h->cfg, S, L, L);
    if (ws == nullptr || ws_bytes < p.total)
        PSD_FAIL(PSD_ERR_WORKSPACE, "workspace of %lld bytes, cached forward over %d x %d rows needs %lld", (long long)ws_bytes,
                 S, L, (long long)p.total);
    if ((reinterpret_cast<uintptr_t>(ws) & 255) != 0) PSD_FAIL(PSD_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    if (!kv.dual && kv.len != block_start)
        PSD_FAIL(PSD_ERR_SHAPE, "the cache holds %d positions, the block starts at %d", kv.len, block_start);
    if (kv.dual && (kv.len != N - L || kv.append)) PSD_FAIL(PSD_ERR_SHAPE, "a cache of the %d positions outside the block", N - L);
    if (kv.len + (kv.dual ? 0 : L) > kv.capacity) PSD_FAIL(PSD_ERR_SHAPE, "cache of %d positions is too small", kv.capacity);
    if (kv.append && kv.seqs_per_cache != 1) PSD_FAIL(PSD_ERR_INVALID_ARG, "appending needs one sequence per cache");
    int32_t rc;
    if (h->cfg.dtype == PSD_DTYPE_BF16)
        rc = forward_cached_impl<bf16_t>(h, tokens, seq_rows, S, N, block_start, L, kv, (char *)ws, st);
    else
        rc = forward_cached_impl<float>(h, tokens, seq_rows, S, N, block_start, L, kv, (char *)ws, st);
    if (rc != PSD_OK) return rc;
    PSD_HIP(hipGetLastError());
    return PSD_OK;
}

int32_t run_forward_hidden(psd_handle *h, const int32_t *tokens, const int32_t *seq_rows, int S, int N, BlockStart block_start,
                           int L, void *ws, int64_t ws_bytes, hipStream_t st, const KvCacheArg *store) {
    const ForwardPlan p = plan_forward(h->cfg, S, N, L);
    if (ws == nullptr || ws_bytes < p.total)
        PSD_FAIL(PSD_ERR_WORKSPACE, "workspace of %lld bytes, forward over %d x %d tokens needs %lld", (long long)ws_bytes,
                 S, N, (long long)p.total);
    if ((reinterpret_cast<uintptr_t>(ws) & 255) != 0) PSD_FAIL(PSD_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    if (store && (!store->base || !store->dual || store->capacity < N - L))
        PSD_FAIL(PSD_ERR_SHAPE, "storing the keys and values outside the block needs a cache of %d positions", N - L);
    if (store && block_start.per_seq) PSD_FAIL(PSD_ERR_UNSUPPORTED, "the approximate cache needs one block start for the whole batch");
    int32_t rc;
    if (h->cfg.dtype == PSD_DTYPE_BF16)
        rc = forward_hidden_impl<bf16_t>(h, tokens, seq_rows, S, N, block_start, L, (char *)ws, st, store);
    else
        rc = forward_hidden_impl<float>(h, tokens, seq_rows, S, N, block_start, L, (char *)ws, st, store);
    if (rc != PSD_OK) return rc;
    PSD_HIP(hipGetLastError());
    return PSD_OK;
}

int32_t run_head_confidence(psd_handle *h, const int32_t *tokens, const int32_t *seq_rows, int S, int N, BlockStart block_start,
                            int L, int32_t *top1, float *conf, const int32_t *out_rows, void *ws_, hipStream_t st, int plan_N) {
    const psd_model_config &c = h->cfg;
    const ForwardPlan p = plan_forward(c, S, plan_N > 0 ? plan_N : N, L);
    char *ws = (char *)ws_;
    const int rows = S * L;
    float *row_sum = (float *)(ws + p.off_rowsum);
    int32_t *row_arg = (int32_t *)(ws + p.off_rowarg);
    psd_handle::Probe &pr = h->probe_head;
    const bool timed = pr.enabled && pr.used + 2 <= pr.ev.size();
    struct StopOnExit {   // closes the timed bracket on every return path
        psd_handle::Probe &pr;
        bool on;
        hipStream_t st;
        double bytes;
        int64_t rows;
        ~StopOnExit() {
            if (!on) return;
            (void)hipEventRecord(pr.ev[pr.used + 1], st);
            pr.used += 2;
            pr.flops += bytes;
            pr.note(rows, 0);
        }
    } stop{pr, timed, st, (double)c.vocab * c.d_model * (c.dtype == PSD_DTYPE_BF16 ? 2.0 : 4.0) +
                              (double)rows * c.d_model * (c.dtype == PSD_DTYPE_BF16 ? 2.0 : 4.0) + rows * 8.0, rows};
    if (timed) (void)hipEventRecord(pr.ev[pr.used], st);
    if (c.dtype == PSD_DTYPE_BF16 && !(h->plain_mask & 4) && h->lm_head_packed && head_stream_supported(rows, c.d_model)) {
        // y was already written in fragment order by the final norm; the merge writes (top1, conf) directly
        HeadFinish fin = {tokens, seq_rows, out_rows, S, N, block_start, L, top1, conf};
        launch_head_stream_finish_bf16((const bf16_t *)(ws + p.off_ypack), (const bf16_t *)h->lm_head_packed, rows, c.vocab,
                                       c.d_model, c.logit_scale, c.mask_id, ws + p.off_part, fin, st);
        PSD_HIP(hipGetLastError());
        return PSD_OK;
    } else if (c.dtype == PSD_DTYPE_BF16 && !(h->plain_mask & 4)) {
        launch_head_confidence_bf16((const bf16_t *)(ws + p.off_y), (const bf16_t *)h->lm_head, rows, c.vocab, c.d_model,
                                    c.logit_scale, c.mask_id, ws + p.off_part, row_sum, row_arg, st);
    } else {
        float *logits = (float *)(ws + p.off_part);
        if (c.dtype == PSD_DTYPE_BF16)
            launch_plain_gemm<bf16_t, float>((const bf16_t *)(ws + p.off_y), (const bf16_t *)h->lm_head, nullptr, rows,
                                             c.vocab, c.d_model, c.d_model, c.d_model, EPI_STORE, nullptr, c.logit_scale, logits, nullptr, c.vocab,
                                             st);
        else
            launch_plain_gemm<float, float>((const float *)(ws + p.off_y), (const float *)h->lm_head, nullptr, rows, c.vocab,
                                            c.d_model, c.d_model, c.d_model, EPI_STORE, nullptr, c.logit_scale, logits, nullptr, c.vocab, st);
        launch_logits_top1(logits, rows, c.vocab, c.mask_id, row_sum, row_arg, st);
    }
    launch_head_finish(row_sum, row_arg, tokens, seq_rows, out_rows, S, N, block_start, L, c.mask_id, c.vocab, top1, conf, st);
    PSD_HIP(hipGetLastError());
    return PSD_OK;
}

int32_t run_head_logits(psd_handle *h, int S, int N, int L, float *logits, void *ws_, hipStream_t st) {
    const psd_model_config &c = h->cfg;
    const ForwardPlan p = plan_forward(c, S, N, L);
    char *ws = (char *)ws_;
    const int rows = S * L;
    if (c.dtype == PSD_DTYPE_BF16)
        launch_plain_gemm<bf16_t, float>((const bf16_t *)(ws + p.off_y), (const bf16_t *)h->lm_head, nullptr, rows, c.vocab,
                                         c.d_model, c.d_model, c.d_model, EPI_STORE, nullptr, c.logit_scale, logits, nullptr, c.vocab, st);
    else
        launch_plain_gemm<float, float>((const float *)(ws + p.off_y), (const float *)h->lm_head, nullptr, rows, c.vocab,
                                        c.d_model, c.d_model, c.d_model, EPI_STORE, nullptr, c.logit_scale, logits, nullptr, c.vocab, st);
    PSD_HIP(hipGetLastError());
    return PSD_OK;
}
