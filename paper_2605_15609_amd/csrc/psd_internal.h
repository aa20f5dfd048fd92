// Internal declarations shared by the translation units of libpsd (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <vector>

#include "psd.h"

struct bf16_t {
    uint16_t bits;
};

struct psd_handle {
    psd_model_config cfg;
    const void *tok_emb, *lm_head;
    const float *final_norm, *rope_cos, *rope_sin;
    struct Layer {
        const float *attn_norm, *ffn_norm, *bq, *bk, *bv;
        const void *wq, *wk, *wv, *wo, *w_gate, *w_up, *w_down;
    };
    std::vector<Layer> layers;
    int w_down_stride;       // row stride of every w_down (elements)
    int device;
    int plain_mask;          // debug: bit 0 plain GEMM, bit 1 plain attention, bit 2 plain LM-head, bit 3 rotary / V transpose as a separate kernel
    void *lm_head_packed;    // bf16 models: fragment-order copy of lm_head owned by the handle (streaming LM-head)
    int32_t *host_counts;    // pinned host staging for psd_decode_block
    int host_counts_cap;
    // optional HIP-event timing of one contraction kernel (epilogue kind + tile config)
    struct Probe {
        int enabled = 0, epi = -1, tile = -1;
        std::vector<hipEvent_t> ev;     // pairs (start, stop)
        size_t used = 0;                // events handed out
        double flops = 0.0;             // algorithmic work of the timed launches (FLOPs; bytes for the LM-head pass)
        std::vector<int64_t> a, b;      // per timed launch: rows and output columns of a contraction; rows of an LM-head
                                        // pass; sequences and drafts per sequence (1 = stage-1 call) of a model call
        void note(int64_t x, int64_t y) {
            a.push_back(x);
            b.push_back(y);
        }
    } probe, probe_head, probe_call;
    // Model calls of the block loops replayed as HIP graphs (launch-bound small models: ~90 kernels of a few
    // microseconds each).  A call is identified by everything its kernels' arguments are derived from; the first time
    // a key is seen the call runs eagerly (which also does the one-time set-up of its kernels), the second time it is
    // captured on capture_stream and instantiated, from then on replayed on the caller's stream.
    struct GraphKey {
        const void *src, *rows, *top1, *conf, *ws, *starts;
        int64_t ws_bytes;
        int S, N, L, start_common, rows_per_seq, epoch;
        bool operator==(const GraphKey &o) const {
            return src == o.src && rows == o.rows && top1 == o.top1 && conf == o.conf && ws == o.ws && starts == o.starts &&
                   ws_bytes == o.ws_bytes && S == o.S && N == o.N && L == o.L && start_common == o.start_common &&
                   rows_per_seq == o.rows_per_seq && epoch == o.epoch;
        }
    };
    struct GraphEntry {
        GraphKey key;
        hipGraphExec_t exec = nullptr;
        bool failed = false;        // capture or instantiation was refused: this call stays eager
        uint64_t last_use = 0;
    };
    std::vector<GraphEntry> graphs;   // at most kMaxGraphs, least recently used replaced
    static constexpr size_t kMaxGraphs = 24;
    hipStream_t capture_stream = nullptr;
    int graphs_enabled = 0;   // off unless asked for: measured to gain nothing where it was expected to (see psd_debug_set_graphs)
    uint64_t graph_clock = 0, graph_replays = 0;
};
// bumped by every debug switch that changes which kernels a model call launches: captured graphs of an older epoch are stale
int kernel_choice_epoch();
void bump_kernel_choice_epoch();

void psd_set_error(const char *fmt, ...);

#define PSD_FAIL(code, ...)         \
    do {                            \
        psd_set_error(__VA_ARGS__); \
        return (code);              \
    } while (0)

#define PSD_HIP(expr)                                                                                  \
    do {                                                                                               \
        hipError_t e_ = (expr);                                                                        \
        if (e_ != hipSuccess) PSD_FAIL(PSD_ERR_DEVICE, "%s: %s", #expr, hipGetErrorString(e_));        \
    } while (0)

static inline int64_t align_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

// ---------------------------------------------------------------- decision kernels (decide.hip)
#define PSD_DEVSTAT_POLICY 0
#define PSD_DEVSTAT_DRAFT 1
#define PSD_DEVSTAT_POST 2
#define PSD_DEVSTAT_EOS 3        // 1 + block position of the first EOS token once the sequence stopped on it, else 0
#define PSD_DEVSTAT_ENTRY 4      // two words: which block positions were masked on entry (bit j = position j)
#define PSD_DEVSTAT_COUNTED 6    // positions resolved at or before the EOS position (all resolved ones without an EOS)
#define PSD_DEVSTAT_HIST 7
#define PSD_DEVSTAT_WORDS (7 + PSD_MAX_NODES + PSD_MAX_BLOCK + 1)

// Where the active block of a sequence begins: one position common to the whole batch, or one per sequence (device
// array indexed by sequence).  Kernels that walk batch slots map a slot to its row of the token matrix first; the
// sequence is that row divided by rows_per_seq (1 for the sequences themselves, K for their drafts [B, K, N]).
struct BlockStart {
    int common;
    const int32_t *per_seq;
    int rows_per_seq;
    BlockStart(int c = 0) : common(c), per_seq(nullptr), rows_per_seq(1) {}
    BlockStart(const int32_t *arr, int rps) : common(0), per_seq(arr), rows_per_seq(rps) {}
    __host__ __device__ int of_row(int64_t row) const { return per_seq ? per_seq[row / rows_per_seq] : common; }
};

struct GraphArg {
    int32_t K;
    uint64_t rank_set[PSD_MAX_NODES];
};

// Raises a kernel's dynamic LDS limit once per device (bit d of `done` = device d has it).  Callable from several
// threads: two that race both set the same value.
inline void ensure_dynamic_lds(const void *kernel, int bytes, std::atomic<uint64_t> &done) {
    int dev = 0;
    (void)hipGetDevice(&dev);
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return;
    (void)hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    done.fetch_or(bit, std::memory_order_release);
}

void launch_eos_stop(const int32_t *tokens, int B, int N, BlockStart block_start, int L, int32_t eos_id, int32_t *n_left, int32_t *m,
                     int32_t *devstats, hipStream_t st);
// only[b] != 0 selects the sequences to finish (NULL: all); their counters of resolved positions are ADDED to
void launch_finish_counts(const int32_t *tokens, int B, int N, BlockStart block_start, int L, int32_t mask_id, int32_t eos_stop,
                          int32_t eos_id, int32_t *devstats, const int32_t *only, hipStream_t st);
// only[b] != 0 selects the sequences the policy is applied to (NULL: all); the others keep tokens and n_left
void launch_select_unmask(int32_t *tokens, int B, int N, BlockStart block_start, int L, const int32_t *top1,
                          const float *conf, psd_policy policy, int32_t mask_id, uint8_t *transfer_mask,
                          int32_t *n_selected, int32_t *n_left, int32_t *devstats, const int32_t *only, hipStream_t st);
void launch_build_drafts(const int32_t *tokens, int B, int N, BlockStart block_start, int L, const int32_t *top1,
                         const float *conf, const GraphArg &g, int32_t mask_id, int32_t *sigma, int32_t *m,
                         int32_t *drafts, hipStream_t st);
void launch_accept(int32_t *tokens, const int32_t *drafts, int B, int N, BlockStart block_start, int L,
                   const int32_t *sigma, const int32_t *m, const GraphArg &g, psd_policy policy, int32_t mask_id,
                   const int32_t *v_top1, const float *v_conf, int32_t *k_star, uint8_t *accepted,
                   int32_t *n_left, int32_t *devstats, int32_t *adopt_top1, float *adopt_conf, hipStream_t st);
// (adopt_top1 / adopt_conf [B, L], or NULL: receive the verifier output of the accepted draft k* of every sequence with m > 0)

// ---------------------------------------------------------------- forward (forward.hip)
// workspace for the K-split partial sums of a residual contraction: at most 7 parts of at most 128 rows
inline int64_t ksplit_bytes(const psd_model_config &c) { return 7ll * 128 * c.d_model * 4; }
struct ForwardPlan {
    int64_t off_h, off_a, off_qkv, off_vt, off_o, off_act, off_ksplit, off_oc, off_hc, off_y, off_ypack, off_rowsum, off_rowarg, off_part, total;
};
ForwardPlan plan_forward(const psd_model_config &cfg, int64_t S, int64_t N, int64_t L);

// Layer stack + final norm on the block rows; leaves y [S*L, d] in the workspace.
// seq_rows (device, may be NULL) maps batch slot s -> row of `tokens` to read.
// store (may be NULL): also leave every layer's rotated keys and values of the positions outside the block in the
// sequences' caches (store->dual), compacted: prefix positions first, then the suffix.
struct KvCacheArg;
int32_t run_forward_hidden(psd_handle *h, const int32_t *tokens, const int32_t *seq_rows, int S, int N,
                           BlockStart block_start, int L, void *ws, int64_t ws_bytes, hipStream_t st,
                           const KvCacheArg *store = nullptr);
// LM-head + top-1 confidence on y; out_rows (device, may be NULL) maps slot s -> row of top1/conf.
int32_t run_head_confidence(psd_handle *h, const int32_t *tokens, const int32_t *seq_rows, int S, int N,
                            BlockStart block_start, int L, int32_t *top1, float *conf, const int32_t *out_rows,
                            void *ws, hipStream_t st, int plan_N = -1 /* sequence length the workspace was planned
                            for, if not N (the cached forward plans for L rows per sequence) */);
// forward over the L block rows of S sequences against their KV caches (context-causal block attention)
int32_t run_forward_cached(psd_handle *h, const int32_t *tokens, const int32_t *seq_rows, int S, int N, int block_start, int L,
                           const KvCacheArg &kv, void *ws, int64_t ws_bytes, hipStream_t st);
int32_t run_head_logits(psd_handle *h, int S, int N, int L, float *logits, void *ws, hipStream_t st);
// debug: layer `layer` alone on the caller's residual stream [S*N, d_model] (in place); see psd_debug_layer
int32_t run_debug_layer(psd_handle *h, int layer, float *hidden, int S, int N, int L, int stop_after, void *ws, int64_t ws_bytes,
                        hipStream_t st);
int64_t act_row_stride(const psd_model_config &cfg);

// Keys and values that precede a sequence's own rows in attention: a KV cache of `len` positions, shared by
// seqs_per_cache consecutive sequences (the K drafts of one verification batch share their sequence's prefix).
// K rows [len][n_kv_heads*d_head] with row stride ld_k; values transposed, [n_kv_heads*d_head][ld_vt] with the keys
// of every group of 16 in the order 0-3, 8-11, 4-7, 12-15 (the contraction-slot order of the second attention
// MFMA) and zeros behind position len.  Caches are stride_k / stride_vt elements apart.  len = 0: no prefix.
struct KvPrefix {
    const void *k = nullptr, *vt = nullptr;
    int len = 0, ld_k = 0, ld_vt = 0;
    int64_t stride_k = 0, stride_vt = 0;
    const int32_t *seq_rows = nullptr;   // cache of sequence s = (seq_rows ? seq_rows[s] : s) / seqs_per_cache
    int seqs_per_cache = 1;
};
// position of key i inside a transposed value row
__host__ __device__ inline int vt_key_slot(int i) {
    const int piece = (i >> 2) & 3;
    return (i & ~15) | ((((piece & 1) << 1) | (piece >> 1)) << 2) | (i & 3);
}
// One sequence's KV cache of `capacity` positions: per layer the K rows, then the transposed values.
struct KvLayout {
    int64_t k_elems, vt_elems, ld_k, ld_vt, per_seq;   // elements
};
inline KvLayout kv_layout(const psd_model_config &c, int capacity) {
    KvLayout l;
    l.ld_k = (int64_t)c.n_kv_heads * c.d_head;
    l.ld_vt = (capacity + 63) / 64 * 64;
    l.k_elems = capacity * l.ld_k;
    l.vt_elems = l.ld_k * l.ld_vt;
    l.per_seq = c.n_layers * (l.k_elems + l.vt_elems);
    return l;
}
// what a model call may attend to besides its own rows
struct KvCacheArg {
    void *base = nullptr;      // NULL: no cache (the call runs over whole sequences)
    int capacity = 0, len = 0, seqs_per_cache = 1;
    bool append = false;       // store the rows' keys and values behind position len (seqs_per_cache must be 1)
    bool dual = false;         // approximate cache of a bidirectional model: the len = N - L entries are the positions
                               // OUTSIDE the block (prefix, then suffix), frozen by the whole-sequence call that
                               // entered the block; the block rows keep their positions block_start ..
};

// ---------------------------------------------------------------- kernel launchers
// elementwise.hip
template <typename T>
void launch_embed(const int32_t *tokens, const int32_t *seq_rows, int S, int N, const T *emb, int vocab, int d, float *h,
                  hipStream_t st);
// the same for the L block rows of each sequence only: h [S*L, d]
template <typename T>
void launch_embed_block(const int32_t *tokens, const int32_t *seq_rows, int S, int N, int block_start, int L, const T *emb,
                        int vocab, int d, float *h, hipStream_t st);
// keys (rotated) and values of rows row_first .. row_first+count-1 of every sequence of qkv [S*rows_per_seq, ...] into the
// caches of their sequences, cache positions at.len .. at.len+count-1
template <typename T>
void launch_kv_store(const T *qkv, int ld_qkv, int S, int rows_per_seq, int row_first, int count, int n_heads, int n_kv_heads,
                     int d_head, T *k_cache, T *vt_cache, const KvPrefix &at, hipStream_t st);
// K-split partial sums that still have to be added to the residual stream h [rows, d]: partial[s] has the
// same shape, s = 0 .. n-1, `stride` floats apart.  The norm that reads h next adds them (and stores h).
struct PendingSums {
    const float *partial = nullptr;
    int n = 0;
    int64_t stride = 0;
};
template <typename T>
void launch_rmsnorm(float *h, int64_t rows, int d, const float *gain, float eps, T *out, PendingSums pend, hipStream_t st);
template <typename T>
void launch_rmsnorm_block(float *h, const int32_t *seq_rows, int S, int N, BlockStart block_start, int L, int d, const float *gain,
                          float eps, T *out, T *packed /* fragment-order copy, may be NULL */, PendingSums pend,
                          hipStream_t st);
// dst [S*L, width] <- the L block rows of each of the S sequences of src [S*N, width]
template <typename T>
void launch_gather_block_rows(const T *src, T *dst, int width, const int32_t *seq_rows, int S, int N, BlockStart block_start, int L,
                              hipStream_t st);
template <typename T>
void launch_rope(T *qkv, int ld /* row stride */, int64_t tokens, int N, int pos0 /* position of row 0 of each sequence */, int n_heads, int n_kv_heads, int d_head, const float *cos_t,
                 const float *sin_t, hipStream_t st);
// Row strides of the workspace matrices.  Padding rows by 64 elements keeps consecutive rows out of the same
// cache channel; it pays for the SwiGLU output (24 KB rows feeding the down projection) and was measured
// to make no difference for qkv and vT, which stay dense.
inline int64_t padded_row_stride(int64_t width) { return width + 64; }
inline int64_t qkv_row_stride(int64_t w) { return w; }
inline int64_t vt_row_stride(int64_t N) { return (N + 63) / 64 * 64; }
// vT[s][kvh][c][i] <- V part of qkv[s*N + i] (rows of vt_row_stride(N) elements); the MFMA attention reads values key-contiguous
// rotary in place on q and k (position pos0 + row index inside the sequence) and V transposed into vT, one launch;
// d_head % 16 == 0
void launch_rope_transpose_v(bf16_t *qkv, int ld_qkv, int S, int N, int pos0, int n_heads, int n_kv_heads, int d_head,
                             const float *cos_t, const float *sin_t, bf16_t *vT, hipStream_t st);
void launch_transpose_v(const bf16_t *qkv, int ld_qkv, int S, int N, int n_heads, int n_kv_heads, int d_head, bf16_t *vT,
                        hipStream_t st);

// plain_kernels.hip (debug path, any shape)
enum Epilogue { EPI_STORE = 0, EPI_BIAS = 1, EPI_RESIDUAL = 2, EPI_SWIGLU = 3 };
template <typename T, typename TO>
void launch_plain_gemm(const T *A, const T *W, const T *W2, int64_t M, int Nout, int Kin, int lda, int ldw, int epi, const float *bias,
                       float scale, TO *out, float *resid, int ldo, hipStream_t st);
// block_len > 0: context-causal blocks among the own rows (key j visible to query i iff j / block_len <= i / block_len)
template <typename T>
void launch_plain_attention(const T *qkv, int ld, int S, int N, int n_heads, int n_kv_heads, int d_head, T *out,
                            const KvPrefix &pre, int block_len,
                            hipStream_t st);
void launch_logits_top1(const float *logits, int rows, int V, int mask_id, float *row_sum, int32_t *row_arg,
                        hipStream_t st);
void launch_head_finish(const float *row_sum, const int32_t *row_arg, const int32_t *tokens, const int32_t *seq_rows,
                        const int32_t *out_rows, int S, int N, BlockStart block_start, int L, int mask_id, int vocab, int32_t *top1,
                        float *conf, hipStream_t st);

// gemm_mfma.hip (bf16; Nout, Kin multiples of 64)
// index of the tile configuration the dispatcher picks for a shape; gemm_bf16_tile_name(i) describes configuration i
// (workgroup tile, wavefronts, LDS ring depths), 0 <= i < gemm_bf16_tile_count()
int gemm_bf16_tile(int64_t M, int Nout, int epi, int Kin = 0);   // Kin = 0: not known (matters for residual contractions only)
int gemm_bf16_tile_count();
// QKV projection that also applies the rotary embedding to the q / k heads and stores V transposed into vT (what
// launch_rope_transpose_v does in a second pass), bit-identical to the two-pass form.  gemm_bf16_qkv_tile returns the tile
// to pass on, or -1 when the shape has no tile that holds whole heads of one kind (then the two-pass form runs).
// rows_per_seq: rows of A per sequence (a multiple of 16); v_start: first V column; pos0: position of a sequence's row 0.
int gemm_bf16_qkv_tile(int64_t M, int Nout, int d_head, int v_start, int rows_per_seq);
void launch_gemm_bf16_qkv(const bf16_t *A, const bf16_t *W, int64_t M, int Nout, int Kin, int lda, int ldw, const float *bias, bf16_t *qkv,
                          int ld_qkv, int d_head, int v_start, int rows_per_seq, int pos0, const float *cos_t, const float *sin_t,
                          bf16_t *vT, int ld_vt, int tile, hipStream_t st);
// K-split of a residual contraction (1 = none).  With s > 1 parts, launch_gemm_bf16_split adds part 0 into
// resid and stores parts 1..s-1 to partial [s-1][M][Nout] fp32; the next reader of resid adds them in order.
int gemm_bf16_splits(int64_t M, int Nout, int Kin);
void launch_gemm_bf16_split(const bf16_t *A, const bf16_t *W, int64_t M, int Nout, int Kin, int lda, int ldw, float *resid, int ldo,
                            float *partial, int splits, hipStream_t st);
void launch_fold_partials(float *resid, int64_t rows, int cols, int ldo, const float *partial, int n_partial, hipStream_t st);
const char *gemm_bf16_tile_name(int tile);
// debug, process-wide (not per handle; not for use while another thread launches): -1 = automatic; otherwise bits 0-7
// the tile (0xff = automatic), bits 8-15 the K-split of residual contractions (0 = automatic), bits 16-23 the band
// height of the tile order (0 = unchanged)
void gemm_bf16_force_tile(int tile);
// 256 workgroups x 4 wavefronts x iters x 16 MFMAs (32x32x16 bf16) on the given operand data; sink >= 4 MiB
void launch_mfma_rate(const void *operands, int n_vec16, int iters, void *sink, hipStream_t st);
// A [M, Kin] with row stride lda, W / W2 [Nout, Kin] with row stride ldw (elements)
void launch_gemm_bf16(const bf16_t *A, const bf16_t *W, const bf16_t *W2, int64_t M, int Nout, int Kin, int lda, int ldw, int epi,
                      const float *bias, bf16_t *out, float *resid, int ldo, hipStream_t st);
// attention_mfma.hip (bf16, d_head 64 or 128): q, k from qkv (rotary applied), values from vT
void launch_attention_bf16(const bf16_t *qkv, int ld_qkv, const bf16_t *vT, int S, int N, int n_heads, int n_kv_heads, int d_head,
                           bf16_t *out, const KvPrefix &pre, hipStream_t st);
// lm_head.hip (bf16): LM-head fused with the online top-1 / sum-exp reduction
int64_t head_partial_bytes(int rows, int V);
// fragment-order copies: [ceil(R/32)][K/16][64 lanes][8 bf16]
int64_t packed_rows_bytes(int64_t R, int K);
void launch_pack_rows(const bf16_t *src, int64_t R, int K, bf16_t *dst, hipStream_t st);
bool head_stream_supported(int rows, int d);
void launch_head_stream_bf16(const bf16_t *y_packed, const bf16_t *W_packed, int rows, int V, int d, float scale, int mask_id,
                             void *partials, float *row_sum, int32_t *row_arg, hipStream_t st);
// where the streamed head's result goes: (row_sum, row_arg) and/or the final (top1, conf) tables with sentinels
struct HeadFinish {
    const int32_t *tokens, *seq_rows, *out_rows;
    int S, N;
    BlockStart block_start;
    int L;
    int32_t *top1;
    float *conf;
};
void launch_head_stream_finish_bf16(const bf16_t *y_packed, const bf16_t *W_packed, int rows, int V, int d, float scale,
                                    int mask_id, void *partials, const HeadFinish &fin, hipStream_t st);
void launch_head_confidence_bf16(const bf16_t *y, const bf16_t *W, int rows, int V, int d, float scale, int mask_id,
                                 void *partials, float *row_sum, int32_t *row_arg, hipStream_t st);
