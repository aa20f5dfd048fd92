/*
 * psd.h -- C ABI of the MI355X (gfx950) library for the Parallel Speculative Decoding
 * (PSD) denoising step of masked-diffusion language models.
 *
 * One loop iteration of the paper's Alg. 1 is
 *     stage 1  forward -> (x_hat, c) on the masked positions of the active block  (Sec. 3.1)
 *              T = pi(x, c); commit x_hat on T                                      (Eq. 1)
 *     stage 2  sigma = residual masks by step-t confidence; K drafts               (Eq. 2)
 *     stage 3  one batched forward over the K drafts; hierarchical acceptance over
 *              the draft DAG; advance to the deepest accepted draft                 (Sec. 3.2)
 * and every step runs in hand-written HIP kernels behind the calls below.
 *
 * Conventions
 *   - Every function returns an int32 status: PSD_OK (0) or a negative PSD_ERR_*.
 *     Arguments are validated on the host before anything is enqueued; on error nothing
 *     is launched and no output is written.  psd_last_error() gives a message.
 *   - "device" pointers are HIP device memory owned by the caller (any allocator).
 *     "host" pointers are ordinary host memory.  The library allocates device memory only
 *     inside psd_create (for bf16 models a second copy of the LM-head matrix in MFMA-fragment
 *     order, vocab*d_model*2 bytes) and frees it in psd_destroy.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     enqueue asynchronously and do not synchronise, except psd_decode_block, which
 *     returns host statistics and reads small counters back once per iteration.
 *   - Layouts are row-major.  tokens int32 [B, N]; the active block is positions
 *     block_start .. block_start+L-1 of every sequence (1 <= L <= 64; the step calls take one block_start for
 *     the batch, psd_decode_block and psd_decode one per sequence).  Per-block tables
 *     are top1 int32 [B, L] and conf float [B, L]: a masked position carries the
 *     prediction, any other position the sentinel (its own token, -1.0f).
 *   - Sequences of a batch are independent.  In the whole-sequence calls batching never changes a sequence's
 *     logits or top-1 tokens; the confidence normaliser is summed in an order that depends on the number of rows
 *     in the call, so confidences can differ in the last fp32 bit between batch shapes.  The block-row calls
 *     (psd_*_cached, psd_*_approx) cut the output and down projections along K when a call has at most 128 rows,
 *     so there a sequence's fp32 sums, and with near-tied confidences its decisions, can depend on how many
 *     sequences or drafts share the call; results agree to fp32 rounding of those sums.
 *   - Token ids outside [0, vocab) are invalid input: they read a zero embedding row (no fault).  A block row
 *     whose logits are all non-finite has no prediction: it yields (token 0, confidence 0).
 */
#ifndef PSD_H
#define PSD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PSD_OK               0
#define PSD_ERR_INVALID_ARG -1
#define PSD_ERR_SHAPE       -2
#define PSD_ERR_WORKSPACE   -3
#define PSD_ERR_DEVICE      -4
#define PSD_ERR_UNSUPPORTED -5

#define PSD_MAX_NODES 32   /* K, root included */
#define PSD_MAX_BLOCK 64   /* L */

#define PSD_DTYPE_FP32 0   /* debug path: fp32 storage and arithmetic, plain kernels */
#define PSD_DTYPE_BF16 1   /* bf16 storage, MFMA contractions with fp32 accumulation */
#define PSD_ATTN_BIDIRECTIONAL 0
#define PSD_ATTN_BLOCK_CAUSAL 1

typedef struct psd_handle psd_handle;

/* Model layout.  The paper only requires a bidirectional transformer that yields a
 * distribution per position (Sec. 3.1); this is the pre-norm RMSNorm / rotary / SwiGLU
 * decoder stack of the benchmarked 7-8B models, run without a causal mask. */
typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, d_head, d_ffn, vocab;
    int32_t mask_id;       /* id of [M]; it has an embedding row but is never predicted */
    float   rms_eps;
    int32_t qkv_bias;      /* 1: bq/bk/bv present */
    int32_t dtype;         /* PSD_DTYPE_*: type of every weight matrix */
    float   logit_scale;   /* logits = logit_scale * (y W_lm^T); 1.0 normally */
    int32_t max_seq;       /* rows of the rotary tables */
    int32_t attention;     /* PSD_ATTN_*: bidirectional (default 0), or context-causal blocks (App. A: full
                            * attention inside a block of the decoding block length, causal across blocks) */
} psd_model_config;

/* Device pointers, borrowed for the life of the handle.  Matrices are [out, in] in the
 * model dtype; norm gains, biases and rotary tables are fp32.  The per-layer members are
 * host arrays of n_layers device pointers (copied by psd_create). */
typedef struct {
    const void  *tok_emb;      /* [vocab, d_model] */
    const float *final_norm;   /* [d_model] */
    const void  *lm_head;      /* [vocab, d_model] */
    const float *rope_cos;     /* [max_seq, d_head/2], cos(pos * theta^(-2j/d_head)) */
    const float *rope_sin;     /* [max_seq, d_head/2]; pairs are (j, j + d_head/2) */
    const float *const *attn_norm;   /* [d_model] */
    const void  *const *wq;          /* [n_heads*d_head, d_model] */
    const void  *const *wk;          /* [n_kv_heads*d_head, d_model] */
    const void  *const *wv;          /* [n_kv_heads*d_head, d_model] */
    const float *const *bq, *const *bk, *const *bv;   /* NULL arrays when qkv_bias == 0 */
    const void  *const *wo;          /* [d_model, n_heads*d_head] */
    const float *const *ffn_norm;    /* [d_model] */
    const void  *const *w_gate;      /* [d_ffn, d_model] */
    const void  *const *w_up;        /* [d_ffn, d_model] */
    const void  *const *w_down;      /* [d_model, d_ffn], row stride w_down_stride */
    int32_t w_down_stride;           /* elements between rows of w_down; 0 = d_ffn (dense).  A multiple of 8.
                                      * Rows padded by 64 elements avoid cache-channel conflicts on MI355X
                                      * when a dense row is a multiple of 8 KB (d_ffn = 12288). */
} psd_weights;

/* Transfer policy pi (Sec. 3.2 stage 1; App. B.2): over the masked positions of the block,
 * ordered by confidence descending (ties: lower position first), commit every position
 * with c > tau plus the k_min most confident; if k_max > 0 at most the k_max most
 * confident of those.  Greedy decoding: tau = +inf, k_min = 1.  Confidence Parallel
 * Decoding: tau = 0.9, k_min = 1.  The same rule is the acceptance criterion A_pi. */
typedef struct {
    float   tau;
    int32_t k_min;
    int32_t k_max;   /* 0 = unbounded */
    /* EOS early stopping of psd_decode_block / psd_decode_block_cached (evaluation protocol of
     * App. B.1; the other calls ignore both fields).  eos_stop = 0: off.  eos_stop = 1: a sequence
     * stops as soon as an EOS token has been produced: after every update of its state (the stage-1
     * commit; the advance with its post-verification commit) its block is searched for eos_id, and
     * if it is there the sequence takes part in no further model call, whatever is still masked. */
    int32_t eos_stop;
    int32_t eos_id;  /* 0 <= eos_id < vocab, not the mask token (checked when eos_stop = 1) */
    /* Block loops only (psd_decode, psd_decode_block, psd_decode_block_cached); 0 = the literal Alg. 1.
     * 1 = a variant that is NOT the literal Alg. 1 and gives different results in general: the last line
     * of stage 3 commits, by pi, predictions of the accepted draft k* -- the literal loop then calls the
     * model again on the committed state (stage 1 of the next iteration).  The variant takes that
     * post-verification commit as the next iteration's stage-1 commit and draws the next speculative
     * ordering and drafts from k*'s verifier output (x_hat_k*, c_k*), the model's exact prediction on the
     * state just before that commit.  An iteration then costs one model call, the batched verification;
     * only the call that enters a block is a stage-1 call.  Every committed token still comes from an
     * exact forward of an exact state.  The tables live for one library call: each call starts with a
     * stage-1 call for every sequence (so max_iterations = 1 gains nothing). */
    int32_t single_forward;
} psd_policy;

/* Draft DAG (Sec. 3.2 stage 2).  Node k speculates on the ranks of the speculative
 * ordering sigma whose bits are set in rank_set[k] (bit r <-> sigma_{r+1}); node 0 is the
 * root with rank_set[0] = 0.  Edges are implied: (p, k) is an edge iff S_p is a strict
 * subset of S_k.  Ranks >= m (the number of residual masks) are ignored. */
typedef struct {
    int32_t  K;
    uint64_t rank_set[PSD_MAX_NODES];
} psd_graph;

/* Per-sequence counters of psd_decode_block.  TPF = tokens / invocations with
 * tokens = tokens_policy + tokens_draft + tokens_postverify; a batched verification
 * counts as one invocation (Sec. 4.1 "Metrics"). */
typedef struct {
    int64_t invocations;
    int64_t tokens_policy;       /* committed by pi in stage 1 */
    int64_t tokens_draft;        /* |S_k*| of the accepted drafts */
    int64_t tokens_postverify;   /* committed by pi on k*'s verifier output */
    int32_t depth_hist[PSD_MAX_NODES + PSD_MAX_BLOCK + 1];   /* histogram of |S_k*| */
    /* App. B.1: tokens up to and including the EOS position.  tokens_counted grows by the number of
     * block positions the call resolved at or before the first EOS token of the block (tokens
     * unmasked beyond it are discarded, whenever they were unmasked); by all it resolved when the
     * call did not stop on an EOS.  stopped is set to 1 and eos_pos to the sequence position of that
     * first EOS token when it did; both are left alone otherwise. */
    int64_t tokens_counted;
    int32_t stopped;
    int32_t eos_pos;
} psd_stats;

const char *psd_status_string(int32_t status);
/* sizeof of the structures above as this library was built, in the order psd_model_config, psd_weights,
 * psd_policy, psd_graph, psd_stats, psd_work, psd_graph_score, psd_debug_layout (the first n of them into out; returns how many
 * there are): lets a foreign-language binding check its own declarations. */
int32_t psd_struct_sizes(int32_t *out, int32_t n);
/* Message of the last error raised on the calling thread ("" if none). */
const char *psd_last_error(void);

/* Creates a handle on the current HIP device.  Fails with PSD_ERR_DEVICE when no gfx950
 * device is present, PSD_ERR_SHAPE / PSD_ERR_UNSUPPORTED on layouts the kernels do not
 * cover (bf16 needs d_head in {64, 128} and d_model, d_ffn multiples of 64; fp32 takes
 * any even d_head). */
int32_t psd_create(const psd_model_config *cfg, const psd_weights *w, psd_handle **out);
int32_t psd_destroy(psd_handle *h);

/* Bytes of device workspace that a forward over up to max_seqs sequences of length N with
 * block length L needs (psd_verify_accept and psd_decode_block run max_seqs = B*K).
 * Negative status on bad arguments. */
int64_t psd_workspace_bytes(const psd_model_config *cfg, int32_t max_seqs, int32_t N, int32_t L);

/* Prefix chain: node k speculates on the k*width most confident residual positions. */
int32_t psd_graph_chain(int32_t K, int32_t width, psd_graph *out);
/* Subset lattice: one node for every subset of the `depth` most confident residual positions
 * (2^depth nodes, ordered by size): the densest multi-parent DAG over those positions -- a
 * deeper draft can be reached through every order of unmasking (Sec. 3.2 stage 2).  depth 0..5. */
int32_t psd_graph_lattice(int32_t depth, psd_graph *out);

/* Model call (Sec. 3.1; Alg. 1 stage 1 and the batched pass of stage 3): forward S
 * sequences over all N positions with bidirectional attention, then on the L block rows of
 * each the top-1 token x_hat = argmax_v p(v) and confidence c = max_v p(v), p the softmax
 * of the logits over the vocabulary without [M].  Ties go to the lowest token id.  The
 * logits are reduced on the fly and never stored.
 *   tokens device int32 [S, N] (read); top1 device int32 [S, L], conf device float [S, L]
 *   (written); ws device, ws_bytes >= psd_workspace_bytes(cfg, S, N, L). */
int32_t psd_forward_confidence(psd_handle *h, const int32_t *tokens, int32_t S, int32_t N,
                               int32_t block_start, int32_t L, int32_t *top1, float *conf,
                               void *ws, int64_t ws_bytes, void *stream);

/* Debug companion of psd_forward_confidence: writes the raw block logits
 * logit_scale * (y W_lm^T), [M] column included, as float [S*L, vocab] (device).  Only for
 * numeric parity checks; the decode path never materialises logits. */
int32_t psd_forward_logits(psd_handle *h, const int32_t *tokens, int32_t S, int32_t N,
                           int32_t block_start, int32_t L, float *logits,
                           void *ws, int64_t ws_bytes, void *stream);

/* Debug switch for numeric cross-checks: bit 0 runs the layer contractions, bit 1 the
 * attention, bit 2 the LM-head on the plain (non-MFMA) kernels; bit 3 keeps the rotary embedding and the
 * transpose of V in a kernel of their own instead of the QKV projection's epilogue (same bits either way).
 * 0 (default) = MFMA path. */
int32_t psd_debug_set_plain(psd_handle *h, int32_t mask);

/* Debug hook for parity checks of one layer at full width: runs layer `layer` of the model alone on a residual
 * stream supplied by the caller -- hidden, device float [S*N, d_model], updated in place as one layer of the forward
 * would (Sec. 3.1 only asks for a bidirectional transformer; the layer is RMSNorm, QKV, rotary, attention over the
 * sequence's N rows, output projection, RMSNorm, SwiGLU, down projection, with the kernels and tiles the forward picks
 * for S*N rows).  stop_after = 1 stops once the attention output is written and leaves hidden untouched.  The
 * intermediates stay in the workspace, where psd_debug_workspace_layout says (byte offsets; row strides in elements
 * of the model dtype): a = output of the last norm that ran [S*N, d_model]; qkv = projections with rotary applied
 * [S*N, ld_qkv]; vT = values transposed, [S, n_kv_heads*d_head, ld_vt] with the keys of every group of 16 in the
 * order 0-3, 8-11, 4-7, 12-15; o = attention output [S*N, n_heads*d_head]; act = SwiGLU output [S*N, ld_act].
 * ws as for psd_forward_confidence(S, N, L).  Honours psd_debug_set_plain. */
typedef struct {
    int64_t off_a, off_qkv, off_vt, off_o, off_act;
    int32_t ld_qkv, ld_act, ld_vt, reserved;
} psd_debug_layout;
int32_t psd_debug_workspace_layout(const psd_model_config *cfg, int32_t S, int32_t N, int32_t L, psd_debug_layout *out);
int32_t psd_debug_layer(psd_handle *h, int32_t layer, float *hidden, int32_t S, int32_t N, int32_t L, int32_t stop_after,
                        void *ws, int64_t ws_bytes, void *stream);

/* Debug / tuning: forces the workgroup tile of the layer contractions (see psd_probe_begin
 * and psd_kernel_gemm_tile_name for the numbering; -1 = pick per shape; a tile that cannot run the
 * epilogue asked for is ignored).  Process-wide. */
int32_t psd_debug_force_gemm_tile(int32_t tile);
/* Optional: the block loops (psd_decode, psd_decode_block) replay the whole-sequence model calls of a shape they have
 * seen twice as HIP graphs.  Results are bit-identical to eager launches.  Off by default: on the one workload where
 * a model call is ~75 kernels of 4-11 microseconds (8 layers, d_model 512) the queue already runs them back to back and
 * the graph changes nothing (119 ms per decode either way); the time goes to the kernels' own floor, not to launches.
 * enabled = 1 / 0 switches it on / off for the handle, a negative value leaves it; replays (may be NULL) receives the
 * number of graph launches so far.  A graph holds the addresses the call was captured with (tokens, tables, workspace):
 * up to 24 distinct calls are kept, least recently used replaced.  Calls that are being timed by psd_probe_begin and
 * the KV-cached calls always launch eagerly. */
int32_t psd_debug_set_graphs(psd_handle *h, int32_t enabled, int64_t *replays);

/* Stage 1 commit (Eq. 1): applies pi to every sequence in place.
 *   tokens device int32 [B, N] (updated); top1/conf device [B, L] (read);
 *   transfer_mask device uint8 [B, L] (1 where committed); n_selected device int32 [B]. */
int32_t psd_select_unmask(psd_handle *h, int32_t *tokens, int32_t B, int32_t N, int32_t block_start,
                          int32_t L, const int32_t *top1, const float *conf, const psd_policy *policy,
                          uint8_t *transfer_mask, int32_t *n_selected, void *stream);

/* Stage 2 (Eq. 2): from the post-commit tokens and the step-t (top1, conf): the
 * speculative ordering sigma (block-local positions, confidence descending, ties lower
 * position first, padded with -1), the residual count m, and the K drafts.
 *   tokens device int32 [B, N] (read); sigma device int32 [B, L]; m device int32 [B];
 *   drafts device int32 [B, K, N] (written). */
int32_t psd_build_drafts(psd_handle *h, const int32_t *tokens, int32_t B, int32_t N, int32_t block_start,
                         int32_t L, const int32_t *top1, const float *conf, const psd_graph *graph,
                         int32_t *sigma, int32_t *m, int32_t *drafts, void *stream);

/* Hierarchical acceptance and state advance on given verifier outputs (Alg. 1 stage 3
 * without the model call).  Node k is accepted iff some accepted p with S_p a strict
 * subset of S_k has, on every position i of S_k \ S_p, v_top1[p, i] equal to the drafted
 * token and i committed by pi applied to p's verifier output.  k* is the accepted node
 * with the largest S (ties: lowest index); tokens <- draft k*, then pi is applied once more
 * on k*'s verifier output.  Sequences with m == 0 are left untouched (k_star = 0).
 *   tokens device int32 [B, N] (written); drafts device int32 [B, K, N]; sigma device
 *   [B, L]; m device [B]; v_top1 / v_conf device [B, K, L]; k_star device int32 [B];
 *   accepted device uint8 [B, K]. */
int32_t psd_accept(psd_handle *h, int32_t *tokens, const int32_t *drafts, int32_t B, int32_t N,
                   int32_t block_start, int32_t L, const int32_t *sigma, const int32_t *m,
                   const psd_graph *graph, const psd_policy *policy, const int32_t *v_top1,
                   const float *v_conf, int32_t *k_star, uint8_t *accepted, void *stream);

/* Stage 3 whole (Sec. 3.2): one batched forward over the B*K drafts (one invocation),
 * then psd_accept on its outputs, which are also returned in v_top1 / v_conf [B, K, L].
 * ws_bytes >= psd_workspace_bytes(cfg, B*K, N, L). */
int32_t psd_verify_accept(psd_handle *h, int32_t *tokens, const int32_t *drafts, int32_t B, int32_t N,
                          int32_t block_start, int32_t L, const int32_t *sigma, const int32_t *m,
                          const psd_graph *graph, const psd_policy *policy, int32_t *k_star,
                          uint8_t *accepted, int32_t *v_top1, float *v_conf,
                          void *ws, int64_t ws_bytes, void *stream);

/* Alg. 1 on one block of each of B sequences: sequence b decodes the block [block_start[b], block_start[b]+L) until
 * it has no masked position left (block_start: host int32 [B]; the sequences need not be on the same block).  An
 * iteration is one stage-1 model call over the sequences still running and one batched verification call over the K
 * drafts of those that keep masks after the stage-1 commit; sequences that finish early drop out of the model calls.
 * Blocks until done.  tokens device int32 [B, N] (updated in place);
 * stats host psd_stats [B], counters are ADDED to what it holds (zero it first);
 * ws_bytes >= psd_workspace_bytes(cfg, B*K, N, L) + psd_decode_scratch_bytes(B, N, L, K). */
int32_t psd_decode_block(psd_handle *h, int32_t *tokens, int32_t B, int32_t N, const int32_t *block_start,
                         int32_t L, const psd_policy *policy, const psd_graph *graph, psd_stats *stats,
                         void *ws, int64_t ws_bytes, void *stream);
/* The whole semi-autoregressive generation (Alg. 1 per block; App. B.1: blocks left to right, the next block of a
 * sequence starts once its current one is fully resolved; with policy->eos_stop a sequence ends with the block in
 * which an EOS token was produced).  block_start: host int32 [B], in and out: the first position of every sequence's
 * current block on entry (N - block_start[b] a multiple of L; block_start[b] >= N: nothing left to do), and where
 * the sequence stands on return (>= N when it reached the end).  Every sequence advances through its own blocks: a
 * sequence that resolves its block moves on in the next iteration while the others continue, so the model calls
 * keep all running sequences in one batch.  max_iterations > 0 returns after that many iterations of the batch
 * (0: until every sequence is done); *iterations_done (host, may be NULL) receives the number run.  A later call
 * continues from tokens and block_start as they stand.  Workspace and stats as for psd_decode_block; with
 * max_iterations > 0 and EOS stopping, tokens_counted of a call counts what that call resolved at or before the
 * first EOS its block holds by the end of the call. */
int32_t psd_decode(psd_handle *h, int32_t *tokens, int32_t B, int32_t N, int32_t *block_start, int32_t L,
                   const psd_policy *policy, const psd_graph *graph, psd_stats *stats, int32_t max_iterations,
                   int32_t *iterations_done, void *ws, int64_t ws_bytes, void *stream);
int64_t psd_decode_scratch_bytes(int32_t B, int32_t N, int32_t L, int32_t K);

/* ---- Context-causal block attention with an exact prefix KV cache ------------------------------
 * One model family of the paper (App. A, the continually pretrained block-diffusion model) attends
 * fully inside a block and causally across blocks.  With config.attention = PSD_ATTN_BLOCK_CAUSAL
 * (blocks = the decoding blocks, from position 0; prompt length a multiple of the block length):
 *   - the calls above still work on whole sequences (masked attention on the plain kernels: the
 *     on-device reference for this mode);
 *   - the calls below run the model on the L rows of the active block only.  Everything before the
 *     block is finished, so its keys and values are exact in a cache, and nothing after it is
 *     visible.  The K drafts of a verification batch share their sequence's cache (the "KV-cache
 *     sharing" of Sec. 3.2 stage 3, lossless here).
 * The cache is caller-owned device memory, psd_kv_cache_bytes(cfg, capacity) bytes per sequence,
 * sequences back to back, 256-byte aligned; per layer it holds the rotated keys
 * [capacity, n_kv_heads*d_head] and the values transposed.  It must be zeroed (psd_kv_reset) before a
 * sequence starts.  Its length is not stored: a call's block_start says how many positions it holds,
 * and psd_kv_prefill / psd_decode_block_cached extend it block by block.  Block lengths must be
 * multiples of 16.  Workspace: psd_workspace_bytes(cfg, sequences, L, L) (+ the decode scratch).
 *   psd_kv_prefill: forwards positions [0, n_prompt) of tokens [B, N] block by block and fills the caches.
 *   psd_forward_confidence_cached: tokens device int32 [S, N], only positions block_start .. +L are
 *     read; sequence s uses cache s / seqs_per_cache; writes top1/conf [S, L] (both or neither) and,
 *     if logits != NULL, the raw block logits [S*L, vocab] (debug).
 *   psd_decode_block_cached: psd_decode_block with cached model calls; afterwards the finished block
 *     is appended to the caches (one more forward over the B blocks, not counted as an invocation:
 *     it decodes nothing). */
int64_t psd_kv_cache_bytes(const psd_model_config *cfg, int32_t capacity);
int32_t psd_kv_reset(psd_handle *h, void *cache, int32_t n_seqs, int32_t capacity, void *stream);
int32_t psd_kv_prefill(psd_handle *h, const int32_t *tokens, int32_t B, int32_t N, int32_t n_prompt, int32_t L,
                       void *cache, int32_t capacity, void *ws, int64_t ws_bytes, void *stream);
int32_t psd_forward_confidence_cached(psd_handle *h, const int32_t *tokens, int32_t S, int32_t N, int32_t block_start,
                                      int32_t L, int32_t seqs_per_cache, const void *cache, int32_t capacity,
                                      int32_t *top1, float *conf, float *logits, void *ws, int64_t ws_bytes,
                                      void *stream);
int32_t psd_decode_block_cached(psd_handle *h, int32_t *tokens, int32_t B, int32_t N, int32_t block_start, int32_t L,
                                const psd_policy *policy, const psd_graph *graph, psd_stats *stats, void *cache,
                                int32_t capacity, void *ws, int64_t ws_bytes, void *stream);

/* ---- Approximate KV cache for fully bidirectional models -----------------------------------------
 * Sec. 3.2 stage 3 notes that KV-cache sharing can cut redundant computation; with bidirectional
 * attention any cache is an approximation, and the paper fixes no scheme.  The one offered here is the
 * published prefix + suffix ("dual") cache of block-wise diffusion decoding: the model call that enters a
 * block runs over the whole sequences (exact) and freezes, per layer, the rotated keys and the values of the
 * N - L positions outside the block; every later call on that block runs on the L block rows alone and
 * attends to the frozen entries, which are stale by then.  Results differ from the exact calls above (they
 * are those of the same procedure under this approximation; the test oracle has the same mode).
 * config.attention must be PSD_ATTN_BIDIRECTIONAL, L a multiple of 16.  The cache is laid out like the exact
 * one (psd_kv_cache_bytes(cfg, capacity) per sequence, capacity >= N - L, zeroed once with psd_kv_reset).
 *   psd_forward_confidence_approx: refresh = 1: exact call over the S whole sequences, fills cache s for
 *     sequence s (seqs_per_cache must be 1); refresh = 0: block rows against the caches, sequence s using
 *     cache s / seqs_per_cache (the K drafts of a verification batch share their sequence's cache).
 *     Outputs as psd_forward_confidence_cached; ws as psd_workspace_bytes(cfg, S, refresh ? N : L, L).
 *   psd_decode_block_approx: Alg. 1 on the block; the first stage-1 call refreshes, all other calls use the
 *     caches.  cache for B sequences; ws_bytes >= max(psd_workspace_bytes(cfg, B, N, L),
 *     psd_workspace_bytes(cfg, B*K, L, L)) + psd_decode_scratch_bytes(B, N, L, K). */
int32_t psd_forward_confidence_approx(psd_handle *h, const int32_t *tokens, int32_t S, int32_t N, int32_t block_start,
                                      int32_t L, int32_t refresh, int32_t seqs_per_cache, void *cache, int32_t capacity,
                                      int32_t *top1, float *conf, float *logits, void *ws, int64_t ws_bytes,
                                      void *stream);
int32_t psd_decode_block_approx(psd_handle *h, int32_t *tokens, int32_t B, int32_t N, int32_t block_start, int32_t L,
                                const psd_policy *policy, const psd_graph *graph, psd_stats *stats, void *cache,
                                int32_t capacity, void *ws, int64_t ws_bytes, void *stream);

/* Offline calibration of the draft graph (Sec. 3.2 stage 2: the topology is fixed before inference so
 * as to maximise empirical throughput).  The calibration batch -- tokens device int32 [B, N], the first
 * n_prompt positions of every row resolved, the rest [M] -- is decoded block by block once per candidate
 * (on a copy in work_tokens, device int32 [B, N]; tokens itself is only read), timed with HIP events on
 * `stream`; scores[c] (host) receives the candidate's decode time, decoded tokens per second, TPF, tokens
 * and invocations summed over the batch, and *best the index with the highest tokens per second (lowest
 * index on ties).  cache = NULL: whole-sequence model calls; otherwise the block-causal cached path
 * (cache as for psd_decode_block_cached, for B sequences; it is reset and prefilled from the prompt before
 * every candidate, outside the timed region).  ws as for psd_decode_block with the largest K among the
 * candidates.  EOS early stopping is not applied (policy->eos_stop is ignored).  Blocks until done. */
typedef struct {
    double  seconds, tokens_per_s, tpf;
    int64_t tokens, invocations;
} psd_graph_score;
int32_t psd_calibrate_graph(psd_handle *h, const int32_t *tokens, int32_t *work_tokens, int32_t B, int32_t N,
                            int32_t n_prompt, int32_t L, const psd_policy *policy, const psd_graph *candidates,
                            int32_t n_candidates, psd_graph_score *scores, int32_t *best, void *cache,
                            int32_t capacity, void *ws, int64_t ws_bytes, void *stream);

/* Per-handle timing of the last psd_decode_block / forward calls is not kept; callers time
 * with HIP events on `stream`.  For roofline accounting the library reports the algorithmic
 * work of one forward: FLOPs of the layer contractions, of attention, and of the LM-head,
 * and the bytes the LM-head pass must move (weights once + hidden rows + outputs). */
typedef struct {
    double gemm_flops, attn_flops, head_flops, head_bytes, weight_bytes;
} psd_work;
int32_t psd_forward_work(const psd_model_config *cfg, int32_t S, int32_t N, int32_t L, psd_work *out);

/* Kernel-level hooks for parity tests and timing at full shapes without a model: the same
 * launchers the forward uses, on caller-provided device buffers (bf16 = raw 16-bit).
 *   gemm:  epilogue 0/1: out[m, n] = bf16(sum_k A[m,k] W[n,k] (+ bias[n]));
 *          2: resid[m, n] += sum (fp32);  3: out = bf16(silu(A W^T) * (A W2^T)).
 *          A [M, Kin] with row stride lda, W / W2 [Nout, Kin] with row stride ldw (elements, multiples
 *          of 8); Nout, Kin multiples of 64; ldo = row stride of out / resid.
 *   attention: qkv [S*N, (n_heads + 2 n_kv_heads) * d_head] with row stride ld_qkv (elements, multiple of 8),
 *          rotary already applied; vT is scratch of psd_kernel_attention_scratch_bytes; out
 *          [S*N, n_heads*d_head] dense.
 *   head:  y [rows, d], W [vocab, d] -> row_sum[r] = sum_v exp(z_v - max_v z), row_arg[r] =
 *          argmax_v z_v over v != mask_id, z = scale * y W^T; scratch from
 *          psd_kernel_head_scratch_bytes. */
int32_t psd_kernel_gemm_bf16(const void *A, const void *W, const void *W2, int64_t M, int32_t Nout, int32_t Kin,
                             int32_t lda, int32_t ldw, int32_t epilogue, const float *bias, void *out, float *resid,
                             int32_t ldo, void *stream);
/* The residual contraction (epilogue 2, dense A, W and resid) cut into k_splits parts along K (0 = the choice
 * the forward makes for this shape, possibly 1; otherwise 1..8 with Kin a multiple of 64*k_splits): part 0
 * adds into resid, the others go to `partial` (device, (k_splits-1)*M*Nout floats) and are then added
 * to resid in order by a second kernel, so that resid ends as resid + A W^T.  *used_splits (host, may be
 * NULL) receives the number of parts. */
int32_t psd_kernel_gemm_residual_splitk(const void *A, const void *W, int64_t M, int32_t Nout, int32_t Kin,
                                        float *resid, float *partial, int64_t partial_bytes, int32_t k_splits,
                                        int32_t *used_splits, void *stream);
int64_t psd_kernel_attention_scratch_bytes(int32_t S, int32_t N, int32_t n_kv_heads, int32_t d_head);
int32_t psd_kernel_attention_bf16(const void *qkv, int32_t ld_qkv, int32_t S, int32_t N, int32_t n_heads,
                                  int32_t n_kv_heads, int32_t d_head, void *vT, void *out, void *stream);
int64_t psd_kernel_head_scratch_bytes(int32_t rows, int32_t vocab);
/*   streaming head (what the forward runs for <= 192 rows): both operands in MFMA-fragment order,
 *          [ceil(R/32)][K/16][64 lanes][8 bf16]; psd_kernel_pack_rows builds that copy of a row-major
 *          [R, K] matrix into dst of psd_kernel_packed_bytes(R, K) bytes.  Same outputs and scratch as
 *          psd_kernel_head_confidence_bf16 (the tiled kernel, which the forward keeps for more rows). */
int64_t psd_kernel_packed_bytes(int64_t R, int32_t K);
int32_t psd_kernel_pack_rows(const void *src, int64_t R, int32_t K, void *dst, void *stream);
int32_t psd_kernel_head_stream_bf16(const void *y_packed, const void *W_packed, int32_t rows, int32_t vocab, int32_t d,
                                    float scale, int32_t mask_id, void *scratch, float *row_sum, int32_t *row_arg,
                                    void *stream);
int32_t psd_kernel_head_confidence_bf16(const void *y, const void *W, int32_t rows, int32_t vocab, int32_t d, float scale,
                                        int32_t mask_id, void *scratch, float *row_sum, int32_t *row_arg, void *stream);
/* psd_kernel_head_stream_bf16 for callers that cannot allocate device memory or size a scratch buffer: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs and kernels; the
 * per-slab partial results go to a static device array inside the library (11 796 480 bytes, held by every GPU the
 * library runs on until the process ends) instead of `scratch`.  Limits: rows <= 192, vocab <= 163 840
 * (PSD_ERR_WORKSPACE beyond them; nothing is launched).  Allocates nothing and frees nothing.  All calls on one GPU
 * share that array: calls that overlap on one GPU (different streams or threads) race; calls on one stream do not. */
int32_t psd_kernel_head_stream_static_bf16(const void *y_packed, const void *W_packed, int32_t rows, int32_t vocab,
                                           int32_t d, float scale, int32_t mask_id, float *row_sum, int32_t *row_arg,
                                           void *stream);

/* Calibration kernel: 256 workgroups of 4 wavefronts, each running `iters` rounds of 16 independent
 * v_mfma_f32_32x32x16_bf16 on operand data read from `operands` (device, bf16 values, >= 16 bytes)
 * and rotated between rounds; nothing else.  Returns in *flops the FLOPs of the launch; the
 * caller times it with events on `stream`.  The MFMA clock is power-managed, so the rate on real
 * data (not zeros) is the sustained ceiling for a contraction on this device.  sink: device, 4 MiB. */
int32_t psd_kernel_mfma_rate(const void *operands, int64_t operand_bytes, int32_t iters, void *sink, int64_t sink_bytes,
                             double *flops, void *stream);

/* Kernel timing for roofline accounting.  Between psd_probe_begin and psd_probe_end every
 * launch of the layer-contraction kernel with the given epilogue (0 store, 1 bias,
 * 2 residual, 3 SwiGLU) and workgroup tile configuration (an index below
 * psd_kernel_gemm_tile_count; psd_kernel_gemm_tile_name describes it: tile extent, wavefronts,
 * depths of the two LDS rings) is bracketed by HIP events on the stream it is launched on (up to
 * max_launches; later ones go untimed).  Kind 4 selects the LM-head confidence pass instead
 * (all its kernels, tile ignored), kind 5 every model call (forward + confidence pass) made by
 * psd_decode_block / psd_decode; both can be timed together with one contraction kernel.
 * psd_probe_end waits for those events and returns their summed duration, the number of timed
 * launches and their algorithmic work: FLOPs (2*M*N*K, twice that for SwiGLU) for a contraction,
 * bytes (vocab*d*2 + rows*d*2 + rows*8) for the LM-head pass, 0 for model calls (psd_forward_work gives it).
 * psd_probe_read (after psd_probe_end) copies the first max_n timed launches one by one: ms[i] their duration and
 * (a[i], b[i]) = (rows, output columns) of a contraction, (rows, 0) of an LM-head pass, (sequences, drafts per
 * sequence: 1 for a stage-1 call, K for a verification call) of a model call; returns how many it wrote.
 * psd_kernel_gemm_tile tells which tile the dispatcher picks for a shape. */
int32_t psd_probe_begin(psd_handle *h, int32_t epilogue, int32_t tile, int32_t max_launches);
int32_t psd_probe_end(psd_handle *h, int32_t epilogue, double *total_ms, int64_t *launches, double *work);
int32_t psd_probe_read(psd_handle *h, int32_t epilogue, int32_t max_n, float *ms, int64_t *a, int64_t *b);
int32_t psd_kernel_gemm_tile(int64_t M, int32_t Nout, int32_t epilogue);
/* Number of tile configurations (valid tile ids are 0 .. count-1) and a static description of one. */
int32_t psd_kernel_gemm_tile_count(void);
const char *psd_kernel_gemm_tile_name(int32_t tile);

#ifdef __cplusplus
}
#endif
#endif /* PSD_H */
