// Decision kernels of the PSD step: transfer policy (Eq. 1), speculative ordering and
// draft assembly (Eq. 2), hierarchical acceptance and state advance (Alg. 1, stage 3);
// EOS early stopping and the truncated token count of the evaluation protocol (App. B.1).
//
// One 64-lane wavefront owns one sequence's block (L <= 64): lane j is block position j.
// Rankings are rank-by-counting with wavefront shuffles -- position j's rank among the
// masked positions is the number of masked positions that come before it in the order
// (confidence descending, lower position first on ties) -- so no sort is needed and ties
// are resolved identically everywhere.  All comparisons are on the fp32 confidences as
// stored, the precision the decisions are defined in.
#include "psd_internal.h"

namespace {

constexpr int WAVE = 64;

// rank of lane j among lanes with live == true by (c desc, lane asc); meaningful for live lanes
__device__ __forceinline__ int rank_by_confidence(bool live, float c) {
    const int lane = threadIdx.x & (WAVE - 1);
    int r = 0;
#pragma unroll 8
    for (int i = 0; i < WAVE; ++i) {
        const float ci = __shfl(c, i, WAVE);
        const int li = __shfl((int)live, i, WAVE);
        r += (li && (ci > c || (ci == c && i < lane))) ? 1 : 0;
    }
    return r;
}

// would the policy commit a live lane of this rank and confidence?
__device__ __forceinline__ bool policy_commits(bool live, int rank, float c, const psd_policy &p) {
    bool ok = live && (c > p.tau || rank < p.k_min);
    if (p.k_max > 0) ok = ok && rank < p.k_max;
    return ok;
}

// ------------------------------------------------------------------ stage 1 commit (Eq. 1)
__global__ __launch_bounds__(WAVE) void select_unmask_kernel(int32_t *__restrict__ tokens, int N, BlockStart bs, int L,
                                                             const int32_t *__restrict__ top1,
                                                             const float *__restrict__ conf, psd_policy policy,
                                                             int32_t mask_id, uint8_t *__restrict__ transfer_mask,
                                                             int32_t *__restrict__ n_selected,
                                                             int32_t *__restrict__ n_left,
                                                             int32_t *__restrict__ devstats,
                                                             const int32_t *__restrict__ only) {
    const int b = blockIdx.x;
    const int j = threadIdx.x;
    if (only && only[b] == 0) return;   // uniform per workgroup: this sequence had no stage-1 call
    const int block_start = bs.of_row(b);
    int32_t *row = tokens + (int64_t)b * N + block_start;
    const bool in = j < L;
    // a sequence that stopped on an EOS token keeps its masks: its predictions are stale, nothing is committed
    const bool stopped = devstats && devstats[(int64_t)b * PSD_DEVSTAT_WORDS + PSD_DEVSTAT_EOS] > 0;
    const bool live = in && !stopped && row[j] == mask_id;
    const float c = in ? conf[(int64_t)b * L + j] : -2.0f;
    const int rank = rank_by_confidence(live, c);
    const bool take = policy_commits(live, rank, c, policy);
    if (take) row[j] = top1[(int64_t)b * L + j];
    if (in && transfer_mask) transfer_mask[(int64_t)b * L + j] = take ? 1 : 0;
    const int n_take = __popcll(__ballot(take));
    const int n_live = __popcll(__ballot(live));
    if (j == 0) {
        if (n_selected) n_selected[b] = n_take;
        if (n_left) n_left[b] = n_live - n_take;
        if (devstats) devstats[(int64_t)b * PSD_DEVSTAT_WORDS + PSD_DEVSTAT_POLICY] += n_take;
    }
}

// ------------------------------------------------------------------ stage 2 drafts (Eq. 2)
// grid (K, B): every (sequence, node) pair recomputes the ranking (64 shuffles) and writes
// its own draft row with coalesced 4-byte stores.
__global__ __launch_bounds__(WAVE) void build_drafts_kernel(const int32_t *__restrict__ tokens, int N, BlockStart bs,
                                                            int L, const int32_t *__restrict__ top1,
                                                            const float *__restrict__ conf, GraphArg g, int32_t mask_id,
                                                            int32_t *__restrict__ sigma, int32_t *__restrict__ m_out,
                                                            int32_t *__restrict__ drafts) {
    const int k = blockIdx.x;
    const int b = blockIdx.y;
    const int j = threadIdx.x;
    const int block_start = bs.of_row(b);
    const int32_t *row = tokens + (int64_t)b * N;
    int32_t *out = drafts + ((int64_t)b * g.K + k) * N;
    const bool in = j < L;
    const int32_t tok = in ? row[block_start + j] : 0;
    const bool live = in && tok == mask_id;
    const float c = in ? conf[(int64_t)b * L + j] : -2.0f;
    const int rank = rank_by_confidence(live, c);
    const int m = __popcll(__ballot(live));
    // copy the sequence, then overwrite the block with the speculated tokens
    for (int i = j; i < N; i += WAVE)
        if (i < block_start || i >= block_start + L) out[i] = row[i];
    if (in) {
        const bool spec = live && rank < m && ((g.rank_set[k] >> rank) & 1ull);
        out[block_start + j] = spec ? top1[(int64_t)b * L + j] : tok;
    }
    if (k == 0) {   // uniform per workgroup
        __shared__ int s_pos[WAVE];
        if (live) s_pos[rank] = j;
        __syncthreads();
        if (in) sigma[(int64_t)b * L + j] = (j < m) ? s_pos[j] : -1;
        if (j == 0) m_out[b] = m;
    }
}

// ------------------------------------------------------------------ stage 3 acceptance + advance
__global__ __launch_bounds__(WAVE) void accept_kernel(int32_t *__restrict__ tokens, const int32_t *__restrict__ drafts,
                                                      int N, BlockStart bs, int L, const int32_t *__restrict__ sigma,
                                                      const int32_t *__restrict__ m_in, GraphArg g, psd_policy policy,
                                                      int32_t mask_id, const int32_t *__restrict__ v_top1,
                                                      const float *__restrict__ v_conf, int32_t *__restrict__ k_star_out,
                                                      uint8_t *__restrict__ accepted_out, int32_t *__restrict__ n_left,
                                                      int32_t *__restrict__ devstats, int32_t *__restrict__ adopt_top1,
                                                      float *__restrict__ adopt_conf) {
    __shared__ int s_rank[WAVE];              // block position -> rank in sigma, or -1
    __shared__ uint64_t s_S[PSD_MAX_NODES];   // S_k as a bit set over block positions
    __shared__ uint64_t s_ok[PSD_MAX_NODES][PSD_MAX_NODES];   // [p][k]: positions where edge test passes
    __shared__ uint64_t s_commit[PSD_MAX_NODES];               // positions pi commits on p's output
    __shared__ int s_order[PSD_MAX_NODES];
    __shared__ int s_acc[PSD_MAX_NODES];

    const int b = blockIdx.x;
    const int j = threadIdx.x;
    const int block_start = bs.of_row(b);
    const int K = g.K;
    const int m = m_in[b];
    const bool in = j < L;
    if (m <= 0) {   // nothing was speculated for this sequence: leave its state alone
        if (j == 0) {
            if (k_star_out) k_star_out[b] = 0;
        }
        if (accepted_out && j < K) accepted_out[(int64_t)b * K + j] = (j == 0) ? 1 : 0;
        return;
    }
    s_rank[j] = -1;
    __syncthreads();
    if (j < m && j < L) {
        const int pos = sigma[(int64_t)b * L + j];
        if (pos >= 0 && pos < L) s_rank[pos] = j;
    }
    __syncthreads();
    const int my_rank = s_rank[j];
    const int32_t *dbase = drafts + (int64_t)b * K * N + block_start;

    // node sets, policy outcome on every node's verifier output, per-edge token agreement
    for (int p = 0; p < K; ++p) {
        const bool spec = my_rank >= 0 && ((g.rank_set[p] >> my_rank) & 1ull);
        const uint64_t Sp = __ballot(spec);
        const int32_t dtok = in ? dbase[(int64_t)p * N + j] : 0;
        const bool live = in && dtok == mask_id;
        const float c = in ? v_conf[((int64_t)b * K + p) * L + j] : -2.0f;
        const int rank = rank_by_confidence(live, c);
        const uint64_t commit = __ballot(policy_commits(live, rank, c, policy));
        if (j == 0) {
            s_S[p] = Sp;
            s_commit[p] = commit;
        }
        const int32_t vt = in ? v_top1[((int64_t)b * K + p) * L + j] : -1;
        for (int k = 0; k < K; ++k) {
            const int32_t ktok = in ? dbase[(int64_t)k * N + j] : -2;
            const uint64_t agree = __ballot(in && vt == ktok);
            if (j == 0) s_ok[p][k] = agree & commit;
        }
    }
    __syncthreads();

    // topological order: |S_k| ascending, ties by node index
    if (j < K) {
        const int mine = __popcll(s_S[j]);
        int pos = 0;
        for (int n = 0; n < K; ++n) {
            const int other = __popcll(s_S[n]);
            pos += (other < mine || (other == mine && n < j)) ? 1 : 0;
        }
        s_order[pos] = j;
        s_acc[j] = (j == 0) ? 1 : 0;
    }
    __syncthreads();

    if (j == 0) {
        for (int t = 0; t < K; ++t) {
            const int k = s_order[t];
            if (k == 0) continue;
            const uint64_t Sk = s_S[k];
            int ok = 0;
            for (int p = 0; p < K && !ok; ++p) {
                if (!s_acc[p]) continue;
                const uint64_t Sp = s_S[p];
                const bool strict_subset = (Sp & ~Sk) == 0 && Sp != Sk;
                if (strict_subset && ((Sk & ~Sp) & ~s_ok[p][k]) == 0) ok = 1;
            }
            s_acc[k] = ok;
        }
        int best = 0, best_n = -1;
        for (int k = 0; k < K; ++k) {
            const int n = __popcll(s_S[k]);
            if (s_acc[k] && n > best_n) {
                best = k;
                best_n = n;
            }
        }
        s_order[0] = best;
    }
    __syncthreads();
    const int k_star = s_order[0];
    if (accepted_out && j < K) accepted_out[(int64_t)b * K + j] = (uint8_t)s_acc[j];

    // advance: x <- draft k*, then pi once more on k*'s verifier output
    const int32_t dtok = in ? dbase[(int64_t)k_star * N + j] : 0;
    const bool live = in && dtok == mask_id;
    const bool take = live && ((s_commit[k_star] >> j) & 1ull);
    if (in) tokens[(int64_t)b * N + block_start + j] = take ? v_top1[((int64_t)b * K + k_star) * L + j] : dtok;
    // single-forward loop: k*'s verifier output becomes the table the next drafts are drawn from
    if (adopt_top1 && in) {
        adopt_top1[(int64_t)b * L + j] = v_top1[((int64_t)b * K + k_star) * L + j];
        adopt_conf[(int64_t)b * L + j] = v_conf[((int64_t)b * K + k_star) * L + j];
    }
    const int n_live = __popcll(__ballot(live));
    const int n_take = __popcll(__ballot(take));
    if (j == 0) {
        const int depth = __popcll(s_S[k_star]);
        if (k_star_out) k_star_out[b] = k_star;
        if (n_left) n_left[b] = n_live - n_take;
        if (devstats) {
            int32_t *ds = devstats + (int64_t)b * PSD_DEVSTAT_WORDS;
            ds[PSD_DEVSTAT_DRAFT] += depth;
            ds[PSD_DEVSTAT_POST] += n_take;
            ds[PSD_DEVSTAT_HIST + depth] += 1;
        }
    }
}

// ------------------------------------------------------------------ EOS early stopping (App. B.1)
// After a state update: a sequence whose block holds the EOS token is finished, whatever is still masked.
// Its mask counts are zeroed, which is what takes it out of the following model calls, and the position is
// flagged in its counters, which is what keeps the stage-1 commit from touching it again.
__global__ __launch_bounds__(WAVE) void eos_stop_kernel(const int32_t *__restrict__ tokens, int N, BlockStart bs, int L,
                                                        int32_t eos_id, int32_t *__restrict__ n_left,
                                                        int32_t *__restrict__ m, int32_t *__restrict__ devstats) {
    const int b = blockIdx.x, j = threadIdx.x;
    const int block_start = bs.of_row(b);
    const bool hit = j < L && tokens[(int64_t)b * N + block_start + j] == eos_id;
    const uint64_t hits = __ballot(hit);
    if (hits != 0ull && j == 0) {
        if (n_left) n_left[b] = 0;
        if (m) m[b] = 0;
        devstats[(int64_t)b * PSD_DEVSTAT_WORDS + PSD_DEVSTAT_EOS] = __ffsll((unsigned long long)hits);
    }
}

// A sequence leaves its block (resolved, stopped on an EOS token, or the call ends): the first EOS position of the
// block (when stopping on EOS is on) and the number of positions resolved since the block was entered at or before
// it -- all resolved positions without an EOS -- are added to the sequence's counters.  The positions masked on
// entry are in the counters as a 64-bit set.  only != NULL: just the sequences b with only[b] != 0.
__global__ __launch_bounds__(WAVE) void finish_counts_kernel(const int32_t *__restrict__ tokens, int N, BlockStart bs, int L,
                                                             int32_t mask_id, int32_t eos_stop, int32_t eos_id,
                                                             int32_t *__restrict__ devstats, const int32_t *__restrict__ only) {
    const int b = blockIdx.x, j = threadIdx.x;
    if (only && only[b] == 0) return;
    const int block_start = bs.of_row(b);
    const int32_t tok = j < L ? tokens[(int64_t)b * N + block_start + j] : mask_id;
    const uint64_t hits = __ballot(eos_stop && j < L && tok == eos_id);
    const uint64_t resolved = __ballot(j < L && tok != mask_id);
    if (j == 0) {
        int32_t *ds = devstats + (int64_t)b * PSD_DEVSTAT_WORDS;
        const int eos = hits ? __ffsll((unsigned long long)hits) - 1 : -1;
        const int limit = eos >= 0 ? eos : L - 1;
        const uint64_t upto = limit >= 63 ? ~0ull : ((1ull << (limit + 1)) - 1ull);
        const uint64_t entry = (uint64_t)(uint32_t)ds[PSD_DEVSTAT_ENTRY] | ((uint64_t)(uint32_t)ds[PSD_DEVSTAT_ENTRY + 1] << 32);
        ds[PSD_DEVSTAT_EOS] = eos + 1;
        ds[PSD_DEVSTAT_COUNTED] += __popcll(entry & resolved & upto);
    }
}

}   // namespace

void launch_eos_stop(const int32_t *tokens, int B, int N, BlockStart block_start, int L, int32_t eos_id, int32_t *n_left, int32_t *m,
                     int32_t *devstats, hipStream_t st) {
    hipLaunchKernelGGL(eos_stop_kernel, dim3(B), dim3(WAVE), 0, st, tokens, N, block_start, L, eos_id, n_left, m, devstats);
}

void launch_finish_counts(const int32_t *tokens, int B, int N, BlockStart block_start, int L, int32_t mask_id, int32_t eos_stop,
                          int32_t eos_id, int32_t *devstats, const int32_t *only, hipStream_t st) {
    hipLaunchKernelGGL(finish_counts_kernel, dim3(B), dim3(WAVE), 0, st, tokens, N, block_start, L, mask_id, eos_stop, eos_id,
                       devstats, only);
}

void launch_select_unmask(int32_t *tokens, int B, int N, BlockStart block_start, int L, const int32_t *top1, const float *conf,
                          psd_policy policy, int32_t mask_id, uint8_t *transfer_mask, int32_t *n_selected,
                          int32_t *n_left, int32_t *devstats, const int32_t *only, hipStream_t st) {
    hipLaunchKernelGGL(select_unmask_kernel, dim3(B), dim3(WAVE), 0, st, tokens, N, block_start, L, top1, conf, policy,
                       mask_id, transfer_mask, n_selected, n_left, devstats, only);
}

void launch_build_drafts(const int32_t *tokens, int B, int N, BlockStart block_start, int L, const int32_t *top1,
                         const float *conf, const GraphArg &g, int32_t mask_id, int32_t *sigma, int32_t *m,
                         int32_t *drafts, hipStream_t st) {
    hipLaunchKernelGGL(build_drafts_kernel, dim3(g.K, B), dim3(WAVE), 0, st, tokens, N, block_start, L, top1, conf, g,
                       mask_id, sigma, m, drafts);
}

void launch_accept(int32_t *tokens, const int32_t *drafts, int B, int N, BlockStart block_start, int L, const int32_t *sigma,
                   const int32_t *m, const GraphArg &g, psd_policy policy, int32_t mask_id, const int32_t *v_top1,
                   const float *v_conf, int32_t *k_star, uint8_t *accepted, int32_t *n_left, int32_t *devstats,
                   int32_t *adopt_top1, float *adopt_conf, hipStream_t st) {
    hipLaunchKernelGGL(accept_kernel, dim3(B), dim3(WAVE), 0, st, tokens, drafts, N, block_start, L, sigma, m, g, policy,
                       mask_id, v_top1, v_conf, k_star, accepted, n_left, devstats, adopt_top1, adopt_conf);
}
