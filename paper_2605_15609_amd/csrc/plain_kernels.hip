// Debug path: plain kernels for any shape and either storage type, fp32 arithmetic, no
// MFMA.  The fp32 model configuration runs entirely on these; for bf16 models they are the
// on-device cross-check of the MFMA kernels (same rounding points, different algorithm).
#include "psd_internal.h"
#include "device_types.h"

namespace {

constexpr int GT = 64;   // block tile (GT x GT outputs), 256 threads, 4x4 outputs per thread
constexpr int GK = 16;

template <typename T, typename TO>
__global__ __launch_bounds__(256) void plain_gemm_kernel(const T *__restrict__ A, const T *__restrict__ W,
                                                         const T *__restrict__ W2, int64_t M, int Nout, int Kin, int lda, int ldw, int epi,
                                                         const float *__restrict__ bias, float scale,
                                                         TO *__restrict__ out, float *__restrict__ resid, int ldo) {
    __shared__ float As[GK][GT + 1];
    __shared__ float Ws[GK][GT + 1];
    __shared__ float W2s[GK][GT + 1];
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    const int64_t m0 = (int64_t)blockIdx.y * GT;
    const int n0 = blockIdx.x * GT;
    float acc[4][4] = {}, acc2[4][4] = {};
    const bool dual = epi == EPI_SWIGLU;
    for (int k0 = 0; k0 < Kin; k0 += GK) {
        for (int e = threadIdx.x; e < GT * GK; e += 256) {
            const int r = e / GK, c = e % GK;
            const int k = k0 + c;
            As[c][r] = (m0 + r < M && k < Kin) ? to_float(A[(m0 + r) * lda + k]) : 0.f;
            Ws[c][r] = (n0 + r < Nout && k < Kin) ? to_float(W[(int64_t)(n0 + r) * ldw + k]) : 0.f;
            if (dual) W2s[c][r] = (n0 + r < Nout && k < Kin) ? to_float(W2[(int64_t)(n0 + r) * ldw + k]) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < GK; ++c) {
            float a[4], w[4], w2[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[i] = As[c][ty * 4 + i];
                w[i] = Ws[c][tx * 4 + i];
                w2[i] = dual ? W2s[c][tx * 4 + i] : 0.f;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
                    acc2[i][j] = fmaf(a[i], w2[j], acc2[i][j]);
                }
        }
        __syncthreads();
    }
    for (int i = 0; i < 4; ++i) {
        const int64_t m = m0 + ty * 4 + i;
        if (m >= M) continue;
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= Nout) continue;
            float v = acc[i][j] * scale;
            if (epi == EPI_BIAS) v += bias[n];
            if (epi == EPI_SWIGLU) v = v / (1.0f + expf(-v)) * acc2[i][j];
            if (epi == EPI_RESIDUAL)
                resid[m * ldo + n] += v;
            else
                out[m * ldo + n] = from_float<TO>(v);
        }
    }
}

// one wavefront per (query, head, sequence); scores of all keys kept in LDS.  Keys = the prefix (KV cache, all
// visible) followed by the sequence's own N rows, among which block_len > 0 hides the blocks after the query's
template <typename T>
__global__ __launch_bounds__(64) void plain_attention_kernel(const T *__restrict__ qkv, int ld, int N, int n_heads,
                                                             int n_kv_heads, int d_head, T *__restrict__ out, KvPrefix pre,
                                                             int block_len) {
    extern __shared__ float smem[];
    float *qs = smem;            // [d_head]
    float *sc = smem + d_head;   // [pre.len + N]
    const int i = blockIdx.x, hd = blockIdx.y, s = blockIdx.z;
    const int lane = threadIdx.x;
    const int row_w = ld;
    const int kvh = hd / (n_heads / n_kv_heads);
    const T *base = qkv + (int64_t)s * N * row_w;
    const T *q = base + (int64_t)i * row_w + hd * d_head;
    const int64_t cache = pre.len ? (pre.seq_rows ? pre.seq_rows[s] : s) / pre.seqs_per_cache : 0;
    const T *kc = (const T *)pre.k + cache * pre.stride_k + kvh * d_head;
    const T *vc = (const T *)pre.vt + cache * pre.stride_vt + (int64_t)kvh * d_head * pre.ld_vt;
    const int n_keys = pre.len + N;
    for (int c = lane; c < d_head; c += 64) qs[c] = to_float(q[c]);
    __syncthreads();
    const float scale = 1.0f / sqrtf((float)d_head);
    float mx = -INFINITY;
    for (int jj = lane; jj < n_keys; jj += 64) {
        const int own = jj - pre.len;
        const T *k = own < 0 ? kc + (int64_t)jj * pre.ld_k : base + (int64_t)own * row_w + (n_heads + kvh) * d_head;
        float dot = 0.f;
        for (int c = 0; c < d_head; ++c) dot = fmaf(qs[c], to_float(k[c]), dot);
        dot *= scale;
        if (own >= 0 && block_len > 0 && own / block_len > i / block_len) dot = -INFINITY;
        sc[jj] = dot;
        mx = fmaxf(mx, dot);
    }
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    float sum = 0.f;
    for (int jj = lane; jj < n_keys; jj += 64) {
        const float e = expf(sc[jj] - mx);
        sc[jj] = e;
        sum += e;
    }
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
    __syncthreads();
    const float inv = 1.0f / sum;
    T *o = out + ((int64_t)s * N + i) * (n_heads * d_head) + hd * d_head;
    for (int c = lane; c < d_head; c += 64) {
        float acc = 0.f;
        for (int jj = 0; jj < pre.len; ++jj) acc = fmaf(sc[jj], to_float(vc[(int64_t)c * pre.ld_vt + vt_key_slot(jj)]), acc);
        for (int jj = 0; jj < N; ++jj) {
            const T *v = base + (int64_t)jj * row_w + (n_heads + n_kv_heads + kvh) * d_head;
            acc = fmaf(sc[pre.len + jj], to_float(v[c]), acc);
        }
        o[c] = from_float<T>(acc * inv);
    }
}

// top-1 over stored logits (debug path): argmax with ties to the lowest id, the mask column
// excluded; row_sum = sum_v exp(z_v - z_max), so that the confidence is 1 / row_sum
__global__ __launch_bounds__(256) void logits_top1_kernel(const float *__restrict__ logits, int V, int mask_id,
                                                          float *__restrict__ row_sum, int32_t *__restrict__ row_arg) {
    __shared__ float s_v[256];
    __shared__ int s_i[256];
    const int r = blockIdx.x;
    const float *z = logits + (int64_t)r * V;
    float best = -INFINITY;
    int arg = 0x7fffffff;
    for (int v = threadIdx.x; v < V; v += 256) {
        if (v == mask_id) continue;
        const float x = z[v];
        if (x > best || (x == best && v < arg)) {
            best = x;
            arg = v;
        }
    }
    s_v[threadIdx.x] = best;
    s_i[threadIdx.x] = arg;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (threadIdx.x < off) {
            const float ov = s_v[threadIdx.x + off];
            const int oi = s_i[threadIdx.x + off];
            if (ov > s_v[threadIdx.x] || (ov == s_v[threadIdx.x] && oi < s_i[threadIdx.x])) {
                s_v[threadIdx.x] = ov;
                s_i[threadIdx.x] = oi;
            }
        }
        __syncthreads();
    }
    best = s_v[0];
    arg = s_i[0];
    __syncthreads();
    float sum = 0.f;
    for (int v = threadIdx.x; v < V; v += 256)
        if (v != mask_id) sum += expf(z[v] - best);
    s_v[threadIdx.x] = sum;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (threadIdx.x < off) s_v[threadIdx.x] += s_v[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        row_sum[r] = s_v[0];
        row_arg[r] = arg;
    }
}

// (top1, conf) from (row_arg, row_sum): masked block positions get the prediction, the
// others the sentinel (own token, -1)
__global__ void head_finish_kernel(const float *__restrict__ row_sum, const int32_t *__restrict__ row_arg,
                                   const int32_t *__restrict__ tokens, const int32_t *__restrict__ seq_rows,
                                   const int32_t *__restrict__ out_rows, int S, int N, BlockStart block_start, int L,
                                   int mask_id, int vocab, int32_t *__restrict__ top1, float *__restrict__ conf) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= S * L) return;
    const int s = idx / L, j = idx % L;
    const int64_t src = seq_rows ? seq_rows[s] : s;
    const int64_t dst = out_rows ? out_rows[s] : s;
    const int32_t tok = tokens[src * N + block_start.of_row(src) + j];
    const bool masked = tok == mask_id;
    // a row without one finite logit (a model call on invalid input) has no prediction: token 0, confidence 0
    const int32_t arg = row_arg[idx];
    const float sum = row_sum[idx];
    const bool valid = (uint32_t)arg < (uint32_t)vocab && sum >= 1.0f;
    top1[dst * L + j] = masked ? (valid ? arg : 0) : tok;
    conf[dst * L + j] = masked ? (valid ? 1.0f / sum : 0.0f) : -1.0f;
}

}   // namespace

template <typename T, typename TO>
void launch_plain_gemm(const T *A, const T *W, const T *W2, int64_t M, int Nout, int Kin, int lda, int ldw, int epi, const float *bias,
                       float scale, TO *out, float *resid, int ldo, hipStream_t st) {
    dim3 grid((Nout + GT - 1) / GT, (unsigned)((M + GT - 1) / GT));
    hipLaunchKernelGGL((plain_gemm_kernel<T, TO>), grid, dim3(256), 0, st, A, W, W2, M, Nout, Kin, lda, ldw, epi, bias, scale, out,
                       resid, ldo);
}

template <typename T>
void launch_plain_attention(const T *qkv, int ld, int S, int N, int n_heads, int n_kv_heads, int d_head, T *out,
                            const KvPrefix &pre, int block_len, hipStream_t st) {
    const size_t smem = (size_t)(d_head + pre.len + N) * sizeof(float);
    hipLaunchKernelGGL(plain_attention_kernel<T>, dim3(N, n_heads, S), dim3(64), smem, st, qkv, ld, N, n_heads, n_kv_heads,
                       d_head, out, pre, block_len);
}

void launch_logits_top1(const float *logits, int rows, int V, int mask_id, float *row_sum, int32_t *row_arg,
                        hipStream_t st) {
    hipLaunchKernelGGL(logits_top1_kernel, dim3(rows), dim3(256), 0, st, logits, V, mask_id, row_sum, row_arg);
}

void launch_head_finish(const float *row_sum, const int32_t *row_arg, const int32_t *tokens, const int32_t *seq_rows,
                        const int32_t *out_rows, int S, int N, BlockStart block_start, int L, int mask_id, int vocab, int32_t *top1,
                        float *conf, hipStream_t st) {
    const int n = S * L;
    hipLaunchKernelGGL(head_finish_kernel, dim3((n + 255) / 256), dim3(256), 0, st, row_sum, row_arg, tokens, seq_rows,
                       out_rows, S, N, block_start, L, mask_id, vocab, top1, conf);
}

template void launch_plain_gemm<float, float>(const float *, const float *, const float *, int64_t, int, int, int, int, int,
                                              const float *, float, float *, float *, int, hipStream_t);
template void launch_plain_gemm<bf16_t, bf16_t>(const bf16_t *, const bf16_t *, const bf16_t *, int64_t, int, int, int, int, int,
                                                const float *, float, bf16_t *, float *, int, hipStream_t);
template void launch_plain_gemm<bf16_t, float>(const bf16_t *, const bf16_t *, const bf16_t *, int64_t, int, int, int, int, int,
                                               const float *, float, float *, float *, int, hipStream_t);
template void launch_plain_attention<float>(const float *, int, int, int, int, int, int, float *, const KvPrefix &, int,
                                            hipStream_t);
template void launch_plain_attention<bf16_t>(const bf16_t *, int, int, int, int, int, int, bf16_t *, const KvPrefix &, int,
                                             hipStream_t);
