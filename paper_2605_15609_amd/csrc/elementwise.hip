// Token-wise kernels of the forward pass: embedding gather, RMSNorm, rotary embedding.
// All are HBM-bound streaming kernels: one workgroup per row, 16-byte accesses where the
// layout allows, fp32 arithmetic, the residual stream h kept in fp32.
#include "psd_internal.h"
#include "device_types.h"
#include "rope_device.h"

namespace {

template <typename T>
__global__ __launch_bounds__(256) void embed_kernel(const int32_t *__restrict__ tokens,
                                                    const int32_t *__restrict__ seq_rows, int N, int first, int count,
                                                    const T *__restrict__ emb, int vocab, int d, float *__restrict__ h) {
    const int64_t t = blockIdx.x;   // slot-major row index s*count + i: position first + i of sequence s
    const int s = (int)(t / count), i = (int)(t % count);
    const int64_t src_row = seq_rows ? seq_rows[s] : s;
    const int32_t tok = tokens[src_row * N + first + i];
    // an id outside the embedding table (invalid input, e.g. a prediction taken from a model call that produced
    // non-finite logits) reads nothing: its row of the stream is zero
    const bool known = (uint32_t)tok < (uint32_t)vocab;
    const T *e = emb + (int64_t)(known ? tok : 0) * d;
    float *o = h + t * d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) o[c] = known ? to_float(e[c]) : 0.f;
}

__device__ __forceinline__ float block_sum(float v, float *smem) {
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    if ((threadIdx.x & 63) == 0) smem[w] = v;
    __syncthreads();
    float tot = 0.f;
    for (int i = 0; i < nw; ++i) tot += smem[i];
    __syncthreads();
    return tot;
}

// out[r, :] = h[src(r), :] * rsqrt(mean(h^2) + eps) * gain ; src(r) = r, or the block rows of each sequence.
// Pending K-split partial sums of the contraction that wrote h last are added first, in order, and the row of
// h is brought up to date.
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(float *__restrict__ h, int d, const float *__restrict__ gain,
                                                      float eps, T *__restrict__ out, int N, BlockStart block_start, int L,
                                                      T *__restrict__ packed, PendingSums pend,
                                                      const int32_t *__restrict__ seq_rows) {
    __shared__ float smem[4];
    const int64_t r = blockIdx.x;
    int64_t src = r;
    if (L > 0) src = (r / L) * N + block_start.of_row(seq_rows ? seq_rows[r / L] : r / L) + (r % L);
    float *x = h + src * d;
    float ss = 0.f;
    for (int c = threadIdx.x; c < d; c += blockDim.x) {
        float v = x[c];
        if (pend.n > 0) {
            for (int s = 0; s < pend.n; ++s) v += pend.partial[s * pend.stride + src * d + c];
            x[c] = v;
        }
        ss += v * v;
    }
    ss = block_sum(ss, smem);
    const float inv = 1.0f / sqrtf(ss / (float)d + eps);
    T *o = out + r * d;
    const int nks = d / 16;
    for (int c = threadIdx.x; c < d; c += blockDim.x) {
        const T v = from_float<T>(x[c] * inv * gain[c]);
        o[c] = v;
        // second copy in MFMA-fragment order [row / 32][c / 16][64 lanes][8] for the streaming LM-head
        if (packed) packed[(((r >> 5) * nks + (c >> 4)) * 64 + ((c >> 3) & 1) * 32 + (r & 31)) * 8 + (c & 7)] = v;
    }
}

// the norms of the bf16 path: one workgroup per row, the row (d <= 8192) held in registers between the
// two passes, 32-byte loads and 16-byte stores.  L > 0: output row r is block row r % L of sequence r / L;
// packed: second copy in MFMA-fragment order (a thread's 8 values are one 16-byte operand slot there too)
__global__ __launch_bounds__(256) void rmsnorm_bf16_vec_kernel(float *__restrict__ h, int d, const float *__restrict__ gain,
                                                               float eps, bf16_t *__restrict__ out, PendingSums pend, int N,
                                                               BlockStart block_start, int L, bf16_t *__restrict__ packed,
                                                               const int32_t *__restrict__ seq_rows) {
    __shared__ float smem[4];
    const int64_t r_out = blockIdx.x;
    const int64_t r = L > 0 ? (r_out / L) * N + block_start.of_row(seq_rows ? seq_rows[r_out / L] : r_out / L) + (r_out % L) : r_out;
    float4 *x = reinterpret_cast<float4 *>(h + r * d);
    const float4 *g = reinterpret_cast<const float4 *>(gain);
    constexpr int MAXV = 4;                 // 8 floats per chunk, up to 4 chunks per thread: d <= 8192
    float4 v[MAXV][2];
    float ss = 0.f;
    const int nchunk = d / 8;
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
        const int c = i * 256 + threadIdx.x;
        if (c < nchunk) {
            v[i][0] = x[2 * c];
            v[i][1] = x[2 * c + 1];
            if (pend.n > 0) {
                // all partial sums are fetched before the first is added (one round trip to memory instead of one
                // per part: these launches have a few dozen rows and nothing else to hide the latency); the adds
                // keep the order of the parts
                constexpr int MAXP = 7;     // a contraction is cut into at most 8 parts
                float4 q[MAXP][2];
#pragma unroll
                for (int s = 0; s < MAXP; ++s)
                    if (s < pend.n) {
                        const float4 *qp = reinterpret_cast<const float4 *>(pend.partial + s * pend.stride + r * d);
                        q[s][0] = qp[2 * c];
                        q[s][1] = qp[2 * c + 1];
                    }
#pragma unroll
                for (int s = 0; s < MAXP; ++s)
                    if (s < pend.n) {
                        v[i][0].x += q[s][0].x; v[i][0].y += q[s][0].y; v[i][0].z += q[s][0].z; v[i][0].w += q[s][0].w;
                        v[i][1].x += q[s][1].x; v[i][1].y += q[s][1].y; v[i][1].z += q[s][1].z; v[i][1].w += q[s][1].w;
                    }
                x[2 * c] = v[i][0];
                x[2 * c + 1] = v[i][1];
            }
            ss += v[i][0].x * v[i][0].x + v[i][0].y * v[i][0].y + v[i][0].z * v[i][0].z + v[i][0].w * v[i][0].w;
            ss += v[i][1].x * v[i][1].x + v[i][1].y * v[i][1].y + v[i][1].z * v[i][1].z + v[i][1].w * v[i][1].w;
        }
    }
    ss = block_sum(ss, smem);
    const float inv = 1.0f / sqrtf(ss / (float)d + eps);
    uint4 *o = reinterpret_cast<uint4 *>(out + r_out * d);
    uint4 *op = reinterpret_cast<uint4 *>(packed);
    const int64_t nks = d / 16;
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
        const int c = i * 256 + threadIdx.x;
        if (c < nchunk) {
            const float4 g0 = g[2 * c], g1 = g[2 * c + 1];
            uint4 w;
            w.x = pack_bf16x2(v[i][0].x * inv * g0.x, v[i][0].y * inv * g0.y);
            w.y = pack_bf16x2(v[i][0].z * inv * g0.z, v[i][0].w * inv * g0.w);
            w.z = pack_bf16x2(v[i][1].x * inv * g1.x, v[i][1].y * inv * g1.y);
            w.w = pack_bf16x2(v[i][1].z * inv * g1.z, v[i][1].w * inv * g1.w);
            o[c] = w;
            // fragment order [row / 32][k / 16][64 lanes][8]: lane = (k / 8 % 2) * 32 + row % 32, chunk c = k / 8
            if (packed) op[((r_out >> 5) * nks + (c >> 1)) * 64 + (c & 1) * 32 + (r_out & 31)] = w;
        }
    }
}

// rotate-half rotary embedding in place on the q and k heads of qkv [tokens, (H + 2 Hkv) * dh], row stride ld
template <typename T>
__global__ __launch_bounds__(256) void rope_kernel(T *__restrict__ qkv, int ld, int N, int pos0, int n_heads, int n_kv_heads, int d_head,
                                                   const float *__restrict__ cos_t, const float *__restrict__ sin_t) {
    const int64_t t = blockIdx.x;
    const int pos = pos0 + (int)(t % N);
    const int half = d_head >> 1;
    const int rot_heads = n_heads + n_kv_heads;
    T *row = qkv + t * (int64_t)ld;
    for (int idx = threadIdx.x; idx < rot_heads * half; idx += blockDim.x) {
        const int hd = idx / half, j = idx % half;
        T *p = row + hd * d_head;
        const float c = cos_t[(int64_t)pos * half + j], s = sin_t[(int64_t)pos * half + j];
        const float x1 = to_float(p[j]), x2 = to_float(p[j + half]);
        p[j] = from_float<T>(x1 * c - x2 * s);
        p[j + half] = from_float<T>(x2 * c + x1 * s);
    }
}

// bf16 rotary, one workgroup per token
__global__ __launch_bounds__(256) void rope_bf16_vec_kernel(bf16_t *__restrict__ qkv, int ld, int N, int pos0, int n_heads, int n_kv_heads,
                                                            int d_head, const float *__restrict__ cos_t,
                                                            const float *__restrict__ sin_t) {
    const int64_t t = blockIdx.x;
    rope_bf16_vec_token(qkv + t * (int64_t)ld, pos0 + (int)(t % N), n_heads, n_kv_heads, d_head, cos_t, sin_t);
}

}   // namespace

namespace {
// dst[r, :] = src[(r / L) * N + block_start + r % L, :]: the block rows of every sequence, packed
template <typename T>
__global__ __launch_bounds__(256) void gather_block_rows_kernel(const T *__restrict__ src, T *__restrict__ dst, int width, int N,
                                                                BlockStart block_start, int L,
                                                                const int32_t *__restrict__ seq_rows) {
    const int64_t r = blockIdx.x;
    const T *s = src + ((r / L) * N + block_start.of_row(seq_rows ? seq_rows[r / L] : r / L) + (r % L)) * width;
    T *d = dst + r * width;
    for (int c = threadIdx.x; c < width; c += blockDim.x) d[c] = s[c];
}
}   // namespace

template <typename T>
void launch_gather_block_rows(const T *src, T *dst, int width, const int32_t *seq_rows, int S, int N, BlockStart block_start, int L,
                              hipStream_t st) {
    hipLaunchKernelGGL(gather_block_rows_kernel<T>, dim3((unsigned)(S * L)), dim3(256), 0, st, src, dst, width, N, block_start, L,
                       seq_rows);
}
template void launch_gather_block_rows<float>(const float *, float *, int, const int32_t *, int, int, BlockStart, int, hipStream_t);
template void launch_gather_block_rows<bf16_t>(const bf16_t *, bf16_t *, int, const int32_t *, int, int, BlockStart, int, hipStream_t);

template <typename T>
void launch_embed(const int32_t *tokens, const int32_t *seq_rows, int S, int N, const T *emb, int vocab, int d, float *h,
                  hipStream_t st) {
    hipLaunchKernelGGL(embed_kernel<T>, dim3((unsigned)((int64_t)S * N)), dim3(256), 0, st, tokens, seq_rows, N, 0, N, emb, vocab, d,
                       h);
}
template <typename T>
void launch_embed_block(const int32_t *tokens, const int32_t *seq_rows, int S, int N, int block_start, int L, const T *emb,
                        int vocab, int d, float *h, hipStream_t st) {
    hipLaunchKernelGGL(embed_kernel<T>, dim3((unsigned)((int64_t)S * L)), dim3(256), 0, st, tokens, seq_rows, N, block_start, L,
                       emb, vocab, d, h);
}

namespace {
// one workgroup per stored row (s, j): the rotated keys of row row_first + j of sequence s go to K row len + j of the
// sequence's cache, its values into column vt_key_slot(len + j) of the transposed value rows
template <typename T>
__global__ __launch_bounds__(256) void kv_store_kernel(const T *__restrict__ qkv, int ld_qkv, int rows_per_seq, int row_first,
                                                       int count, int n_heads, int n_kv_heads, int d_head,
                                                       T *__restrict__ k_cache, T *__restrict__ vt_cache, KvPrefix at) {
    const int64_t r = blockIdx.x;
    const int s = (int)(r / count), j = (int)(r % count);
    const int64_t cache = (at.seq_rows ? at.seq_rows[s] : s) / at.seqs_per_cache;
    const int w = n_kv_heads * d_head;
    const T *krow = qkv + ((int64_t)s * rows_per_seq + row_first + j) * ld_qkv + n_heads * d_head, *vrow = krow + w;
    T *kdst = k_cache + cache * at.stride_k + (int64_t)(at.len + j) * at.ld_k;
    T *vdst = vt_cache + cache * at.stride_vt + vt_key_slot(at.len + j);
    for (int c = threadIdx.x; c < w; c += blockDim.x) {
        kdst[c] = krow[c];
        vdst[(int64_t)c * at.ld_vt] = vrow[c];
    }
}
}   // namespace

template <typename T>
void launch_kv_store(const T *qkv, int ld_qkv, int S, int rows_per_seq, int row_first, int count, int n_heads, int n_kv_heads,
                     int d_head, T *k_cache, T *vt_cache, const KvPrefix &at, hipStream_t st) {
    if (count <= 0 || S <= 0) return;
    hipLaunchKernelGGL(kv_store_kernel<T>, dim3((unsigned)(S * count)), dim3(256), 0, st, qkv, ld_qkv, rows_per_seq, row_first,
                       count, n_heads, n_kv_heads, d_head, k_cache, vt_cache, at);
}
template void launch_kv_store<float>(const float *, int, int, int, int, int, int, int, int, float *, float *, const KvPrefix &,
                                     hipStream_t);
template void launch_kv_store<bf16_t>(const bf16_t *, int, int, int, int, int, int, int, int, bf16_t *, bf16_t *, const KvPrefix &,
                                      hipStream_t);
template <typename T>
void launch_rmsnorm(float *h, int64_t rows, int d, const float *gain, float eps, T *out, PendingSums pend, hipStream_t st) {
    hipLaunchKernelGGL(rmsnorm_kernel<T>, dim3((unsigned)rows), dim3(256), 0, st, h, d, gain, eps, out, 0, BlockStart(), 0, (T *)nullptr,
                       pend, (const int32_t *)nullptr);
}
template <>
void launch_rmsnorm<bf16_t>(float *h, int64_t rows, int d, const float *gain, float eps, bf16_t *out, PendingSums pend,
                            hipStream_t st) {
    if (d % 8 == 0 && d <= 8192)
        hipLaunchKernelGGL(rmsnorm_bf16_vec_kernel, dim3((unsigned)rows), dim3(256), 0, st, h, d, gain, eps, out, pend, 0, BlockStart(), 0,
                           (bf16_t *)nullptr, (const int32_t *)nullptr);
    else
        hipLaunchKernelGGL(rmsnorm_kernel<bf16_t>, dim3((unsigned)rows), dim3(256), 0, st, h, d, gain, eps, out, 0, BlockStart(), 0,
                           (bf16_t *)nullptr, pend, (const int32_t *)nullptr);
}
template <typename T>
void launch_rmsnorm_block(float *h, const int32_t *seq_rows, int S, int N, BlockStart block_start, int L, int d, const float *gain,
                          float eps, T *out, T *packed, PendingSums pend, hipStream_t st) {
    hipLaunchKernelGGL(rmsnorm_kernel<T>, dim3((unsigned)(S * L)), dim3(256), 0, st, h, d, gain, eps, out, N, block_start, L,
                       packed, pend, seq_rows);
}
template <>
void launch_rmsnorm_block<bf16_t>(float *h, const int32_t *seq_rows, int S, int N, BlockStart block_start, int L, int d,
                                  const float *gain, float eps, bf16_t *out, bf16_t *packed, PendingSums pend, hipStream_t st) {
    if (d % 16 == 0 && d <= 8192)
        hipLaunchKernelGGL(rmsnorm_bf16_vec_kernel, dim3((unsigned)(S * L)), dim3(256), 0, st, h, d, gain, eps, out, pend, N,
                           block_start, L, packed, seq_rows);
    else
        hipLaunchKernelGGL(rmsnorm_kernel<bf16_t>, dim3((unsigned)(S * L)), dim3(256), 0, st, h, d, gain, eps, out, N, block_start,
                           L, packed, pend, seq_rows);
}

namespace {
__global__ __launch_bounds__(256) void fold_partials_kernel(float *__restrict__ resid, int cols, int ldo,
                                                            const float *__restrict__ partial, int n_partial, int64_t stride) {
    const int64_t r = blockIdx.x;
    for (int c = threadIdx.x; c < cols; c += blockDim.x) {
        float v = resid[r * ldo + c];
        for (int s = 0; s < n_partial; ++s) v += partial[s * stride + r * cols + c];
        resid[r * ldo + c] = v;
    }
}
}   // namespace

void launch_fold_partials(float *resid, int64_t rows, int cols, int ldo, const float *partial, int n_partial, hipStream_t st) {
    if (n_partial > 0)
        hipLaunchKernelGGL(fold_partials_kernel, dim3((unsigned)rows), dim3(256), 0, st, resid, cols, ldo, partial, n_partial,
                           rows * (int64_t)cols);
}
template <typename T>
void launch_rope(T *qkv, int ld, int64_t tokens, int N, int pos0, int n_heads, int n_kv_heads, int d_head, const float *cos_t,
                 const float *sin_t, hipStream_t st) {
    hipLaunchKernelGGL(rope_kernel<T>, dim3((unsigned)tokens), dim3(256), 0, st, qkv, ld, N, pos0, n_heads, n_kv_heads, d_head,
                       cos_t, sin_t);
}
template <>
void launch_rope<bf16_t>(bf16_t *qkv, int ld, int64_t tokens, int N, int pos0, int n_heads, int n_kv_heads, int d_head, const float *cos_t,
                         const float *sin_t, hipStream_t st) {
    if (d_head % 16 == 0)
        hipLaunchKernelGGL(rope_bf16_vec_kernel, dim3((unsigned)tokens), dim3(256), 0, st, qkv, ld, N, pos0, n_heads, n_kv_heads, d_head,
                           cos_t, sin_t);
    else
        hipLaunchKernelGGL(rope_kernel<bf16_t>, dim3((unsigned)tokens), dim3(256), 0, st, qkv, ld, N, pos0, n_heads, n_kv_heads, d_head,
                           cos_t, sin_t);
}

#define INSTANTIATE(T)                                                                                              \
    template void launch_embed<T>(const int32_t *, const int32_t *, int, int, const T *, int, int, float *, hipStream_t); \
    template void launch_rmsnorm<T>(float *, int64_t, int, const float *, float, T *, PendingSums, hipStream_t);    \
    template void launch_rmsnorm_block<T>(float *, const int32_t *, int, int, BlockStart, int, int, const float *, float, T *, T *, \
                                          PendingSums, hipStream_t);                                                \
    template void launch_rope<T>(T *, int, int64_t, int, int, int, int, int, const float *, const float *, hipStream_t);      \
    template void launch_embed_block<T>(const int32_t *, const int32_t *, int, int, int, int, const T *, int, int, float *, \
                                        hipStream_t);
INSTANTIATE(float)
template void launch_embed<bf16_t>(const int32_t *, const int32_t *, int, int, const bf16_t *, int, int, float *, hipStream_t);
template void launch_embed_block<bf16_t>(const int32_t *, const int32_t *, int, int, int, int, const bf16_t *, int, int, float *,
                                         hipStream_t);

