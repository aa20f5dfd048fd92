// LM-head fused with softmax top-1 (Sec. 3.1: x_hat = argmax_v p(v), c = max_v p(v)).
//
// The vocabulary is streamed once: W_lm [V, d] is the ROW operand of the MFMA kernel, the
// hidden rows y [rows, d] the column operand, so a lane holds 16 vocabulary entries of one
// hidden row per 32x32 tile and reduces them in registers.  Every workgroup owns a slab of
// 256 (or 128) vocabulary ids for a tile of hidden rows and emits one (max, argmax, sum-exp)
// triple per row; a second tiny kernel merges the slabs in ascending id order, so ties keep
// the lowest token id and the result does not depend on scheduling.  Full logits never
// reach HBM.  The [M] column is excluded from both the max and the normaliser.
#include <mutex>

#include "gemm_mfma.h"

namespace {

using namespace mfma;

constexpr int SLAB_BIG = 256, SLAB_SMALL = 128;

int slab_rows(int rows) { return rows <= 32 ? SLAB_SMALL : SLAB_BIG; }

// one wavefront per hidden row: merge the per-slab triples; row_sum = sum_v exp(z_v - z_max)
__global__ __launch_bounds__(64) void head_merge_kernel(const float *__restrict__ pmax, const float *__restrict__ psum,
                                                        const int32_t *__restrict__ parg, int slabs, int rows,
                                                        float *__restrict__ row_sum, int32_t *__restrict__ row_arg) {
    const int r = blockIdx.x, lane = threadIdx.x;
    float best = -INFINITY, sum = 0.f;
    int arg = 0x7fffffff;
    for (int sl = lane; sl < slabs; sl += 64) {
        const int64_t o = (int64_t)sl * rows + r;
        top1_merge(best, arg, sum, pmax[o], parg[o], psum[o]);
    }
    for (int off = 32; off > 0; off >>= 1) {
        const float b2 = __shfl_xor(best, off, 64);
        const int a2 = __shfl_xor(arg, off, 64);
        const float s2 = __shfl_xor(sum, off, 64);
        top1_merge(best, arg, sum, b2, a2, s2);
    }
    if (lane == 0) {
        row_sum[r] = sum;
        row_arg[r] = arg;
    }
}


// ---------------------------------------------------------------------------------------------
// Streaming head for few hidden rows (<= 192): the pass is HBM-bound, so it is built as a pure
// stream.  W_lm is kept in a second copy laid out in MFMA-fragment order -- for every block of 32
// vocabulary rows and 16 k, the 64 lanes' 16-byte operands back to back (1 KB) -- so that a
// wavefront that owns TMV*32 vocabulary ids reads its share of the matrix as one linear run of
// fully coalesced 1 KB loads, straight into registers: no LDS, no barriers, no workgroup-level
// coupling.  The hidden rows are packed the same way (a few hundred KB, L2-resident, re-read by
// every wavefront).  A ring of D k-steps of operand registers keeps D KB per operand row-block in
// flight per wavefront.  The epilogue is the same in-register (max, lowest argmax, sum-exp)
// reduction as the tiled kernel; one triple per (row, wavefront slab) goes to the merge kernel.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int TMV, int TNR, int D, int DB = D>
__global__ __launch_bounds__(256) void head_stream_kernel(const bf16_t *__restrict__ Wp, const bf16_t *__restrict__ Yp, int V,
                                                          int rows, int Kin, int n_slabs, Top1Args t1) {
    const int slab = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + (threadIdx.x >> 6));
    if (slab >= n_slabs) return;
    const int lane = threadIdx.x & 63, lrow = lane & 31, lhalf = lane >> 5;
    const int nks = Kin / 16;
    const int64_t frag_row_bytes = (int64_t)nks * 1024;   // one 32-row block over all of K
    // descriptors cover only the row blocks that exist; fetches of a missing block are rejected and read as zero
    const int w_blocks = min(TMV, (V + 31) / 32 - slab * TMV), y_blocks = min(TNR, (rows + 31) / 32);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(Wp) + (int64_t)slab * TMV * nks * 512, 0, (int)(w_blocks * frag_row_bytes), 0x00020000);
    const __amdgpu_buffer_rsrc_t ry =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(Yp), 0, (int)(y_blocks * frag_row_bytes), 0x00020000);
    const int voff = lane * 16;

    floatx16 acc[TMV][TNR];
#pragma unroll
    for (int i = 0; i < TMV; ++i)
#pragma unroll
        for (int j = 0; j < TNR; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // operand rings: D k-steps of weight fragments (HBM latency) and DB <= D of hidden-row fragments (L2 latency)
    static_assert(D % DB == 0, "the hidden-row ring must divide the weight ring");
    u32x4 ra[D][TMV], rb[DB][TNR];
#define PSD_HEAD_FETCH_A(u, ks)                                                                                \
    {                                                                                                         \
        _Pragma("unroll") for (int i = 0; i < TMV; ++i)                                                       \
            ra[u][i] = __builtin_amdgcn_raw_buffer_load_b128(rw, voff, (i * nks + (ks)) * 1024, 0);           \
    }
#define PSD_HEAD_FETCH_B(u, ks)                                                                                \
    {                                                                                                         \
        _Pragma("unroll") for (int j = 0; j < TNR; ++j)                                                       \
            rb[u][j] = __builtin_amdgcn_raw_buffer_load_b128(ry, voff, (j * nks + (ks)) * 1024, 0);           \
    }
#pragma unroll
    for (int u = 0; u < D; ++u) {
        PSD_HEAD_FETCH_A(u, u)
        if (u < DB) PSD_HEAD_FETCH_B(u, u)
    }
    for (int ks0 = 0; ks0 < nks; ks0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
#pragma unroll
            for (int i = 0; i < TMV; ++i)
#pragma unroll
                for (int j = 0; j < TNR; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ra[u][i]),
                                                                        __builtin_bit_cast(bf16x8, rb[u % DB][j]), acc[i][j], 0, 0,
                                                                        0);
            // refill the slots for D / DB k-steps ahead (past the end: the last k-step again, never consumed)
            PSD_HEAD_FETCH_A(u, min(ks0 + u + D, nks - 1))
            PSD_HEAD_FETCH_B(u % DB, min(ks0 + u + DB, nks - 1))
        }
    }
#undef PSD_HEAD_FETCH_A
#undef PSD_HEAD_FETCH_B

#pragma unroll
    for (int j = 0; j < TNR; ++j) {
        float best = -INFINITY;
        int arg = 0x7fffffff;
#pragma unroll
        for (int i = 0; i < TMV; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = (slab * TMV + i) * 32 + 8 * (v >> 2) + 4 * lhalf + (v & 3);
                float z = acc[i][j][v] * t1.scale;
                if (m >= V || m == t1.mask_id) z = -INFINITY;
                acc[i][j][v] = z;
                if (z > best) {
                    best = z;
                    arg = m;
                }
            }
        float sum = 0.f;
        if (best > -INFINITY) {
#pragma unroll
            for (int i = 0; i < TMV; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) sum += __expf(acc[i][j][v] - best);
        }
        const float b2 = __shfl_xor(best, 32, 64);
        const int a2 = __shfl_xor(arg, 32, 64);
        const float s2 = __shfl_xor(sum, 32, 64);
        top1_merge(best, arg, sum, b2, a2, s2);
        const int col = j * 32 + lrow;
        if (lhalf == 0 && col < rows) {
            const int64_t o = (int64_t)slab * t1.cols_total + col;
            t1.pmax[o] = best;
            t1.psum[o] = sum;
            t1.parg[o] = arg;
        }
    }
}

// row-major [R, K] -> fragment order [ceil(R/32)][K/16][64 lanes][8]; rows past R are zero
__global__ __launch_bounds__(256) void pack_rows_kernel(const bf16_t *__restrict__ src, int R, int K, u32x4 *__restrict__ dst,
                                                        int64_t n_vec) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;   // one 16-byte operand per thread
    if (idx >= n_vec) return;
    const int lane = (int)(idx & 63);
    const int64_t frag = idx >> 6;
    const int nks = K / 16;
    const int ks = (int)(frag % nks);
    const int64_t rb = frag / nks;
    const int64_t r = rb * 32 + (lane & 31);
    const int k = ks * 16 + (lane >> 5) * 8;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (r < R) v = *reinterpret_cast<const u32x4 *>(src + r * K + k);
    dst[idx] = v;
}

template <int TMV, int TNR, int D, int DB = D>
void launch_stream(const bf16_t *Wp, const bf16_t *Yp, int V, int rows, int d, Top1Args t1, hipStream_t st) {
    const int n_slabs = (V + 32 * TMV - 1) / (32 * TMV);
    hipLaunchKernelGGL((head_stream_kernel<TMV, TNR, D, DB>), dim3((n_slabs + 3) / 4), dim3(256), 0, st, Wp, Yp, V, rows, d, n_slabs,
                       t1);
}

// one workgroup per hidden row: merge the slab triples and write the block tables (prediction on masked
// positions, sentinel (own token, -1) elsewhere)
__global__ __launch_bounds__(256) void head_merge_finish_kernel(const float *__restrict__ pmax, const float *__restrict__ psum,
                                                                const int32_t *__restrict__ parg, int slabs, int rows,
                                                                HeadFinish fin, int mask_id, int vocab) {
    __shared__ float s_b[4], s_s[4];
    __shared__ int s_a[4];
    const int r = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    float best = -INFINITY, sum = 0.f;
    int arg = 0x7fffffff;
    for (int sl = tid; sl < slabs; sl += 256) {
        const int64_t o = (int64_t)sl * rows + r;
        top1_merge(best, arg, sum, pmax[o], parg[o], psum[o]);
    }
    for (int off = 32; off > 0; off >>= 1) {
        const float b2 = __shfl_xor(best, off, 64);
        const int a2 = __shfl_xor(arg, off, 64);
        const float s2 = __shfl_xor(sum, off, 64);
        top1_merge(best, arg, sum, b2, a2, s2);
    }
    if (lane == 0) {
        s_b[w] = best;
        s_a[w] = arg;
        s_s[w] = sum;
    }
    __syncthreads();
    if (tid == 0) {
        for (int i = 1; i < 4; ++i) top1_merge(best, arg, sum, s_b[i], s_a[i], s_s[i]);
        const int s = r / fin.L, j = r % fin.L;
        const int64_t src = fin.seq_rows ? fin.seq_rows[s] : s;
        const int64_t dst = fin.out_rows ? fin.out_rows[s] : s;
        const int32_t tok = fin.tokens[src * fin.N + fin.block_start.of_row(src) + j];
        const bool masked = tok == mask_id;
        // a row without one finite logit (a model call on invalid input) has no prediction: token 0, confidence 0
        const bool valid = (uint32_t)arg < (uint32_t)vocab && sum >= 1.0f;
        fin.top1[dst * fin.L + j] = masked ? (valid ? arg : 0) : tok;
        fin.conf[dst * fin.L + j] = masked ? (valid ? 1.0f / sum : 0.0f) : -1.0f;
    }
}

}   // namespace

int64_t head_partial_bytes(int rows, int V) {
    const int64_t slabs = (V + 31) / 32;   // finest slab any path uses
    return 3 * align_up(slabs * (int64_t)rows * 4, 256);
}

int64_t packed_rows_bytes(int64_t R, int K) { return (R + 31) / 32 * 32 * (int64_t)K * 2; }

void launch_pack_rows(const bf16_t *src, int64_t R, int K, bf16_t *dst, hipStream_t st) {
    const int64_t n_vec = (R + 31) / 32 * (int64_t)(K / 16) * 64;
    hipLaunchKernelGGL(pack_rows_kernel, dim3((unsigned)((n_vec + 255) / 256)), dim3(256), 0, st, src, (int)R, K, (u32x4 *)dst,
                       n_vec);
}

bool head_stream_supported(int rows, int d) { return rows <= 192 && d % 64 == 0; }

static int stream_partials(const bf16_t *y_packed, const bf16_t *W_packed, int rows, int V, int d, float scale, int mask_id,
                           void *partials, Top1Args &t1, hipStream_t st) {
    const int64_t stride = align_up((int64_t)((V + 31) / 32) * rows * 4, 256);
    t1.scale = scale;
    t1.mask_id = mask_id;
    t1.pmax = (float *)partials;
    t1.psum = (float *)((char *)partials + stride);
    t1.parg = (int32_t *)((char *)partials + 2 * stride);
    t1.cols_total = rows;
    // wavefront shapes: as many vocabulary blocks per wavefront as the accumulators allow, so the hidden
    // rows (re-read from L2 by every wavefront) cost a fraction of the weight stream
    const bool deep = (d / 16) % 8 == 0;
    int slabs;
    if (rows <= 32) {
        slabs = (V + 127) / 128;
        if (deep) launch_stream<4, 1, 8>(W_packed, y_packed, V, rows, d, t1, st);
        else launch_stream<4, 1, 4>(W_packed, y_packed, V, rows, d, t1, st);
    } else if (rows <= 64) {
        slabs = (V + 127) / 128;
        launch_stream<4, 2, 4>(W_packed, y_packed, V, rows, d, t1, st);
    } else if (rows <= 128) {
        slabs = (V + 127) / 128;
        launch_stream<4, 4, 4>(W_packed, y_packed, V, rows, d, t1, st);
    } else {
        slabs = (V + 63) / 64;
        launch_stream<2, 6, 4>(W_packed, y_packed, V, rows, d, t1, st);
    }
    return slabs;
}

void launch_head_stream_bf16(const bf16_t *y_packed, const bf16_t *W_packed, int rows, int V, int d, float scale, int mask_id,
                             void *partials, float *row_sum, int32_t *row_arg, hipStream_t st) {
    Top1Args t1;
    const int slabs = stream_partials(y_packed, W_packed, rows, V, d, scale, mask_id, partials, t1, st);
    hipLaunchKernelGGL(head_merge_kernel, dim3(rows), dim3(64), 0, st, t1.pmax, t1.psum, t1.parg, slabs, rows, row_sum,
                       row_arg);
}

void launch_head_stream_finish_bf16(const bf16_t *y_packed, const bf16_t *W_packed, int rows, int V, int d, float scale,
                                    int mask_id, void *partials, const HeadFinish &fin, hipStream_t st) {
    Top1Args t1;
    const int slabs = stream_partials(y_packed, W_packed, rows, V, d, scale, mask_id, partials, t1, st);
    hipLaunchKernelGGL(head_merge_finish_kernel, dim3(rows), dim3(256), 0, st, t1.pmax, t1.psum, t1.parg, slabs, rows, fin,
                       mask_id, V);
}

void launch_head_confidence_bf16(const bf16_t *y, const bf16_t *W, int rows, int V, int d, float scale, int mask_id,
                                 void *partials, float *row_sum, int32_t *row_arg, hipStream_t st) {
    const int slab = slab_rows(rows);
    const int slabs = (V + slab - 1) / slab;
    const int64_t stride = align_up((int64_t)((V + 31) / 32) * rows * 4, 256);
    Top1Args t1;
    t1.scale = scale;
    t1.mask_id = mask_id;
    t1.pmax = (float *)partials;
    t1.psum = (float *)((char *)partials + stride);
    t1.parg = (int32_t *)((char *)partials + 2 * stride);
    t1.cols_total = rows;
    // row operand = W_lm (M := V), column operand = y (Nout := rows)
    if (rows <= 32)
        launch_cfg<SLAB_SMALL, 32, 4, 1, EPI_TOP1, 2>(W, y, nullptr, V, rows, d, d, d, nullptr, nullptr, nullptr, 0, t1, st);
    else if (rows <= 64)
        launch_cfg<SLAB_BIG, 64, 4, 1, EPI_TOP1, 2>(W, y, nullptr, V, rows, d, d, d, nullptr, nullptr, nullptr, 0, t1, st);
    else
        launch_cfg<SLAB_BIG, 128, 2, 2, EPI_TOP1, 2>(W, y, nullptr, V, rows, d, d, d, nullptr, nullptr, nullptr, 0, t1, st);
    hipLaunchKernelGGL(head_merge_kernel, dim3(rows), dim3(64), 0, st, t1.pmax, t1.psum, t1.parg, slabs, rows, row_sum,
                       row_arg);
}

// ---------------------------------------------------------------------------------------------
// The streaming head for callers that cannot allocate (HIP graph capture, tight serving loops): the per-slab
// (max, sum-exp, argmax) triples go to a file-scope device array instead of a caller-provided scratch buffer.
// Every GPU holds its own copy of the array at its own address; the address is looked up once per device and
// that pointer, never the array's name, is what host code hands to the kernels.
namespace {

constexpr int kStaticMaxRows = 192;         // the streaming kernel's own limit
constexpr int kStaticMaxVocab = 163840;     // 5120 slabs of 32 ids
constexpr size_t kStaticScratchBytes = 3ull * (kStaticMaxVocab / 32) * kStaticMaxRows * 4;   // 11 796 480 bytes

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device (looked up on the first call there)
int32_t static_scratch(void **out) {
    int dev = -1;
    PSD_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) PSD_FAIL(PSD_ERR_DEVICE, "device index %d outside 0..%d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        PSD_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) PSD_FAIL(PSD_ERR_DEVICE, "hipGetSymbolAddress returned a NULL address for the static scratch array");
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return PSD_OK;
}

}   // namespace

extern "C" int32_t psd_kernel_head_stream_static_bf16(const void *y_packed, const void *W_packed, int32_t rows, int32_t vocab,
                                                      int32_t d, float scale, int32_t mask_id, float *row_sum, int32_t *row_arg,
                                                      void *stream) {
    if (!y_packed || !W_packed || !row_sum || !row_arg || rows < 1 || vocab < 2) PSD_FAIL(PSD_ERR_INVALID_ARG, "bad arguments");
    if (!head_stream_supported(rows, d)) PSD_FAIL(PSD_ERR_SHAPE, "streaming head takes at most 192 rows and d a multiple of 64");
    if (rows > kStaticMaxRows || vocab > kStaticMaxVocab)
        PSD_FAIL(PSD_ERR_WORKSPACE, "the static scratch array holds the partial results of at most %d rows x %d vocabulary ids, not %d x %d",
                 kStaticMaxRows, kStaticMaxVocab, rows, vocab);
    void *ptr = nullptr;
    const int32_t rc = static_scratch(&ptr);
    if (rc != PSD_OK) return rc;
    // every (row, slab) triple the merge reads is written by the stream kernel of this same call: nothing to clear
    launch_head_stream_bf16((const bf16_t *)y_packed, (const bf16_t *)W_packed, rows, vocab, d, scale, mask_id, ptr, row_sum,
                            row_arg, (hipStream_t)stream);
    PSD_HIP(hipGetLastError());
    return PSD_OK;
}
