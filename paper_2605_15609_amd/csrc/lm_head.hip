// LM-head fused with softmax top-1 (Sec. 3.1: x_hat = argmax_v p(v), c = max_v p(v)).
//
// The vocabulary is streamed once: W_lm [V, d] is the ROW operand of the MFMA kernel, the
// hidden rows y [rows, d] the column operand, so a lane holds 16 vocabulary entries of one
// hidden row per 32x32 tile and reduces them in registers.  Every workgroup owns a slab of
// 256 (or 128) vocabulary ids for a tile of hidden rows and emits one (max, argmax, sum-exp)
// triple per row; a second tiny kernel merges the slabs in ascending id order, so ties keep
// the lowest token id and the result does not depend on scheduling.  Full logits never
// reach HBM.  The [M] column is excluded from both the max and the normaliser.
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

}   // namespace

int64_t head_partial_bytes(int rows, int V) {
    const int64_t slabs = (V + SLAB_SMALL - 1) / SLAB_SMALL;
    return 3 * align_up(slabs * (int64_t)rows * 4, 256);
}

void launch_head_confidence_bf16(const bf16_t *y, const bf16_t *W, int rows, int V, int d, float scale, int mask_id,
                                 void *partials, float *row_sum, int32_t *row_arg, hipStream_t st) {
    const int slab = slab_rows(rows);
    const int slabs = (V + slab - 1) / slab;
    const int64_t stride = align_up((int64_t)((V + SLAB_SMALL - 1) / SLAB_SMALL) * rows * 4, 256);
    Top1Args t1;
    t1.scale = scale;
    t1.mask_id = mask_id;
    t1.pmax = (float *)partials;
    t1.psum = (float *)((char *)partials + stride);
    t1.parg = (int32_t *)((char *)partials + 2 * stride);
    t1.cols_total = rows;
    // row operand = W_lm (M := V), column operand = y (Nout := rows)
    if (rows <= 32)
        launch_cfg<SLAB_SMALL, 32, 4, 1, EPI_TOP1>(W, y, nullptr, V, rows, d, nullptr, nullptr, nullptr, 0, t1, st);
    else if (rows <= 64)
        launch_cfg<SLAB_BIG, 64, 4, 1, EPI_TOP1>(W, y, nullptr, V, rows, d, nullptr, nullptr, nullptr, 0, t1, st);
    else
        launch_cfg<SLAB_BIG, 128, 2, 2, EPI_TOP1>(W, y, nullptr, V, rows, d, nullptr, nullptr, nullptr, 0, t1, st);
    hipLaunchKernelGGL(head_merge_kernel, dim3(rows), dim3(64), 0, st, t1.pmax, t1.psum, t1.parg, slabs, rows, row_sum,
                       row_arg);
}
