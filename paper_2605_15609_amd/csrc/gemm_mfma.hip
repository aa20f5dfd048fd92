// Layer contractions of the forward pass (QKV, O, SwiGLU gate/up, down) on the MFMA kernel
// template of gemm_mfma.h: activations are the row operand, weights [out, in] the column
// operand.  The workgroup tile is picked per shape so that the grid fills the 256 CUs: big
// square tiles (least LDS traffic per FLOP) when there are enough of them, smaller ones for
// the short-M stage-1 pass and the narrow O / down projections.
#include "gemm_mfma.h"

namespace {

using namespace mfma;

struct TileCfg {
    int bm, bn;
};
// index = value returned by gemm_bf16_tile
constexpr TileCfg kTiles[] = {{128, 128}, {256, 256}, {256, 128}, {128, 64}, {128, 192}, {128, 64}, {128, 128}, {64, 64}, {256, 256}, {256, 256}};
constexpr int kNumTiles = sizeof(kTiles) / sizeof(kTiles[0]);

template <int EPI>
void dispatch(const bf16_t *A, const bf16_t *W, const bf16_t *W2, int M, int Nout, int Kin, const float *bias,
              bf16_t *out, float *resid, int ldo, hipStream_t st) {
    Top1Args none = {};
    switch (gemm_bf16_tile(M, Nout, EPI)) {
        case 1: launch_cfg<256, 256, 2, 2, EPI>(A, W, W2, M, Nout, Kin, bias, out, resid, ldo, none, st); break;
        case 2: launch_cfg<256, 128, 2, 2, EPI>(A, W, W2, M, Nout, Kin, bias, out, resid, ldo, none, st); break;
        case 3:   // (never chosen for SwiGLU: the gate and up halves need whole subtiles per wave)
            if constexpr (EPI != EPI_SWIGLU) {
                launch_cfg<128, 64, 2, 2, EPI>(A, W, W2, M, Nout, Kin, bias, out, resid, ldo, none, st);
                break;
            }
            [[fallthrough]];
        case 4:
            if constexpr (EPI != EPI_SWIGLU) {
                launch_cfg<128, 192, 2, 2, EPI>(A, W, W2, M, Nout, Kin, bias, out, resid, ldo, none, st);
                break;
            }
            [[fallthrough]];
        case 5:   // deep LDS ring: a lone workgroup per CU needs its fetches several stages ahead
            if constexpr (EPI != EPI_SWIGLU) {
                launch_cfg<128, 64, 2, 2, EPI, 4>(A, W, W2, M, Nout, Kin, bias, out, resid, ldo, none, st);
                break;
            }
            [[fallthrough]];
        case 6: launch_cfg<128, 128, 2, 2, EPI, 4>(A, W, W2, M, Nout, Kin, bias, out, resid, ldo, none, st); break;
        case 7:
            if constexpr (EPI != EPI_SWIGLU) {
                launch_cfg<64, 64, 2, 2, EPI, 4>(A, W, W2, M, Nout, Kin, bias, out, resid, ldo, none, st);
                break;
            }
            [[fallthrough]];
        case 8: launch_cfg<256, 256, 2, 4, EPI>(A, W, W2, M, Nout, Kin, bias, out, resid, ldo, none, st); break;
        case 9: launch_cfg<256, 256, 4, 2, EPI>(A, W, W2, M, Nout, Kin, bias, out, resid, ldo, none, st); break;
        default: launch_cfg<128, 128, 2, 2, EPI>(A, W, W2, M, Nout, Kin, bias, out, resid, ldo, none, st); break;
    }
}

}   // namespace

static int g_force_tile = -1;
void gemm_bf16_force_tile(int tile) { g_force_tile = tile; }

int gemm_bf16_tile(int64_t M, int Nout, int epi) {
    if (g_force_tile >= 0 && g_force_tile < kNumTiles) {
        const bool ok = epi != EPI_SWIGLU || (kTiles[g_force_tile].bn / 2) % 64 == 0;
        if (ok) return g_force_tile;
    }
    // Rules read off a sweep of every tile over the layer shapes of the benchmark configurations
    // (MI355X): the 256x256 tile has the least LDS traffic per FLOP but runs one workgroup per CU, so
    // it only pays with enough rounds of them (or for SwiGLU, whose two weight operands share the
    // activation tile); short-M contractions with a narrow output need the small tile to reach every
    // CU; otherwise 128x128 with two workgroups per CU hides latency best.
    const bool dual = epi == EPI_SWIGLU;
    const int64_t cols = dual ? 2 * (int64_t)Nout : Nout;
    const int64_t t256 = ((M + 255) / 256) * ((cols + 255) / 256);
    // the 256x256 tile runs as 8 wavefronts (two per SIMD, each 64x128): same LDS traffic per FLOP as four
    // 128x128 wavefronts would need fewer fragment reads, but the second wavefront per SIMD hides the
    // latencies that a lone one exposes
    if (dual) return t256 >= 128 ? 9 : 0;
    if (t256 >= 768 || (t256 >= 384 && Nout >= 8192)) return 9;
    const int64_t t128 = ((M + 127) / 128) * ((cols + 127) / 128);
    const int64_t t12864 = ((M + 127) / 128) * ((cols + 63) / 64);
    if (t128 <= 256) {   // at most one 128x128 workgroup per CU: latency-bound, use the deep LDS ring
        if (t12864 <= 128) return 7;
        return t12864 <= 256 ? 5 : 6;
    }
    if (t128 <= 320) return 3;
    if (epi != EPI_RESIDUAL && Nout % 192 == 0 && t128 >= 1024) return 4;
    return 0;
}

void launch_gemm_bf16(const bf16_t *A, const bf16_t *W, const bf16_t *W2, int64_t M, int Nout, int Kin, int epi,
                      const float *bias, bf16_t *out, float *resid, int ldo, hipStream_t st) {
    const int m = (int)M;
    switch (epi) {
        case EPI_STORE: dispatch<EPI_STORE>(A, W, W2, m, Nout, Kin, bias, out, resid, ldo, st); break;
        case EPI_BIAS: dispatch<EPI_BIAS>(A, W, W2, m, Nout, Kin, bias, out, resid, ldo, st); break;
        case EPI_RESIDUAL: dispatch<EPI_RESIDUAL>(A, W, W2, m, Nout, Kin, bias, out, resid, ldo, st); break;
        default: dispatch<EPI_SWIGLU>(A, W, W2, m, Nout, Kin, bias, out, resid, ldo, st); break;
    }
}

// ---------------------------------------------------------------------------------------------
// Calibration: what a loop of nothing but v_mfma_f32_32x32x16_bf16 sustains on this device when
// the operands are real data (16 independent accumulators per wavefront, 4 wavefronts per CU,
// operand registers rotated every iteration).  The MFMA clock is power-managed, so this is well
// below the rate the same loop reaches on all-zero operands; it is the ceiling a contraction
// kernel can be judged against besides the published peak.
namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void mfma_rate_kernel(const u32x4_t *__restrict__ src, int n_src, int iters,
                                                        floatx16 *__restrict__ sink) {
    bf16x8 a[4], b[4];
    for (int i = 0; i < 4; ++i) {
        a[i] = __builtin_bit_cast(bf16x8, src[(threadIdx.x * 8 + i) % n_src]);
        b[i] = __builtin_bit_cast(bf16x8, src[(threadIdx.x * 8 + 4 + i) % n_src]);
    }
    floatx16 acc[4][4];
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 4; ++j)
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        bf16x8 t = a[0];
        a[0] = a[1]; a[1] = a[2]; a[2] = a[3]; a[3] = t;
        t = b[0];
        b[0] = b[1]; b[1] = b[2]; b[2] = b[3]; b[3] = t;
    }
    floatx16 s = acc[0][0];
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 4; ++j)
            if (i || j) s += acc[i][j];
    sink[blockIdx.x * 256 + threadIdx.x] = s;
}

}   // namespace

void launch_mfma_rate(const void *operands, int n_vec16, int iters, void *sink, hipStream_t st) {
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(256), dim3(256), 0, st, (const u32x4_t *)operands, n_vec16, iters,
                       (floatx16 *)sink);
}
