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
constexpr TileCfg kTiles[] = {{128, 128}, {256, 256}, {256, 128}, {128, 64}, {128, 192}, {128, 64}, {128, 128}, {64, 64}};
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
    // it only pays with at least two full rounds of them (or for SwiGLU, whose two weight operands
    // share the activation tile); short-M contractions with a narrow output need the small tile to
    // reach every CU; otherwise 128x128 with two workgroups per CU hides latency best.
    const bool dual = epi == EPI_SWIGLU;
    const int64_t cols = dual ? 2 * (int64_t)Nout : Nout;
    const int64_t t256 = ((M + 255) / 256) * ((cols + 255) / 256);
    if (dual) return t256 >= 128 ? 1 : 0;
    if (t256 >= 512 && epi != EPI_RESIDUAL) return 1;
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
