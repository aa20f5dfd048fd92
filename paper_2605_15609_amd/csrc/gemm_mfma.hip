// Layer contractions of the forward pass (QKV, O, SwiGLU gate/up, down) on the MFMA kernel
// template of gemm_mfma.h: activations are the row operand, weights [out, in] the column
// operand.
#include "gemm_mfma.h"

namespace {

using namespace mfma;

template <int EPI>
void dispatch(const bf16_t *A, const bf16_t *W, const bf16_t *W2, int M, int Nout, int Kin, const float *bias,
              bf16_t *out, float *resid, int ldo, hipStream_t st) {
    Top1Args none = {};
    if (gemm_bf16_tile(M, Nout, EPI) == 1)
        launch_cfg<256, 256, 2, 2, EPI>(A, W, W2, M, Nout, Kin, bias, out, resid, ldo, none, st);
    else
        launch_cfg<128, 128, 2, 2, EPI>(A, W, W2, M, Nout, Kin, bias, out, resid, ldo, none, st);
}

}   // namespace

int gemm_bf16_tile(int64_t M, int Nout, int epi) {
    // big tiles once they still give every CU work; smaller ones for short M or narrow N
    const int64_t cols = (epi == EPI_SWIGLU) ? 2 * (int64_t)Nout : Nout;
    const int64_t t256 = ((M + 255) / 256) * ((cols + 255) / 256);
    return t256 >= 256 ? 1 : 0;
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
