// Layer contractions of the forward pass (QKV, O, SwiGLU gate/up, down) on the MFMA kernel
// template of gemm_mfma.h: activations are the row operand, weights [out, in] the column
// operand.  The workgroup tile is picked per shape so that the grid fills the 256 CUs: big
// tiles (least LDS traffic per FLOP) when whole rounds of them come out, smaller ones for
// the short-M stage-1 pass and the narrow O / down projections.
#include "gemm_mfma.h"

namespace {

using namespace mfma;

// Main-loop schedule of the 8- and 4-wavefront tiles (bits as in gemm_bf16_kernel)
#ifndef PSD_SCHED_8W
#define PSD_SCHED_8W (2 | 4 | 8)
#endif
#ifndef PSD_SCHED_4W
#define PSD_SCHED_4W 8
#endif
constexpr int S8 = PSD_SCHED_8W, S4 = PSD_SCHED_4W;

struct TileCfg {
    int bm, bn;
    const char *name;
};
// index = value returned by gemm_bf16_tile
constexpr TileCfg kTiles[] = {
    // (tiles 0 and 1 run in the 32x32x16 or the 16x16x32 MFMA form, whichever was measured faster for the epilogue; 8 and 9
    // force the 16x16x32 form)
    {128, 128, "128x128, 4 wavefronts, LDS rings 2/3"},   // two workgroups per CU
    {256, 256, "256x256, 8 wavefronts, LDS rings 2/3"},   // least LDS traffic per FLOP; fills the 160 KB
    {256, 192, "256x192, 8 wavefronts, LDS rings 2/4"},
    {128, 192, "128x192, 4 wavefronts, LDS rings 2/2"},   // two workgroups per CU
    {128, 64, "128x64, 4 wavefronts, LDS rings 4/4"},     // lone workgroup per CU: fetches several stages ahead
    {128, 128, "128x128, 4 wavefronts, LDS rings 4/4"},
    {64, 64, "64x64, 4 wavefronts, LDS rings 4/4"},
    {256, 128, "256x128, 8 wavefronts, LDS rings 2/4"},   // one full round of 256 workgroups for 2048 x 4096 outputs
    {256, 256, "256x256, 8 wavefronts, 16x16x32 MFMAs, LDS rings 2/3"},
    {128, 128, "128x128, 4 wavefronts, 16x16x32 MFMAs, LDS rings 2/3"},
};
constexpr int kNumTiles = sizeof(kTiles) / sizeof(kTiles[0]);

template <int EPI>
void dispatch(const bf16_t *A, const bf16_t *W, const bf16_t *W2, int M, int Nout, int Kin, int lda, int ldw, const float *bias,
              bf16_t *out, float *resid, int ldo, hipStream_t st) {
    Top1Args none = {};
    const int tile = gemm_bf16_tile(M, Nout, EPI, Kin);
    // SwiGLU needs an even number of 32-column subtiles per wavefront (gate and up halves); gemm_bf16_tile
    // never returns the others for it
    if constexpr (EPI != EPI_SWIGLU) {
        switch (tile) {
            case 2: return launch_cfg<256, 192, 4, 2, EPI, 2, 4, S8>(A, W, W2, M, Nout, Kin, lda, ldw, bias, out, resid, ldo, none, st);
            case 3: return launch_cfg<128, 192, 2, 2, EPI, 2, 2, S4>(A, W, W2, M, Nout, Kin, lda, ldw, bias, out, resid, ldo, none, st);
            case 4: return launch_cfg<128, 64, 2, 2, EPI, 4, 4, S4>(A, W, W2, M, Nout, Kin, lda, ldw, bias, out, resid, ldo, none, st);
            case 6: return launch_cfg<64, 64, 2, 2, EPI, 4, 4, S4>(A, W, W2, M, Nout, Kin, lda, ldw, bias, out, resid, ldo, none, st);
            case 7: return launch_cfg<256, 128, 4, 2, EPI, 2, 4, S8>(A, W, W2, M, Nout, Kin, lda, ldw, bias, out, resid, ldo, none, st);
            default: break;
        }
    }
    switch (tile) {
        case 1:
            // the 16x16x32 MFMA form of the same tile is 3 - 9 % faster on the store epilogues and on residual
            // contractions with short K (measured at 2048 - 163 840 rows), level to 5 % faster on SwiGLU (512 rows), 4 - 7 %
            // slower on residual contractions at K = 12288
            if (EPI != EPI_RESIDUAL || Kin <= 4096)
                return launch_cfg<256, 256, 4, 2, EPI, 2, 3, S8, 16>(A, W, W2, M, Nout, Kin, lda, ldw, bias, out, resid, ldo, none, st);
            return launch_cfg<256, 256, 4, 2, EPI, 2, 3, S8>(A, W, W2, M, Nout, Kin, lda, ldw, bias, out, resid, ldo, none, st);
        case 5: return launch_cfg<128, 128, 2, 2, EPI, 4, 4, S4>(A, W, W2, M, Nout, Kin, lda, ldw, bias, out, resid, ldo, none, st);
        case 8: return launch_cfg<256, 256, 4, 2, EPI, 2, 3, S8, 16>(A, W, W2, M, Nout, Kin, lda, ldw, bias, out, resid, ldo, none, st);
        case 9: return launch_cfg<128, 128, 2, 2, EPI, 2, 3, S4, 16>(A, W, W2, M, Nout, Kin, lda, ldw, bias, out, resid, ldo, none, st);
        default:
            // (128x128 in the 16x16x32 form: SwiGLU 1.07 -> 1.29 PFLOP/s at 163 840 rows, the stores + 3 %, residual
            // contractions 81 -> 73 us at K = 4096 and level at K = 12288)
            if (EPI != EPI_RESIDUAL || Kin <= 4096)
                return launch_cfg<128, 128, 2, 2, EPI, 2, 3, S4, 16>(A, W, W2, M, Nout, Kin, lda, ldw, bias, out, resid, ldo, none, st);
            return launch_cfg<128, 128, 2, 2, EPI, 2, 3, S4>(A, W, W2, M, Nout, Kin, lda, ldw, bias, out, resid, ldo, none, st);
    }
}

bool tile_fits(int tile, int epi) { return epi != EPI_SWIGLU || tile == 0 || tile == 1 || tile == 5 || tile == 8 || tile == 9; }

}   // namespace

static int g_force_tile = -1, g_force_splits = 0, g_group_m = 4;
// tile < 0: automatic.  Otherwise bits 0-7 the tile, bits 8-15 the K-split of the residual hook, bits 16-23 the band
// height of the tile order (0 = leave it)
void gemm_bf16_force_tile(int tile) {
    g_force_tile = tile < 0 ? -1 : (tile & 0xff) == 0xff ? -1 : (tile & 0xff);
    g_force_splits = tile < 0 ? 0 : ((tile >> 8) & 0xff);
    if (tile < 0) g_group_m = 4;
    else if ((tile >> 16) & 0xff) g_group_m = (tile >> 16) & 0xff;
}
int gemm_tile_group_m() { return g_group_m; }
int gemm_bf16_tile_count() { return kNumTiles; }
const char *gemm_bf16_tile_name(int tile) { return tile >= 0 && tile < kNumTiles ? kTiles[tile].name : "?"; }

int gemm_bf16_tile(int64_t M, int Nout, int epi, int Kin) {
    if (g_force_tile >= 0 && g_force_tile < kNumTiles && tile_fits(g_force_tile, epi)) return g_force_tile;
    const bool dual = epi == EPI_SWIGLU;
    const int64_t cols = dual ? 2 * (int64_t)Nout : Nout;
    auto tiles = [&](int bm, int bn) { return ((M + bm - 1) / bm) * ((cols + bn - 1) / bn); };
    // SwiGLU reads two weight operands against one activation tile: the big tile as soon as it
    // reaches half of the CUs
    // (a single row tile is a pure weight stream: the deep equal rings keep more of it in flight)
    if (dual) return tiles(256, 256) >= 128 ? 1 : (M <= 128 ? 5 : 0);
    // At most one 128x128 workgroup per CU: the contraction is bound by fetch latency, not by the
    // matrix cores; small tiles reach every CU and the deep rings keep several stages in flight.
    if (tiles(128, 128) <= 256) {
        const int64_t t = tiles(128, 64);
        return t <= 128 ? 6 : t <= 256 ? 4 : 5;
    }
    // Otherwise: rounds of workgroups over the 256 CUs times the work of one round, weighted by the
    // rate each tile sustains on a full machine (PFLOP/s with weights streamed cold from HBM, from a
    // sweep over the layer shapes of the benchmark configurations).  A tile that runs two workgroups per
    // CU does a round of 512 in the time of two.
    struct Cand {
        int tile, per_round;
        double rate;
    };
    // Residual contractions (fp32 read-modify-write epilogue), measured at 2048 x 4096 and 6144 x 3584 outputs: 256x192 beats
    // 128x192 by 2 - 8 %; with a long K (12288: 215 against 235 us) one full round of 256x128 tiles beats two 128x128
    // workgroups per CU, with K = 4096 it does not (the 128x128 tile in its 16x16x32 form: 73 against 77 us).  Kin = 0:
    // unknown, taken as long.  Store epilogues: per round of workgroups the 256x128 tile is 5 - 15 % ahead of 128x128 (512 x 12288
    // outputs: 57 against 69 us) and behind 256x192.
    const bool resid = epi == EPI_RESIDUAL;
    const Cand cand[] = {{1, 256, 1.25}, {2, 256, 1.16}, {3, 512, resid ? 1.12 : 1.15}, {0, 512, 1.00},
                         {7, 256, !resid ? 1.03 : (Kin == 0 || Kin > 4096) ? 1.08 : 0.90}};
    int best = 0;
    double best_cost = 0;
    for (const Cand &c : cand) {
        const int64_t n = tiles(kTiles[c.tile].bm, kTiles[c.tile].bn);
        const int64_t rounds = (n + c.per_round - 1) / c.per_round;
        const double cost = (double)rounds * (c.per_round / 256) * kTiles[c.tile].bm * kTiles[c.tile].bn / c.rate;
        if (best_cost == 0 || cost < best_cost) {
            best_cost = cost;
            best = c.tile;
        }
    }
    return best;
}

// A residual contraction over at most 128 rows is a weight stream with one row tile and few column tiles: far too
// few workgroups to keep HBM busy.  It is cut along K instead, one 128x128 workgroup (rings 4/4) per (column tile,
// K part), up to 256 workgroups; every part keeps at least 8 K stages.  Part 0 adds into resid, the others store
// partial sums that the next reader of resid adds in order (at most 7 * 128 rows: cheap at this size; for taller
// contractions the extra pass costs more than the split gains, measured).
int gemm_bf16_splits(int64_t M, int Nout, int Kin) {
    int splits = 1;
    if (g_force_splits > 0) {
        splits = g_force_splits;
    } else if (g_force_tile < 0 && M <= 128) {
        const int64_t tiles = (Nout + 127) / 128;
        for (int s = 8; s >= 2; s >>= 1)
            if (tiles * s <= 256 && Kin / s >= 8 * BK && Kin % (s * BK) == 0) {
                splits = s;
                break;
            }
    }
    if (splits > 8 || splits < 1 || Kin % (splits * BK) != 0) splits = 1;
    return splits;
}

void launch_gemm_bf16_split(const bf16_t *A, const bf16_t *W, int64_t M, int Nout, int Kin, int lda, int ldw, float *resid, int ldo,
                            float *partial, int splits, hipStream_t st) {
    Top1Args none = {};
    launch_cfg<128, 128, 2, 2, EPI_RESIDUAL, 4, 4, S4>(A, W, nullptr, (int)M, Nout, Kin, lda, ldw, nullptr, nullptr, resid, ldo, none, st,
                                                     splits, partial);
}

// QKV projection with rotary and the V transpose in its epilogue (EPI_QKV).  The tile is the one the plain store
// would get, provided every tile then holds whole heads of one kind: the tile width a multiple of d_head and the first
// V column a multiple of the tile width.  -1: no such tile, run the store epilogue and the separate kernel instead.
int gemm_bf16_qkv_tile(int64_t M, int Nout, int d_head, int v_start, int rows_per_seq) {
    if ((d_head != 64 && d_head != 128) || rows_per_seq % 16 != 0 || Nout % 8 != 0) return -1;
    int tile = gemm_bf16_tile(M, Nout, EPI_STORE);
    // the 192-column tiles cut heads in two: the 256x256 tile takes over where the plain store would have picked one of
    // them (2048 x 6144 outputs: 87 us + 24 us for the separate rotary / transpose kernel against 95 us in one)
    if (tile == 2 || tile == 3) tile = 1;
    const int bn = kTiles[tile].bn;
    if (bn % d_head != 0 || v_start % bn != 0) return -1;
    return tile;
}

void launch_gemm_bf16_qkv(const bf16_t *A, const bf16_t *W, int64_t M, int Nout, int Kin, int lda, int ldw, const float *bias, bf16_t *qkv,
                          int ld_qkv, int d_head, int v_start, int rows_per_seq, int pos0, const float *cos_t, const float *sin_t,
                          bf16_t *vT, int ld_vt, int tile, hipStream_t st) {
    Top1Args none = {};
    QkvArgs qa;
    qa.d_head = d_head;
    qa.v_start = v_start;
    qa.N = rows_per_seq;
    qa.pos0 = pos0;
    qa.cos_t = cos_t;
    qa.sin_t = sin_t;
    qa.vT = vT;
    qa.ld_vt = ld_vt;
    const int m = (int)M;
    switch (tile) {
        case 1:   // (the 16x16x32 MFMA form: see dispatch)
        case 8: return launch_cfg<256, 256, 4, 2, EPI_QKV, 2, 3, S8, 16>(A, W, nullptr, m, Nout, Kin, lda, ldw, bias, qkv, nullptr, ld_qkv, none, st, 1, nullptr, qa);
        case 4: return launch_cfg<128, 64, 2, 2, EPI_QKV, 4, 4, S4>(A, W, nullptr, m, Nout, Kin, lda, ldw, bias, qkv, nullptr, ld_qkv, none, st, 1, nullptr, qa);
        case 5: return launch_cfg<128, 128, 2, 2, EPI_QKV, 4, 4, S4>(A, W, nullptr, m, Nout, Kin, lda, ldw, bias, qkv, nullptr, ld_qkv, none, st, 1, nullptr, qa);
        case 6: return launch_cfg<64, 64, 2, 2, EPI_QKV, 4, 4, S4>(A, W, nullptr, m, Nout, Kin, lda, ldw, bias, qkv, nullptr, ld_qkv, none, st, 1, nullptr, qa);
        case 7: return launch_cfg<256, 128, 4, 2, EPI_QKV, 2, 4, S8>(A, W, nullptr, m, Nout, Kin, lda, ldw, bias, qkv, nullptr, ld_qkv, none, st, 1, nullptr, qa);
        case 9:
        default: return launch_cfg<128, 128, 2, 2, EPI_QKV, 2, 3, S4, 16>(A, W, nullptr, m, Nout, Kin, lda, ldw, bias, qkv, nullptr, ld_qkv, none, st, 1, nullptr, qa);
    }
}

void launch_gemm_bf16(const bf16_t *A, const bf16_t *W, const bf16_t *W2, int64_t M, int Nout, int Kin, int lda, int ldw, int epi,
                      const float *bias, bf16_t *out, float *resid, int ldo, hipStream_t st) {
    const int m = (int)M;
    switch (epi) {
        case EPI_STORE: dispatch<EPI_STORE>(A, W, W2, m, Nout, Kin, lda, ldw, bias, out, resid, ldo, st); break;
        case EPI_BIAS: dispatch<EPI_BIAS>(A, W, W2, m, Nout, Kin, lda, ldw, bias, out, resid, ldo, st); break;
        case EPI_RESIDUAL: dispatch<EPI_RESIDUAL>(A, W, W2, m, Nout, Kin, lda, ldw, bias, out, resid, ldo, st); break;
        default: dispatch<EPI_SWIGLU>(A, W, W2, m, Nout, Kin, lda, ldw, bias, out, resid, ldo, st); break;
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
