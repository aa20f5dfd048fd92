// bf16 contraction D[i, j] = sum_k X[i, k] * Y[j, k] on the gfx950 matrix cores
// (v_mfma_f32_32x32x16_bf16, fp32 accumulation).  Both operands are K-contiguous ("NT"
// form, row strides ldx / ldy elements), the natural MFMA feed: every lane fetches 8 consecutive k
// (16 bytes) of one row.
//
// Tiling: a workgroup of 4 or 8 wavefronts owns a BM x BN tile; K advances 64 at a time.  Each
// operand tile has its own ring of LDS stages (NSA for X, NSB for Y) filled by direct global -> LDS
// loads, one barrier per stage.  The rings differ in depth because the operands differ in where
// they come from: activations were just written and sit in cache, weights arrive cold from HBM and
// need their fetches several stages ahead.
// LDS rows are 128 bytes; the 16-byte chunk c of row r sits at chunk slot c ^ ((r >> 1) & 7),
// so the 32 rows a wavefront touches per fragment fetch spread over all 64 banks.  Workgroup ids are remapped so
// that each of the 8 XCDs (which receive consecutive ids round-robin) works on a compact
// range of tiles and its private L2 sees the operand reuse.
//
// After the K loop a lane holds, for every 32x32 subtile, column j = lane % 32 and the 16
// rows i = 8*(v/4) + 4*(lane/32) + v%4.  The epilogue is a template policy:
//   EPI_STORE / EPI_BIAS   out = bf16(acc (+ bias[j]))                     QKV projection
//   EPI_RESIDUAL           resid[i, j] += acc           (fp32 stream)       O and down projections
//                          With k_splits > 1 the K range is cut into equal parts, one workgroup per (tile,
//                          part): part 0 adds into resid, part s > 0 stores its sum to partial[s - 1] (same
//                          shape, dense rows), and whoever reads the stream next adds the partials in order.
//   EPI_SWIGLU             out = bf16(silu(X Yg^T) * (X Yu^T))              gate and up in one pass
//   EPI_TOP1               per column j: running (max, argmax, sum-exp) over the rows i
//                          (LM-head with X = W_lm, Y = hidden rows; logits never stored)
//   EPI_QKV                QKV projection with what used to be a second pass over its output folded in: the tile
//                          (+ bias) is rounded to bf16 into LDS (the operand rings are free by then); a tile of q / k
//                          heads is read back row-wise, rotated (rotary position of row m: pos0 + m % N) and stored
//                          with 16-byte accesses; a tile of V heads is read back column-wise and stored transposed,
//                          key-contiguous, in the slot order the attention kernel's second MFMA wants.  Same values
//                          as EPI_STORE / EPI_BIAS followed by the separate rotary / transpose kernel, bit for bit.
#pragma once
#include "psd_internal.h"
#include "device_types.h"
#include "rope_device.h"

// With two wavefronts per SIMD in one workgroup (the 8-wavefront tiles) the one inside an MFMA cluster gets issue
// priority over its sibling's loads and address arithmetic (measured: SwiGLU 362 -> 352 us at 2048 tokens; the
// 4-wavefront tiles, whose SIMD siblings belong to another workgroup, lose 4 % with it).
#ifndef PSD_NO_SETPRIO
#define PSD_PRIO_HI if constexpr (NW == 8 && !NOPRIO) __builtin_amdgcn_s_setprio(1);
#define PSD_PRIO_LO if constexpr (NW == 8 && !NOPRIO) __builtin_amdgcn_s_setprio(0);
#else
#define PSD_PRIO_HI
#define PSD_PRIO_LO
#endif
// row tiles per band of the tile order (see the kernel); 4 unless a tuning run changes it (measured over the layer
// contractions of the 8B shapes at 2048 - 163 840 rows: bands of 4 and 8 within 1 %, 1 and 16 about 5 % slower)
int gemm_tile_group_m();

namespace mfma {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int EPI_TOP1 = 4;
constexpr int EPI_QKV = 5;
constexpr int BK = 64;                  // k extent per stage (bf16) = 128 bytes per LDS row

struct Top1Args {
    float scale;        // logits = scale * acc
    int mask_id;        // row (vocab id) that is never predicted
    float *pmax;        // [slabs, cols] partial maxima
    float *psum;        // [slabs, cols] partial sum exp(z - pmax)
    int32_t *parg;      // [slabs, cols] partial argmax (lowest id on ties)
    int cols_total;
};

struct QkvArgs {
    int d_head;           // 64 or 128; every tile holds whole heads (BN % d_head == 0)
    int v_start;          // columns [0, v_start) are q and k heads, [v_start, Nout) V heads; a multiple of BN
    int N, pos0;          // rows per sequence (a multiple of 16) and the rotary position of a sequence's first row
    const float *cos_t, *sin_t;   // [positions, d_head / 2]
    bf16_t *vT;           // [sequences][Nout - v_start][ld_vt]
    int ld_vt;
};

// Swizzle key of an LDS row: 64 banks x 4 bytes = 256 bytes per bank line, rows are 128 bytes, so rows r and r+1 cover
// the two halves of a bank line and the chunk slot is rotated by (r >> 1) over the 8 slots of a row: 16 consecutive rows
// fetching the same logical 16-byte chunk hit 16 distinct bank groups.
__device__ __forceinline__ int row_key(int row) { return (row >> 1) & 7; }

// merge two (max, argmax, sum-exp) triples; ties go to the lower index
__device__ __forceinline__ void top1_merge(float &b, int &a, float &s, float b2, int a2, float s2) {
    const float bn = fmaxf(b, b2);
    const float s_new = (bn == -INFINITY) ? 0.f : s * __expf(b - bn) + s2 * __expf(b2 - bn);
    if (b2 > b || (b2 == b && a2 < a)) a = a2;
    b = bn;
    s = s_new;
}

template <int MI, typename Acc>
__device__ __forceinline__ Acc mfma_step(bf16x8 a, bf16x8 b, Acc c) {
    if constexpr (MI == 32) return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// Scheduling hint for one k-step: spread NR LDS reads (front-loaded over the first half, so they land
// before the next k-step needs them), NW LDS writes and NV global loads evenly between NM MFMAs.
template <int I, int NM, int NR, int NW, int NV>
__device__ __forceinline__ void sched_mix() {
    if constexpr (I < NM) {
        // LDS writes cannot be reordered before LDS reads that precede them in program order, so the
        // reads take the first half of the k-step and the writes (with the global loads that refill
        // their registers) the second half
        constexpr int half = (NM + 1) / 2, rest = NM - half;
        constexpr int r = (I < half) ? ((I + 1) * NR / half - I * NR / half) : 0;
        constexpr int J = I - half;
        constexpr int w = (I >= half) ? ((J + 1) * NW / rest - J * NW / rest) : 0;
        constexpr int v = (I >= half) ? ((J + 1) * NV / rest - J * NV / rest) : 0;
        if constexpr (r > 0) __builtin_amdgcn_sched_group_barrier(0x100, r, 0);
        if constexpr (w > 0) __builtin_amdgcn_sched_group_barrier(0x200, w, 0);
        if constexpr (v > 0) __builtin_amdgcn_sched_group_barrier(0x020, v, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        sched_mix<I + 1, NM, NR, NW, NV>();
    }
}

template <int BM, int BN, int WGM, int WGN, int EPI, int NSA, int NSB, int SCHED = 0, int MI = 32>
__global__ __launch_bounds__(WGM * WGN * 64) void gemm_bf16_kernel(const bf16_t *__restrict__ X, const bf16_t *__restrict__ Y,
                                                        const bf16_t *__restrict__ Y2, int M, int Nout, int Kin, int ldx, int ldy,
                                                        const float *__restrict__ bias, bf16_t *__restrict__ out,
                                                        float *__restrict__ resid, int ldo, int tiles_n, int n_tiles,
                                                        Top1Args t1, int k_splits, float *__restrict__ partial, int group_m,
                                                        QkvArgs qa) {
    extern __shared__ __align__(16) unsigned char lds[];
    // Schedule of the main loop.  Bit 1: only the lower half of the wavefronts issues fetches, for itself and for
    // wavefront w + NW/2 (its sibling on the same SIMD when there are 8): a fetch instruction holds its wavefront up for
    // some 20 cycles, and two siblings that both fetch right after the stage barrier leave the matrix core idle.
    // Bit 2: no issue priority around the MFMA groups (the compiler then interleaves them with the LDS reads and the
    // fetches as the scheduling hints ask).  Bit 3: the fetches of a stage spread over its first three k-steps instead
    // of all in the first.  Measured over the layer shapes of the benchmark configurations: 2 | 4 | 8 on the
    // 8-wavefront tiles and 8 on the 4-wavefront tiles take 2 - 8 % off (bit 1 costs the small 4-wavefront tiles 2 - 8 %).
    constexpr bool ASYM = (SCHED & 2) != 0, NOPRIO = (SCHED & 4) != 0, SPREAD = (SCHED & 8) != 0;
    static_assert((SCHED & 1) == 0, "schedule bits");
    constexpr int ROW_BYTES = BK * 2;                     // an LDS row: one tile row of one stage
    constexpr int LPR = ROW_BYTES / 16, RPI = 64 / LPR;   // lanes per LDS row (8) and rows per DMA instruction (8: 1 KB)
    constexpr bool DUAL = EPI == EPI_SWIGLU;
    constexpr int BN_OUT = DUAL ? BN / 2 : BN;            // output columns per tile
    constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BN * ROW_BYTES, B_RING = NSA * A_BYTES;   // X ring first, then the Y ring
    // MFMA instruction: MI = 32 is v_mfma_f32_32x32x16_bf16, MI = 16 is v_mfma_f32_16x16x32_bf16.  Same flops per cycle;
    // under the chip's power limit the 16x16x32 form sustains 8 - 15 % more on random operands (a loop of nothing but
    // MFMAs: 1.62 against 1.41 PFLOP/s with 4 wavefronts per CU, 1.81 against 1.67 with 8).  An operand fragment is
    // MI rows x (16 or 32) k with every lane holding 8 consecutive k of row lane % MI, k-chunk lane / MI; a lane of the
    // MI x MI result holds column lane % MI and NV rows.
    static_assert(MI == 32 || MI == 16, "MFMA shape");
    constexpr int WTM = BM / WGM, WTN = BN / WGN, TM = WTM / MI, TN = WTN / MI;
    constexpr int NV = MI * MI / 64;                 // accumulator values per lane and subtile
    constexpr int KSTEP = MI == 32 ? 16 : 32;        // k extent of one MFMA
    constexpr int KSTEPS = BK / KSTEP;               // k-steps per stage
    static_assert(KSTEPS == 2 || KSTEPS == 4, "k-steps per stage");
    typedef float accv_t __attribute__((ext_vector_type(NV)));
    constexpr int NW = WGM * WGN;   // wavefronts per workgroup
    static_assert((NW == 4 || NW == 8) && TM >= 1 && TN >= 1 && (!DUAL || TN % 2 == 0), "tile shape");
    static_assert(BM % (RPI * NW) == 0 && BN % (RPI * NW) == 0, "every wavefront moves whole row groups of both tiles");

    // XCD-aware tile id: ids i, i+8, i+16 ... land on the same XCD; give that XCD a contiguous tile range
    int pid = blockIdx.x, split = 0;
    if (EPI == EPI_RESIDUAL && k_splits > 1) {
        split = pid / n_tiles;
        pid -= split * n_tiles;
    }
    const int k_len = Kin / k_splits, k_beg = split * k_len;   // this workgroup's K range
    if (n_tiles % 8 == 0) pid = (pid % 8) * (n_tiles / 8) + pid / 8;
    // Each XCD has its own L2 and runs about 32 consecutive tile ids of its range at a time, all walking K roughly in
    // step, so those 32 tiles should share operand tiles both ways: ids are laid out in bands of `group_m` row tiles,
    // column-major inside a band, which makes 32 consecutive ids a patch of group_m x (32 / group_m) tiles (every
    // activation K-slice is fetched once for 32 / group_m workgroups, every weight K-slice once for group_m).  With
    // at most group_m row tiles this is the plain "rows fastest" order.
    const int tiles_m = n_tiles / tiles_n;
    const int band = group_m * tiles_n;
    const int first_m = (pid / band) * group_m;
    const int rows_in_band = min(tiles_m - first_m, group_m);
    const int tile_m = first_m + (pid % band) % rows_in_band;
    const int tile_n = (pid % band) / rows_in_band;
    const int m0 = tile_m * BM, n0 = tile_n * BN_OUT;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;

    accv_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < NV; ++v) acc[i][j][v] = 0.f;

    // Operand tiles go from global memory straight into LDS (buffer_load ... lds): no staging
    // registers and no ds_write traffic on the wavefronts' issue ports.  One such instruction moves
    // 64 lanes x 16 bytes = 8 tile rows x 128 bytes into 1 KB of consecutive LDS, lane l landing at
    // offset 16*l, i.e. row l/8, chunk slot l%8.  The XOR swizzle therefore lives on the global
    // side: the lane fetches logical chunk (l%8) ^ key(row), key(row) = (row >> 1) & 7.  Row groups
    // are dealt to the NW wavefronts round-robin (group g = NW*j + wave), which makes the key a
    // per-lane constant: ((wave & 1) * 4 + l/16) & 7.  The per-lane byte offset is one VGPR; the
    // group and K position are wave-uniform and ride in a scalar offset.  Rows past the matrix edge
    // are rejected by the descriptor's range check (they only feed outputs that are never stored).
    const int rows_x = min(BM, M - m0), rows_y = min(BN_OUT, Nout - n0);
    const __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(X) + (int64_t)m0 * ldx + k_beg, 0, ((rows_x - 1) * ldx + Kin - k_beg) * 2, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_y = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(Y) + (int64_t)n0 * ldy + k_beg, 0, ((rows_y - 1) * ldy + Kin - k_beg) * 2, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_y2 = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(DUAL ? Y2 : Y) + (int64_t)n0 * ldy + k_beg, 0, ((rows_y - 1) * ldy + Kin - k_beg) * 2, 0x00020000);
    const int uwave = __builtin_amdgcn_readfirstlane(wave);
    const int dma_key = (((uwave & 1) << 2) + (lane >> 4)) & 7;
    const int voff_x = (lane / LPR) * ldx * 2 + (((lane % LPR) ^ dma_key) << 4);
    const int voff_y = (lane / LPR) * ldy * 2 + (((lane % LPR) ^ dma_key) << 4);
    constexpr int GA = BM / RPI / NW, GB = BN / RPI / NW;   // row groups per wavefront, A and B tile
    constexpr int NLD = GA + GB;                      // DMA instructions per wavefront per stage
    typedef __attribute__((address_space(3))) void lds_void;

// global -> LDS: one stage of the X tile / of the Y tile, K position k0, into ring slot `slot`
// `half`: -1 the whole stage, 0 / 1 the first / second half of this wavefront's row groups (an odd group goes first).
// With ASYM the lower NW/2 wavefronts fetch for themselves and for wavefront w + NW/2, the others do nothing.
#define PSD_GEMM_DMA_A_PART(slot, k0, half)                                                                   \
    if (!ASYM || uwave < NW / 2) {                                                                            \
        _Pragma("unroll") for (int hh = 0; hh < (ASYM ? 2 : 1); ++hh) {                                       \
            const int uw_ = uwave + hh * (NW / 2);                                                            \
            unsigned char *sa_ = lds + (slot) * A_BYTES + uw_ * 1024;                                         \
            _Pragma("unroll") for (int j = 0; j < GA; ++j)                                                    \
                if ((half) < 0 || (j < (GA + 1) / 2) == ((half) == 0))                                        \
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_x, (lds_void *)(sa_ + j * (NW * 1024)), 16, voff_x, \
                                                             ((j * NW + uw_) * RPI * ldx + (k0)) * 2, 0, 0);  \
        }                                                                                                     \
    }
#define PSD_GEMM_DMA_B_PART(slot, k0, half)                                                                   \
    if (!ASYM || uwave < NW / 2) {                                                                            \
        _Pragma("unroll") for (int hh = 0; hh < (ASYM ? 2 : 1); ++hh) {                                       \
            const int uw_ = uwave + hh * (NW / 2);                                                            \
            unsigned char *sb_ = lds + B_RING + (slot) * B_BYTES + uw_ * 1024;                                \
            _Pragma("unroll") for (int j = 0; j < GB; ++j) {                                                  \
                if (!((half) < 0 || (j < (GB + 1) / 2) == ((half) == 0))) continue;                           \
                if (DUAL && j * (RPI * NW) >= BN / 2)                                                         \
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_y2, (lds_void *)(sb_ + j * (NW * 1024)), 16, voff_y, \
                                                             (((j * NW + uw_) * RPI - BN / 2) * ldy + (k0)) * 2, 0, 0); \
                else                                                                                          \
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_y, (lds_void *)(sb_ + j * (NW * 1024)), 16, voff_y, \
                                                             ((j * NW + uw_) * RPI * ldy + (k0)) * 2, 0, 0);  \
            }                                                                                                 \
        }                                                                                                     \
    }
#define PSD_GEMM_DMA_A(slot, k0) PSD_GEMM_DMA_A_PART(slot, k0, -1)
#define PSD_GEMM_DMA_B(slot, k0) PSD_GEMM_DMA_B_PART(slot, k0, -1)
// Every iteration issues the fetch of the shallower ring first.  Memory returns in issue order, so
// once the counter says that at most WAIT younger DMA instructions are in flight, both tiles of the
// next stage have landed: with the X ring shallower, its stage kt+1 was issued NSA-2 iterations ago
// and only that iteration's Y fetch plus NSA-2 whole iterations are younger (and mirrored).
#define PSD_GEMM_ISSUE(sa, sb, kt_)                                                                           \
    {                                                                                                         \
        if constexpr (NSA <= NSB) {                                                                           \
            PSD_GEMM_DMA_A(sa, ((kt_) + NSA - 1) * BK)                                                        \
            PSD_GEMM_DMA_B(sb, ((kt_) + NSB - 1) * BK)                                                        \
        } else {                                                                                              \
            PSD_GEMM_DMA_B(sb, ((kt_) + NSB - 1) * BK)                                                        \
            PSD_GEMM_DMA_A(sa, ((kt_) + NSA - 1) * BK)                                                        \
        }                                                                                                     \
    }
    constexpr int WAIT = (ASYM ? 2 : 1) * (NSA < NSB ? (NSA - 2) * NLD + GB : NSA > NSB ? (NSB - 2) * NLD + GA : (NSA - 2) * NLD);
// the DMAs of the next stage have landed; then all wavefronts agree (s_barrier), and the compiler must
// not move LDS accesses across the point
#define PSD_GEMM_STAGE_SYNC(n)                                                                                \
    {                                                                                                         \
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(n) : "memory");                                              \
        __builtin_amdgcn_s_barrier();                                                                         \
        asm volatile("" ::: "memory");                                                                        \
    }

    const int nk = k_len / BK;
    const int lrow = lane & (MI - 1), lhalf = lane / MI;   // row of this lane's fragments inside a subtile, and its k-chunk (0..1 or 0..3)
    // row inside a subtile of accumulator value v of this lane
    auto vrow = [&](int v) { return MI == 32 ? 8 * (v >> 2) + 4 * lhalf + (v & 3) : 4 * lhalf + v; };

    // LDS byte offsets of this lane's fragment rows (k-step 0); k-step kk flips the chunk index by 2*kk
    int offa[TM], offb[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) offa[i] = (wm * WTM + i * MI + lrow) * ROW_BYTES;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        int r;
        if constexpr (DUAL) {   // first half of the subtiles: gate rows, second half: up rows of the same columns
            const int jj = j % (TN / 2);
            r = (j >= TN / 2 ? BN / 2 : 0) + wn * (WTN / 2) + jj * MI + lrow;
        } else {
            r = wn * WTN + j * MI + lrow;
        }
        offb[j] = B_RING + r * ROW_BYTES;
    }
    const int rsw = row_key(lrow);   // swizzle key of every fragment row of this lane: rows differ by multiples of 32

// fragments of k-step kk of an LDS stage into register set `set`
#define PSD_GEMM_LOAD_FRAGS(sa, sb, kk, set)                                                                  \
    {                                                                                                         \
        const unsigned char *a_ = lds + (sa) * A_BYTES, *b_ = lds + (sb) * B_BYTES;                           \
        const int co_ = ((((kk) * (KSTEP / 8) + lhalf) ^ rsw) << 4);                                          \
        _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                        \
            fa[set][i] = *reinterpret_cast<const bf16x8 *>(a_ + offa[i] + co_);                               \
        _Pragma("unroll") for (int j = 0; j < TN; ++j)                                                        \
            fb[set][j] = *reinterpret_cast<const bf16x8 *>(b_ + offb[j] + co_);                               \
    }
#define PSD_GEMM_MFMA(set)                                                                                    \
    {                                                                                                         \
        PSD_PRIO_HI                                                                                           \
        _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                        \
            _Pragma("unroll") for (int j = 0; j < TN; ++j)                                                    \
                acc[i][j] = mfma_step<MI>(fa[set][i], fb[set][j], acc[i][j]);                                 \
        PSD_PRIO_LO                                                                                           \
    }

    constexpr int NFRAG = TM + TN, NMFMA = TM * TN;
    static_assert(NSA >= 2 && NSB >= 2 && (ASYM ? 2 : 1) * ((NSA - 1) * GA + (NSB - 1) * GB) <= 63, "DMA groups in flight must fit the vmcnt counter");
    static_assert(!ASYM || (NW / 2) % 2 == 0, "wavefronts w and w + NW/2 share the swizzle key of their row groups");
    bf16x8 fa[2][TM], fb[2][TN];

#pragma unroll
    for (int p = 0; p < NSA - 1; ++p) PSD_GEMM_DMA_A(p, p * BK)
#pragma unroll
    for (int p = 0; p < NSB - 1; ++p) PSD_GEMM_DMA_B(p, p * BK)
    PSD_GEMM_STAGE_SYNC(0)
    PSD_GEMM_LOAD_FRAGS(0, 0, 0, 0)

    // Per K-stage: the DMAs that refill the ring slots every wavefront left at the last barrier go
    // out during k-step 0 (X stage kt+NSA-1, Y stage kt+NSB-1).  k-steps 0..2 compute with
    // the next k-step's fragments in flight; after the stage barrier k-step 3 computes while the first
    // fragments of the next stage arrive.  The body is branch-free: fetches past the end of K stay
    // inside the buffer range (or are rejected) and land in ring slots that are never consumed.
    int ca = 0, cb = 0;
    for (int kt = 0; kt < nk; ++kt) {
        const int na = (ca + 1 == NSA) ? 0 : ca + 1, nb = (cb + 1 == NSB) ? 0 : cb + 1;
        const int fill_a = (ca == 0) ? NSA - 1 : ca - 1, fill_b = (cb == 0) ? NSB - 1 : cb - 1;
        PSD_GEMM_LOAD_FRAGS(ca, cb, 1, 1)
        if constexpr (SPREAD && KSTEPS == 4) {
            // the shallower ring's stage in two halves during k-steps 0 and 1, the deeper ring's during k-step 2: the
            // same issue order as PSD_GEMM_ISSUE, so the wait below counts the same
            constexpr int MUL = ASYM ? 2 : 1;
            constexpr int G1 = NSA <= NSB ? GA : GB, G2 = NSA <= NSB ? GB : GA;
            if constexpr (NSA <= NSB) { PSD_GEMM_DMA_A_PART(fill_a, (kt + NSA - 1) * BK, 0) } else { PSD_GEMM_DMA_B_PART(fill_b, (kt + NSB - 1) * BK, 0) }
            PSD_GEMM_MFMA(0)
            sched_mix<0, NMFMA, NFRAG, 0, MUL * ((G1 + 1) / 2)>();
            PSD_GEMM_LOAD_FRAGS(ca, cb, 2, 0)
            if constexpr (NSA <= NSB) { PSD_GEMM_DMA_A_PART(fill_a, (kt + NSA - 1) * BK, 1) } else { PSD_GEMM_DMA_B_PART(fill_b, (kt + NSB - 1) * BK, 1) }
            PSD_GEMM_MFMA(1)
            sched_mix<0, NMFMA, NFRAG, 0, MUL * (G1 / 2)>();
            PSD_GEMM_LOAD_FRAGS(ca, cb, 3, 1)
            if constexpr (NSA <= NSB) { PSD_GEMM_DMA_B(fill_b, (kt + NSB - 1) * BK) } else { PSD_GEMM_DMA_A(fill_a, (kt + NSA - 1) * BK) }
            PSD_GEMM_MFMA(0)
            sched_mix<0, NMFMA, NFRAG, 0, MUL * G2>();
        } else {
            PSD_GEMM_ISSUE(fill_a, fill_b, kt)
            PSD_GEMM_MFMA(0)
            sched_mix<0, NMFMA, NFRAG, 0, (ASYM ? 2 : 1) * NLD>();
            if constexpr (KSTEPS == 4) {
                PSD_GEMM_LOAD_FRAGS(ca, cb, 2, 0)
                PSD_GEMM_MFMA(1)
                sched_mix<0, NMFMA, NFRAG, 0, 0>();
                PSD_GEMM_LOAD_FRAGS(ca, cb, 3, 1)
                PSD_GEMM_MFMA(0)
                sched_mix<0, NMFMA, NFRAG, 0, 0>();
            }
        }
        // (with two k-steps per stage the second one computes behind the barrier)
        PSD_GEMM_STAGE_SYNC(WAIT)
        PSD_GEMM_LOAD_FRAGS(na, nb, 0, 0)
        PSD_GEMM_MFMA(1)
        sched_mix<0, NMFMA, NFRAG, 0, 0>();
        ca = na;
        cb = nb;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // no DMA may outlive the loop
#undef PSD_GEMM_LOAD_FRAGS
#undef PSD_GEMM_MFMA
#undef PSD_GEMM_DMA_A
#undef PSD_GEMM_DMA_B
#undef PSD_GEMM_DMA_A_PART
#undef PSD_GEMM_DMA_B_PART
#undef PSD_GEMM_ISSUE
#undef PSD_GEMM_STAGE_SYNC

    if constexpr (EPI == EPI_TOP1) {
        // per column j: (max, lowest argmax, sum exp) over this tile's rows; rows ascend with (i, v)
        // inside a lane, so a strict comparison keeps the lowest index on ties
        __shared__ float s_b[WGM][BN];
        __shared__ float s_s[WGM][BN];
        __shared__ int s_a[WGM][BN];
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            float best = -INFINITY;
            int arg = 0x7fffffff;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    const int m = m0 + wm * WTM + i * MI + vrow(v);
                    float z = acc[i][j][v] * t1.scale;
                    if (m >= M || m == t1.mask_id) z = -INFINITY;
                    acc[i][j][v] = z;
                    if (z > best) {
                        best = z;
                        arg = m;
                    }
                }
            float sum = 0.f;
            if (best > -INFINITY) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int v = 0; v < NV; ++v) sum += __expf(acc[i][j][v] - best);
            }
            // the 64 / MI lanes that hold this column own disjoint row sets
#pragma unroll
            for (int off = 32; off >= MI; off >>= 1) {
                const float b2 = __shfl_xor(best, off, 64);
                const int a2 = __shfl_xor(arg, off, 64);
                const float s2 = __shfl_xor(sum, off, 64);
                top1_merge(best, arg, sum, b2, a2, s2);
            }
            if (lhalf == 0) {
                const int col = wn * WTN + j * MI + lrow;
                s_b[wm][col] = best;
                s_a[wm][col] = arg;
                s_s[wm][col] = sum;
            }
        }
        __syncthreads();
        if (tid < BN && n0 + tid < Nout) {
            float best = s_b[0][tid], sum = s_s[0][tid];
            int arg = s_a[0][tid];
#pragma unroll
            for (int w = 1; w < WGM; ++w) top1_merge(best, arg, sum, s_b[w][tid], s_a[w][tid], s_s[w][tid]);
            const int64_t o = (int64_t)tile_m * t1.cols_total + n0 + tid;
            t1.pmax[o] = best;
            t1.psum[o] = sum;
            t1.parg[o] = arg;
        }
    } else if constexpr (EPI == EPI_QKV) {
        constexpr int NT = NW * 64;
        constexpr int LDC = BN * 2 + 16;   // bytes per row of the row-major staging tile: the two half-waves (rows r, r + 4) land 64 bytes apart in the banks
        constexpr int LDT = BM * 2 + 8;    // bytes per column of the column-major one: 32 lanes x 8 bytes cover all banks once
        static_assert(BM * LDC <= (NSA * BM + NSB * BN) * ROW_BYTES && BN * LDT <= (NSA * BM + NSB * BN) * ROW_BYTES, "staging tile fits the rings");
        __syncthreads();                   // every wavefront is done with the operand rings
        if (n0 < qa.v_start) {
            // ---- q / k heads: stage row-major, rotate pairs (j, j + d_head / 2), store 16 bytes per access
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int col = wn * WTN + j * MI + lrow;
                    const float bn = bias ? bias[min(n0 + col, Nout - 1)] : 0.f;
#pragma unroll
                    for (int v = 0; v < NV; ++v) {
                        const int row = wm * WTM + i * MI + vrow(v);
                        *reinterpret_cast<uint16_t *>(lds + row * LDC + col * 2) = from_float<bf16_t>(acc[i][j][v] + bn).bits;
                    }
                }
            __syncthreads();
            const int half = qa.d_head >> 1, groups = half >> 3, heads = BN / qa.d_head;
            const int units = BM * heads * groups;   // 8 pair indices of one head of one row each
            for (int u = tid; u < units; u += NT) {
                const int g = u % groups, hd = (u / groups) % heads, row = u / (groups * heads);
                const int m = m0 + row, n = n0 + hd * qa.d_head + g * 8;
                if (m >= M || n >= Nout) continue;
                const unsigned char *src = lds + row * LDC + (hd * qa.d_head + g * 8) * 2;
                const uint4 a = *reinterpret_cast<const uint4 *>(src), b = *reinterpret_cast<const uint4 *>(src + half * 2);
                const int64_t t = (int64_t)(qa.pos0 + m % qa.N) * half + g * 8;
                const float4 c0 = *reinterpret_cast<const float4 *>(qa.cos_t + t), c1 = *reinterpret_cast<const float4 *>(qa.cos_t + t + 4);
                const float4 s0 = *reinterpret_cast<const float4 *>(qa.sin_t + t), s1 = *reinterpret_cast<const float4 *>(qa.sin_t + t + 4);
                uint4 ra, rb;
                rope_rotate8(a, b, c0, c1, s0, s1, ra, rb);
                bf16_t *dst = out + (int64_t)m * ldo + n;
                *reinterpret_cast<uint4 *>(dst) = ra;
                *reinterpret_cast<uint4 *>(dst + half) = rb;
            }
        } else {
            // ---- V heads: stage column-major (a lane's 4 consecutive rows are one 8-byte piece), store transposed.
            // Inside every group of 16 keys the slots hold keys 0-3, 8-11, 4-7, 12-15.
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int col = wn * WTN + j * MI + lrow;
                    const float bn = bias ? bias[min(n0 + col, Nout - 1)] : 0.f;
#pragma unroll
                    for (int q = 0; q < NV / 4; ++q) {
                        const int row = wm * WTM + i * MI + vrow(4 * q);
                        uint2 w;
                        w.x = pack_bf16x2(acc[i][j][4 * q + 0] + bn, acc[i][j][4 * q + 1] + bn);
                        w.y = pack_bf16x2(acc[i][j][4 * q + 2] + bn, acc[i][j][4 * q + 3] + bn);
                        *reinterpret_cast<uint2 *>(lds + col * LDT + row * 2) = w;
                    }
                }
            __syncthreads();
            constexpr int G16 = BM / 16;
            const int n_v = Nout - qa.v_start;
            for (int u = tid; u < BN * G16 * 2; u += NT) {
                const int h = u & 1, g = (u >> 1) % G16, col = u / (2 * G16);
                const int m = m0 + g * 16, n = n0 + col;
                if (m >= M || n >= Nout) continue;
                const unsigned char *src = lds + col * LDT + (g * 16 + 4 * h) * 2;
                const uint2 lo = *reinterpret_cast<const uint2 *>(src), hi = *reinterpret_cast<const uint2 *>(src + 16);
                const int sq = m / qa.N, i0 = m % qa.N;   // N % 16 == 0: the 16 keys belong to one sequence
                bf16_t *dst = qa.vT + ((int64_t)sq * n_v + (n - qa.v_start)) * qa.ld_vt + i0 + 8 * h;
                *reinterpret_cast<uint4 *>(dst) = make_uint4(lo.x, lo.y, hi.x, hi.y);
            }
        }
    } else {
        constexpr int TN_OUT = DUAL ? TN / 2 : TN;
        constexpr int WTN_OUT = DUAL ? WTN / 2 : WTN;
        if constexpr (EPI == EPI_RESIDUAL) {
            // fp32 read-modify-write of the stream.  16 values (a 32x32 subtile, or four 16x16 ones) are fetched before the first is
            // written back: written as one load-add-store per element, every load would wait for the store before it
            // (the compiler cannot tell rows m * ldo apart) and the epilogue becomes a chain of memory round trips
            // (measured: 6.45 -> 5.67 ms for the output projection at 163 840 rows; a whole row of subtiles per round trip
            // gains nothing more and spills registers on the 128x192 tile).
            float *dst = (split == 0) ? resid : partial + (int64_t)(split - 1) * M * Nout;
            const int ldd = (split == 0) ? ldo : Nout;
            // subtiles per round trip: up to 16 values in flight per lane
            constexpr int JB = NV >= 16 ? 1 : (TN % 4 == 0 ? 4 : TN % 2 == 0 ? 2 : 1);
            static_assert(TN % JB == 0 && JB * NV <= 16, "subtile batches");
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j0 = 0; j0 < TN; j0 += JB) {
                    float old[JB][NV];
#pragma unroll
                    for (int jj = 0; jj < JB; ++jj) {
                        const int n = n0 + wn * WTN + (j0 + jj) * MI + lrow;
#pragma unroll
                        for (int v = 0; v < NV; ++v) {
                            const int m = m0 + wm * WTM + i * MI + vrow(v);
                            old[jj][v] = (split == 0 && n < Nout && m < M) ? dst[(int64_t)m * ldd + n] : 0.f;
                        }
                    }
#pragma unroll
                    for (int jj = 0; jj < JB; ++jj) {
                        const int n = n0 + wn * WTN + (j0 + jj) * MI + lrow;
#pragma unroll
                        for (int v = 0; v < NV; ++v) {
                            const int m = m0 + wm * WTM + i * MI + vrow(v);
                            if (n < Nout && m < M) dst[(int64_t)m * ldd + n] = old[jj][v] + acc[i][j0 + jj][v];
                        }
                    }
                }
            return;
        }
        // bf16 outputs.  A lane holds single columns: written straight to memory that is 2-byte stores, 64 bytes per row
        // and instruction.  Where rows allow 16-byte accesses the tile is staged in LDS instead (the operand rings are
        // free; row-major, rows padded by 16 bytes so that the two half-waves land 64 bytes apart in the banks) and
        // stored with 16 bytes per lane (measured in one process at 163 840 rows: store epilogue 13.78 -> 13.52 ms, SwiGLU
        // 26.57 -> 26.2 ms; within noise below 2048 rows).
        constexpr int BNO = BN_OUT, LDC = BNO * 2 + 16, NT = NW * 64;
        static_assert(BM * LDC <= (NSA * BM + NSB * BN) * ROW_BYTES, "staging tile fits the rings");
        if ((ldo & 7) == 0 && (Nout & 7) == 0 && (reinterpret_cast<uintptr_t>(out) & 15) == 0) {   // uniform
            __syncthreads();   // every wavefront is done with the operand rings
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN_OUT; ++j) {
                    const int col = wn * WTN_OUT + j * MI + lrow;
                    const float bn = (EPI == EPI_BIAS) ? bias[min(n0 + col, Nout - 1)] : 0.f;
#pragma unroll
                    for (int v = 0; v < NV; ++v) {
                        const int row = wm * WTM + i * MI + vrow(v);
                        float x = acc[i][j][v];
                        if (EPI == EPI_BIAS) x += bn;
                        if (DUAL) {
                            const float u = acc[i][j + TN / 2][v];
                            x = x * __builtin_amdgcn_rcpf(1.0f + __expf(-x)) * u;
                        }
                        *reinterpret_cast<uint16_t *>(lds + row * LDC + col * 2) = from_float<bf16_t>(x).bits;
                    }
                }
            __syncthreads();
            for (int u = tid; u < BM * (BNO / 8); u += NT) {
                const int c8 = u % (BNO / 8), row = u / (BNO / 8);
                const int m = m0 + row, n = n0 + c8 * 8;
                if (m < M && n < Nout)
                    *reinterpret_cast<uint4 *>(out + (int64_t)m * ldo + n) = *reinterpret_cast<const uint4 *>(lds + row * LDC + c8 * 16);
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN_OUT; ++j) {
                const int n = n0 + wn * WTN_OUT + j * MI + lrow;
                if (n >= Nout) continue;
                const float bn = (EPI == EPI_BIAS) ? bias[n] : 0.f;
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    const int m = m0 + wm * WTM + i * MI + vrow(v);
                    if (m >= M) continue;
                    float x = acc[i][j][v];
                    if (EPI == EPI_BIAS) x += bn;
                    if (DUAL) {
                        const float u = acc[i][j + TN / 2][v];
                        x = x * __builtin_amdgcn_rcpf(1.0f + __expf(-x)) * u;   // silu(x) * u; v_rcp_f32 (1 ulp) instead of a full division
                    }
                    out[(int64_t)m * ldo + n] = from_float<bf16_t>(x);
                }
            }
    }
}

template <int BM, int BN, int WGM, int WGN, int EPI, int NSA = 2, int NSB = NSA, int SCHED = 0, int MI = 32>
void launch_cfg(const bf16_t *X, const bf16_t *Y, const bf16_t *Y2, int M, int Nout, int Kin, int ldx, int ldy, const float *bias,
                bf16_t *out, float *resid, int ldo, Top1Args t1, hipStream_t st, int k_splits = 1, float *partial = nullptr,
                QkvArgs qa = QkvArgs()) {
    constexpr int BN_OUT = (EPI == EPI_SWIGLU) ? BN / 2 : BN;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (Nout + BN_OUT - 1) / BN_OUT;
    const int n_tiles = tiles_m * tiles_n;
    constexpr int smem = (NSA * BM + NSB * BN) * BK * 2;
    static_assert(smem <= 160 * 1024, "LDS ring exceeds the 160 KB of a CU");
    auto kern = gemm_bf16_kernel<BM, BN, WGM, WGN, EPI, NSA, NSB, SCHED, MI>;
    static std::atomic<uint64_t> lds_raised{0};   // one per instantiation
    ensure_dynamic_lds(reinterpret_cast<const void *>(kern), smem, lds_raised);
    if (EPI != EPI_RESIDUAL) k_splits = 1;
    hipLaunchKernelGGL(kern, dim3(n_tiles * k_splits), dim3(WGM * WGN * 64), smem, st, X, Y, Y2, M, Nout, Kin, ldx, ldy, bias, out, resid,
                       ldo, tiles_n, n_tiles, t1, k_splits, partial, gemm_tile_group_m(), qa);
}

}   // namespace mfma
