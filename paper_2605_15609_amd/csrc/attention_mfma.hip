// Bidirectional (non-causal) flash-style attention on the gfx950 matrix cores, bf16 in,
// fp32 softmax statistics and accumulation.  No mask: every query sees all N keys (the
// dLLM forward of Sec. 3.1 conditions each position on the whole sequence).
//
// The kernel works on the transposed problem so that each query lives in one lane column:
//   S^T[key, q] = K Q^T          A operand = K rows (LDS), B operand = Q rows (registers)
//   O^T[c, q]  += V^T P^T        A operand = V^T rows (LDS), B operand = P^T (registers)
// With v_mfma_f32_32x32x16_bf16 a lane then holds 16 keys of ONE query per 32x32 tile, so
// the running max / sum of the online softmax need no cross-lane traffic beyond one
// exchange between the two half-waves, and the probabilities P^T are already in the
// register layout the second MFMA wants as its B operand: they never touch LDS.  The
// contraction index of the second MFMA is a permutation of the keys (slot (half, e) <->
// key 8*(e/4) + 4*half + e%4 of each group of 16); V^T tiles are stored in LDS in that same
// permuted key order, so a lane's 8 values are one 16-byte read.
//
// One workgroup = 4 (or 2) wavefronts = 128 (64) queries of one (sequence, head); K and V^T tiles
// of 64 keys go global -> LDS directly (buffer_load ... lds) into double-buffered, XOR-swizzled LDS.  Grouped KV heads: the
// query heads of a group simply read the same K / V^T tiles (they hit L2).
#include <type_traits>

#include "psd_internal.h"
#include "device_types.h"
#include "rope_device.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BKV = 64;    // keys per stage

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 u) { return __builtin_bit_cast(bf16x8, u); }

typedef __attribute__((address_space(3))) void lds_void;

// NW wavefronts (32 queries each) per workgroup; ld_qkv / ld_vt = row strides (elements) of qkv and of vT,
// whose rows hold N rounded up to 64 keys (tail zero)
//
// pre: keys and values that precede the sequence's own N rows (a KV cache of pre.len positions, shared by
// pre.seqs_per_cache consecutive sequences).  Every query sees all of them and all N own keys: with the own rows
// being one block, that is context-causal block attention.  pre.len = 0: plain bidirectional attention.
//
// KSP > 1 (= NW): key-split mode for a single block of 32 queries.  The NW wavefronts all take the same queries
// and deal the key tiles round-robin; each runs the tile loop on its own, with a ring of its own in LDS (no
// barrier inside the loop), and the partial (max, sum, O^T) are merged in wavefront order at the end.  A lone
// wavefront per (sequence, head) walks its tiles as one serial chain of fetch, MFMA, softmax, MFMA; the split
// shortens that chain, which is all the time there is on the block-row path.
template <int DH, int NW, int NSTG, int KSP = 1>
__global__ __launch_bounds__(NW * 64, 2) void attention_kernel(const bf16_t *__restrict__ qkv, int ld_qkv,
                                                            const bf16_t *__restrict__ vT, int ld_vt, int N, int n_heads,
                                                            int n_kv_heads, bf16_t *__restrict__ out, KvPrefix pre) {
    constexpr int KROW = DH * 2;                 // bytes per K row in LDS
    constexpr int K_BYTES = BKV * KROW;
    constexpr int VROW = BKV * 2;                // bytes per V^T row in LDS (128)
    constexpr int V_BYTES = DH * VROW;
    constexpr int STAGE = K_BYTES + V_BYTES;
    constexpr int CT = DH / 32;                  // output subtiles along the head dimension
    constexpr int KS = DH / 16;                  // k-steps of the score contraction
    constexpr int KRPI = 1024 / KROW;            // K rows moved by one DMA instruction (4 or 8)
    static_assert(KSP == 1 || KSP == NW, "key-split mode: every wavefront of the workgroup takes part");
    constexpr int NWD = KSP > 1 ? 1 : NW;        // wavefronts that share the fetch of one tile
    constexpr int KG = BKV / KRPI / NWD;         // K-tile DMA instructions per wavefront
    constexpr int VG = DH / 8 / NWD;             // V^T-tile DMA instructions per wavefront (8 rows each)
    extern __shared__ __align__(16) unsigned char lds_all[];
    // Swizzle key of a K row.  The 64 LDS banks span 256 bytes: 128-byte rows (d_head 64) alternate between the
    // two halves, so rows r and r+1 may share a chunk slot and the key is (r >> 1) & 7 as in the GEMM tiles;
    // 256-byte rows (d_head 128) all start at bank 0 and need 16 different slots for 16 consecutive rows.
    auto kkey = [](int r) { return DH == 128 ? (r & 15) : ((r >> 1) & 7); };

    // Workgroups go to the 8 XCDs round-robin in launch order (x fastest).  Every query block of every head of one KV group
    // reads the same keys and values, so they should meet in one XCD's L2: the (KV head, sequence) units are dealt to
    // the XCDs, and an XCD walks its units one after the other (measured at 128 x 1280, 32 heads: 23.5 GB fetched per
    // launch with the plain order, the keys and values of a head once per query block).
    int qblk = blockIdx.x, head = blockIdx.y, s = blockIdx.z;
    {
        const int group = n_heads / n_kv_heads, units = n_kv_heads * (int)gridDim.z, per_unit = (int)gridDim.x * group;
        if (units % 8 == 0) {
            const int pid = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
            const int slot = pid >> 3, unit = (slot / per_unit) * 8 + (pid & 7), within = slot % per_unit;
            qblk = within % (int)gridDim.x;
            head = (unit % n_kv_heads) * group + within / (int)gridDim.x;
            s = unit / n_kv_heads;
        }
    }
    const int kvh = head / (n_heads / n_kv_heads);
    const int row_w = ld_qkv;
    const int tid = threadIdx.x, lane = tid & 63, wave_id = __builtin_amdgcn_readfirstlane(tid >> 6);
    // key-split: one query block per workgroup, a private ring per wavefront, every wavefront fetches whole tiles
    const int q_base = KSP > 1 ? qblk * 32 : qblk * (32 * NW) + wave_id * 32;   // this wavefront's first query
    const int wave = KSP > 1 ? 0 : wave_id;      // index among the wavefronts that share a tile's fetch
    unsigned char *lds = lds_all + (KSP > 1 ? wave_id * (NSTG * STAGE) : 0);
    const int lrow = lane & 31, lhalf = lane >> 5;
    const bf16_t *seq = qkv + (int64_t)s * N * row_w;

    // Q fragments: lane (q = lrow, half) holds Q[q][16*ks + 8*half .. +7]
    bf16x8 qf[KS];
    {
        const int q = q_base + lrow;
        const bf16_t *qp = seq + (int64_t)q * row_w + head * DH;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            u32x4 t = {0u, 0u, 0u, 0u};
            if (q < N) t = *reinterpret_cast<const u32x4 *>(qp + ks * 16 + lhalf * 8);
            qf[ks] = as_bf16x8(t);
        }
    }

    // K and V^T tiles go global -> LDS directly (buffer_load ... lds), 1 KB per instruction, with the XOR
    // swizzle applied on the global side: the lane that lands at (row, slot) fetches chunk slot ^ key(row),
    // key(row) = kkey(row) for K rows and (row >> 1) & 7 for the 128-byte V^T rows.  Row groups are dealt round-robin to the wavefronts.  Keys past the end of
    // the sequence are rejected by the descriptor (K); value slots past it are zeroed in registers in the last tile.
    const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(seq) + (n_heads + kvh) * DH, 0, (int)(((int64_t)N * row_w - (n_heads + kvh) * DH) * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>(vT) + ((int64_t)s * n_kv_heads + kvh) * DH * (int64_t)ld_vt, 0, DH * ld_vt * 2, 0x00020000);
    // the prefix (cache) of this sequence; empty descriptors when there is none
    const int n_pre = (pre.len + BKV - 1) / BKV;
    const int64_t cache = n_pre ? (pre.seq_rows ? pre.seq_rows[s] : s) / pre.seqs_per_cache : 0;
    const __amdgpu_buffer_rsrc_t rk_pre = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>((const bf16_t *)pre.k) + cache * pre.stride_k + kvh * DH, 0, n_pre ? (pre.len * pre.ld_k - kvh * DH) * 2 : 0,
        0x00020000);
    const __amdgpu_buffer_rsrc_t rv_pre = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t *>((const bf16_t *)pre.vt) + cache * pre.stride_vt + (int64_t)kvh * DH * pre.ld_vt, 0,
        n_pre ? DH * pre.ld_vt * 2 : 0, 0x00020000);
    constexpr int KLPR = 64 / KRPI;              // lanes per K row in one DMA instruction (16 or 8)
#define PSD_ATT_DMA_FROM(stage, rk_, ldk_, rv_, ldv_, k0)                                                        \
    {                                                                                                            \
        unsigned char *sk_ = lds + (stage) * STAGE + wave * 1024, *sv_ = lds + (stage) * STAGE + K_BYTES + wave * 1024; \
        _Pragma("unroll") for (int j = 0; j < KG; ++j) {                                                         \
            const int row = (j * NWD + wave) * KRPI + lane / KLPR;                                                \
            const int voff = (lane / KLPR) * (ldk_) * 2 + (((lane % KLPR) ^ kkey(row)) << 4);                     \
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rk_, (lds_void *)(sk_ + j * (NWD * 1024)), 16, voff,         \
                                                     (((k0) + (j * NWD + wave) * KRPI) * (ldk_)) * 2, 0, 0);       \
        }                                                                                                        \
        _Pragma("unroll") for (int j = 0; j < VG; ++j) {                                                         \
            const int row = (j * NWD + wave) * 8 + (lane >> 3);                                                   \
            const int voff = (lane >> 3) * (ldv_) * 2 + (((lane & 7) ^ ((row >> 1) & 7)) << 4);                  \
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rv_, (lds_void *)(sv_ + j * (NWD * 1024)), 16, voff,         \
                                                     ((j * NWD + wave) * 8 * (ldv_) + (k0)) * 2, 0, 0);            \
        }                                                                                                        \
    }
// tile tt of the key sequence: prefix tiles first, then the own rows
#define PSD_ATT_DMA(stage, tt)                                                                                   \
    {                                                                                                            \
        if ((tt) < n_pre) PSD_ATT_DMA_FROM(stage, rk_pre, pre.ld_k, rv_pre, pre.ld_vt, (tt) * BKV)               \
        else PSD_ATT_DMA_FROM(stage, rk, row_w, rv, ld_vt, ((tt) - n_pre) * BKV)                                 \
    }
#define PSD_ATT_SYNC()                                                                                           \
    {                                                                                                            \
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NSTG - 2) * (KG + VG)) : "memory");                            \
        if constexpr (KSP == 1) __builtin_amdgcn_s_barrier();   /* a private ring needs no agreement */          \
        asm volatile("" ::: "memory");                                                                           \
    }

    floatx16 acc_o[CT];
#pragma unroll
    for (int i = 0; i < CT; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc_o[i][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const float sl2 = 1.4426950408889634f / sqrtf((float)DH);   // softmax scale folded into exp2

    // Ring of NSTG tile stages: the fetch of tile t + NSTG - 1 goes out before tile t is computed, so a tile has
    // NSTG - 1 tile times to arrive (one tile of MFMA work is shorter than a round trip to memory).  Memory
    // returns in issue order: once at most (NSTG - 2) tiles' worth of this wavefront's fetches are in flight,
    // the next tile has landed.
    static_assert(NSTG >= 2 && (NSTG - 1) * (KG + VG) <= 63, "DMA groups in flight must fit the vmcnt counter");
    const int n_tiles = n_pre + (N + BKV - 1) / BKV;
    // this wavefront's tiles: all of them, or every KSP-th one
    constexpr int TSTEP = KSP;
    const int t_first = KSP > 1 ? wave_id : 0;
#pragma unroll
    for (int p = 0; p < NSTG - 1; ++p) PSD_ATT_DMA(p, t_first + p * TSTEP)
    PSD_ATT_SYNC()

    int stage = 0;
    for (int t = t_first; t < n_tiles; t += TSTEP) {
        // first key of the tile within its segment, and the number of keys that segment has
        const int k0 = (t < n_pre ? t : t - n_pre) * BKV, limit = t < n_pre ? pre.len : N;
        // refill the slot every wavefront left at the last barrier; past the last tile the fetch is rejected or
        // reads padding and is never consumed
        const int fill = (stage == 0) ? NSTG - 1 : stage - 1;
        PSD_ATT_DMA(fill, t + (NSTG - 1) * TSTEP)
        const unsigned char *sk = lds + stage * STAGE, *sv = sk + K_BYTES;

        // scores, transposed: acc_s[kt][v] <-> key 32*kt + 8*(v/4) + 4*half + v%4, query lrow
        floatx16 acc_s[2];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
            for (int v = 0; v < 16; ++v) acc_s[kt][v] = 0.f;
            const int r = kt * 32 + lrow;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const int c = ks * 2 + lhalf;
                const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(sk + r * KROW + ((c ^ kkey(r)) << 4));
                acc_s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], acc_s[kt], 0, 0, 0);
            }
        }
        // keys past the end of the segment do not exist
        if (k0 + BKV > limit) {
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = k0 + kt * 32 + 8 * (v >> 2) + 4 * lhalf + (v & 3);
                    if (key >= limit) acc_s[kt][v] = -INFINITY;
                }
        }
        // online softmax for this lane's query
        float mx = acc_s[0][0];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, acc_s[kt][v]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        // exp(x - m) as the bare v_exp_f32 of (x * sl2 - m * sl2): one fused multiply-add per score, no
        // denormal handling (a probability below 2^-126 is zero)
        const float m_new = fmaxf(m_run, mx);
        const float m_s = m_new * sl2;
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * sl2);
        float psum = 0.f;
        bf16x8 pf[4];   // P^T as B operands, one per group of 16 keys
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            float p[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                p[v] = __builtin_amdgcn_exp2f(__builtin_fmaf(acc_s[kt][v], sl2, -m_s));
                psum += p[v];
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                u32x4 f;
                f.x = pack_bf16x2(p[8 * u + 0], p[8 * u + 1]);
                f.y = pack_bf16x2(p[8 * u + 2], p[8 * u + 3]);
                f.z = pack_bf16x2(p[8 * u + 4], p[8 * u + 5]);
                f.w = pack_bf16x2(p[8 * u + 6], p[8 * u + 7]);
                pf[kt * 2 + u] = as_bf16x8(f);
            }
        }
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc_o[ct][v] *= alpha;
        // O^T += V^T P^T.  In the last, partial tile of a segment the value slots past its end hold whatever the memory
        // held (the tail of a cache row, row padding): their probabilities are zero, but 0 x NaN is NaN, so those slots
        // are zeroed in registers.  The two versions of the loop sit in two branches of a wave-uniform test so that
        // full tiles run the bare one.
        auto pv = [&](auto masked) {
#pragma unroll
            for (int kg = 0; kg < 4; ++kg) {
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) {
                    const int r = ct * 32 + lrow;
                    const int c = kg * 2 + lhalf;
                    bf16x8 vf = *reinterpret_cast<const bf16x8 *>(sv + r * VROW + ((c ^ ((r >> 1) & 7)) << 4));
                    if constexpr (decltype(masked)::value) {
                        // slot order inside a group of 16 keys: this lane's elements 0-3 are keys 4*half + 0..3, elements
                        // 4-7 keys 8 + 4*half + 0..3
                        const int n_lo = limit - (k0 + kg * 16 + 4 * lhalf), n_hi = n_lo - 8;
                        u32x4 w = __builtin_bit_cast(u32x4, vf);
                        w.x &= n_lo >= 2 ? 0xffffffffu : n_lo == 1 ? 0x0000ffffu : 0u;
                        w.y &= n_lo >= 4 ? 0xffffffffu : n_lo == 3 ? 0x0000ffffu : 0u;
                        w.z &= n_hi >= 2 ? 0xffffffffu : n_hi == 1 ? 0x0000ffffu : 0u;
                        w.w &= n_hi >= 4 ? 0xffffffffu : n_hi == 3 ? 0x0000ffffu : 0u;
                        vf = as_bf16x8(w);
                    }
                    acc_o[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kg], acc_o[ct], 0, 0, 0);
                }
            }
        };
        if (k0 + BKV > limit) pv(std::true_type());
        else pv(std::false_type());
        PSD_ATT_SYNC()
        stage = (stage + 1 == NSTG) ? 0 : stage + 1;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // no fetch may outlive the loop
#undef PSD_ATT_DMA
#undef PSD_ATT_DMA_FROM
#undef PSD_ATT_SYNC

    // the two half-waves of a query hold disjoint key subsets of the sum
    l_run += __shfl_xor(l_run, 32, 64);
    if constexpr (KSP > 1) {
        // merge the wavefronts' partial results in wavefront order: the others leave (max, sum, O^T) in their own
        // ring, wavefront 0 rescales everything to the common maximum and stores.  Field f of lane l sits at
        // word f * 64 + l.  A wavefront without tiles contributes max = -inf, sum = 0.
        float *mine = reinterpret_cast<float *>(lds);
        if (wave_id > 0) {
            mine[lane] = m_run;
            mine[64 + lane] = l_run;
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int v = 0; v < 16; ++v) mine[(2 + ct * 16 + v) * 64 + lane] = acc_o[ct][v];
        }
        __syncthreads();
        if (wave_id > 0) return;
        for (int w = 1; w < KSP; ++w) {
            const float *other = reinterpret_cast<const float *>(lds_all + w * (NSTG * STAGE));
            const float m_o = other[lane], l_o = other[64 + lane];
            const float m_new = fmaxf(m_run, m_o);
            const float a_me = __builtin_amdgcn_exp2f((m_run - m_new) * sl2), a_o = __builtin_amdgcn_exp2f((m_o - m_new) * sl2);
            l_run = l_run * a_me + l_o * a_o;
            m_run = m_new;
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc_o[ct][v] = acc_o[ct][v] * a_me + other[(2 + ct * 16 + v) * 64 + lane] * a_o;
        }
    }
    const float inv = 1.0f / l_run;
    const int q = q_base + lrow;
    if (q < N) {
        bf16_t *op = out + ((int64_t)s * N + q) * (n_heads * DH) + head * DH;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int c = ct * 32 + 8 * g + 4 * lhalf;
                uint2 w;
                w.x = pack_bf16x2(acc_o[ct][4 * g + 0] * inv, acc_o[ct][4 * g + 1] * inv);
                w.y = pack_bf16x2(acc_o[ct][4 * g + 2] * inv, acc_o[ct][4 * g + 3] * inv);
                *reinterpret_cast<uint2 *>(op + c) = w;
            }
    }
}

// vT[s][kvh][c][pi(i)] = qkv[s*N + i][(H + Hkv + kvh)*dh + c], 64x64 tiles through LDS.  Rows of vT (stride ld_vt)
// hold N rounded up to 64 keys, the tail zero.  Inside every group of 16 keys the order is 0-3, 8-11, 4-7, 12-15: the
// contraction-slot order of the second attention MFMA, so that a lane's 8 values are one 16-byte piece.
__device__ __forceinline__ void transpose_v_tile(const bf16_t *__restrict__ qkv, int ld_qkv, int N, int n_heads, int n_kv_heads,
                                                 int d_head, bf16_t *__restrict__ vT, int ld_vt, int i0, int cg, int s) {
    __shared__ uint16_t tile[64][66];
    const int row_w = ld_qkv;
    const int col0 = cg * 64;                                          // within the V part; cg indexes 64-wide column groups of all KV heads
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int r = ty; r < 64; r += 4) {
        const int i = i0 + r;
        tile[r][tx] = (i < N) ? qkv[((int64_t)s * N + i) * row_w + (n_heads + n_kv_heads) * d_head + col0 + tx].bits : 0;
    }
    __syncthreads();
    // destination key slot tx holds source key: swap the middle two 4-key pieces of each 16-group
    const int piece = (tx >> 2) & 3;
    const int src_key = (tx & ~15) | ((((piece & 1) << 1) | (piece >> 1)) << 2) | (tx & 3);
    for (int r = ty; r < 64; r += 4) {
        const int c = col0 + r;   // = kvh * d_head + channel
        vT[((int64_t)s * n_kv_heads * d_head + c) * ld_vt + i0 + tx].bits = tile[src_key][r];
    }
}

__global__ __launch_bounds__(256) void transpose_v_kernel(const bf16_t *__restrict__ qkv, int ld_qkv, int N, int n_heads,
                                                          int n_kv_heads, int d_head, bf16_t *__restrict__ vT, int ld_vt) {
    transpose_v_tile(qkv, ld_qkv, N, n_heads, n_kv_heads, d_head, vT, ld_vt, blockIdx.x * 64, blockIdx.y, blockIdx.z);
}

// Rotary on the q and k heads and the transpose of V touch disjoint columns of the same qkv rows: one launch does
// both.  Workgroups [0, tokens) rotate one token each, the rest move one 64x64 tile of V (tile index: key tile
// fastest, then column group, then sequence).
__global__ __launch_bounds__(256) void rope_transpose_v_kernel(bf16_t *__restrict__ qkv, int ld_qkv, int N, int pos0, int n_heads,
                                                               int n_kv_heads, int d_head, const float *__restrict__ cos_t,
                                                               const float *__restrict__ sin_t, bf16_t *__restrict__ vT, int ld_vt,
                                                               int tokens, int tiles_i, int tiles_c) {
    if ((int)blockIdx.x < tokens) {
        const int64_t t = blockIdx.x;
        rope_bf16_vec_token(qkv + t * (int64_t)ld_qkv, pos0 + (int)(t % N), n_heads, n_kv_heads, d_head, cos_t, sin_t);
    } else {
        const int idx = (int)blockIdx.x - tokens;
        transpose_v_tile(qkv, ld_qkv, N, n_heads, n_kv_heads, d_head, vT, ld_vt, (idx % tiles_i) * 64, (idx / tiles_i) % tiles_c,
                         idx / (tiles_i * tiles_c));
    }
}

}   // namespace

void launch_transpose_v(const bf16_t *qkv, int ld_qkv, int S, int N, int n_heads, int n_kv_heads, int d_head, bf16_t *vT,
                        hipStream_t st) {
    const int N_pad = (N + 63) / 64 * 64;
    hipLaunchKernelGGL(transpose_v_kernel, dim3(N_pad / 64, n_kv_heads * d_head / 64, S), dim3(256), 0, st, qkv, ld_qkv, N,
                       n_heads, n_kv_heads, d_head, vT, (int)vt_row_stride(N));
}

void launch_rope_transpose_v(bf16_t *qkv, int ld_qkv, int S, int N, int pos0, int n_heads, int n_kv_heads, int d_head,
                             const float *cos_t, const float *sin_t, bf16_t *vT, hipStream_t st) {
    const int tiles_i = (N + 63) / 64, tiles_c = n_kv_heads * d_head / 64, tokens = S * N;
    hipLaunchKernelGGL(rope_transpose_v_kernel, dim3((unsigned)(tokens + tiles_i * tiles_c * S)), dim3(256), 0, st, qkv, ld_qkv, N,
                       pos0, n_heads, n_kv_heads, d_head, cos_t, sin_t, vT, (int)vt_row_stride(N), tokens, tiles_i, tiles_c);
}

template <int DH, int NW, int NSTG, int KSP = 1>
static void launch_att(const bf16_t *qkv, int ld_qkv, const bf16_t *vT, int S, int N, int n_heads, int n_kv_heads, bf16_t *out,
                       const KvPrefix &pre, hipStream_t st) {
    constexpr int smem = KSP * NSTG * (BKV * DH * 2 + DH * BKV * 2);
    static_assert(smem <= 160 * 1024, "LDS rings exceed the 160 KB of a CU");
    static_assert(KSP == 1 || (2 + DH / 32 * 16) * 64 * 4 <= NSTG * (BKV * DH * 2 + DH * BKV * 2), "merge data fit a ring");
    auto kern = attention_kernel<DH, NW, NSTG, KSP>;
    static std::atomic<uint64_t> lds_raised{0};   // one per instantiation
    ensure_dynamic_lds(reinterpret_cast<const void *>(kern), smem, lds_raised);
    constexpr int q_per_wg = KSP > 1 ? 32 : 32 * NW;
    dim3 grid((N + q_per_wg - 1) / q_per_wg, n_heads, S);
    hipLaunchKernelGGL(kern, grid, dim3(NW * 64), smem, st, qkv, ld_qkv, vT, (int)vt_row_stride(N), N, n_heads, n_kv_heads, out,
                       pre);
}

// LDS ring depth of the K / V^T tiles; deeper rings (3, 4 stages) were measured 3-7 % slower: the kernel is not
// bound by fetch latency
constexpr int NSTG = 2;
void launch_attention_bf16(const bf16_t *qkv, int ld_qkv, const bf16_t *vT, int S, int N, int n_heads, int n_kv_heads, int d_head,
                           bf16_t *out, const KvPrefix &pre, hipStream_t st) {
    // 128 queries per workgroup when that still gives two workgroups per CU, else 64; a single block of 32
    // queries (block-row path) is split along the keys over as many wavefronts as have room for a ring each
    const int64_t blocks128 = (int64_t)((N + 127) / 128) * n_heads * S;
    const bool small = blocks128 < 512;
    if (d_head == 128) {
        if (N <= 32) launch_att<128, 2, NSTG, 2>(qkv, ld_qkv, vT, S, N, n_heads, n_kv_heads, out, pre, st);
        else if (small) launch_att<128, 2, NSTG>(qkv, ld_qkv, vT, S, N, n_heads, n_kv_heads, out, pre, st);
        else launch_att<128, 4, NSTG>(qkv, ld_qkv, vT, S, N, n_heads, n_kv_heads, out, pre, st);
    } else {
        if (N <= 32) launch_att<64, 4, NSTG, 4>(qkv, ld_qkv, vT, S, N, n_heads, n_kv_heads, out, pre, st);
        else if (small) launch_att<64, 2, NSTG>(qkv, ld_qkv, vT, S, N, n_heads, n_kv_heads, out, pre, st);
        else launch_att<64, 4, NSTG>(qkv, ld_qkv, vT, S, N, n_heads, n_kv_heads, out, pre, st);
    }
}
