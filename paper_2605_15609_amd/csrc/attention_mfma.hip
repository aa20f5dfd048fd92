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
// One workgroup = 4 wavefronts = 128 queries of one (sequence, head); K and V^T tiles of
// 64 keys are staged through double-buffered, XOR-swizzled LDS.  Grouped KV heads: the
// query heads of a group simply read the same K / V^T tiles (they hit L2).
#include "psd_internal.h"
#include "device_types.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BQ = 128;    // queries per workgroup
constexpr int BKV = 64;    // keys per stage

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 u) { return __builtin_bit_cast(bf16x8, u); }

template <int DH>
__global__ __launch_bounds__(256) void attention_kernel(const bf16_t *__restrict__ qkv, const bf16_t *__restrict__ vT, int N,
                                                        int n_heads, int n_kv_heads, bf16_t *__restrict__ out) {
    constexpr int KROW = DH * 2;                 // bytes per K row in LDS
    constexpr int K_BYTES = BKV * KROW;
    constexpr int VROW = BKV * 2;                // bytes per V^T row in LDS (128)
    constexpr int V_BYTES = DH * VROW;
    constexpr int STAGE = K_BYTES + V_BYTES;
    constexpr int KCH = BKV * (DH / 8) / 256;    // 16-byte chunks per thread, K tile
    constexpr int VCH = DH * 8 / 256;            // 16-byte chunks per thread, V^T tile
    constexpr int CT = DH / 32;                  // output subtiles along the head dimension
    constexpr int KS = DH / 16;                  // k-steps of the score contraction
    __shared__ __align__(16) unsigned char lds[2 * STAGE];

    const int q0 = blockIdx.x * BQ, head = blockIdx.y, s = blockIdx.z;
    const int kvh = head / (n_heads / n_kv_heads);
    const int row_w = (n_heads + 2 * n_kv_heads) * DH;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lrow = lane & 31, lhalf = lane >> 5;
    const bf16_t *seq = qkv + (int64_t)s * N * row_w;
    const bf16_t *vt_head = vT + ((int64_t)s * n_kv_heads + kvh) * DH * (int64_t)N;
    const uint4 zero4 = make_uint4(0, 0, 0, 0);

    // Q fragments: lane (q = lrow, half) holds Q[q][16*ks + 8*half .. +7]
    bf16x8 qf[KS];
    {
        const int q = q0 + wave * 32 + lrow;
        const bf16_t *qp = seq + (int64_t)q * row_w + head * DH;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            u32x4 t = {0u, 0u, 0u, 0u};
            if (q < N) t = *reinterpret_cast<const u32x4 *>(qp + ks * 16 + lhalf * 8);
            qf[ks] = as_bf16x8(t);
        }
    }

    uint4 rk[KCH], rv[VCH];
// global -> registers for the key tile starting at k0 (keys past the end read as zero)
#define PSD_ATT_LOAD_GLOBAL(k0)                                                                                  \
    {                                                                                                            \
        _Pragma("unroll") for (int i = 0; i < KCH; ++i) {                                                        \
            const int qd = i * 256 + tid, r = qd / (DH / 8), c = qd % (DH / 8);                                  \
            const int key = (k0) + r;                                                                            \
            rk[i] = zero4;                                                                                       \
            if (key < N)                                                                                         \
                rk[i] = *reinterpret_cast<const uint4 *>(seq + (int64_t)key * row_w + (n_heads + kvh) * DH + c * 8); \
        }                                                                                                        \
        _Pragma("unroll") for (int i = 0; i < VCH; ++i) {                                                        \
            const int qd = i * 256 + tid, r = qd >> 3, c = qd & 7;                                               \
            const int key = (k0) + c * 8;                                                                        \
            rv[i] = zero4;                                                                                       \
            if (key < N) rv[i] = *reinterpret_cast<const uint4 *>(vt_head + (int64_t)r * N + key);               \
        }                                                                                                        \
    }
// registers -> LDS.  V^T chunk c holds keys 8c..8c+7 of a row; keys 4w..4w+3 of each 8-key half u of a
// 16-key group kg go to chunk (2*kg + w), 8-byte slot u: the permuted key order of the second MFMA
#define PSD_ATT_STORE_LDS(stage)                                                                                 \
    {                                                                                                            \
        unsigned char *sk_ = lds + (stage) * STAGE, *sv_ = sk_ + K_BYTES;                                        \
        _Pragma("unroll") for (int i = 0; i < KCH; ++i) {                                                        \
            const int qd = i * 256 + tid, r = qd / (DH / 8), c = qd % (DH / 8);                                  \
            *reinterpret_cast<uint4 *>(sk_ + r * KROW + ((c ^ ((r >> 1) & 7)) << 4)) = rk[i];                           \
        }                                                                                                        \
        _Pragma("unroll") for (int i = 0; i < VCH; ++i) {                                                        \
            const int qd = i * 256 + tid, r = qd >> 3, c = qd & 7;                                               \
            const int kg = c >> 1, u = c & 1;                                                                    \
            *reinterpret_cast<uint2 *>(sv_ + r * VROW + (((kg * 2 + 0) ^ ((r >> 1) & 7)) << 4) + u * 8) =               \
                make_uint2(rv[i].x, rv[i].y);                                                                    \
            *reinterpret_cast<uint2 *>(sv_ + r * VROW + (((kg * 2 + 1) ^ ((r >> 1) & 7)) << 4) + u * 8) =               \
                make_uint2(rv[i].z, rv[i].w);                                                                    \
        }                                                                                                        \
    }

    floatx16 acc_o[CT];
#pragma unroll
    for (int i = 0; i < CT; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc_o[i][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const float sl2 = 1.4426950408889634f / sqrtf((float)DH);   // softmax scale folded into exp2

    const int n_tiles = (N + BKV - 1) / BKV;
    PSD_ATT_LOAD_GLOBAL(0)
    PSD_ATT_STORE_LDS(0)
    __syncthreads();

    for (int t = 0; t < n_tiles; ++t) {
        const int stage = t & 1, k0 = t * BKV;
        if (t + 1 < n_tiles) PSD_ATT_LOAD_GLOBAL(k0 + BKV)
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
                const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(sk + r * KROW + ((c ^ ((r >> 1) & 7)) << 4));
                acc_s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], acc_s[kt], 0, 0, 0);
            }
        }
        // keys past the end of the sequence do not exist
        if (k0 + BKV > N) {
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = k0 + kt * 32 + 8 * (v >> 2) + 4 * lhalf + (v & 3);
                    if (key >= N) acc_s[kt][v] = -INFINITY;
                }
        }
        // online softmax for this lane's query
        float mx = acc_s[0][0];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, acc_s[kt][v]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run, mx);
        const float alpha = exp2f((m_run - m_new) * sl2);
        float psum = 0.f;
        bf16x8 pf[4];   // P^T as B operands, one per group of 16 keys
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            float p[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                p[v] = exp2f((acc_s[kt][v] - m_new) * sl2);
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
        // O^T += V^T P^T
#pragma unroll
        for (int kg = 0; kg < 4; ++kg) {
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                const int r = ct * 32 + lrow;
                const int c = kg * 2 + lhalf;
                const bf16x8 vf = *reinterpret_cast<const bf16x8 *>(sv + r * VROW + ((c ^ ((r >> 1) & 7)) << 4));
                acc_o[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kg], acc_o[ct], 0, 0, 0);
            }
        }
        if (t + 1 < n_tiles) PSD_ATT_STORE_LDS(stage ^ 1)
        __syncthreads();
    }

#undef PSD_ATT_LOAD_GLOBAL
#undef PSD_ATT_STORE_LDS
    // the two half-waves of a query hold disjoint key subsets of the sum
    l_run += __shfl_xor(l_run, 32, 64);
    const float inv = 1.0f / l_run;
    const int q = q0 + wave * 32 + lrow;
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

// vT[s][kvh][c][i] = qkv[s*N + i][(H + Hkv + kvh)*dh + c], 64x64 tiles through LDS
__global__ __launch_bounds__(256) void transpose_v_kernel(const bf16_t *__restrict__ qkv, int N, int n_heads, int n_kv_heads,
                                                          int d_head, bf16_t *__restrict__ vT) {
    __shared__ uint16_t tile[64][66];
    const int i0 = blockIdx.x * 64, cg = blockIdx.y, s = blockIdx.z;   // cg indexes 64-wide column groups of all KV heads
    const int row_w = (n_heads + 2 * n_kv_heads) * d_head;
    const int col0 = cg * 64;                                          // within the V part
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int r = ty; r < 64; r += 4) {
        const int i = i0 + r;
        tile[r][tx] = (i < N) ? qkv[((int64_t)s * N + i) * row_w + (n_heads + n_kv_heads) * d_head + col0 + tx].bits : 0;
    }
    __syncthreads();
    for (int r = ty; r < 64; r += 4) {
        const int c = col0 + r;   // = kvh * d_head + channel
        const int i = i0 + tx;
        if (i < N) vT[((int64_t)s * n_kv_heads * d_head + c) * N + i].bits = tile[tx][r];
    }
}

}   // namespace

void launch_transpose_v(const bf16_t *qkv, int S, int N, int n_heads, int n_kv_heads, int d_head, bf16_t *vT,
                        hipStream_t st) {
    hipLaunchKernelGGL(transpose_v_kernel, dim3((N + 63) / 64, n_kv_heads * d_head / 64, S), dim3(256), 0, st, qkv, N,
                       n_heads, n_kv_heads, d_head, vT);
}

void launch_attention_bf16(const bf16_t *qkv, const bf16_t *vT, int S, int N, int n_heads, int n_kv_heads, int d_head,
                           bf16_t *out, hipStream_t st) {
    dim3 grid((N + BQ - 1) / BQ, n_heads, S);
    if (d_head == 128)
        hipLaunchKernelGGL(attention_kernel<128>, grid, dim3(256), 0, st, qkv, vT, N, n_heads, n_kv_heads, out);
    else
        hipLaunchKernelGGL(attention_kernel<64>, grid, dim3(256), 0, st, qkv, vT, N, n_heads, n_kv_heads, out);
}
