// Decode-size projections with everything that follows them fused into the epilogue
// (the q/k/v and output projections of the policy pi_theta, Section 3.1, for batches of up to 512 rows):
//
//   skinny_qkv   q/k/v = A W^T, rotary positions applied to q and k, q written in the activation type,
//                k and v appended to the paged cache             (one launch instead of GEMM + RoPE/append)
//   skinny_o     h += A W^T, plus the new residual row times the next RMSNorm's gain in the activation type
//                and the per-row sums of squares that norm needs: the projection behind it multiplies by
//                rsqrt(mean h^2 + eps) in its own epilogue, (h g rs) W^T = rs ((h g) W^T)
//                                                                 (one launch instead of GEMM + RMSNorm)
//
// C[M,N] = A[M,K] W[N,K]^T with N of a few thousand and K of a few thousand: 5-40 MB of weights, a handful of
// microseconds.  A block owns a 64 x 32 output tile over the WHOLE of K, so no partial sums ever leave the
// block; its four waves each take a quarter of K and add up through LDS at the end.  Every wave runs its own
// pipeline without any block barrier: 64-deep K steps of its quarter go global memory -> LDS directly
// (global_load_lds, 16 bytes per lane, whole 128-byte rows per eight lanes: fragment loads straight from
// global memory would ask the load unit for 64 separate 16-byte pieces per instruction and are bound by its
// request rate), three steps in flight, XOR-swizzled so that the 16-byte fragment reads hit distinct banks.
// The m blocks that share a weight strip run back to back on one die.
#include "pc_internal.h"

namespace pc {

static constexpr int SK_BM = 64, SK_BN = 32, SK_WAVES = 4;
static constexpr int SK_BK = 64, SK_NS = 3;                            // K step, steps in flight per wave
static constexpr int SK_STEP_ELEMS = (SK_BM + SK_BN) * SK_BK;          // one step of one wave: A rows, then W rows
static constexpr int SK_LOADS = (SK_BM + SK_BN) / 8;                   // wave-wide 1 KB loads per step (8 rows each)
static constexpr size_t SK_SMEM = (size_t)SK_WAVES * SK_NS * SK_STEP_ELEMS * 2;   // 144 KB of 16-bit elements
static constexpr int SK_STRIDE = 36;                                   // LDS row stride of the wave partials (floats)

typedef __attribute__((ext_vector_type(4))) uint32_t sk_u32x4;

struct SkinnyQkv {
    const int32_t *row_slot, *slot_len;
    const float *rope_cos, *rope_sin;
    KvGeom kv;
    int layer, hq;
    void *q_out;
};
struct SkinnyO {
    float *h;        // fp32 residual stream [M, N], updated in place
    const float *gain;   // [N]: gain of the RMSNorm that follows
    void *h_act;     // the new rows times that gain, in the activation type [M, N] (the norm's scale comes later)
    float *ssq;      // [N / 32][M]: sum of squares of the new row over this block's 32 columns
};

template <typename T> __device__ inline typename Mma<T>::frag sk_ld(const T *p) {
    return __builtin_bit_cast(typename Mma<T>::frag, *(const sk_u32x4 *)p);
}

// MODE 0: q/k/v + RoPE + append (weights rows of every q and k head permuted so that a 32-column block holds
//         16 dims of the first half of the head and their 16 rotation partners, see pack_qkv_rows)
// MODE 1: residual update + activation copy + sums of squares
template <typename T, int MODE>
__global__ __launch_bounds__(64 * SK_WAVES) void gemm_skinny_kernel(const T *__restrict__ A, const T *__restrict__ W,
                                                                  int M, int N, int K, int mb, int nb, SkinnyQkv qa,
                                                                  SkinnyO oa, uint32_t *__restrict__ sat) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char sk_smem[];
    const int id = blockIdx.x, die = id % 8, j = id / 8;
    const int bn = (j / mb) * 8 + die;
    if (bn >= nb) return;
    const int bm = j % mb;
    const int m0 = bm * SK_BM, n0 = bn * SK_BN;
    const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64, i = lane % 16, g = lane / 16;
    const int steps = K / (SK_BK * SK_WAVES);          // K steps of 64 per wave
    const int kwave = wave * steps * SK_BK;
    T *ring = (T *)sk_smem + (size_t)wave * SK_NS * SK_STEP_ELEMS;     // this wave's own stages

    // ---- global -> LDS: a wave-wide load fills 8 rows of 64 k; lane -> (row lr, 16-byte slot); slot c of row r
    // receives chunk c ^ swz(r), swz(r) = (r / 2) & 7
    const int lr = lane / 8, lslot = lane % 8;
    const T *src[SK_LOADS];
#pragma unroll
    for (int l = 0; l < SK_LOADS; ++l) {
        const int row = 8 * l + lr;                    // rows 0..63: A, 64..95: W
        const int chunk = lslot ^ ((row / 2) & 7);
        src[l] = (row < SK_BM ? A + (int64_t)min(m0 + row, M - 1) * K : W + (int64_t)(n0 + row - SK_BM) * K) + kwave +
                 chunk * 8;
    }
    auto issue = [&](int st, int stage) {
        const int koff = min(st, steps - 1) * SK_BK;   // past the end: a redundant reload that keeps the count constant
        T *dst = ring + stage * SK_STEP_ELEMS;
#pragma unroll
        for (int l = 0; l < SK_LOADS; ++l)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src[l] + koff),
                                             (__attribute__((address_space(3))) void *)(dst + 8 * l * SK_BK), 16, 0, 0);
    };

    typedef typename Mma<T>::frag frag_t;
    f32x4_t acc[4][2];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) acc[mt][nt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};

    // fragment addressing: lane (i, g) reads chunk 4 kk + g of row 16 t + i, stored at slot chunk ^ swz(row)
    int foff[6][2];
#pragma unroll
    for (int t = 0; t < 6; ++t) {
        const int row = 16 * t + i;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) foff[t][kk] = row * SK_BK + (((4 * kk + g) ^ ((row / 2) & 7)) * 8);
    }

#pragma unroll
    for (int st = 0; st < SK_NS - 1; ++st) issue(st, st);
    int stage = 0;
    for (int st = 0; st < steps; ++st) {
        const int refill = (stage == 0) ? SK_NS - 1 : stage - 1;   // consumed in the previous iteration
        issue(st + SK_NS - 1, refill);
        // at most the loads of the two younger steps are still in flight: this step has landed in LDS
        __builtin_amdgcn_s_waitcnt((((SK_NS - 1) * SK_LOADS) & 0xF) | ((((SK_NS - 1) * SK_LOADS) >> 4) << 14) | (0x7 << 4) |
                                   (0xF << 8));
        asm volatile("" ::: "memory");
        const T *base = ring + stage * SK_STEP_ELEMS;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            frag_t fa[4], fb[2];
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) fa[mt] = *(const frag_t *)(base + foff[mt][kk]);
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) fb[nt] = *(const frag_t *)(base + foff[4 + nt][kk]);
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int nt = 0; nt < 2; ++nt) acc[mt][nt] = Mma<T>::m16(fa[mt], fb[nt], acc[mt][nt]);
        }
        asm volatile("" ::: "memory");
        stage = (stage + 1 == SK_NS) ? 0 : stage + 1;
    }
    __builtin_amdgcn_s_waitcnt((0x7 << 4) | (0xF << 8));   // vmcnt(0): nothing may still be writing LDS
    __syncthreads();                                       // every wave is done with its stages: reuse them
    float (*part)[SK_BM][SK_STRIDE] = (float (*)[SK_BM][SK_STRIDE])sk_smem;

    // ---- the four K quarters meet in LDS: acc[mt][nt][v] is C[16 mt + 4 g + v][16 nt + i] of the tile
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int v = 0; v < 4; ++v) part[wave][16 * mt + 4 * g + v][16 * nt + i] = acc[mt][nt][v];
    __syncthreads();
    // thread -> row r of the tile, columns 8 cg .. 8 cg + 7
    const int r = tid / 4, cg = tid % 4, row = m0 + r;
    float v8[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        float s = part[0][r][8 * cg + e];
#pragma unroll
        for (int w = 1; w < SK_WAVES; ++w) s += part[w][r][8 * cg + e];   // fixed order: deterministic
        v8[e] = s;
    }
    const bool live = row < M;

    if (MODE == 1) {
        float ss = 0.f;
        if (live) {
            float *hp = oa.h + (int64_t)row * N + n0 + 8 * cg;
            float4 h0 = ((float4 *)hp)[0], h1 = ((float4 *)hp)[1];
            h0.x += v8[0]; h0.y += v8[1]; h0.z += v8[2]; h0.w += v8[3];
            h1.x += v8[4]; h1.y += v8[5]; h1.z += v8[6]; h1.w += v8[7];
            ((float4 *)hp)[0] = h0;
            ((float4 *)hp)[1] = h1;
            const float4 g0 = ((const float4 *)(oa.gain + n0 + 8 * cg))[0], g1 = ((const float4 *)(oa.gain + n0 + 8 * cg))[1];
            sk_u32x4 pk = {pack2_sat<T>(h0.x * g0.x, h0.y * g0.y, sat), pack2_sat<T>(h0.z * g0.z, h0.w * g0.w, sat),
                           pack2_sat<T>(h1.x * g1.x, h1.y * g1.y, sat), pack2_sat<T>(h1.z * g1.z, h1.w * g1.w, sat)};
            *(sk_u32x4 *)((T *)oa.h_act + (int64_t)row * N + n0 + 8 * cg) = pk;
            ss = h0.x * h0.x + h0.y * h0.y + h0.z * h0.z + h0.w * h0.w + h1.x * h1.x + h1.y * h1.y + h1.z * h1.z +
                 h1.w * h1.w;
        }
        ss += __shfl_xor(ss, 1, 64);
        ss += __shfl_xor(ss, 2, 64);
        if (live && cg == 0) oa.ssq[(int64_t)bn * M + row] = ss;
        return;
    }

    // ---- MODE 0: which part of the q | k | v row this block holds (block-uniform)
    const int hd = qa.kv.head_dim, half = hd / 2;          // hd = 128 here
    const int qd = qa.hq * hd, kvd = qa.kv.n_kv_heads * hd;
    // the rotation partner of this thread's 8 values sits two threads further (cg ^ 2): exchange first, every
    // lane takes part
    float p8[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) p8[e] = __shfl_xor(v8[e], 2, 64);
    if (!live) return;
    const int slot = qa.row_slot[row];
    const int pos = qa.slot_len[slot];
    if (n0 < qd + kvd) {   // a q or k head: rotate
        const bool is_q = n0 < qd;
        const int c0 = is_q ? n0 : n0 - qd;
        const int head = c0 / hd, b = (c0 % hd) / 32;
        const int jj = 16 * b + 8 * (cg & 1);                  // first of this thread's 8 pair indices
        const float4 *cp = (const float4 *)(qa.rope_cos + (int64_t)pos * half + jj);
        const float4 *sp = (const float4 *)(qa.rope_sin + (int64_t)pos * half + jj);
        const float4 c_lo = cp[0], c_hi = cp[1], s_lo = sp[0], s_hi = sp[1];
        const float cs[8] = {c_lo.x, c_lo.y, c_lo.z, c_lo.w, c_hi.x, c_hi.y, c_hi.z, c_hi.w};
        const float sn[8] = {s_lo.x, s_lo.y, s_lo.z, s_lo.w, s_hi.x, s_hi.y, s_hi.z, s_hi.w};
        float o8[8];
#pragma unroll
        for (int e = 0; e < 8; ++e)
            o8[e] = (cg < 2) ? (v8[e] * cs[e] - p8[e] * sn[e])      // x1' = x1 cos - x2 sin
                             : (v8[e] * cs[e] + p8[e] * sn[e]);     // x2' = x2 cos + x1 sin
        const int dim = jj + (cg < 2 ? 0 : half);
        sk_u32x4 pk = {pack2_sat<T>(o8[0], o8[1], sat), pack2_sat<T>(o8[2], o8[3], sat), pack2_sat<T>(o8[4], o8[5], sat),
                       pack2_sat<T>(o8[6], o8[7], sat)};
        if (is_q) {
            *(sk_u32x4 *)((T *)qa.q_out + ((int64_t)row * qa.hq + head) * hd + dim) = pk;
        } else {
            const int bs = qa.kv.block_size;
            const int blk = qa.kv.block_table[(int64_t)slot * qa.kv.max_blocks_per_slot + pos / bs];
            T *kd = (T *)qa.kv.pool + (int64_t)qa.layer * qa.kv.layer_stride + (int64_t)blk * qa.kv.block_elems() +
                    (int64_t)head * qa.kv.head_elems() + qa.kv.k_index(pos % bs, dim);   // 8 dims: 16 contiguous bytes
            *(sk_u32x4 *)kd = pk;
        }
    } else {               // a v head
        const int c0 = n0 - qd - kvd;
        const int head = c0 / hd, d0 = c0 % hd + 8 * cg;
        const int bs = qa.kv.block_size;
        const int blk = qa.kv.block_table[(int64_t)slot * qa.kv.max_blocks_per_slot + pos / bs];
        T *vd = (T *)qa.kv.pool + (int64_t)qa.layer * qa.kv.layer_stride + (int64_t)blk * qa.kv.block_elems() +
                (int64_t)head * qa.kv.head_elems();
#pragma unroll
        for (int e = 0; e < 8; ++e) vd[qa.kv.v_index(pos % bs, d0 + e)] = from_f32_sat<T>(v8[e], sat);
    }
}

bool skinny_ok(int M, int N, int K, int head_dim) {
    return M > 0 && M <= 512 && N % SK_BN == 0 && K % (SK_BK * SK_WAVES) == 0 && head_dim == 128;
}

void skinny_init() {   // once per process: the kernels use more dynamic LDS than the default limit
    (void)hipFuncSetAttribute((const void *)gemm_skinny_kernel<bf16_t, 0>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)SK_SMEM);
    (void)hipFuncSetAttribute((const void *)gemm_skinny_kernel<bf16_t, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)SK_SMEM);
    (void)hipFuncSetAttribute((const void *)gemm_skinny_kernel<f16_t, 0>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)SK_SMEM);
    (void)hipFuncSetAttribute((const void *)gemm_skinny_kernel<f16_t, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)SK_SMEM);
}

template <typename T, int MODE>
static void skinny_launch(const void *A, const void *W, int M, int N, int K, const SkinnyQkv &qa, const SkinnyO &oa,
                          uint32_t *sat, hipStream_t s) {
    const int mb = (M + SK_BM - 1) / SK_BM, nb = N / SK_BN;
    const unsigned grid = (unsigned)((nb + 7) / 8 * 8 * mb);
    gemm_skinny_kernel<T, MODE><<<grid, 64 * SK_WAVES, SK_SMEM, s>>>((const T *)A, (const T *)W, M, N, K, mb, nb, qa, oa, sat);
}

void launch_skinny_qkv(int dtype, const void *A, const void *W, int M, int K, const int32_t *row_slot,
                       const int32_t *slot_len, const float *rope_cos, const float *rope_sin, int hq, KvGeom kv, int layer,
                       void *q_out, uint32_t *sat, hipStream_t s) {
    SkinnyQkv qa{row_slot, slot_len, rope_cos, rope_sin, kv, layer, hq, q_out};
    SkinnyO oa{nullptr, nullptr, nullptr, nullptr};
    const int N = (hq + 2 * kv.n_kv_heads) * kv.head_dim;
    if (dtype == KD_BF16) skinny_launch<bf16_t, 0>(A, W, M, N, K, qa, oa, sat, s);
    else skinny_launch<f16_t, 0>(A, W, M, N, K, qa, oa, sat, s);
}

void launch_skinny_o(int dtype, const void *A, const void *W, int M, int N, int K, float *h, const float *gain, void *h_act,
                     float *ssq, uint32_t *sat, hipStream_t s) {
    SkinnyQkv qa{};
    SkinnyO oa{h, gain, h_act, ssq};
    if (dtype == KD_BF16) skinny_launch<bf16_t, 1>(A, W, M, N, K, qa, oa, sat, s);
    else skinny_launch<f16_t, 1>(A, W, M, N, K, qa, oa, sat, s);
}

}  // namespace pc
