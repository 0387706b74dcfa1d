// Grouped-query causal attention over the paged KV cache (the attention of the
// policy pi_theta(o_t | q, o_<t), Section 3.1).
//
//   attention_simt_kernel      plain ALU, any dtype / head_dim <= 256: the fp32 model path
//   attention_prefill_mfma     bf16, head_dim 128: 16 query positions of one head per wave
//   attention_decode_mfma      bf16, head_dim 128: the query heads that share a kv head (<= 16)
//                              of one sequence per block, split over the context, + merge pass
//
// The matrix-core kernels share one inner loop.  Per 32-token tile it forms
//   S^T[token][column] = K[token][:] . Q[column][:]      (two 16x16x32 products per 32 of head_dim)
//   O[column][:]      += P[column][token] V[token][:]    (eight 16x16x32 products)
// where a "column" is a query row: a head (decode) or a position (prefill).
// Inside each block K and V are stored in the order of the products' operand
// fragments (KvGeom), so both products read 16 contiguous bytes per lane and one
// contiguous kilobyte per wave straight from global memory; no LDS staging is
// needed because every K/V byte is used by exactly one wave.
#include <algorithm>

#include "pc_internal.h"

namespace pc {

static constexpr int WAVE = 64;

__device__ inline float wave_max_f(float v) {
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
    return v;
}
__device__ inline float wave_sum_f(float v) {
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}

// =====================================================================================
// plain-ALU attention: one wave per (row, query head)
// =====================================================================================
template <typename T>
__global__ __launch_bounds__(64) void attention_simt_kernel(const T *__restrict__ q,
                                                            const int32_t *__restrict__ row_slot,
                                                            const int32_t *__restrict__ row_pos,
                                                            const int32_t *__restrict__ slot_len, int hq, KvGeom kv,
                                                            int layer, T *__restrict__ out, uint32_t *__restrict__ sat) {
    __shared__ float qs[256];
    __shared__ float ps[WAVE];
    const int head = blockIdx.x, r = blockIdx.y, lane = threadIdx.x;
    const int hd = kv.head_dim, bs = kv.block_size;
    const int slot = row_slot[r];
    const int pos = row_pos ? row_pos[r] : slot_len[slot];
    const int ctx = pos + 1;
    const int g = head / (hq / kv.n_kv_heads);
    const float scale = 1.0f / sqrtf((float)hd);
    for (int i = lane; i < hd; i += WAVE) qs[i] = to_f32(q[((int64_t)r * hq + head) * hd + i]) * scale;
    __syncthreads();
    const T *base = (const T *)kv.pool + (int64_t)layer * kv.layer_stride + (int64_t)g * kv.head_elems();
    const int32_t *table = kv.block_table + (int64_t)slot * kv.max_blocks_per_slot;
    float m = -INFINITY, l = 0.f;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int c0 = 0; c0 < ctx; c0 += WAVE) {
        const int key = c0 + lane;
        float s = -INFINITY;
        if (key < ctx) {
            const T *kp = base + (int64_t)table[key / bs] * kv.block_elems();
            float d = 0.f;
            for (int i = 0; i < hd; ++i) d = fmaf(qs[i], to_f32(kp[kv.k_index(key % bs, i)]), d);
            s = d;
        }
        const float m_new = fmaxf(m, wave_max_f(s));
        const float p = (key < ctx) ? expf(s - m_new) : 0.f;
        const float corr = expf(m - m_new);
        l = l * corr + wave_sum_f(p);
        m = m_new;
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] *= corr;
        ps[lane] = p;
        __syncthreads();
        const int nk = min(WAVE, ctx - c0);
        for (int j = 0; j < nk; ++j) {
            const int kj = c0 + j;
            const T *vp = base + (int64_t)table[kj / bs] * kv.block_elems();
            const float pj = ps[j];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int c = lane + WAVE * i;
                if (c < hd) acc[i] = fmaf(pj, to_f32(vp[kv.v_index(kj % bs, c)]), acc[i]);
            }
        }
        __syncthreads();
    }
    const float inv = 1.0f / l;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int c = lane + WAVE * i;
        if (c < hd) out[((int64_t)r * hq + head) * hd + c] = from_f32_sat<T>(acc[i] * inv, sat);
    }
}

void launch_attention_simt(int dtype, const void *q, const int32_t *row_slot, const int32_t *row_pos,
                           const int32_t *slot_len, int rows, int hq, KvGeom kv, int layer, void *out,
                           uint32_t *sat, hipStream_t s) {
    if (rows <= 0) return;
    dim3 grid(hq, rows);
    if (dtype == KD_F32)
        attention_simt_kernel<float><<<grid, 64, 0, s>>>((const float *)q, row_slot, row_pos, slot_len, hq, kv, layer,
                                                         (float *)out, sat);
    else if (dtype == KD_BF16)
        attention_simt_kernel<bf16_t><<<grid, 64, 0, s>>>((const bf16_t *)q, row_slot, row_pos, slot_len, hq, kv,
                                                          layer, (bf16_t *)out, sat);
    else
        attention_simt_kernel<f16_t><<<grid, 64, 0, s>>>((const f16_t *)q, row_slot, row_pos, slot_len, hq, kv, layer,
                                                         (f16_t *)out, sat);
}

// =====================================================================================
// matrix-core attention, head_dim = 128
// =====================================================================================
typedef f32x4_t f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

static constexpr int HD = 128;
static constexpr float LOG2E = 1.4426950408889634f;

// 16x16x32 operand layout (wave of 64 lanes, i = lane%16, g = lane/16):
//   a: A[row i][k = 8g .. 8g+7]     b: B[k = 8g .. 8g+7][col i]     d[v]: D[row 4g+v][col i]
struct AttnState {
    float m;        // running max of column lane%16 (same on the 4 lanes of a column)
    float l;        // this lane's share of the running sum of column lane%16
    f32x4 o[8];     // O[column 4g+v][16*nn + i]
};

template <typename T> __device__ inline typename Mma<T>::frag ld_frag(const T *p) {
    u32x4 t = *(const u32x4 *)p;
    return __builtin_bit_cast(typename Mma<T>::frag, t);
}
template <typename T> __device__ inline typename Mma<T>::frag zero_frag() {
    return __builtin_bit_cast(typename Mma<T>::frag, (u32x4){0, 0, 0, 0});
}

template <typename T> struct KvTile {
    typename Mma<T>::frag ka[2][4], vf[8];
};

// The K and V fragments of the 32-token tile that starts at token t0 (a multiple of 32).  The cache stores them
// fragment-major (KvGeom): every fragment is one contiguous kilobyte, lane l reads its 16 bytes at offset 16 l.
template <typename T>
__device__ inline void load_kv_tile(const T *__restrict__ head_base, int64_t block_elems,
                                    const int32_t *__restrict__ table, int bs, int t0, KvTile<T> &kt) {
    const int lane = threadIdx.x % WAVE;
    const int tile = (t0 % bs) >> 5;
    const T *kb = head_base + (int64_t)table[t0 / bs] * block_elems + lane * 8;
    const T *vb = kb + (int64_t)bs * HD;
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) kt.ka[u][kk] = ld_frag(kb + (((tile * 2 + u) * 4 + kk) << 9));
#pragma unroll
    for (int nn = 0; nn < 8; ++nn) kt.vf[nn] = ld_frag(vb + ((tile * 8 + nn) << 9));
}

// One tile's update of the running softmax state of NH query-head groups that share the kv head.
// Tokens > col_limit (this lane's column) or >= tok_end are masked.
template <typename T, int NH>
__device__ inline void attend_tile(const KvTile<T> &kt, const typename Mma<T>::frag (&qf)[NH][4], int t0, int tok_end,
                                   int col_limit, float scale_log2, AttnState (&st)[NH]) {
    const int lane = threadIdx.x % WAVE, g = lane / 16;
    bool ok[2][4];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int tok = t0 + 8 * g + 4 * u + v;
            ok[u][v] = (tok <= col_limit) && (tok < tok_end);
        }
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        f32x4 s[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            s[u] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) s[u] = Mma<T>::m16(kt.ka[u][kk], qf[h][kk], s[u]);
        }
        // lane (column i, g) holds the scores of tokens t0 + 8g + 4u + v
        float mx = -INFINITY;
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (ok[u][v]) mx = fmaxf(mx, s[u][v]);
        mx = fmaxf(mx, __shfl_xor(mx, 16, WAVE));
        mx = fmaxf(mx, __shfl_xor(mx, 32, WAVE));
        const float m_new = fmaxf(st[h].m, mx);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float corr = exp2f((st[h].m - m_use) * scale_log2);   // st.m = -inf -> 0
        float p[2][4], psum = 0.f;
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                p[u][v] = ok[u][v] ? exp2f((s[u][v] - m_use) * scale_log2) : 0.f;
                psum += p[u][v];
            }
        st[h].l = st[h].l * corr + psum;
        st[h].m = m_new;
        float c4[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) c4[v] = __shfl(corr, 4 * g + v, WAVE);
        u32x4 pw = {pack2<T>(p[0][0], p[0][1]), pack2<T>(p[0][2], p[0][3]), pack2<T>(p[1][0], p[1][1]),
                    pack2<T>(p[1][2], p[1][3])};
        const typename Mma<T>::frag pa = __builtin_bit_cast(typename Mma<T>::frag, pw);
#pragma unroll
        for (int nn = 0; nn < 8; ++nn) {
#pragma unroll
            for (int v = 0; v < 4; ++v) st[h].o[nn][v] *= c4[v];
            st[h].o[nn] = Mma<T>::m16(pa, kt.vf[nn], st[h].o[nn]);
        }
    }
}

// Consumes the 32-token tiles t0 = tile_begin, tile_begin + tile_step, ... < tok_end, for NH query-head groups
// that share the kv head: the K and V fragments of a tile are loaded once and used for every group.
// AHEAD: the next tile is requested before the current one is consumed (two fragment sets in registers);
// pays where a wave has few tiles and nothing else on its SIMD hides their latency.
template <typename T, int NH, bool AHEAD = false>
__device__ inline void attend_tiles(const T *__restrict__ head_base, int64_t block_elems,
                                    const int32_t *__restrict__ table, int bs,
                                    const typename Mma<T>::frag (&qf)[NH][4], int tile_begin, int tile_step, int tok_end,
                                    int col_limit, float scale_log2, AttnState (&st)[NH]) {
    if (AHEAD) {
        KvTile<T> a, b;
        int ta = tile_begin;
        if (ta >= tok_end) return;
        load_kv_tile<T>(head_base, block_elems, table, bs, ta, a);
        for (;;) {
            const int tb = ta + tile_step;
            if (tb < tok_end) load_kv_tile<T>(head_base, block_elems, table, bs, tb, b);
            attend_tile<T, NH>(a, qf, ta, tok_end, col_limit, scale_log2, st);
            if (tb >= tok_end) break;
            ta = tb + tile_step;
            if (ta < tok_end) load_kv_tile<T>(head_base, block_elems, table, bs, ta, a);
            attend_tile<T, NH>(b, qf, tb, tok_end, col_limit, scale_log2, st);
            if (ta >= tok_end) break;
        }
        return;
    }
    for (int t0 = tile_begin; t0 < tok_end; t0 += tile_step) {
        KvTile<T> kt;
        load_kv_tile<T>(head_base, block_elems, table, bs, t0, kt);
        attend_tile<T, NH>(kt, qf, t0, tok_end, col_limit, scale_log2, st);
    }
}

__device__ inline void state_init(AttnState &st) {
    st.m = -INFINITY;
    st.l = 0.f;
#pragma unroll
    for (int nn = 0; nn < 8; ++nn) st.o[nn] = (f32x4){0.f, 0.f, 0.f, 0.f};
}

// ---------------------------------------------------------------- prefill
// One wave per block: 16 query positions of NH query heads (that share a kv head) of one prompt; the K/V
// fragments of a tile are loaded once for the NH heads.  1-D grid laid out die by die (workgroup i runs on die
// i % 8): all blocks of a (prompt, kv head) pair -- its query-head groups times its query tiles -- run back to
// back on ONE die, so that pair's K/V is fetched from HBM once and then served from that die's L2 (the K/V
// of a whole chunk does not fit an L2, and in plain order every die would stream all of it).
template <typename T, int NH>
__global__ __launch_bounds__(64) void attention_prefill_mfma_kernel(const T *__restrict__ q,
                                                                    const int32_t *__restrict__ cu_rows,
                                                                    const int32_t *__restrict__ prompt_slot, int hq,
                                                                    KvGeom kv, int layer, int n_prompts, int n_qt,
                                                                    T *__restrict__ out, uint32_t *__restrict__ sat) {
    const int rep_h = hq / kv.n_kv_heads, items = (rep_h / NH) * n_qt;
    const int b = blockIdx.x, die = b % 8, j = b / 8;
    const int unit = (j / items) * 8 + die;                      // (prompt, kv head)
    if (unit >= n_prompts * kv.n_kv_heads) return;
    const int item = j % items;
    const int p = unit / kv.n_kv_heads;
    const int kvh = unit % kv.n_kv_heads;
    const int head0 = kvh * rep_h + (item / n_qt) * NH;          // first of this wave's NH heads
    const int q0 = (n_qt - 1 - item % n_qt) * 16;                // long causal ranges first
    const int row0 = cu_rows[p], len = cu_rows[p + 1] - row0;
    if (q0 >= len) return;
    const int lane = threadIdx.x, i = lane % 16, g = lane / 16;
    const int slot = prompt_slot[p];
    const T *head_base = (const T *)kv.pool + (int64_t)layer * kv.layer_stride + (int64_t)kvh * kv.head_elems();
    const int32_t *table = kv.block_table + (int64_t)slot * kv.max_blocks_per_slot;
    const bool col_ok = (q0 + i) < len;
    typename Mma<T>::frag qf[NH][4];
    AttnState st[NH];
#pragma unroll
    for (int h = 0; h < NH; ++h) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            if (col_ok)
                qf[h][kk] = ld_frag(q + ((int64_t)(row0 + q0 + i) * hq + head0 + h) * HD + 32 * kk + 8 * g);
            else
                qf[h][kk] = zero_frag<T>();
        }
        state_init(st[h]);
    }
    const int tok_end = min(q0 + 16, len);
    attend_tiles<T, NH>(head_base, kv.block_elems(), table, kv.block_size, qf, 0, 32, tok_end, col_ok ? q0 + i : -1,
                        LOG2E / sqrtf((float)HD), st);
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        float l = st[h].l;
        l += __shfl_xor(l, 16, WAVE);
        l += __shfl_xor(l, 32, WAVE);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int col = 4 * g + v;
            const float lc = __shfl(l, col, WAVE);
            if (q0 + col < len) {
                const float inv = 1.0f / lc;
                T *o = out + ((int64_t)(row0 + q0 + col) * hq + head0 + h) * HD;
#pragma unroll
                for (int nn = 0; nn < 8; ++nn) o[16 * nn + i] = from_f32_sat<T>(st[h].o[nn][v] * inv, sat);
            }
        }
    }
}

template <typename T, int NH>
static void prefill_launch(const void *q, const int32_t *cu_rows, const int32_t *prompt_slot, int n_prompts, int max_len,
                           int hq, KvGeom kv, int layer, void *out, uint32_t *sat, hipStream_t s) {
    const int n_qt = (max_len + 15) / 16, items = (hq / kv.n_kv_heads / NH) * n_qt;
    const int units = n_prompts * kv.n_kv_heads;
    const unsigned grid = (unsigned)((units + 7) / 8 * 8) * (unsigned)items;
    attention_prefill_mfma_kernel<T, NH><<<grid, 64, 0, s>>>((const T *)q, cu_rows, prompt_slot, hq, kv, layer, n_prompts,
                                                             n_qt, (T *)out, sat);
}

template <typename T>
static void prefill_launch_t(const void *q, const int32_t *cu_rows, const int32_t *prompt_slot, int n_prompts,
                             int max_len, int hq, KvGeom kv, int layer, void *out, uint32_t *sat, hipStream_t s) {
    const int rep = hq / kv.n_kv_heads;   // heads per wave: as many as divide the group, up to three
    if (rep % 3 == 0) prefill_launch<T, 3>(q, cu_rows, prompt_slot, n_prompts, max_len, hq, kv, layer, out, sat, s);
    else if (rep % 2 == 0) prefill_launch<T, 2>(q, cu_rows, prompt_slot, n_prompts, max_len, hq, kv, layer, out, sat, s);
    else prefill_launch<T, 1>(q, cu_rows, prompt_slot, n_prompts, max_len, hq, kv, layer, out, sat, s);
}

void launch_attention_prefill_mfma(int dtype, const void *q, const int32_t *cu_rows, const int32_t *prompt_slot,
                                   int n_prompts, int max_len, int hq, KvGeom kv, int layer, void *out, uint32_t *sat,
                                   hipStream_t s) {
    if (n_prompts <= 0 || max_len <= 0) return;
    if (dtype == KD_BF16) prefill_launch_t<bf16_t>(q, cu_rows, prompt_slot, n_prompts, max_len, hq, kv, layer, out, sat, s);
    else prefill_launch_t<f16_t>(q, cu_rows, prompt_slot, n_prompts, max_len, hq, kv, layer, out, sat, s);
}

// ---------------------------------------------------------------- decode
// A block has 4 waves when the batch alone fills the chip twice over (two blocks per CU), 8 waves when
// there are too few (row, kv head) pairs for that: one block per CU then, and every wave walks half as
// many tiles, which is what counts when the launch is bound by latency rather than by bandwidth.
static int decode_waves(int rows, int n_kv_heads) { return rows * n_kv_heads <= 256 ? 8 : 4; }

// Number of context splits: enough blocks to fill the chip, none when the batch alone nearly does
// (a merge pass costs more than a partly filled chip).
int attention_decode_splits(int rows, int n_kv_heads, int max_ctx) {
    const int blocks = rows * n_kv_heads;
    if (blocks >= 192) return 1;
    const int round = 32 * decode_waves(rows, n_kv_heads);
    int s = (384 + blocks - 1) / blocks;
    s = std::min(s, std::max(1, (max_ctx + round - 1) / round));
    return std::max(1, std::min(s, 16));
}

// scratch per (row, q head, split): (max, sum) and the unnormalised output [HD].
// rows * splits(rows) never exceeds rows + 512 (splits > 1 only while rows * kv heads < 192, and then
// splits <= 384 / (rows * kv heads) + 1).
size_t attention_decode_scratch_floats(int max_rows, int hq, int hd) {
    return (size_t)(max_rows + 512) * hq * (hd + 2);
}

// Every row cuts ITS context into n_splits equal pieces (rounded up to whole passes of `round` tokens).
__device__ inline int split_len(int ctx, int n_splits, int round) {
    return ((ctx + n_splits - 1) / n_splits + round - 1) / round * round;
}

// One block per (row, kv head, context split), NW waves; wave w takes the tiles w, w+NW, ... of the split.
// DIRECT (one split): the block normalises and writes the attention output itself.
// Block order: `group` consecutive rows are the rollouts of one prompt and read the same prefix blocks;
// the 1-D grid is laid out so that those blocks run back to back on ONE die (workgroup i runs on die
// i % 8), which then fetches the shared prefix from HBM once and serves the other rollouts from its L2.
template <typename T, bool DIRECT, int NW>
__global__ __launch_bounds__(64 * NW) void attention_decode_mfma_kernel(const T *__restrict__ q,
                                                                       const int32_t *__restrict__ row_slot,
                                                                       const int32_t *__restrict__ slot_len, int hq,
                                                                       KvGeom kv, int layer, int rows, int n_splits,
                                                                       int group, float *__restrict__ part_ml,
                                                                       float *__restrict__ part_o,
                                                                       T *__restrict__ out, uint32_t *__restrict__ sat) {
    constexpr int ROUND = 32 * NW;   // tokens one block consumes per pass of its waves
    constexpr int NSLOT = 4;         // waves that hand their output to the final sum (8 waves: pairs add up first)
    __shared__ float sm[NW][16], sl[NW][16];
    __shared__ float so[NSLOT][16][HD];
    const int b = blockIdx.x, die = b % 8, j = b / 8;
    const int unit = (j / group) * 8 + die;              // (prompt, kv head, split)
    const int per_prompt = kv.n_kv_heads * n_splits;
    if (unit >= (rows / group) * per_prompt) return;
    const int r = (unit / per_prompt) * group + j % group;
    const int kvh = (unit / n_splits) % kv.n_kv_heads, sp = unit % n_splits;
    const int slot = row_slot[r];
    const int ctx = slot_len[slot] + 1;
    const int len = split_len(ctx, n_splits, ROUND);
    const int beg = sp * len;
    if (beg >= ctx) return;
    const int end = min(ctx, beg + len);
    const int tid = threadIdx.x, lane = tid % WAVE, wave = tid / WAVE, i = lane % 16, g = lane / 16;
    const int rep = hq / kv.n_kv_heads;
    const T *head_base = (const T *)kv.pool + (int64_t)layer * kv.layer_stride + (int64_t)kvh * kv.head_elems();
    const int32_t *table = kv.block_table + (int64_t)slot * kv.max_blocks_per_slot;
    typename Mma<T>::frag qf[1][4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        if (i < rep)
            qf[0][kk] = ld_frag(q + ((int64_t)r * hq + kvh * rep + i) * HD + 32 * kk + 8 * g);
        else
            qf[0][kk] = zero_frag<T>();
    }
    AttnState st1[1];
    state_init(st1[0]);
    AttnState &st = st1[0];
    const float scale_log2 = LOG2E / sqrtf((float)HD);
    attend_tiles<T, 1, NW == 8>(head_base, kv.block_elems(), table, kv.block_size, qf, beg + 32 * wave, ROUND, end,
                                ctx - 1, scale_log2, st1);
    // ---- combine the waves
    float l = st.l;
    l += __shfl_xor(l, 16, WAVE);
    l += __shfl_xor(l, 32, WAVE);
    if (g == 0) {
        sm[wave][i] = st.m;
        sl[wave][i] = l;
    }
    __syncthreads();
    // every wave brings its output to the block's common maximum
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int col = 4 * g + v;
        float M = sm[0][col];
#pragma unroll
        for (int w = 1; w < NW; ++w) M = fmaxf(M, sm[w][col]);
        const float mw = sm[wave][col];
        const float fw = (mw == -INFINITY) ? 0.f : exp2f((mw - M) * scale_log2);
#pragma unroll
        for (int nn = 0; nn < 8; ++nn) st.o[nn][v] *= fw;
    }
    if (NW == 8) {   // odd waves pass their output to the even wave below them
        if (wave % 2 == 1) {
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int nn = 0; nn < 8; ++nn) so[wave / 2][4 * g + v][16 * nn + i] = st.o[nn][v];
        }
        __syncthreads();
        if (wave % 2 == 0) {
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int nn = 0; nn < 8; ++nn) st.o[nn][v] += so[wave / 2][4 * g + v][16 * nn + i];
        }
        __syncthreads();
    }
    if (NW == 4 || wave % 2 == 0) {
        const int slot_w = NW == 4 ? wave : wave / 2;
#pragma unroll
        for (int v = 0; v < 4; ++v)
#pragma unroll
            for (int nn = 0; nn < 8; ++nn) so[slot_w][4 * g + v][16 * nn + i] = st.o[nn][v];
    }
    __syncthreads();
    // rep columns x 128 values over the block's threads; a thread's values all belong to one column per pass
    for (int e = tid; e < rep * HD; e += 64 * NW) {
        const int col = e / HD, c = e % HD;
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < NSLOT; ++w) v += so[w][col][c];
        if (DIRECT) {
            float M = sm[0][col];
#pragma unroll
            for (int w = 1; w < NW; ++w) M = fmaxf(M, sm[w][col]);
            float L = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const float mw = sm[w][col];
                L += (mw == -INFINITY) ? 0.f : sl[w][col] * exp2f((mw - M) * scale_log2);
            }
            out[((int64_t)r * hq + kvh * rep + col) * HD + c] = from_f32_sat<T>(v / L, sat);
        } else {
            const int64_t idx = ((int64_t)r * hq + kvh * rep + col) * n_splits + sp;
            part_o[idx * HD + c] = v;
        }
    }
    if (!DIRECT && tid < rep) {
        const int col = tid;
        float M = sm[0][col];
#pragma unroll
        for (int w = 1; w < NW; ++w) M = fmaxf(M, sm[w][col]);
        float L = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float mw = sm[w][col];
            L += (mw == -INFINITY) ? 0.f : sl[w][col] * exp2f((mw - M) * scale_log2);
        }
        const int64_t idx = ((int64_t)r * hq + kvh * rep + col) * n_splits + sp;
        part_ml[2 * idx] = M;
        part_ml[2 * idx + 1] = L;
    }
}

// grid (q heads, rows), 128 threads: one per head_dim column
template <typename T>
__global__ __launch_bounds__(128) void attention_decode_merge_kernel(const int32_t *__restrict__ row_slot,
                                                                     const int32_t *__restrict__ slot_len, int hq,
                                                                     int n_splits, int round,
                                                                     const float *__restrict__ part_ml,
                                                                     const float *__restrict__ part_o,
                                                                     T *__restrict__ out, uint32_t *__restrict__ sat) {
    const int head = blockIdx.x, r = blockIdx.y, c = threadIdx.x;
    const int ctx = slot_len[row_slot[r]] + 1;
    const int len = split_len(ctx, n_splits, round);
    const int ns = (ctx + len - 1) / len;            // the splits that found tokens
    const int64_t base = ((int64_t)r * hq + head) * n_splits;
    const float scale_log2 = LOG2E / sqrtf((float)HD);
    float M = -INFINITY;
    for (int s = 0; s < ns; ++s) M = fmaxf(M, part_ml[2 * (base + s)]);
    float L = 0.f, acc = 0.f;
    for (int s = 0; s < ns; ++s) {
        const float f = exp2f((part_ml[2 * (base + s)] - M) * scale_log2);
        L += f * part_ml[2 * (base + s) + 1];
        acc += f * part_o[(base + s) * HD + c];
    }
    out[((int64_t)r * hq + head) * HD + c] = from_f32_sat<T>(acc / L, sat);
}

template <typename T, int NW>
static void decode_launch_nw(const T *q, const int32_t *row_slot, const int32_t *slot_len, int rows, int hq, KvGeom kv,
                             int layer, int n_splits, int group, float *part_ml, float *part_o, T *out, unsigned grid,
                             uint32_t *sat, hipStream_t s) {
    if (n_splits == 1)
        attention_decode_mfma_kernel<T, true, NW><<<grid, 64 * NW, 0, s>>>(q, row_slot, slot_len, hq, kv, layer, rows,
                                                                           n_splits, group, part_ml, part_o, out, sat);
    else
        attention_decode_mfma_kernel<T, false, NW><<<grid, 64 * NW, 0, s>>>(q, row_slot, slot_len, hq, kv, layer, rows,
                                                                            n_splits, group, part_ml, part_o, out, sat);
}

template <typename T>
static void decode_launch(const void *q, const int32_t *row_slot, const int32_t *slot_len, int rows, int hq, KvGeom kv,
                          int layer, int n_splits, int group, float *scratch, void *out, uint32_t *sat, hipStream_t s) {
    float *part_ml = scratch;
    float *part_o = scratch + (size_t)rows * hq * n_splits * 2;
    if (group < 1 || rows % group) group = 1;
    const int units = (rows / group) * kv.n_kv_heads * n_splits;
    const unsigned grid = (unsigned)((units + 7) / 8 * 8 * group);
    if (decode_waves(rows, kv.n_kv_heads) == 8)
        decode_launch_nw<T, 8>((const T *)q, row_slot, slot_len, rows, hq, kv, layer, n_splits, group, part_ml, part_o,
                               (T *)out, grid, sat, s);
    else
        decode_launch_nw<T, 4>((const T *)q, row_slot, slot_len, rows, hq, kv, layer, n_splits, group, part_ml, part_o,
                               (T *)out, grid, sat, s);
}

void launch_attention_decode_mfma(int dtype, const void *q, const int32_t *row_slot, const int32_t *slot_len, int rows,
                                  int hq, KvGeom kv, int layer, int n_splits, int group, float *scratch, void *out,
                                  uint32_t *sat, hipStream_t s) {
    if (rows <= 0) return;
    if (dtype == KD_BF16)
        decode_launch<bf16_t>(q, row_slot, slot_len, rows, hq, kv, layer, n_splits, group, scratch, out, sat, s);
    else
        decode_launch<f16_t>(q, row_slot, slot_len, rows, hq, kv, layer, n_splits, group, scratch, out, sat, s);
}

// only needed when n_splits > 1
void launch_attention_decode_merge(int dtype, const int32_t *row_slot, const int32_t *slot_len, int rows, int hq,
                                   int n_kv_heads, int n_splits, float *scratch, void *out, uint32_t *sat,
                                   hipStream_t s) {
    if (rows <= 0 || n_splits <= 1) return;
    const float *part_ml = scratch;
    const float *part_o = scratch + (size_t)rows * hq * n_splits * 2;
    const int round = 32 * decode_waves(rows, n_kv_heads);
    dim3 mgrid(hq, rows);
    if (dtype == KD_BF16)
        attention_decode_merge_kernel<bf16_t><<<mgrid, 128, 0, s>>>(row_slot, slot_len, hq, n_splits, round, part_ml,
                                                                    part_o, (bf16_t *)out, sat);
    else
        attention_decode_merge_kernel<f16_t><<<mgrid, 128, 0, s>>>(row_slot, slot_len, hq, n_splits, round, part_ml,
                                                                   part_o, (f16_t *)out, sat);
}

}  // namespace pc
