// Row-wise kernels of the decoder forward (Section 3.1 policy pi_theta):
// embedding gather, RMSNorm, rotary positions + KV append, and the small
// bookkeeping kernels of the paged cache.  All are HBM/latency bound.
#include "pc_internal.h"

namespace pc {

static constexpr int WAVE = 64;

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}

// ------------------------------------------------------------------ embed
template <typename T>
__global__ void embed_kernel(const T *__restrict__ table, const int32_t *__restrict__ tokens, int d, int vocab,
                             float *__restrict__ h) {
    int r = blockIdx.x;
    int tok = tokens[r];
    if (tok < 0 || tok >= vocab) tok = 0;
    const T *src = table + (int64_t)tok * d;
    float *dst = h + (int64_t)r * d;
    for (int i = threadIdx.x; i < d; i += blockDim.x) dst[i] = to_f32(src[i]);
}

void launch_embed(int dtype, const void *table, const int32_t *tokens, int rows, int d, int vocab, float *h,
                  hipStream_t s) {
    if (rows <= 0) return;
    if (dtype == PC_DTYPE_F32)
        embed_kernel<float><<<rows, 256, 0, s>>>((const float *)table, tokens, d, vocab, h);
    else
        embed_kernel<bf16_t><<<rows, 256, 0, s>>>((const bf16_t *)table, tokens, d, vocab, h);
}

// ------------------------------------------------------------------ RMSNorm
// out = h * rsqrt(mean(h^2) + eps) * gain; one block per row, statistics in fp32.
template <typename T>
__global__ void rmsnorm_kernel(const float *__restrict__ h, const int32_t *__restrict__ src_row,
                               const float *__restrict__ gain, int d, float eps, T *__restrict__ out) {
    __shared__ float part[16];
    int r = blockIdx.x;
    const float *x = h + (int64_t)(src_row ? src_row[r] : r) * d;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d; i += blockDim.x) {
        float v = x[i];
        ss += v * v;
    }
    ss = wave_sum(ss);
    int wid = threadIdx.x / WAVE, lane = threadIdx.x % WAVE, nw = blockDim.x / WAVE;
    if (lane == 0) part[wid] = ss;
    __syncthreads();
    float tot = 0.f;
    for (int i = 0; i < nw; ++i) tot += part[i];
    float rs = 1.0f / sqrtf(tot / (float)d + eps);
    T *o = out + (int64_t)r * d;
    for (int i = threadIdx.x; i < d; i += blockDim.x) o[i] = from_f32<T>(x[i] * rs * gain[i]);
}

void launch_rmsnorm(int dtype, const float *h, const int32_t *src_row, const float *gain, int rows, int d, float eps,
                    void *out, hipStream_t s) {
    if (rows <= 0) return;
    if (dtype == PC_DTYPE_F32)
        rmsnorm_kernel<float><<<rows, 256, 0, s>>>(h, src_row, gain, d, eps, (float *)out);
    else
        rmsnorm_kernel<bf16_t><<<rows, 256, 0, s>>>(h, src_row, gain, d, eps, (bf16_t *)out);
}

// ------------------------------------------------------------------ RoPE + KV append
// One block per row.  The pair (i, i + hd/2) of every q and k head turns by the
// angle pos * theta^(-2i/hd) (cos/sin tables are built on the host in double).
template <typename T>
__global__ void rope_append_kernel(const float *__restrict__ qkv, const int32_t *__restrict__ row_slot,
                                   const int32_t *__restrict__ row_pos, const int32_t *__restrict__ slot_len,
                                   const float *__restrict__ rope_cos, const float *__restrict__ rope_sin, int hq,
                                   KvGeom kv, int layer, T *__restrict__ q_out) {
    const int r = blockIdx.x;
    const int hd = kv.head_dim, half = hd / 2, hkv = kv.n_kv_heads, bs = kv.block_size;
    const int slot = row_slot[r];
    const int pos = row_pos ? row_pos[r] : slot_len[slot];
    const float *row = qkv + (int64_t)r * (hq + 2 * hkv) * hd;
    const float *cs = rope_cos + (int64_t)pos * half;
    const float *sn = rope_sin + (int64_t)pos * half;
    const int blk = kv.block_table[(int64_t)slot * kv.max_blocks_per_slot + pos / bs];
    const int tin = pos % bs;
    T *pool = (T *)kv.pool + (int64_t)layer * kv.layer_stride + (int64_t)blk * kv.block_elems();

    // q heads
    for (int i = threadIdx.x; i < hq * half; i += blockDim.x) {
        int head = i / half, j = i % half;
        float x1 = row[head * hd + j], x2 = row[head * hd + j + half];
        float c = cs[j], sgn = sn[j];
        q_out[(int64_t)r * hq * hd + head * hd + j] = from_f32<T>(x1 * c - x2 * sgn);
        q_out[(int64_t)r * hq * hd + head * hd + j + half] = from_f32<T>(x2 * c + x1 * sgn);
    }
    // k heads -> K [tok][hd]
    const float *krow = row + hq * hd;
    for (int i = threadIdx.x; i < hkv * half; i += blockDim.x) {
        int head = i / half, j = i % half;
        float x1 = krow[head * hd + j], x2 = krow[head * hd + j + half];
        float c = cs[j], sgn = sn[j];
        T *kd = pool + (int64_t)head * kv.head_elems() + (int64_t)tin * hd;
        kd[j] = from_f32<T>(x1 * c - x2 * sgn);
        kd[j + half] = from_f32<T>(x2 * c + x1 * sgn);
    }
    // v heads -> V^T [hd][tok]
    const float *vrow = krow + hkv * hd;
    for (int i = threadIdx.x; i < hkv * hd; i += blockDim.x) {
        int head = i / hd, j = i % hd;
        T *vd = pool + (int64_t)head * kv.head_elems() + (int64_t)bs * hd;
        vd[(int64_t)j * bs + tin] = from_f32<T>(vrow[head * hd + j]);
    }
}

void launch_rope_append(int dtype, const float *qkv, const int32_t *row_slot, const int32_t *row_pos,
                        const int32_t *slot_len, const float *rope_cos, const float *rope_sin, int rows, int hq,
                        KvGeom kv, int layer, void *q_out, hipStream_t s) {
    if (rows <= 0) return;
    if (dtype == PC_DTYPE_F32)
        rope_append_kernel<float><<<rows, 256, 0, s>>>(qkv, row_slot, row_pos, slot_len, rope_cos, rope_sin, hq, kv,
                                                       layer, (float *)q_out);
    else
        rope_append_kernel<bf16_t><<<rows, 256, 0, s>>>(qkv, row_slot, row_pos, slot_len, rope_cos, rope_sin, hq, kv,
                                                        layer, (bf16_t *)q_out);
}

// ------------------------------------------------------------------ bookkeeping
__global__ void advance_len_kernel(int32_t *slot_len, const int32_t *row_slot, int rows) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < rows) slot_len[row_slot[i]] += 1;   // slots in a step are distinct
}
void launch_advance_len(int32_t *slot_len, const int32_t *row_slot, int rows, hipStream_t s) {
    if (rows <= 0) return;
    advance_len_kernel<<<(rows + 255) / 256, 256, 0, s>>>(slot_len, row_slot, rows);
}

__global__ void fill_i32_kernel(int32_t *p, int32_t v, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}
void launch_fill_i32(int32_t *p, int32_t v, int64_t n, hipStream_t s) {
    if (n <= 0) return;
    fill_i32_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(p, v, n);
}

// copies whole KV blocks (all layers, all kv heads): pairs[2i] -> pairs[2i+1]
template <typename T>
__global__ void copy_block_kernel(KvGeom kv, const int32_t *__restrict__ pairs) {
    int pair = blockIdx.x, layer = blockIdx.y;
    int src = pairs[2 * pair], dst = pairs[2 * pair + 1];
    int64_t n = kv.block_elems();
    const T *s = (const T *)kv.pool + (int64_t)layer * kv.layer_stride + (int64_t)src * n;
    T *d = (T *)kv.pool + (int64_t)layer * kv.layer_stride + (int64_t)dst * n;
    for (int64_t i = threadIdx.x; i < n; i += blockDim.x) d[i] = s[i];
}
void launch_copy_block(int dtype, KvGeom kv, int n_layers, const int32_t *pairs, int n_pairs, hipStream_t s) {
    if (n_pairs <= 0) return;
    dim3 grid(n_pairs, n_layers);
    if (dtype == PC_DTYPE_F32)
        copy_block_kernel<float><<<grid, 256, 0, s>>>(kv, pairs);
    else
        copy_block_kernel<bf16_t><<<grid, 256, 0, s>>>(kv, pairs);
}

// ------------------------------------------------------------------ weight repacking
template <typename T>
__global__ void pack_rows_kernel(const T *__restrict__ src, T *__restrict__ dst, int64_t cols, int64_t dst_row0) {
    int64_t r = blockIdx.x;
    for (int64_t i = threadIdx.x; i < cols; i += blockDim.x) dst[(dst_row0 + r) * cols + i] = src[r * cols + i];
}
void launch_pack_rows(int dtype, const void *src, void *dst, int64_t rows, int64_t cols, int64_t dst_row0,
                      hipStream_t s) {
    if (rows <= 0) return;
    if (dtype == PC_DTYPE_F32)
        pack_rows_kernel<float><<<(unsigned)rows, 256, 0, s>>>((const float *)src, (float *)dst, cols, dst_row0);
    else
        pack_rows_kernel<bf16_t><<<(unsigned)rows, 256, 0, s>>>((const bf16_t *)src, (bf16_t *)dst, cols, dst_row0);
}

// dst row 64t + c      = gate row 32t + c   (c < 32)
// dst row 64t + 32 + c = up   row 32t + c
template <typename T>
__global__ void pack_gate_up_kernel(const T *__restrict__ gate, const T *__restrict__ up, T *__restrict__ dst, int d) {
    int64_t j = blockIdx.x;   // ffn row
    int64_t t = j / 32, c = j % 32;
    for (int i = threadIdx.x; i < d; i += blockDim.x) {
        dst[(64 * t + c) * d + i] = gate[j * d + i];
        dst[(64 * t + 32 + c) * d + i] = up[j * d + i];
    }
}
void launch_pack_gate_up(int dtype, const void *gate, const void *up, void *dst, int d_ff, int d, hipStream_t s) {
    if (dtype == PC_DTYPE_F32)
        pack_gate_up_kernel<float><<<d_ff, 256, 0, s>>>((const float *)gate, (const float *)up, (float *)dst, d);
    else
        pack_gate_up_kernel<bf16_t><<<d_ff, 256, 0, s>>>((const bf16_t *)gate, (const bf16_t *)up, (bf16_t *)dst, d);
}

}  // namespace pc
