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
    if (dtype == KD_F32)   // the table is the caller's: fp32, or bf16 for both 16-bit kernel dtypes
        embed_kernel<float><<<rows, 256, 0, s>>>((const float *)table, tokens, d, vocab, h);
    else
        embed_kernel<bf16_t><<<rows, 256, 0, s>>>((const bf16_t *)table, tokens, d, vocab, h);
}

// ------------------------------------------------------------------ RMSNorm
// out = h * rsqrt(mean(h^2) + eps) * gain; one block per row, statistics in fp32.
// Pending split-K slices of the previous projection are folded into h first (slice order).
// VEC4: d % 4 == 0 and d <= 4 * 256 * RMS_MAXV: the row lives in registers between the two passes.
static constexpr int RMS_MAXV = 6;

template <typename T> __device__ inline void store4(T *p, float4 v, uint32_t *sat);
template <> __device__ inline void store4<float>(float *p, float4 v, uint32_t *) { *(float4 *)p = v; }
template <> __device__ inline void store4<bf16_t>(bf16_t *p, float4 v, uint32_t *) {
    uint2 u = {pack2<bf16_t>(v.x, v.y), pack2<bf16_t>(v.z, v.w)};
    *(uint2 *)p = u;
}
template <> __device__ inline void store4<f16_t>(f16_t *p, float4 v, uint32_t *sat) {
    uint2 u = {pack2_sat<f16_t>(v.x, v.y, sat), pack2_sat<f16_t>(v.z, v.w, sat)};
    *(uint2 *)p = u;
}

template <typename T, bool VEC4>
__global__ __launch_bounds__(256) void rmsnorm_kernel(float *__restrict__ h, const int32_t *__restrict__ src_row,
                                                      const float *__restrict__ gain, int rows, int d, float eps,
                                                      T *__restrict__ out, const float *__restrict__ slices, int S,
                                                      uint32_t *__restrict__ sat) {
    __shared__ float part[4];
    const int r = blockIdx.x, tid = threadIdx.x;
    float *x = h + (int64_t)(src_row ? src_row[r] : r) * d;
    float ss = 0.f;
    float4 keep[RMS_MAXV];
    if (VEC4) {
        const int n4 = d / 4;
#pragma unroll
        for (int j = 0; j < RMS_MAXV; ++j) {
            const int i = tid + 256 * j;
            if (i < n4) {
                float4 v = ((const float4 *)x)[i];
                if (S > 1) {
                    const float4 *sp = (const float4 *)(slices + (int64_t)r * d) + i;
                    const int64_t zs = (int64_t)rows * d / 4;
                    float4 add = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
                    for (int z = 0; z < S; ++z) {
                        const float4 t = sp[z * zs];
                        add.x += t.x; add.y += t.y; add.z += t.z; add.w += t.w;
                    }
                    v.x += add.x; v.y += add.y; v.z += add.z; v.w += add.w;
                    ((float4 *)x)[i] = v;
                }
                keep[j] = v;
                ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
            }
        }
    } else {
        for (int i = tid; i < d; i += 256) {
            float v = x[i];
            if (S > 1) {
                float add = 0.f;
                for (int z = 0; z < S; ++z) add += slices[((int64_t)z * rows + r) * d + i];
                v += add;
                x[i] = v;
            }
            ss += v * v;
        }
    }
    ss = wave_sum(ss);
    if (tid % WAVE == 0) part[tid / WAVE] = ss;
    __syncthreads();
    const float tot = part[0] + part[1] + part[2] + part[3];
    const float rs = 1.0f / sqrtf(tot / (float)d + eps);
    T *o = out + (int64_t)r * d;
    if (VEC4) {
        const int n4 = d / 4;
#pragma unroll
        for (int j = 0; j < RMS_MAXV; ++j) {
            const int i = tid + 256 * j;
            if (i < n4) {
                const float4 g = ((const float4 *)gain)[i];
                float4 v = keep[j];
                v.x = v.x * rs * g.x; v.y = v.y * rs * g.y; v.z = v.z * rs * g.z; v.w = v.w * rs * g.w;
                store4<T>(o + 4 * i, v, sat);
            }
        }
    } else {
        for (int i = tid; i < d; i += 256) o[i] = from_f32_sat<T>(x[i] * rs * gain[i], sat);
    }
}

void launch_rmsnorm(int dtype, float *h, const int32_t *src_row, const float *gain, int rows, int d, float eps,
                    void *out, const float *slices, int S, uint32_t *sat, hipStream_t s) {
    if (rows <= 0) return;
    const bool vec = (d % 4 == 0) && d <= 4 * 256 * RMS_MAXV;
#define PC_RMS(T)                                                                                              \
    do {                                                                                                       \
        if (vec) rmsnorm_kernel<T, true><<<rows, 256, 0, s>>>(h, src_row, gain, rows, d, eps, (T *)out, slices, S, sat);  \
        else rmsnorm_kernel<T, false><<<rows, 256, 0, s>>>(h, src_row, gain, rows, d, eps, (T *)out, slices, S, sat);     \
    } while (0)
    if (dtype == KD_F32) PC_RMS(float);
    else if (dtype == KD_BF16) PC_RMS(bf16_t);
    else PC_RMS(f16_t);
#undef PC_RMS
}

// ------------------------------------------------------------------ RoPE + KV append
// The pair (i, i + hd/2) of every q and k head turns by the angle pos * theta^(-2i/hd) (cos/sin tables are
// built on the host in double).  Grid (rows, item chunks): a row's work items are its q pairs, then its k
// pairs, then its v elements; every thread takes exactly one, so all of a row's loads are in flight at once.
template <typename T>
__global__ __launch_bounds__(256) void rope_append_kernel(const float *__restrict__ qkv, int S, int rows,
                                                          const int32_t *__restrict__ row_slot,
                                                          const int32_t *__restrict__ row_pos,
                                                          const int32_t *__restrict__ slot_len,
                                                          const float *__restrict__ rope_cos,
                                                          const float *__restrict__ rope_sin, int hq, KvGeom kv,
                                                          int layer, T *__restrict__ q_out,
                                                          uint32_t *__restrict__ sat, int perm) {
    const int r = blockIdx.x;
    const int hd = kv.head_dim, half = hd / 2, hkv = kv.n_kv_heads, bs = kv.block_size;
    const int nq = hq * half, nk = hkv * half, nv = hkv * hd;
    const int item = blockIdx.y * 256 + threadIdx.x;
    if (item >= nq + nk + nv) return;
    const int width = (hq + 2 * hkv) * hd;
    const float *row = qkv + (int64_t)r * width;
    const int64_t zs = (int64_t)rows * width;   // distance between K slices
    // perm: the weight rows of every q and k head were packed in the order the fused decode projection wants
    // (qkv_packed_dim): dim j of a head then sits at column qkv_packed_dim(j) of the head
    auto val = [&](int c) {
        float v = row[c];
        for (int z = 1; z < S; ++z) v += row[z * zs + c];
        return v;
    };
    auto qk_col = [&](int j) { return perm ? qkv_packed_dim(j, hd) : j; };
    const int slot = row_slot[r];
    const int pos = row_pos ? row_pos[r] : slot_len[slot];
    if (item < nq) {
        const int head = item / half, j = item % half;
        const float x1 = val(head * hd + qk_col(j)), x2 = val(head * hd + qk_col(j + half));
        const float c = rope_cos[(int64_t)pos * half + j], sgn = rope_sin[(int64_t)pos * half + j];
        T *qd = q_out + (int64_t)r * hq * hd + head * hd;
        qd[j] = from_f32_sat<T>(x1 * c - x2 * sgn, sat);
        qd[j + half] = from_f32_sat<T>(x2 * c + x1 * sgn, sat);
        return;
    }
    const int blk = kv.block_table[(int64_t)slot * kv.max_blocks_per_slot + pos / bs];
    const int tin = pos % bs;
    T *pool = (T *)kv.pool + (int64_t)layer * kv.layer_stride + (int64_t)blk * kv.block_elems();
    if (item < nq + nk) {   // k heads
        const int i = item - nq, head = i / half, j = i % half;
        const int koff = hq * hd;
        const float x1 = val(koff + head * hd + qk_col(j)), x2 = val(koff + head * hd + qk_col(j + half));
        const float c = rope_cos[(int64_t)pos * half + j], sgn = rope_sin[(int64_t)pos * half + j];
        T *kd = pool + (int64_t)head * kv.head_elems();
        kd[kv.k_index(tin, j)] = from_f32_sat<T>(x1 * c - x2 * sgn, sat);
        kd[kv.k_index(tin, j + half)] = from_f32_sat<T>(x2 * c + x1 * sgn, sat);
    } else {                // v heads
        const int i = item - nq - nk, head = i / hd, j = i % hd;
        const int voff = (hq + hkv) * hd;
        T *vd = pool + (int64_t)head * kv.head_elems();
        vd[kv.v_index(tin, j)] = from_f32_sat<T>(val(voff + head * hd + j), sat);
    }
}

void launch_rope_append(int dtype, const float *qkv, int S, const int32_t *row_slot, const int32_t *row_pos,
                        const int32_t *slot_len, const float *rope_cos, const float *rope_sin, int rows, int hq,
                        KvGeom kv, int layer, void *q_out, uint32_t *sat, int perm, hipStream_t s) {
    if (rows <= 0) return;
    const int items = hq * (kv.head_dim / 2) + kv.n_kv_heads * (kv.head_dim / 2) + kv.n_kv_heads * kv.head_dim;
    const dim3 grid(rows, (items + 255) / 256);
    if (dtype == KD_F32)
        rope_append_kernel<float><<<grid, 256, 0, s>>>(qkv, S, rows, row_slot, row_pos, slot_len, rope_cos, rope_sin, hq, kv,
                                                       layer, (float *)q_out, sat, perm);
    else if (dtype == KD_BF16)
        rope_append_kernel<bf16_t><<<grid, 256, 0, s>>>(qkv, S, rows, row_slot, row_pos, slot_len, rope_cos, rope_sin, hq, kv,
                                                        layer, (bf16_t *)q_out, sat, perm);
    else
        rope_append_kernel<f16_t><<<grid, 256, 0, s>>>(qkv, S, rows, row_slot, row_pos, slot_len, rope_cos, rope_sin, hq, kv,
                                                       layer, (f16_t *)q_out, sat, perm);
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
    if (dtype == KD_F32)
        copy_block_kernel<float><<<grid, 256, 0, s>>>(kv, pairs);
    else   // both 16-bit kernel dtypes: raw 16-bit payload
        copy_block_kernel<bf16_t><<<grid, 256, 0, s>>>(kv, pairs);
}

// ------------------------------------------------------------------ weight repacking
// TS: the caller's element type, TD: the kernel dtype of the copy (bf16 -> half is a value conversion)
template <typename TS, typename TD> __device__ inline TD conv(TS v) { return from_f32<TD>(to_f32(v)); }

// head_perm > 0: rows come in heads of head_perm rows, and row j of a head goes to row qkv_packed_dim(j) of it
template <typename TS, typename TD>
__global__ void pack_rows_kernel(const TS *__restrict__ src, TD *__restrict__ dst, int64_t cols, int64_t dst_row0,
                                 int head_perm) {
    int64_t r = blockIdx.x, rd = r;
    if (head_perm > 0) rd = (r / head_perm) * head_perm + qkv_packed_dim((int)(r % head_perm), head_perm);
    for (int64_t i = threadIdx.x; i < cols; i += blockDim.x) dst[(dst_row0 + rd) * cols + i] = conv<TS, TD>(src[r * cols + i]);
}
void launch_pack_rows(int kd, const void *src, void *dst, int64_t rows, int64_t cols, int64_t dst_row0, int head_perm,
                      hipStream_t s) {
    if (rows <= 0) return;
    if (kd == KD_F32)
        pack_rows_kernel<float, float><<<(unsigned)rows, 256, 0, s>>>((const float *)src, (float *)dst, cols, dst_row0, head_perm);
    else if (kd == KD_BF16)
        pack_rows_kernel<bf16_t, bf16_t><<<(unsigned)rows, 256, 0, s>>>((const bf16_t *)src, (bf16_t *)dst, cols, dst_row0, head_perm);
    else
        pack_rows_kernel<bf16_t, f16_t><<<(unsigned)rows, 256, 0, s>>>((const bf16_t *)src, (f16_t *)dst, cols, dst_row0, head_perm);
}

// dst row 64t + c      = gate row 32t + c   (c < 32)
// dst row 64t + 32 + c = up   row 32t + c
template <typename TS, typename TD>
__global__ void pack_gate_up_kernel(const TS *__restrict__ gate, const TS *__restrict__ up, TD *__restrict__ dst, int d) {
    int64_t j = blockIdx.x;   // ffn row
    int64_t t = j / 32, c = j % 32;
    for (int i = threadIdx.x; i < d; i += blockDim.x) {
        dst[(64 * t + c) * d + i] = conv<TS, TD>(gate[j * d + i]);
        dst[(64 * t + 32 + c) * d + i] = conv<TS, TD>(up[j * d + i]);
    }
}
void launch_pack_gate_up(int kd, const void *gate, const void *up, void *dst, int d_ff, int d, hipStream_t s) {
    if (kd == KD_F32)
        pack_gate_up_kernel<float, float><<<d_ff, 256, 0, s>>>((const float *)gate, (const float *)up, (float *)dst, d);
    else if (kd == KD_BF16)
        pack_gate_up_kernel<bf16_t, bf16_t><<<d_ff, 256, 0, s>>>((const bf16_t *)gate, (const bf16_t *)up, (bf16_t *)dst, d);
    else
        pack_gate_up_kernel<bf16_t, f16_t><<<d_ff, 256, 0, s>>>((const bf16_t *)gate, (const bf16_t *)up, (f16_t *)dst, d);
}

}  // namespace pc
