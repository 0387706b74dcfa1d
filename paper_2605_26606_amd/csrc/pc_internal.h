// Internal declarations shared by the library's translation units.
// Not part of the C ABI (see include/pc.h for that).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/pc.h"
#include "index_maps.h"

namespace pc {

// ---------------------------------------------------------------- bf16
struct bf16_t {
    uint16_t x;
};

__host__ __device__ inline float bf16_to_f32(bf16_t v) {
    union { uint32_t u; float f; } c;
    c.u = (uint32_t)v.x << 16;
    return c.f;
}
// round to nearest even (inputs are finite here)
__host__ __device__ inline bf16_t f32_to_bf16(float f) {
    union { uint32_t u; float f; } c;
    c.f = f;
    uint32_t u = c.u + 0x7FFFu + ((c.u >> 16) & 1u);
    bf16_t r;
    r.x = (uint16_t)(u >> 16);
    return r;
}

// ---------------------------------------------------------------- f16 (IEEE half)
struct f16_t {
    uint16_t x;
};
__device__ inline float f16_to_f32(f16_t v) { return (float)__builtin_bit_cast(_Float16, v.x); }
// round to nearest even, saturating at the largest finite half instead of overflowing to infinity
__device__ inline f16_t f32_to_f16(float f) {
    f = fminf(fmaxf(f, -65504.f), 65504.f);
    f16_t r;
    r.x = __builtin_bit_cast(uint16_t, (_Float16)f);
    return r;
}

__device__ inline float to_f32(float v) { return v; }
__device__ inline float to_f32(bf16_t v) { return bf16_to_f32(v); }
__device__ inline float to_f32(f16_t v) { return f16_to_f32(v); }
template <typename T> __device__ inline T from_f32(float f);
template <> __device__ inline float from_f32<float>(float f) { return f; }
template <> __device__ inline bf16_t from_f32<bf16_t>(float f) { return f32_to_bf16(f); }
template <> __device__ inline f16_t from_f32<f16_t>(float f) { return f32_to_f16(f); }
// two values packed into one 32-bit word (low half first)
template <typename T> __device__ inline uint32_t pack2(float a, float b) {
    return (uint32_t)from_f32<T>(a).x | ((uint32_t)from_f32<T>(b).x << 16);
}
// Stores of activations and cache entries: a value that leaves the half range is clamped (f32_to_f16)
// and counted in *sat, so that a caller can tell that its model does not fit IEEE-half activations.
template <typename T> __device__ inline T from_f32_sat(float f, uint32_t *sat) { return from_f32<T>(f); }
template <> __device__ inline f16_t from_f32_sat<f16_t>(float f, uint32_t *sat) {
    if (sat && fabsf(f) > 65504.f) atomicAdd(sat, 1u);
    return f32_to_f16(f);
}
template <typename T> __device__ inline uint32_t pack2_sat(float a, float b, uint32_t *sat) {
    return (uint32_t)from_f32_sat<T>(a, sat).x | ((uint32_t)from_f32_sat<T>(b, sat).x << 16);
}

// Kernel data types: the type of activations, KV cache and the library's weight copies.
//   KD_F32   fp32 models
//   KD_BF16  bf16 models, bf16 activations
//   KD_F16   bf16 models, IEEE-half activations and weight copies (bf16 weights convert to half without
//            loss above 6.1e-5 in magnitude, with an absolute error below 3e-8 under it); three more
//            significand bits than bf16 at the same matrix-core rate
enum KernelDtype { KD_F32 = 0, KD_BF16 = 1, KD_F16 = 2 };

// matrix-core products on 8-element fragments
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
template <typename T> struct Mma;
template <> struct Mma<bf16_t> {
    typedef bf16x8_t frag;
    __device__ static inline f32x16_t m32(frag a, frag b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    __device__ static inline f32x4_t m16(frag a, frag b, f32x4_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
};
template <> struct Mma<f16_t> {
    typedef f16x8_t frag;
    __device__ static inline f32x16_t m32(frag a, frag b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
    __device__ static inline f32x4_t m16(frag a, frag b, f32x4_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
    }
};

// ---------------------------------------------------------------- errors
void set_error(const char *fmt, ...);
#define PC_FAIL(code, ...)          \
    do {                            \
        ::pc::set_error(__VA_ARGS__); \
        return (code);              \
    } while (0)
#define PC_HIP(expr)                                                                        \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess) {                                                             \
            ::pc::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
            return PC_ERR_HIP;                                                              \
        }                                                                                   \
    } while (0)

// ---------------------------------------------------------------- KV cache geometry
// Pool layout: [layer][block][kv_head][K | V], block_size * head_dim elements each.
//
// Fragment-major (head_dim a multiple of 32; block_size always is): inside a block the keys and values are stored
// in the order in which the matrix-core attention kernels consume them, so that every operand fragment (64 lanes
// x 16 bytes) is ONE contiguous kilobyte -- a wave-wide load then touches 8 cache lines instead of 64 separate
// 16-byte pieces, which is what bounds a kernel that reads fragments straight from global memory (the load unit
// takes about one request per two clocks per CU, whatever its size).
//   K  tiles of 32 tokens; a tile is 2 x (head_dim / 32) fragments [u][kk]: lane (i, g) of fragment (u, kk) holds
//      dims 32 kk + 8 g .. + 7 of token 8 (i / 4) + i % 4 + 4 u of the tile (the token order that leaves every lane of
//      the score tile with 8 consecutive tokens, the operand layout of the P.V product)
//   V  tiles of 32 tokens; a tile is head_dim / 16 fragments [nn]: lane (i, g) holds tokens 8 g .. 8 g + 7 of dim
//      16 nn + i
// Plain (any other head_dim): K [block_size][head_dim], V^T [head_dim][block_size].
struct KvGeom {
    void *pool;
    int64_t layer_stride;   // elements between layers
    int32_t block_size;
    int32_t n_kv_heads;
    int32_t head_dim;
    int32_t max_blocks_per_slot;
    const int32_t *block_table;   // device [max_slots][max_blocks_per_slot]
    __host__ __device__ int64_t block_elems() const { return (int64_t)n_kv_heads * 2 * block_size * head_dim; }
    __host__ __device__ int64_t head_elems() const { return (int64_t)2 * block_size * head_dim; }
    __host__ __device__ bool frag_major() const { return (head_dim & 31) == 0; }
    // element offsets of K[token tin][dim d] / V[token tin][dim d] inside one (block, kv head) region
    __host__ __device__ int k_index(int tin, int d) const {
        return frag_major() ? kv_k_index_frag(tin, d, head_dim) : tin * head_dim + d;
    }
    __host__ __device__ int v_index(int tin, int d) const {
        return block_size * head_dim + (frag_major() ? kv_v_index_frag(tin, d, head_dim) : d * block_size + tin);
    }
};

// Order of the weight rows (= output columns) of a q or k head for the fused decode projection: a 32-column
// block holds 16 dims of the head's first half and, behind them, their 16 rotary partners (dim + hd/2), so
// that a block can rotate what it computed.  Dim j of the head sits at column qkv_packed_dim(j).
__host__ __device__ inline int qkv_packed_dim(int j, int hd) {
    const int half = hd / 2;
    return j < half ? 32 * (j / 16) + j % 16 : 32 * ((j - half) / 16) + 16 + j % 16;
}

// Epilogues of the projection GEMMs
enum Epilogue {
    EPI_STORE_F32 = 0,   // C fp32 [M,N]
    EPI_RESID_F32 = 1,   // C fp32 [M,N] += product (residual stream update)
    EPI_SWIGLU = 2,      // rows of W come in chunks of 64: 32 gate rows then the 32 matching up rows;
                         // C (model dtype) [M, N/2] = silu(gate) * up
    EPI_STORE_T = 3,     // C model dtype [M,N]
    EPI_SWIGLU_RS = 4,   // EPI_SWIGLU on rows that carry the RMSNorm gain but not its scale: gate and up are
                         // multiplied by the row's rsqrt(mean(h^2) + eps) first (statistics in GemmRowScale)
};

// Per-row RMSNorm statistics for EPI_SWIGLU_RS: ssq[t][row], t < tiles, are partial sums of squares of the row (as the fused output projection leaves them); scale = rsqrt(sum_t ssq / d + eps).
struct GemmRowScale {
    const float *ssq;
    int tiles, d;
    float eps;
};

// ---------------------------------------------------------------- kernel launchers
// (each validates nothing: callers pass shapes that the context has checked; `dtype` is a KernelDtype)
void launch_embed(int dtype, const void *table, const int32_t *tokens, int rows, int d, int vocab, float *h,
                  hipStream_t s);
// out[r] = norm(h[src_row ? src_row[r] : r]) * gain, in the model dtype.  With S > 1 slices
// [S][rows][d] pending (a split-K product not yet added to the residual stream), h[r] += their sum first
// (written back); src_row must be NULL then.
void launch_rmsnorm(int dtype, float *h, const int32_t *src_row, const float *gain, int rows, int d, float eps,
                    void *out, const float *slices, int S, uint32_t *sat, hipStream_t s);
// C = A[M,K] * W[N,K]^T with the given epilogue.  impl 0: plain ALU, 1: matrix cores (bf16 only)
void gemm_init();   // once per process: raises the dynamic-LDS limit of the matrix-core kernels
// Returns the number of K slices S the product was cut into.  S == 1: C holds the finished result.
// S > 1 (only when `slices` is given, for EPI_STORE_F32 / EPI_RESID_F32 at decode sizes): C is untouched
// and `slices` holds S fp32 partial products [S][M][N]; the consumer adds them in slice order (and, for
// EPI_RESID_F32, adds that sum to the residual stream).
// `sat`: counter of half-range clamps of the epilogues that store activations (may be NULL).
int launch_gemm(int dtype, int impl, const void *A, const void *W, void *C, int M, int N, int K, int epi,
                float *slices, size_t slice_cap_floats, uint32_t *sat, hipStream_t s,
                const GemmRowScale *row_scale = nullptr);
// Fused decode projections (gemm_skinny.hip); skinny_ok says whether the shape is one they take.
bool skinny_ok(int M, int N, int K, int head_dim);
void skinny_init();   // once per process, like gemm_init
void launch_skinny_qkv(int dtype, const void *A, const void *W, int M, int K, const int32_t *row_slot,
                       const int32_t *slot_len, const float *rope_cos, const float *rope_sin, int hq, KvGeom kv, int layer,
                       void *q_out, uint32_t *sat, hipStream_t s);
// h += A W^T; h_act = (new h) * gain in the activation type (the next RMSNorm without its scale);
// ssq[N/32][M]: partial sums of squares of the new rows
void launch_skinny_o(int dtype, const void *A, const void *W, int M, int N, int K, float *h, const float *gain, void *h_act,
                     float *ssq, uint32_t *sat, hipStream_t s);
// Rotates q and k at each row's position, writes q (model dtype) and appends k, v to the cache.
//   qkv fp32 [S][rows, (hq+2hkv)*hd] (S >= 1 K slices, summed here); row_slot [rows];
//   row_pos [rows] or NULL (then pos = slot_len[slot])
void launch_rope_append(int dtype, const float *qkv, int S, const int32_t *row_slot, const int32_t *row_pos,
                        const int32_t *slot_len, const float *rope_cos, const float *rope_sin, int rows, int hq,
                        KvGeom kv, int layer, void *q_out, uint32_t *sat, int perm, hipStream_t s);
// Attention of each row's query heads over its slot's cache, positions 0..pos (plain ALU).
void launch_attention_simt(int dtype, const void *q, const int32_t *row_slot, const int32_t *row_pos,
                           const int32_t *slot_len, int rows, int hq, KvGeom kv, int layer, void *out,
                           uint32_t *sat, hipStream_t s);
// Matrix-core attention (bf16).  Prefill: rows of each prompt are contiguous and start at position 0.
void launch_attention_prefill_mfma(int dtype, const void *q, const int32_t *cu_rows, const int32_t *prompt_slot,
                                   int n_prompts, int max_len, int hq, KvGeom kv, int layer, void *out, uint32_t *sat,
                                   hipStream_t s);
// Decode: one query row per sequence.  n_splits = attention_decode_splits(...): with one split the
// kernel writes `out` itself, otherwise it leaves partial results in `scratch` for the merge pass.
int attention_decode_splits(int rows, int n_kv_heads, int max_ctx);
// `group`: consecutive rows that share a prompt (1 if unknown): they are scheduled on one die.
void launch_attention_decode_mfma(int dtype, const void *q, const int32_t *row_slot, const int32_t *slot_len, int rows,
                                  int hq, KvGeom kv, int layer, int n_splits, int group, float *scratch, void *out,
                                  uint32_t *sat, hipStream_t s);
void launch_attention_decode_merge(int dtype, const int32_t *row_slot, const int32_t *slot_len, int rows, int hq,
                                   int n_kv_heads, int n_splits, float *scratch, void *out, uint32_t *sat,
                                   hipStream_t s);
size_t attention_decode_scratch_floats(int max_rows, int hq, int hd);

void launch_advance_len(int32_t *slot_len, const int32_t *row_slot, int rows, hipStream_t s);
void launch_copy_block(int dtype, KvGeom kv, int n_layers, const int32_t *src_dst_pairs, int n_pairs, hipStream_t s);
void launch_fill_i32(int32_t *p, int32_t v, int64_t n, hipStream_t s);

void launch_sample(const float *logits, const int32_t *logit_row, int n, int vocab, float temperature, float top_p,
                   uint64_t seed, const uint64_t *seq_uid, const int32_t *step, int step_base, int eos_id, float eos_bias,
                   int32_t *tokens_out, float *logprob_out, uint8_t *finished, int32_t *hist_tokens,
                   float *hist_logprob, const int32_t *hist_index, hipStream_t s);
// out[r] = log softmax(logits[r] / T)[tokens[token_index[r] + 1]]
void launch_logprob(const float *logits, int n, int vocab, float temperature, const int32_t *tokens,
                    const int32_t *token_index, float *out, hipStream_t s);
void launch_group_stats(const float *rewards, const int32_t *off, int P, int32_t *n_pos, int32_t *n_tot, float *mean,
                        float *var, hipStream_t s);
void launch_select_commit(const float *p_hat, int P, float lo, float hi, float solve, int b_t, uint8_t *cls,
                          uint8_t *evict, int32_t *commit_idx, int32_t *surplus_idx, int32_t *counts, hipStream_t s);
void launch_select_commit_var(const float *mean, const float *var, int P, float var_hard, float var_easy, float pivot,
                              float solve, int b_t, uint8_t *cls, uint8_t *evict, int32_t *commit_idx, int32_t *surplus_idx,
                              int32_t *counts, hipStream_t s);
void launch_advantages(const float *rewards, const int32_t *off, int P, float eps, float *adv, float *mu, float *sigma,
                       hipStream_t s);

// weight repacking at context creation; the source has the model's dtype, the copy the kernel dtype `kd`
// dst[dst_row0 + r'] = src[r]; head_perm > 0: r' = r with its place inside its head of head_perm rows moved to
// qkv_packed_dim
void launch_pack_rows(int kd, const void *src, void *dst, int64_t rows, int64_t cols, int64_t dst_row0, int head_perm,
                      hipStream_t s);
void launch_pack_gate_up(int kd, const void *gate, const void *up, void *dst, int d_ff, int d, hipStream_t s);

}  // namespace pc
