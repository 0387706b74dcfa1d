// Token sampling o_t ~ softmax(logits / T) (Section 3.1; Section 4.2: T = 1.0,
// top_p = 1.0) by inverse CDF with a Philox4x32-10 uniform.
//
// One block of 16 waves per row.  The row is read from HBM once: every wave
// keeps an online (max, sum) of a contiguous segment, the block locates the
// segment whose cumulative weight crosses u*Z, then narrows it twice more
// (16 sub-segments, then an in-order wavefront scan), re-reading only that
// segment.  Sums are accumulated in double so that the selected token agrees
// with an in-order double-precision CDF except within rounding of a boundary.
//
// Nucleus truncation (top_p < 1): the tokens in order of decreasing probability (ties: lower id first) until their
// cumulative mass reaches top_p keep their weight, the rest get none; the passes above then run on the kept
// tokens.  Decreasing probability is decreasing logit, so the cut is found by a radix select over an
// order-preserving 32-bit key of the logit, four passes of 8 bits, each with a histogram of the MASS per bucket
// (double, one histogram per wave, added up in wave order): the bucket in which the cumulative mass from the top
// crosses top_p * Z is the one to refine.  The row is re-read from L2 for every pass.
#include "pc_internal.h"

namespace pc {

static constexpr int WAVE = 64;
static constexpr int SAMPLE_WAVES = 16;

// Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies
__device__ inline void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1,
                                     uint32_t out[4]) {
    const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
        const uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

__device__ inline double wave_sum_d(double v) {
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}
__device__ inline float wave_max_f32(float v) {
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
    return v;
}

// order-preserving key of a float: a < b  <=>  okey(a) < okey(b)
__device__ inline uint32_t okey(float f) {
    const uint32_t b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// The kept set of a nucleus: logit key above kstar, or equal to it with an id up to tie_limit.
struct Nucleus {
    bool on;
    uint32_t kstar;
    int tie_limit;
    float eos_key_add;   // the EOS bias in logit units (bias * temperature): the key of the EOS id is logit + this
};
__device__ inline uint32_t logit_key(float raw, int idx, int eos_id, float eos_key_add) {
    return okey(idx == eos_id ? raw + eos_key_add : raw);
}

template <int VEC>
__device__ inline void load_scaled(const float *__restrict__ x, int idx, int end, float inv_t, int eos_id,
                                   float eos_bias, float (&v)[VEC], bool (&ok)[VEC], const Nucleus &nu) {
    if (VEC == 4 && idx + 3 < end) {
        const float4 t = *(const float4 *)(x + idx);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
#pragma unroll
        for (int c = 0; c < VEC; ++c) ok[c] = true;
    } else {
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            ok[c] = (idx + c) < end;
            v[c] = ok[c] ? x[idx + c] : 0.f;
        }
    }
    if (nu.on) {
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            const uint32_t key = logit_key(v[c], idx + c, eos_id, nu.eos_key_add);
            ok[c] = ok[c] && (key > nu.kstar || (key == nu.kstar && idx + c <= nu.tie_limit));
        }
    }
#pragma unroll
    for (int c = 0; c < VEC; ++c) {
        v[c] = v[c] * inv_t;
        if (idx + c == eos_id) v[c] += eos_bias;
    }
}

__device__ inline int round_up(int a, int b) { return (a + b - 1) / b * b; }

template <int VEC, bool TOPP>
__global__ __launch_bounds__(SAMPLE_WAVES *WAVE) void sample_kernel(
    const float *__restrict__ logits, const int32_t *__restrict__ logit_row, int vocab, float inv_t, float top_p,
    float eos_key_add, uint64_t seed,
    const uint64_t *__restrict__ seq_uid, const int32_t *__restrict__ step, int step_base, int eos_id, float eos_bias,
    int32_t *__restrict__ tokens_out, float *__restrict__ logprob_out, uint8_t *__restrict__ finished,
    int32_t *__restrict__ hist_tokens, float *__restrict__ hist_logprob, const int32_t *__restrict__ hist_index) {
    __shared__ float s_wm[SAMPLE_WAVES];
    __shared__ double s_ws[SAMPLE_WAVES];
    __shared__ double s_sub[SAMPLE_WAVES];
    __shared__ float s_u;
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid % WAVE, wave = tid / WAVE;
    if (finished && finished[row]) {   // block-uniform
        if (tid == 0) {
            tokens_out[row] = eos_id;
            if (logprob_out) logprob_out[row] = 0.f;
            const int hi = hist_index ? hist_index[row] : row;
            if (hist_tokens) hist_tokens[hi] = eos_id;
            if (hist_logprob) hist_logprob[hi] = 0.f;
        }
        return;
    }
    const float *x = logits + (int64_t)(logit_row ? logit_row[row] : row) * vocab;
    if (tid == 0) {
        const uint64_t uid = seq_uid[row];
        const uint32_t st = (uint32_t)(step_base + (step ? step[row] : 0));
        uint32_t r[4];
        philox4x32_10(st, (uint32_t)uid, (uint32_t)(uid >> 32), 0u, (uint32_t)seed, (uint32_t)(seed >> 32), r);
        s_u = ((float)(r[0] >> 9) + 0.5f) * (1.0f / 8388608.0f);   // exact in fp32, inside (0,1)
    }
    constexpr int STRIDE = WAVE * VEC;
    Nucleus nu{false, 0u, 0x7fffffff, eos_key_add};
    // ---- level 1: online (max, sum) per contiguous wave segment
    const int seg = round_up((vocab + SAMPLE_WAVES - 1) / SAMPLE_WAVES, STRIDE);
    auto level1 = [&]() {
        const int b = min(vocab, wave * seg), e = min(vocab, b + seg);
        float m = -INFINITY;
        double s = 0.0;
        // four strides are fetched before the first is folded in (the fold is a serial chain, and a load
        // per link would leave the memory latency exposed at every step); the order of the arithmetic is
        // that of the plain loop
        constexpr int AHEAD = 4;
        for (int base = b; base < e; base += AHEAD * STRIDE) {
            float v[AHEAD][VEC];
            bool ok[AHEAD][VEC];
#pragma unroll
            for (int u = 0; u < AHEAD; ++u)
                load_scaled<VEC>(x, base + u * STRIDE + lane * VEC, e, inv_t, eos_id, eos_bias, v[u], ok[u], nu);
#pragma unroll
            for (int u = 0; u < AHEAD; ++u) {
                float lm = -INFINITY;
#pragma unroll
                for (int c = 0; c < VEC; ++c)
                    if (ok[u][c]) lm = fmaxf(lm, v[u][c]);
                if (lm > m) {
                    s *= (double)expf(m - lm);   // m = -inf -> 0
                    m = lm;
                }
#pragma unroll
                for (int c = 0; c < VEC; ++c)
                    if (ok[u][c]) s += (double)expf(v[u][c] - m);
            }
        }
        const float wm = wave_max_f32(m);
        const double ws = wave_sum_d(m == -INFINITY ? 0.0 : s * (double)expf(m - wm));
        if (lane == 0) {
            s_wm[wave] = wm;
            s_ws[wave] = ws;
        }
    };
    level1();
    if constexpr (TOPP) {
        // ---- nucleus: the key kstar and the id limit among its ties at which the mass from the top reaches top_p Z
        __shared__ double s_hist[SAMPLE_WAVES][256];
        __shared__ int s_cnt[SAMPLE_WAVES][256];
        __shared__ double s_comb[256];
        __shared__ int s_ccnt[256];
        __shared__ uint32_t s_prefix;
        __shared__ double s_above;
        __shared__ int s_keep_ties, s_tie_limit, s_wcount[SAMPLE_WAVES];
        __syncthreads();
        float M0 = -INFINITY;
#pragma unroll
        for (int w = 0; w < SAMPLE_WAVES; ++w) M0 = fmaxf(M0, s_wm[w]);
        double Z0 = 0.0;
#pragma unroll
        for (int w = 0; w < SAMPLE_WAVES; ++w) Z0 += (s_wm[w] == -INFINITY) ? 0.0 : s_ws[w] * (double)expf(s_wm[w] - M0);
        const double want = (double)top_p * Z0;
        if (tid == 0) {
            s_prefix = 0u;
            s_above = 0.0;
        }
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            for (int bkt = lane; bkt < 256; bkt += WAVE) {
                s_hist[wave][bkt] = 0.0;
                s_cnt[wave][bkt] = 0;
            }
            __syncthreads();
            const uint32_t prefix = s_prefix;
            for (int base = tid * VEC; base < vocab; base += SAMPLE_WAVES * WAVE * VEC) {
                float v[VEC];
                bool ok[VEC];
                float raw[VEC];
#pragma unroll
                for (int c = 0; c < VEC; ++c) raw[c] = (base + c < vocab) ? x[base + c] : 0.f;
                load_scaled<VEC>(x, base, vocab, inv_t, eos_id, eos_bias, v, ok, nu);
#pragma unroll
                for (int c = 0; c < VEC; ++c) {
                    if (!ok[c]) continue;
                    const uint32_t key = logit_key(raw[c], base + c, eos_id, eos_key_add);
                    if (pass > 0 && (key >> (shift + 8)) != prefix) continue;
                    const int bkt = (key >> shift) & 255;
                    atomicAdd(&s_hist[wave][bkt], (double)expf(v[c] - M0));
                    atomicAdd(&s_cnt[wave][bkt], 1);
                }
            }
            __syncthreads();
            if (tid < 256) {   // the waves' histograms in wave order
                double h = 0.0;
                int cn = 0;
#pragma unroll
                for (int w = 0; w < SAMPLE_WAVES; ++w) {
                    h += s_hist[w][tid];
                    cn += s_cnt[w][tid];
                }
                s_comb[tid] = h;
                s_ccnt[tid] = cn;
            }
            __syncthreads();
            if (tid == 0) {   // from the top bucket down: where the cumulative mass reaches the wanted one
                double run = s_above;
                int sel = -1, lowest = 0;
                for (int bkt = 255; bkt >= 0; --bkt) {
                    if (s_ccnt[bkt] == 0) continue;
                    lowest = bkt;
                    if (run + s_comb[bkt] >= want) {
                        sel = bkt;
                        break;
                    }
                    run += s_comb[bkt];
                }
                if (sel < 0) {   // rounding left the total short of top_p Z: every token stays
                    sel = lowest;
                    run -= s_comb[lowest];
                }
                s_above = run;
                s_prefix = (prefix << 8) | (uint32_t)sel;
                if (pass == 3) {   // ties at the cut: as many as it takes, lowest ids first
                    const int c = s_ccnt[sel];
                    const double wt = s_comb[sel] / (double)c;
                    int r = (int)ceil((want - run) / wt);
                    r = max(1, min(r, c));
                    while (r > 1 && run + (double)(r - 1) * wt >= want) --r;
                    while (r < c && run + (double)r * wt < want) ++r;
                    s_keep_ties = (r >= c) ? -1 : r;
                }
            }
            __syncthreads();
        }
        nu.kstar = s_prefix;
        nu.tie_limit = 0x7fffffff;
        const int keep_ties = s_keep_ties;
        if (keep_ties > 0) {   // (block-uniform, rare) only the first keep_ties of the tied ids stay: find the id of the last one
            int seen = 0;      // ties in the ids before this chunk (same value in every thread)
            int limit = -1;
            for (int base = 0; base < vocab && limit < 0; base += SAMPLE_WAVES * WAVE) {
                const int idx = base + tid;
                const bool tie = idx < vocab && logit_key(x[idx], idx, eos_id, eos_key_add) == nu.kstar;
                const unsigned long long bal = __ballot(tie);
                if (lane == 0) s_wcount[wave] = __popcll(bal);
                __syncthreads();
                int before = 0, total = 0;
#pragma unroll
                for (int w = 0; w < SAMPLE_WAVES; ++w) {
                    if (w < wave) before += s_wcount[w];
                    total += s_wcount[w];
                }
                if (seen + total >= keep_ties) {   // the last kept tie is in this chunk
                    const int rank = seen + before + __popcll(bal & ((1ull << lane) - 1ull));   // ties before this id
                    if (tie && rank == keep_ties - 1) s_tie_limit = idx;
                    limit = 0;
                }
                seen += total;
                __syncthreads();
            }
            nu.tie_limit = s_tie_limit;
        }
        nu.on = true;
        __syncthreads();
        level1();   // the same pass over the kept tokens only
    }
    __syncthreads();
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < SAMPLE_WAVES; ++w) M = fmaxf(M, s_wm[w]);
    double Z = 0.0, segw[SAMPLE_WAVES];
#pragma unroll
    for (int w = 0; w < SAMPLE_WAVES; ++w) {
        segw[w] = (s_wm[w] == -INFINITY) ? 0.0 : s_ws[w] * (double)expf(s_wm[w] - M);
        Z += segw[w];
    }
    const double target = (double)s_u * Z;
    int k = -1;
    double before = 0.0, run = 0.0;
#pragma unroll
    for (int w = 0; w < SAMPLE_WAVES; ++w) {
        if (k < 0 && run + segw[w] > target) {
            k = w;
            before = run;
        }
        run += segw[w];
    }
    if (k < 0) {   // rounding left no crossing: the last segment with weight
        run = 0.0;
#pragma unroll
        for (int w = 0; w < SAMPLE_WAVES; ++w) {
            if (segw[w] > 0.0) {
                k = w;
                before = run;
            }
            run += segw[w];
        }
    }
    double rem = target - before;
    const int kb = min(vocab, k * seg), ke = min(vocab, kb + seg);
    // ---- level 2: 16 sub-segments of segment k
    const int sub = round_up((seg + SAMPLE_WAVES - 1) / SAMPLE_WAVES, STRIDE);
    {
        const int b = min(ke, kb + wave * sub), e = min(ke, b + sub);
        double s = 0.0;
        for (int base = b; base < e; base += STRIDE) {
            float v[VEC];
            bool ok[VEC];
            load_scaled<VEC>(x, base + lane * VEC, e, inv_t, eos_id, eos_bias, v, ok, nu);
#pragma unroll
            for (int c = 0; c < VEC; ++c)
                if (ok[c]) s += (double)expf(v[c] - M);
        }
        s = wave_sum_d(s);
        if (lane == 0) s_sub[wave] = s;
    }
    __syncthreads();
    if (wave != 0) return;
    int j = -1;
    before = 0.0;
    run = 0.0;
#pragma unroll
    for (int w = 0; w < SAMPLE_WAVES; ++w) {
        const double sw = s_sub[w];
        if (j < 0 && run + sw > rem) {
            j = w;
            before = run;
        }
        run += sw;
    }
    if (j < 0) {
        run = 0.0;
#pragma unroll
        for (int w = 0; w < SAMPLE_WAVES; ++w) {
            if (s_sub[w] > 0.0) {
                j = w;
                before = run;
            }
            run += s_sub[w];
        }
        if (j < 0) j = 0;
    }
    rem -= before;
    // ---- level 3: wave 0 scans sub-segment j in index order
    const int jb = min(ke, kb + j * sub), je = min(ke, jb + sub);
    double running = 0.0;
    int token = -1, last_pos = -1;
    float tok_x = 0.f;
    for (int base = jb; base < je && token < 0; base += STRIDE) {
        float v[VEC];
        bool ok[VEC];
        const int idx = base + lane * VEC;
        load_scaled<VEC>(x, idx, je, inv_t, eos_id, eos_bias, v, ok, nu);
        double pre[VEC], lsum = 0.0;
        int my_last = -1;
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            const double w = ok[c] ? (double)expf(v[c] - M) : 0.0;
            lsum += w;
            pre[c] = lsum;
            if (w > 0.0) my_last = idx + c;
        }
        double incl = lsum;
#pragma unroll
        for (int o = 1; o < WAVE; o <<= 1) {
            const double t = __shfl_up(incl, o, WAVE);
            if (lane >= o) incl += t;
        }
        const double excl = running + (incl - lsum);
        int cross = -1;
#pragma unroll
        for (int c = VEC - 1; c >= 0; --c)
            if (ok[c] && excl + pre[c] > rem) cross = c;
        const unsigned long long bal = __ballot(cross >= 0);
        if (bal) {
            const int src = __ffsll((long long)bal) - 1;
            const int t = __shfl(idx + (cross < 0 ? 0 : cross), src, WAVE);
            float xv = 0.f;
#pragma unroll
            for (int c = 0; c < VEC; ++c)
                if (c == cross) xv = v[c];
            tok_x = __shfl(xv, src, WAVE);
            token = t;
        }
        running += __shfl(incl, WAVE - 1, WAVE);
        // remember the last index that carried weight, for the no-crossing case
        int ml = my_last;
#pragma unroll
        for (int o = WAVE / 2; o > 0; o >>= 1) ml = max(ml, __shfl_xor(ml, o, WAVE));
        last_pos = max(last_pos, ml);
    }
    if (token < 0) {
        token = last_pos >= 0 ? last_pos : max(0, je - 1);
        tok_x = x[token] * inv_t + (token == eos_id ? eos_bias : 0.f);
    }
    if (lane == 0) {
        tokens_out[row] = token;
        const float lp = (float)((double)tok_x - (double)M - log(Z));
        if (logprob_out) logprob_out[row] = lp;
        if (finished && token == eos_id) finished[row] = 1;
        const int hi = hist_index ? hist_index[row] : row;
        if (hist_tokens) hist_tokens[hi] = token;
        if (hist_logprob) hist_logprob[hi] = lp;
    }
}

void launch_sample(const float *logits, const int32_t *logit_row, int n, int vocab, float temperature, float top_p,
                   uint64_t seed, const uint64_t *seq_uid, const int32_t *step, int step_base, int eos_id, float eos_bias,
                   int32_t *tokens_out, float *logprob_out, uint8_t *finished, int32_t *hist_tokens,
                   float *hist_logprob, const int32_t *hist_index, hipStream_t s) {
    if (n <= 0) return;
    const float inv_t = 1.0f / temperature;
    const bool vec = (vocab % 4 == 0) && (((uintptr_t)logits) % 16 == 0);
    const float key_add = (eos_id >= 0) ? eos_bias * temperature : 0.f;
#define PC_SAMPLE(V, TP)                                                                                          \
    sample_kernel<V, TP><<<n, SAMPLE_WAVES * WAVE, 0, s>>>(logits, logit_row, vocab, inv_t, top_p, key_add, seed, seq_uid, \
                                                           step, step_base, eos_id, eos_bias, tokens_out, logprob_out,      \
                                                           finished, hist_tokens, hist_logprob, hist_index)
    if (top_p < 1.0f) {
        if (vec) PC_SAMPLE(4, true);
        else PC_SAMPLE(1, true);
    } else {
        if (vec) PC_SAMPLE(4, false);
        else PC_SAMPLE(1, false);
    }
#undef PC_SAMPLE
}

// log softmax(logits / T) at a given token per row (teacher-forced scoring: Section 3.1, the per-token
// factors of Eq. 2's ratio).  One block of 16 waves per row, the row is read once: online (max, sum) per
// thread, combined over the block; sums in double.  The target of row r is tokens[token_index[r] + 1]:
// the token that follows the position whose logits the row holds.
template <int VEC>
__global__ __launch_bounds__(SAMPLE_WAVES *WAVE) void logprob_kernel(const float *__restrict__ logits, int vocab,
                                                                      float inv_t,
                                                                      const int32_t *__restrict__ tokens,
                                                                      const int32_t *__restrict__ token_index,
                                                                      float *__restrict__ out) {
    __shared__ float s_wm[SAMPLE_WAVES];
    __shared__ double s_ws[SAMPLE_WAVES];
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid % WAVE, wave = tid / WAVE;
    const float *x = logits + (int64_t)row * vocab;
    float m = -INFINITY;
    double s = 0.0;
    for (int base = tid * VEC; base < vocab; base += SAMPLE_WAVES * WAVE * VEC) {
        float v[VEC];
        bool ok[VEC];
        load_scaled<VEC>(x, base, vocab, inv_t, -1, 0.f, v, ok, Nucleus{false, 0u, 0, 0.f});
        float lm = -INFINITY;
#pragma unroll
        for (int c = 0; c < VEC; ++c)
            if (ok[c]) lm = fmaxf(lm, v[c]);
        if (lm > m) {
            s *= (double)expf(m - lm);
            m = lm;
        }
#pragma unroll
        for (int c = 0; c < VEC; ++c)
            if (ok[c]) s += (double)expf(v[c] - m);
    }
    const float wm = wave_max_f32(m);
    const double ws = wave_sum_d(m == -INFINITY ? 0.0 : s * (double)expf(m - wm));
    if (lane == 0) {
        s_wm[wave] = wm;
        s_ws[wave] = ws;
    }
    __syncthreads();
    if (tid == 0) {
        float M = -INFINITY;
        for (int w = 0; w < SAMPLE_WAVES; ++w) M = fmaxf(M, s_wm[w]);
        double Z = 0.0;
        for (int w = 0; w < SAMPLE_WAVES; ++w) Z += (s_wm[w] == -INFINITY) ? 0.0 : s_ws[w] * (double)expf(s_wm[w] - M);
        const int target = tokens[token_index[row] + 1];
        float lp = -INFINITY;
        if (target >= 0 && target < vocab) lp = (float)((double)(x[target] * inv_t) - (double)M - log(Z));
        out[row] = lp;
    }
}

void launch_logprob(const float *logits, int n, int vocab, float temperature, const int32_t *tokens,
                    const int32_t *token_index, float *out, hipStream_t s) {
    if (n <= 0) return;
    const float inv_t = 1.0f / temperature;
    const bool vec = (vocab % 4 == 0) && (((uintptr_t)logits) % 16 == 0);
    if (vec)
        logprob_kernel<4><<<n, SAMPLE_WAVES * WAVE, 0, s>>>(logits, vocab, inv_t, tokens, token_index, out);
    else
        logprob_kernel<1><<<n, SAMPLE_WAVES * WAVE, 0, s>>>(logits, vocab, inv_t, tokens, token_index, out);
}

}  // namespace pc
