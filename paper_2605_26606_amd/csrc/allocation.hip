// Pilot-Commit allocation on the device: per-prompt reward statistics (Eq. 3,
// Section 3.3 pilot success rate), the pilot filter with eviction flags and the
// stable compaction of the commit set (Section 3.3, Algorithm 1), and
// group-relative advantages (Section 3.1).  KBs of data: latency only.
#include "pc_internal.h"

namespace pc {

static constexpr int WAVE = 64;

// one thread per group; sums in double, index order, two passes
__global__ void group_stats_kernel(const float *__restrict__ rewards, const int32_t *__restrict__ off, int P,
                                   int32_t *__restrict__ n_pos, int32_t *__restrict__ n_tot, float *__restrict__ mean,
                                   float *__restrict__ var) {
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= P) return;
    const int b = off[p], e = off[p + 1], n = e - b;
    int pos = 0;
    double s = 0.0;
    for (int i = b; i < e; ++i) {
        const float r = rewards[i];
        s += (double)r;
        pos += (r != 0.0f);
    }
    double mu = 0.0, v = 0.0;
    if (n > 0) {
        mu = s / (double)n;
        double ss = 0.0;
        for (int i = b; i < e; ++i) {
            const double d = (double)rewards[i] - mu;
            ss += d * d;
        }
        v = ss / (double)n;
    }
    if (n_pos) n_pos[p] = pos;
    if (n_tot) n_tot[p] = n;
    if (mean) mean[p] = (float)mu;
    if (var) var[p] = (float)v;
}

void launch_group_stats(const float *rewards, const int32_t *off, int P, int32_t *n_pos, int32_t *n_tot, float *mean,
                        float *var, hipStream_t s) {
    if (P <= 0) return;
    group_stats_kernel<<<(P + 127) / 128, 128, 0, s>>>(rewards, off, P, n_pos, n_tot, mean, var);
}

// One block walks the batch in chunks of 1024 prompts; the kept prompts are
// compacted in batch order (ballot ranks inside a wave, a 16-entry prefix
// across waves, a running count across chunks).
// VAR: the filter for rewards that are not binary: `p_hat` is the pilot mean, `var` the pilot variance, lo / hi are
// the variance thresholds on the approaching (mean <= pivot) and on the leaving side (mean > pivot).
template <bool VAR>
__global__ __launch_bounds__(1024) void select_commit_kernel(const float *__restrict__ p_hat,
                                                             const float *__restrict__ var, int P, float lo, float hi,
                                                             float pivot, float solve, int b_t, uint8_t *__restrict__ cls,
                                                             uint8_t *__restrict__ evict,
                                                             int32_t *__restrict__ commit_idx,
                                                             int32_t *__restrict__ surplus_idx,
                                                             int32_t *__restrict__ counts) {
    __shared__ int w_keep[16], w_easy[16], w_hard[16];
    const int tid = threadIdx.x, lane = tid % WAVE, wave = tid / WAVE;
    int kept_before = 0, n_easy = 0, n_hard = 0;
    for (int q0 = 0; q0 < P; q0 += 1024) {
        const int q = q0 + tid;
        int c = -1;
        if (q < P) {
            const float ph = p_hat[q];
            if (VAR) {
                const float vr = var[q];
                const bool approaching = ph <= pivot;
                const bool kept = approaching ? (vr >= lo) : (vr >= hi);
                c = kept ? 1 : (approaching ? 0 : 2);
            } else {
                c = (ph > hi) ? 2 : (ph < lo) ? 0 : 1;
            }
            if (cls) cls[q] = (uint8_t)c;
            if (evict) evict[q] = (ph >= solve) ? 1 : 0;
        }
        const unsigned long long bk = __ballot(c == 1), be = __ballot(c == 2), bh = __ballot(c == 0);
        if (lane == 0) {
            w_keep[wave] = __popcll(bk);
            w_easy[wave] = __popcll(be);
            w_hard[wave] = __popcll(bh);
        }
        __syncthreads();
        int wave_off = 0, chunk_keep = 0;
        for (int w = 0; w < 16; ++w) {
            if (w < wave) wave_off += w_keep[w];
            chunk_keep += w_keep[w];
            n_easy += w_easy[w];
            n_hard += w_hard[w];
        }
        if (c == 1) {
            const int rank = kept_before + wave_off + __popcll(bk & ((1ull << lane) - 1ull));
            if (b_t <= 0 || rank < b_t)
                commit_idx[rank] = q;
            else if (surplus_idx)
                surplus_idx[rank - b_t] = q;
        }
        kept_before += chunk_keep;
        __syncthreads();
    }
    if (tid == 0) {
        const int n_commit = (b_t <= 0) ? kept_before : min(kept_before, b_t);
        counts[0] = n_commit;
        counts[1] = kept_before - n_commit;
        counts[2] = n_easy;
        counts[3] = n_hard;
    }
}

void launch_select_commit(const float *p_hat, int P, float lo, float hi, float solve, int b_t, uint8_t *cls,
                          uint8_t *evict, int32_t *commit_idx, int32_t *surplus_idx, int32_t *counts, hipStream_t s) {
    select_commit_kernel<false><<<1, 1024, 0, s>>>(p_hat, nullptr, P, lo, hi, 0.f, solve, b_t, cls, evict, commit_idx,
                                                   surplus_idx, counts);
}

void launch_select_commit_var(const float *mean, const float *var, int P, float var_hard, float var_easy, float pivot,
                              float solve, int b_t, uint8_t *cls, uint8_t *evict, int32_t *commit_idx, int32_t *surplus_idx,
                              int32_t *counts, hipStream_t s) {
    select_commit_kernel<true><<<1, 1024, 0, s>>>(mean, var, P, var_hard, var_easy, pivot, solve, b_t, cls, evict,
                                                  commit_idx, surplus_idx, counts);
}

// one thread per group, double inside
__global__ void advantages_kernel(const float *__restrict__ rewards, const int32_t *__restrict__ off, int P, float eps,
                                  float *__restrict__ adv, float *__restrict__ mu_out, float *__restrict__ sigma_out) {
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= P) return;
    const int b = off[p], e = off[p + 1], n = e - b;
    double mu = 0.0, sigma = 0.0;
    if (n > 0) {
        double s = 0.0;
        for (int i = b; i < e; ++i) s += (double)rewards[i];
        mu = s / (double)n;
        double ss = 0.0;
        for (int i = b; i < e; ++i) {
            const double d = (double)rewards[i] - mu;
            ss += d * d;
        }
        sigma = sqrt(ss / (double)n);
        const double den = sigma + (double)eps;
        for (int i = b; i < e; ++i) {
            const double d = (double)rewards[i] - mu;
            adv[i] = (d == 0.0) ? 0.0f : (float)(d / den);
        }
    }
    if (mu_out) mu_out[p] = (float)mu;
    if (sigma_out) sigma_out[p] = (float)sigma;
}

void launch_advantages(const float *rewards, const int32_t *off, int P, float eps, float *adv, float *mu, float *sigma,
                       hipStream_t s) {
    if (P <= 0) return;
    advantages_kernel<<<(P + 127) / 128, 128, 0, s>>>(rewards, off, P, eps, adv, mu, sigma);
}

}  // namespace pc
