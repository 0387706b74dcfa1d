// Standalone driver for the two kernels that dominate a decode step: it launches the library's own
// decode-attention kernel and projection GEMMs, in the launch configurations of the 1.5B-shaped
// workload, with synthetic cache contents, and times them with HIP events.  Used for tuning and for
// hardware-counter runs (rocprofv3 --pmc), which need a plain process without HIP graphs.
//
//   kernel_bench attn [n_seqs group prompt_len gen_len block_size grouped_only event_study]   (defaults 256 4 256 512 64 0 0)
//       event_study: also brackets single launches with an event pair, as the library's per-launch timing does,
//       next to pairs around nothing / one / two empty kernels and around two launches
//   kernel_bench gemm
//   kernel_bench copy                                       (a plain 1 GiB copy: the counters' known-size reference)
#include <stdio.h>
#include <string.h>

#include <vector>

#include "attention.hip"
#include "gemm.hip"

namespace pc {
void set_error(const char *, ...) {}
}
using namespace pc;

#define CK(x)                                                                          \
    do {                                                                               \
        hipError_t e_ = (x);                                                           \
        if (e_ != hipSuccess) {                                                        \
            fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));                    \
            return 1;                                                                  \
        }                                                                              \
    } while (0)

__global__ void fill_half_kernel(uint16_t *p, size_t n, uint32_t seed) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        uint32_t h = (uint32_t)(i * 2654435761u) ^ seed;
        p[i] = 0x2800 | (h & 0x3FF) | ((h >> 3) & 0x8000);   // +-(0.03 .. 0.06) as IEEE half
    }
}
__global__ void copy_kernel(const float4 *__restrict__ src, float4 *__restrict__ dst, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

__global__ void null_kernel() {}

static int bench_attention(int n, int group, int lp, int gen, int bs, bool grouped_only, bool event_study) {
    const int L = 28, hq = 12, hkv = 2, hd = 128;
    const int P = n / group, ctx = lp + gen;
    const int pre_blocks = lp / bs, own_blocks = (ctx + bs - 1) / bs - pre_blocks, per_slot = pre_blocks + own_blocks;
    const int64_t n_blocks = (int64_t)P * pre_blocks + (int64_t)n * own_blocks;
    const int64_t block_elems = (int64_t)hkv * 2 * bs * hd;
    void *pool;
    CK(hipMalloc(&pool, (size_t)(L * n_blocks * block_elems * 2)));
    fill_half_kernel<<<(unsigned)((L * n_blocks * block_elems + 255) / 256), 256>>>((uint16_t *)pool,
                                                                                    (size_t)(L * n_blocks * block_elems), 9);
    std::vector<int32_t> table((size_t)n * per_slot), len(n, ctx - 1), slot(n);
    for (int s = 0; s < n; ++s) {
        slot[s] = s;
        for (int b = 0; b < pre_blocks; ++b) table[(size_t)s * per_slot + b] = (s / group) * pre_blocks + b;
        for (int b = 0; b < own_blocks; ++b) table[(size_t)s * per_slot + pre_blocks + b] = P * pre_blocks + s * own_blocks + b;
    }
    int32_t *d_table, *d_len, *d_slot;
    CK(hipMalloc(&d_table, table.size() * 4));
    CK(hipMalloc(&d_len, n * 4));
    CK(hipMalloc(&d_slot, n * 4));
    CK(hipMemcpy(d_table, table.data(), table.size() * 4, hipMemcpyHostToDevice));
    CK(hipMemcpy(d_len, len.data(), n * 4, hipMemcpyHostToDevice));
    CK(hipMemcpy(d_slot, slot.data(), n * 4, hipMemcpyHostToDevice));
    void *q, *out;
    float *scratch;
    CK(hipMalloc(&q, (size_t)n * hq * hd * 2));
    CK(hipMalloc(&out, (size_t)n * hq * hd * 2));
    fill_half_kernel<<<(n * hq * hd + 255) / 256, 256>>>((uint16_t *)q, (size_t)n * hq * hd, 3);
    CK(hipMalloc(&scratch, attention_decode_scratch_floats(n, hq, hd) * 4));
    KvGeom kv;
    kv.pool = pool;
    kv.layer_stride = n_blocks * block_elems;
    kv.block_size = bs;
    kv.n_kv_heads = hkv;
    kv.head_dim = hd;
    kv.max_blocks_per_slot = per_slot;
    kv.block_table = d_table;
    const int splits = attention_decode_splits(n, hkv, ctx + 64);
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    for (int g : {group, 1}) {
        if (grouped_only && g != group) continue;
        auto layer = [&](int l) {   // the merge pass only runs when the context is split
            launch_attention_decode_mfma(KD_F16, q, d_slot, d_len, n, hq, kv, l, splits, g, scratch, out, nullptr, 0);
            launch_attention_decode_merge(KD_F16, d_slot, d_len, n, hq, hkv, splits, scratch, out, nullptr, 0);
        };
        for (int l = 0; l < L; ++l) layer(l);
        CK(hipDeviceSynchronize());
        const int reps = 3;
        CK(hipEventRecord(e0, 0));
        for (int r = 0; r < reps; ++r)
            for (int l = 0; l < L; ++l) layer(l);
        CK(hipEventRecord(e1, 0));
        CK(hipEventSynchronize(e1));
        float ms;
        CK(hipEventElapsedTime(&ms, e0, e1));
        const double us = ms * 1e3 / (reps * L);
        const double alg = ((double)P * lp + (double)n * gen) * 2 * hkv * hd * 2;       // prefix once per prompt
        const double raw = (double)n * ctx * 2 * hkv * hd * 2;                          // prefix once per sequence
        printf("attention n=%d group=%d(order %d) block %d ctx=%d+%d splits=%d: %.2f us/launch  algorithmic %.1f MB -> %.0f GB/s  "
               "(per-sequence bytes %.1f MB -> %.0f GB/s)  %s\n",
               n, group, g, bs, lp, gen, splits, us, alg / 1e6, alg / us / 1e3, raw / 1e6, raw / us / 1e3,
               hipGetErrorString(hipGetLastError()));
        if (event_study && g == group) {
            // what an event pair reads around k launches of a kernel, averaged
            auto pair_us = [&](int k, bool attn, double *out_us) -> int {
                const int reps = 3;
                double tot = 0;
                for (int r = 0; r < reps; ++r)
                    for (int l = 0; l < L; ++l) {
                        CK(hipEventRecord(e0, 0));
                        for (int c = 0; c < k; ++c) {
                            if (attn) layer(l);
                            else null_kernel<<<1, 64>>>();
                        }
                        CK(hipEventRecord(e1, 0));
                        CK(hipEventSynchronize(e1));
                        float one;
                        CK(hipEventElapsedTime(&one, e0, e1));
                        tot += one;
                    }
                *out_us = tot * 1e3 / (reps * L);
                return 0;
            };
            double p0, n1, n2, a1, a2;
            if (pair_us(0, false, &p0) || pair_us(1, false, &n1) || pair_us(2, false, &n2) || pair_us(1, true, &a1) ||
                pair_us(2, true, &a2))
                return 1;
            printf("event pair around: nothing %.2f us, one empty kernel %.2f us, two empty kernels %.2f us, "
                   "one attention launch %.2f us, two attention launches %.2f us\n", p0, n1, n2, a1, a2);
            printf("  attention launch: %.2f us by (pair - empty pair), %.2f us by (two launches - one launch)\n", a1 - p0,
                   a2 - a1);
        }
    }
    return 0;
}

template <typename Cfg>
static int run_gemm(const char *name, int M, int N, int K, int epi, int split, std::vector<void *> &Ws, void *A, void *C,
                    float *slices) {
    Cfg::init();
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    const int ring = (int)Ws.size();
    for (int i = 0; i < 3; ++i) Cfg::run(A, Ws[i % ring], split > 1 ? (void *)slices : C, M, N, K, epi, split, nullptr, 0);
    CK(hipDeviceSynchronize());
    const int iters = 24;
    CK(hipEventRecord(e0, 0));
    for (int i = 0; i < iters; ++i) Cfg::run(A, Ws[i % ring], split > 1 ? (void *)slices : C, M, N, K, epi, split, nullptr, 0);
    CK(hipEventRecord(e1, 0));
    CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    const double us = ms * 1000 / iters;
    printf("gemm %-28s M=%5d N=%6d K=%5d slices=%2d: %8.2f us  weights %.2f TB/s  %.1f TFLOP/s  %s\n", name, M, N, K, split,
           us, (double)N * K * 2 / us / 1e6, 2.0 * M * N * K / us / 1e6, hipGetErrorString(hipGetLastError()));
    return 0;
}

static int bench_gemm() {
    typedef f16_t T;
    const size_t NK = (size_t)17920 * 1536;
    void *A, *C;
    float *slices;
    CK(hipMalloc(&A, (size_t)16384 * 8960 * 2));
    fill_half_kernel<<<(unsigned)(((size_t)16384 * 8960 + 255) / 256), 256>>>((uint16_t *)A, (size_t)16384 * 8960, 1);
    std::vector<void *> Ws(12);   // a ring larger than the caches: every launch streams its weights from HBM
    for (size_t i = 0; i < Ws.size(); ++i) {
        CK(hipMalloc(&Ws[i], NK * 2));
        fill_half_kernel<<<(unsigned)((NK + 255) / 256), 256>>>((uint16_t *)Ws[i], NK, 77 + (uint32_t)i);
    }
    CK(hipMalloc(&C, (size_t)16384 * 17920 * 4));
    CK(hipMalloc(&slices, (size_t)32 << 20));
    CK(hipDeviceSynchronize());
    int rc = 0;
    rc |= run_gemm<MfmaCfg<T, 256, 128, 4, 2, 3>>("decode gate/up (SwiGLU)", 256, 17920, 1536, EPI_SWIGLU, 1, Ws, A, C, slices);
    rc |= run_gemm<MfmaCfg<T, 128, 64, 2, 2, 4>>("decode down", 256, 1536, 8960, EPI_STORE_F32, 5, Ws, A, C, slices);
    rc |= run_gemm<MfmaCfg<T, 64, 64, 2, 2, 4>>("decode o-proj", 256, 1536, 1536, EPI_STORE_F32, 2, Ws, A, C, slices);
    rc |= run_gemm<MfmaCfg<T, 64, 64, 2, 2, 4>>("decode qkv", 256, 2048, 1536, EPI_STORE_F32, 2, Ws, A, C, slices);
    rc |= run_gemm<MfmaCfg<T, 256, 256, 4, 2, 4, 32, true>>("prefill gate/up (SwiGLU)", 16384, 17920, 1536, EPI_SWIGLU, 1, Ws, A, C, slices);
    rc |= run_gemm<MfmaCfg<T, 256, 128, 4, 2, 3, 64, true>>("prefill down (+residual)", 16384, 1536, 8960, EPI_RESID_F32, 1, Ws, A, C, slices);
    return rc;
}

static int bench_copy() {
    const size_t bytes = (size_t)1 << 30, n = bytes / 16;
    float4 *src, *dst;
    CK(hipMalloc((void **)&src, bytes));
    CK(hipMalloc((void **)&dst, bytes));
    CK(hipMemset(src, 1, bytes));
    for (int i = 0; i < 3; ++i) copy_kernel<<<(unsigned)((n + 255) / 256), 256>>>(src, dst, n);
    CK(hipDeviceSynchronize());
    printf("copy_kernel: 3 launches, each reads 1 GiB (1048576 KiB) and writes 1 GiB\n");
    return 0;
}

int main(int argc, char **argv) {
    const char *what = argc > 1 ? argv[1] : "attn";
    if (!strcmp(what, "attn")) {
        const int n = argc > 2 ? atoi(argv[2]) : 256, g = argc > 3 ? atoi(argv[3]) : 4;
        const int lp = argc > 4 ? atoi(argv[4]) : 256, gen = argc > 5 ? atoi(argv[5]) : 512;
        const int bs = argc > 6 ? atoi(argv[6]) : 64;
        if (n <= 0 || g <= 0 || n % g || lp <= 0 || (bs != 32 && bs != 64 && bs != 128) || lp % bs || gen <= 0) {
            fprintf(stderr, "bad sizes\n");
            return 2;
        }
        return bench_attention(n, g, lp, gen, bs, argc > 7 && atoi(argv[7]) != 0, argc > 8 && atoi(argv[8]) != 0);
    }
    if (!strcmp(what, "gemm")) return bench_gemm();
    if (!strcmp(what, "copy")) return bench_copy();
    fprintf(stderr, "usage: kernel_bench attn|gemm|copy\n");
    return 2;
}
