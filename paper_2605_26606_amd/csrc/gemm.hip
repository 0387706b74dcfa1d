// Projection GEMMs of the decoder (Section 3.1 policy pi_theta):
//   C[M,N] = A[M,K] * W[N,K]^T, fp32 accumulation, with fused epilogues.
// Two implementations:
//   gemm_simt   plain-ALU tiles, any dtype (the fp32 model path)
//   gemm_mfma   bf16 on the matrix cores (v_mfma_f32_32x32x16_bf16), LDS
//               double-buffered, one barrier per K tile
#include "pc_internal.h"

namespace pc {

__device__ inline float silu_f(float x) { return x / (1.0f + expf(-x)); }

template <typename T> __device__ inline void store_out(T *p, float v) { *p = from_f32<T>(v); }

// =====================================================================================
// plain-ALU GEMM: 64x64 tile, BK = 16, 256 threads, 4x4 outputs per thread at stride 16
// =====================================================================================
template <typename T, int EPI>
__global__ __launch_bounds__(256) void gemm_simt_kernel(const T *__restrict__ A, const T *__restrict__ W,
                                                        void *__restrict__ Cv, int M, int N, int K) {
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float As[BK][BM + 4];
    __shared__ float Ws[BK][BN + 4];
    const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    float acc[4][4] = {};
    const int lr = tid / 4, lk = (tid % 4) * 4;   // load coordinates: row lr, k lk..lk+3
    for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int k = k0 + lk + i;
            int am = m0 + lr, wn = n0 + lr;
            As[lk + i][lr] = (am < M && k < K) ? to_f32(A[(int64_t)am * K + k]) : 0.f;
            Ws[lk + i][lr] = (wn < N && k < K) ? to_f32(W[(int64_t)wn * K + k]) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < BK; ++k) {
            float a[4], w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[i] = As[k][ty + 16 * i];
                w[i] = Ws[k][tx + 16 * i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int row = m0 + ty + 16 * i;
        if (row >= M) continue;
        if (EPI == EPI_SWIGLU) {
            // this tile is one gate/up chunk: columns [0,32) gate, [32,64) the matching up
            T *C = (T *)Cv;
            int ob = (n0 / 64) * 32;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                if (n0 + tx + 16 * j + 32 < N)
                    store_out(&C[(int64_t)row * (N / 2) + ob + tx + 16 * j], silu_f(acc[i][j]) * acc[i][j + 2]);
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                int col = n0 + tx + 16 * j;
                if (col >= N) continue;
                if (EPI == EPI_STORE_F32) ((float *)Cv)[(int64_t)row * N + col] = acc[i][j];
                if (EPI == EPI_RESID_F32) ((float *)Cv)[(int64_t)row * N + col] += acc[i][j];
                if (EPI == EPI_STORE_T) store_out(&((T *)Cv)[(int64_t)row * N + col], acc[i][j]);
            }
        }
    }
}

template <typename T>
static void gemm_simt(const void *A, const void *W, void *C, int M, int N, int K, int epi, hipStream_t s) {
    dim3 grid((N + 63) / 64, (M + 63) / 64);
    const T *a = (const T *)A, *w = (const T *)W;
    switch (epi) {
        case EPI_STORE_F32: gemm_simt_kernel<T, EPI_STORE_F32><<<grid, 256, 0, s>>>(a, w, C, M, N, K); break;
        case EPI_RESID_F32: gemm_simt_kernel<T, EPI_RESID_F32><<<grid, 256, 0, s>>>(a, w, C, M, N, K); break;
        case EPI_SWIGLU: gemm_simt_kernel<T, EPI_SWIGLU><<<grid, 256, 0, s>>>(a, w, C, M, N, K); break;
        default: gemm_simt_kernel<T, EPI_STORE_T><<<grid, 256, 0, s>>>(a, w, C, M, N, K); break;
    }
}

// =====================================================================================
// matrix-core GEMM (bf16 in, fp32 accumulate)
// =====================================================================================
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// One 32x32x16 product per instruction.  Operand layout (wave of 64 lanes):
//   a: lane l holds A[row = l%32][k = 8*(l/32) .. +7]
//   b: lane l holds B[k = 8*(l/32) .. +7][col = l%32]   (= W[n = l%32][k...], contiguous in memory)
//   d: lane l, element v holds D[row = 8*(v/4) + 4*(l/32) + v%4][col = l%32]
template <int BM, int BN, int WM, int WN, int EPI>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(const bf16_t *__restrict__ A, const bf16_t *__restrict__ W,
                                                        void *__restrict__ Cv, int M, int N, int K) {
    constexpr int BK = 64;
    constexpr int LDS_STRIDE = BK + 8;   // elements; 144-byte rows keep 128-bit LDS reads conflict-free
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int A_ITERS = BM / 32, W_ITERS = BN / 32;   // 256 threads move 32 rows of 64 k per pass
    static_assert(WM * WN == 4, "four waves per block");
    static_assert(EPI != EPI_SWIGLU || (BN / WN) == 64, "SwiGLU needs one 64-wide gate/up chunk per wave");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16_t *As = (bf16_t *)smem_raw;                       // [2][BM][LDS_STRIDE]
    bf16_t *Ws = As + 2 * BM * LDS_STRIDE;                 // [2][BN][LDS_STRIDE]

    const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
    const int wm = wave / WN, wn = wave % WN;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int lrow = tid / 8, lchunk = tid % 8;            // global->LDS: row lrow (+32 per pass), 16-byte chunk lchunk
    const int KT = (K + BK - 1) / BK;

    u32x4 ra[A_ITERS], rw[W_ITERS];
    auto load_global = [&](int kt) {
        const int k = kt * BK + lchunk * 8;
#pragma unroll
        for (int i = 0; i < A_ITERS; ++i) {
            int r = m0 + lrow + 32 * i;
            ra[i] = (r < M && k < K) ? *(const u32x4 *)(A + (int64_t)r * K + k) : (u32x4){0, 0, 0, 0};
        }
#pragma unroll
        for (int i = 0; i < W_ITERS; ++i) {
            int r = n0 + lrow + 32 * i;
            rw[i] = (r < N && k < K) ? *(const u32x4 *)(W + (int64_t)r * K + k) : (u32x4){0, 0, 0, 0};
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_ITERS; ++i)
            *(u32x4 *)(As + (buf * BM + lrow + 32 * i) * LDS_STRIDE + lchunk * 8) = ra[i];
#pragma unroll
        for (int i = 0; i < W_ITERS; ++i)
            *(u32x4 *)(Ws + (buf * BN + lrow + 32 * i) * LDS_STRIDE + lchunk * 8) = rw[i];
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    load_global(0);
    store_lds(0);
    __syncthreads();
    const int fr = lane % 32, fg = lane / 32;
    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) load_global(kt + 1);
        const bf16_t *as = As + (buf * BM + wm * (BM / WM) + fr) * LDS_STRIDE + fg * 8;
        const bf16_t *ws = Ws + (buf * BN + wn * (BN / WN) + fr) * LDS_STRIDE + fg * 8;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[i] = *(const bf16x8 *)(as + i * 32 * LDS_STRIDE + kk * 16);
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[j] = *(const bf16x8 *)(ws + j * 32 * LDS_STRIDE + kk * 16);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) store_lds(buf ^ 1);
        __syncthreads();
    }

    // epilogue
    const int col_l = lane % 32;
    const int row_l = 4 * (lane / 32);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int rbase = m0 + wm * (BM / WM) + i * 32 + row_l;
        if (EPI == EPI_SWIGLU) {
            bf16_t *C = (bf16_t *)Cv;
            const int ncol = n0 + wn * 64;                 // start of this wave's gate/up chunk
            const int ocol = (ncol / 64) * 32 + col_l;
            if (ncol + 32 + col_l < N) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    int row = rbase + 8 * (v / 4) + (v % 4);
                    if (row < M) C[(int64_t)row * (N / 2) + ocol] = f32_to_bf16(silu_f(acc[i][0][v]) * acc[i][1][v]);
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = n0 + wn * (BN / WN) + j * 32 + col_l;
                if (col >= N) continue;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    int row = rbase + 8 * (v / 4) + (v % 4);
                    if (row >= M) continue;
                    if (EPI == EPI_STORE_F32) ((float *)Cv)[(int64_t)row * N + col] = acc[i][j][v];
                    if (EPI == EPI_RESID_F32) ((float *)Cv)[(int64_t)row * N + col] += acc[i][j][v];
                    if (EPI == EPI_STORE_T) ((bf16_t *)Cv)[(int64_t)row * N + col] = f32_to_bf16(acc[i][j][v]);
                }
            }
        }
    }
}

template <int BM, int BN, int WM, int WN> struct MfmaCfg {
    static constexpr size_t smem = (size_t)2 * (BM + BN) * (64 + 8) * sizeof(bf16_t);
    template <int E> static void set_attr() {
        (void)hipFuncSetAttribute((const void *)gemm_mfma_kernel<BM, BN, WM, WN, E>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    }
    static void init() {
        set_attr<EPI_STORE_F32>();
        set_attr<EPI_RESID_F32>();
        set_attr<EPI_STORE_T>();
        if constexpr (BN / WN == 64) set_attr<EPI_SWIGLU>();
    }
    static void run(const void *A, const void *W, void *C, int M, int N, int K, int epi, hipStream_t s) {
        dim3 grid((N + BN - 1) / BN, (M + BM - 1) / BM);
        const bf16_t *a = (const bf16_t *)A, *w = (const bf16_t *)W;
        switch (epi) {
            case EPI_STORE_F32: gemm_mfma_kernel<BM, BN, WM, WN, EPI_STORE_F32><<<grid, 256, smem, s>>>(a, w, C, M, N, K); break;
            case EPI_RESID_F32: gemm_mfma_kernel<BM, BN, WM, WN, EPI_RESID_F32><<<grid, 256, smem, s>>>(a, w, C, M, N, K); break;
            case EPI_SWIGLU:
                if constexpr (BN / WN == 64)
                    gemm_mfma_kernel<BM, BN, WM, WN, EPI_SWIGLU><<<grid, 256, smem, s>>>(a, w, C, M, N, K);
                break;
            default: gemm_mfma_kernel<BM, BN, WM, WN, EPI_STORE_T><<<grid, 256, smem, s>>>(a, w, C, M, N, K); break;
        }
    }
};

typedef MfmaCfg<128, 128, 2, 2> CfgLarge;   // wave tile 64x64
typedef MfmaCfg<128, 64, 4, 1> CfgSkinny;   // wave tile 32x64: more blocks when M is small

void gemm_init() {
    CfgLarge::init();
    CfgSkinny::init();
}

static void gemm_mfma(const void *A, const void *W, void *C, int M, int N, int K, int epi, hipStream_t s) {
    if (M > 512)
        CfgLarge::run(A, W, C, M, N, K, epi, s);
    else
        CfgSkinny::run(A, W, C, M, N, K, epi, s);
}

void launch_gemm(int dtype, int impl, const void *A, const void *W, void *C, int M, int N, int K, int epi,
                 hipStream_t s) {
    if (M <= 0 || N <= 0) return;
    if (dtype == PC_DTYPE_F32) {
        gemm_simt<float>(A, W, C, M, N, K, epi, s);
    } else if (impl == 0 || (K % 8) != 0) {
        gemm_simt<bf16_t>(A, W, C, M, N, K, epi, s);
    } else {
        gemm_mfma(A, W, C, M, N, K, epi, s);
    }
}

}  // namespace pc
