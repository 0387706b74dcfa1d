// Projection GEMMs of the decoder (Section 3.1 policy pi_theta):
//   C[M,N] = A[M,K] * W[N,K]^T, fp32 accumulation, with fused epilogues.
// Two implementations:
//   gemm_simt   plain-ALU tiles, any dtype (the fp32 model path)
//   gemm_mfma   bf16 / f16 on the matrix cores (32x32x16 or 16x16x32 products),
//               operands streamed global -> LDS several K tiles ahead, one
//               barrier per K tile, output rows re-formed through LDS
#include <algorithm>

#include <type_traits>

#include "pc_internal.h"

namespace pc {

__device__ inline float silu_f(float x) { return x / (1.0f + expf(-x)); }

template <typename T> __device__ inline void store_out(T *p, float v, uint32_t *sat) { *p = from_f32_sat<T>(v, sat); }

// =====================================================================================
// plain-ALU GEMM: 64x64 tile, BK = 16, 256 threads, 4x4 outputs per thread at stride 16
// =====================================================================================
template <typename T, int EPI>
__global__ __launch_bounds__(256) void gemm_simt_kernel(const T *__restrict__ A, const T *__restrict__ W,
                                                        void *__restrict__ Cv, int M, int N, int K,
                                                        uint32_t *__restrict__ sat) {
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
                    store_out(&C[(int64_t)row * (N / 2) + ob + tx + 16 * j], silu_f(acc[i][j]) * acc[i][j + 2], sat);
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                int col = n0 + tx + 16 * j;
                if (col >= N) continue;
                if (EPI == EPI_STORE_F32) ((float *)Cv)[(int64_t)row * N + col] = acc[i][j];
                if (EPI == EPI_RESID_F32) ((float *)Cv)[(int64_t)row * N + col] += acc[i][j];
                if (EPI == EPI_STORE_T) store_out(&((T *)Cv)[(int64_t)row * N + col], acc[i][j], sat);
            }
        }
    }
}

template <typename T>
static void gemm_simt(const void *A, const void *W, void *C, int M, int N, int K, int epi, uint32_t *sat, hipStream_t s) {
    dim3 grid((N + 63) / 64, (M + 63) / 64);
    const T *a = (const T *)A, *w = (const T *)W;
    switch (epi) {
        case EPI_STORE_F32: gemm_simt_kernel<T, EPI_STORE_F32><<<grid, 256, 0, s>>>(a, w, C, M, N, K, sat); break;
        case EPI_RESID_F32: gemm_simt_kernel<T, EPI_RESID_F32><<<grid, 256, 0, s>>>(a, w, C, M, N, K, sat); break;
        case EPI_SWIGLU: gemm_simt_kernel<T, EPI_SWIGLU><<<grid, 256, 0, s>>>(a, w, C, M, N, K, sat); break;
        default: gemm_simt_kernel<T, EPI_STORE_T><<<grid, 256, 0, s>>>(a, w, C, M, N, K, sat); break;
    }
}

// =====================================================================================
// matrix-core GEMM (bf16 in, fp32 accumulate)
// =====================================================================================
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

static constexpr int N_XCD = 8;   // MI355X: 8 accelerator dies, each with its own L2; workgroup i runs on die i % 8

// One 32x32x16 product per instruction.  Operand layout (wave of 64 lanes):
//   a: lane l holds X[row = l%32][k = 8*(l/32) .. +7]
//   b: lane l holds Y[k = 8*(l/32) .. +7][col = l%32]
//   d: lane l, element v holds D[row = 8*(v/4) + 4*(l/32) + v%4][col = l%32]
// The kernel passes the WEIGHT fragment as a and the activation fragment as b (both are 8 consecutive k of one
// matrix row, contiguous in memory), so d is the transposed output tile: lane l holds output row l%32 and, per
// group of four elements, four consecutive output columns.
//
// Work decomposition: a 1-D grid; workgroup id -> (m block, n block, K slice) such that the m blocks
// that share a weight tile run on the same die back to back (the second one finds the tile in L2).
// K slices (S > 1) write plain fp32 slices [S][M][N] to `Cv`; whoever consumes them adds them up in
// slice order (no atomics, no fences: the kernel boundary orders the two).
//
// Data path: global memory -> LDS directly (global_load_lds_dwordx4, no register staging), NSTAGE
// tiles deep, one barrier per K tile; LDS -> registers one K step ahead of the products, also across tiles.  A wave-wide load lands as 1 KB of consecutive LDS (8 rows of
// 64 k); to keep the 128-bit fragment reads conflict free without padding, the 16-byte chunk c of
// row r is stored at chunk slot c ^ swz(r) (the lane fetches the chunk its slot must hold), where swz
// makes any 16 consecutive rows hit 16 different 16-byte bank groups.  K must be a multiple of 64 here.
template <int N> __device__ inline void wait_vmcnt_le() {
    // s_waitcnt with only the vector-memory counter set (gfx9 encoding: vmcnt = bits 15:14 | 3:0)
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

// M16: the products are 16x16x32 instructions (a: A[row l%16][k = 8*(l/16) .. +7], b likewise,
// d[v]: D[row 4*(l/16) + v][col l%16]) instead of 32x32x16: the same fragment bytes per product volume, four
// times as many accumulator tiles per wave.
template <typename T, int BM, int BN, int WM, int WN, int NSTAGE, int BK, int EPI, bool M16 = false>
__global__ __launch_bounds__(64 * WM * WN) void gemm_mfma_kernel(const T *__restrict__ A, const T *__restrict__ W,
                                                        void *__restrict__ Cv, int M, int N, int K, int mb, int nb,
                                                        int S, int plain, uint32_t *__restrict__ sat,
                                                        GemmRowScale rsc) {
    constexpr bool SWIGLU = (EPI == EPI_SWIGLU || EPI == EPI_SWIGLU_RS);
    constexpr int CPR = BK / 8;                           // 16-byte chunks per tile row
    constexpr int RPL = 64 / CPR;                         // tile rows one wave-wide load covers
    // rows that share a swizzle value (measured with a read-rate probe: 16-row fragment reads of 64-byte
    // rows want a new value every 2 rows, 267 -> 320 GB/s per CU)
    constexpr int SWZ_DIV = (M16 && BK == 32) ? 2 : 16 / CPR;
    constexpr int RT = M16 ? 16 : 32;                     // rows (columns) of one accumulator tile
    constexpr int CG = 64 / RT;                           // 16-byte k chunks one product consumes per row
    constexpr int AV = M16 ? 4 : 16;                      // accumulator values per lane and tile
    constexpr int TM = BM / WM / RT, TN = BN / WN / RT;
    typedef typename std::conditional<M16, f32x4_t, f32x16_t>::type acc_t;
    constexpr int NW = WM * WN;                           // waves per block
    constexpr int A_ITERS = BM / (RPL * NW), W_ITERS = BN / (RPL * NW);   // the waves move RPL*NW rows of BK k per pass
    constexpr int LOADS = A_ITERS + W_ITERS;              // load instructions per thread per K tile
    constexpr int STAGE_ELEMS = (BM + BN) * BK;
    static_assert(BK == 64 || BK == 32, "K tile");
    static_assert(BM % (RPL * NW) == 0 && BN % (RPL * NW) == 0, "whole passes");
    static_assert(!SWIGLU || (BN / WN) % 64 == 0, "SwiGLU needs whole 64-wide gate/up chunks per wave");
    static_assert(NSTAGE * LOADS <= 63, "vmcnt is a 6-bit counter");
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
    T *smem = (T *)smem_raw;                     // [NSTAGE][A tile BM x 64 | W tile BN x 64]

    // ---- which tile
    const int id = blockIdx.x;
    int bm, bn, z;
    if (plain == 2) {
        // many row blocks, a multiple of 8 (prefill): every die owns mb/8 row blocks and walks all column blocks in
        // groups of 8, patch by patch of 4 row blocks x 8 column blocks.  The 32 blocks a die runs at a time then
        // share 4 activation slabs and 8 weight slabs (its L2 serves each K tile to 8 resp. 4 blocks), where plain
        // order gave a die 32 different weight slabs at once.
        if (!gemm_patch_tile(id, mb, nb, &bm, &bn)) return;
        z = 0;
    } else if (plain) {   // many row blocks (prefill): neighbours share the activation rows, plain order
        bn = id % nb;
        bm = id / nb;
        z = 0;
        if (bm >= mb) return;
    } else {
        const int die = id % N_XCD, j = id / N_XCD;
        const int unit = (j / mb) * N_XCD + die;           // (n block, K slice) pair
        if (unit >= nb * S) return;
        bm = j % mb;
        bn = unit % nb;
        z = unit / nb;
    }
    const int m0 = bm * BM, n0 = bn * BN;

    const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
    const int wm = wave / WN, wn = wave % WN;
    // the rows' RMSNorm scale from the partial sums of squares ssq[tile][row]: two threads per row, every load of a
    // thread in flight at once (a lane's neighbours read the neighbouring rows: whole cache lines per request)
    constexpr int RS_MAXT = 24;                        // tiles one thread sums per round
    __shared__ float s_rs[EPI == EPI_SWIGLU_RS ? BM : 1];
    __shared__ float s_rs_part[EPI == EPI_SWIGLU_RS ? BM : 1];
    const int KT = K / BK;
    const int per = (KT + S - 1) / S;
    const int kt0 = z * per, kt1 = min(KT, kt0 + per);

    // ---- global -> LDS: in pass i this wave fills rows (4i + wave)*8 .. +7; lane -> (row, slot)
    const int lr = lane / CPR, slot = lane % CPR;
    const T *pa[A_ITERS], *pw[W_ITERS];
#pragma unroll
    for (int i = 0; i < A_ITERS; ++i) {
        const int row = (NW * i + wave) * RPL + lr;
        const int chunk = slot ^ ((row / SWZ_DIV) & (CPR - 1));
        pa[i] = A + (int64_t)min(m0 + row, M - 1) * K + chunk * 8;   // rows past the end: clamped, results discarded
    }
#pragma unroll
    for (int i = 0; i < W_ITERS; ++i) {
        const int row = (NW * i + wave) * RPL + lr;
        const int chunk = slot ^ ((row / SWZ_DIV) & (CPR - 1));
        pw[i] = W + (int64_t)min(n0 + row, N - 1) * K + chunk * 8;
    }
    auto issue_tile = [&](int kt, int stage) {
        const int koff = min(kt, kt1 - 1) * BK;            // past the end: a redundant reload, keeps the count constant
        T *sa = smem + stage * STAGE_ELEMS;
        T *sw = sa + BM * BK;
#pragma unroll
        for (int i = 0; i < A_ITERS; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(pa[i] + koff),
                                             (__attribute__((address_space(3))) void *)(sa + (NW * i + wave) * RPL * BK), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < W_ITERS; ++i)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(pw[i] + koff),
                                             (__attribute__((address_space(3))) void *)(sw + (NW * i + wave) * RPL * BK), 16, 0, 0);
    };

    auto issue_part = [&](int kt, int stage, int part, int parts) {   // the loads l of a tile with l * parts / LOADS == part
        const int koff = min(kt, kt1 - 1) * BK;            // past the end: a redundant reload, keeps the count constant
        T *sa = smem + stage * STAGE_ELEMS;
        T *sw = sa + BM * BK;
#pragma unroll
        for (int i = 0; i < A_ITERS; ++i)
            if (i * parts / LOADS == part)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(pa[i] + koff),
                                                 (__attribute__((address_space(3))) void *)(sa + (NW * i + wave) * RPL * BK), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < W_ITERS; ++i)
            if ((A_ITERS + i) * parts / LOADS == part)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(pw[i] + koff),
                                                 (__attribute__((address_space(3))) void *)(sw + (NW * i + wave) * RPL * BK), 16, 0, 0);
    };
    acc_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int jj = 0; jj < TN; ++jj)
#pragma unroll
            for (int v = 0; v < AV; ++v) acc[i][jj][v] = 0.f;

    // fragment addressing: lane (fr, fg) reads chunk CG*kk + fg of its row, stored at slot chunk ^ swz(row)
    const int fr = lane % RT, fg = lane / RT;
    int arow[TM], aswz[TM], wrow[TN], wswz[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        arow[i] = wm * (BM / WM) + i * RT + fr;
        aswz[i] = (arow[i] / SWZ_DIV) & (CPR - 1);
    }
#pragma unroll
    for (int jj = 0; jj < TN; ++jj) {
        wrow[jj] = wn * (BN / WN) + jj * RT + fr;
        wswz[jj] = (wrow[jj] / SWZ_DIV) & (CPR - 1);
    }
    typedef typename Mma<T>::frag frag_t;
    auto load_frags = [&](const T *sa, const T *sw, int kk, frag_t (&fa)[TM], frag_t (&fb)[TN]) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[i] = *(const frag_t *)(sa + arow[i] * BK + (((CG * kk + fg) ^ aswz[i]) * 8));
#pragma unroll
        for (int jj = 0; jj < TN; ++jj) fb[jj] = *(const frag_t *)(sw + wrow[jj] * BK + (((CG * kk + fg) ^ wswz[jj]) * 8));
    };
    auto product = [&](frag_t a, frag_t b, acc_t c) -> acc_t {
        if constexpr (M16) return Mma<T>::m16(a, b, c);
        else return Mma<T>::m32(a, b, c);
    };
    // One K step (the products of 8*CG k values of every accumulator tile), software-pipelined ACROSS K tiles: while
    // the products of this step run on the fragments `ca`/`cb` already in registers, the fragments of the next step
    // are read into `na`/`nb` -- the next step of the same tile, or, in a tile's last step, the first step of the next
    // tile.  That read needs the next tile visible, so the block's one barrier per tile sits in front of the last
    // step (not at the top of the tile), and right behind it the stage just consumed is refilled.  No product then
    // waits for an LDS read issued just before it (the first version did, once per tile: with one step per tile the
    // matrix cores idled half the time).
    // Wave tiles of fewer than four accumulator tiles (the 128x64 and 64x64 blocks of the small decode projections)
    // keep the barrier at the top of the tile and prefetch within the tile only: with two products per step there
    // is nothing to hide the hand-over under, and the plain order measured faster there (decode down projection
    // 15.1 against 16.5 us).
    constexpr int KK = BK / (8 * CG);                     // steps per tile
    constexpr bool XT = (TM * TN >= 4);                   // pipelined across tiles
    auto kstep = [&](frag_t (&ca)[TM], frag_t (&cb)[TN], frag_t (&na)[TM], frag_t (&nb)[TN], int kt, int stage, int kk) {
        const T *sa = smem + stage * STAGE_ELEMS;
        const T *sw = sa + BM * BK;
        const int pstage = (stage == 0) ? NSTAGE - 1 : stage - 1;
        if constexpr (!XT) {
            if (kk == 0) {
                wait_vmcnt_le<(NSTAGE - 2) * LOADS>();    // this thread's loads of tile kt have landed
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_barrier();             // ... and everybody's; tile kt-1 is consumed
                asm volatile("" ::: "memory");
                load_frags(sa, sw, 0, ca, cb);
            }
            issue_part(kt - 1 + NSTAGE, pstage, kk, KK);  // the refill of tile kt-1's stage, spread over the steps
            if (kk + 1 < KK) load_frags(sa, sw, kk + 1, na, nb);
        } else if (kk == KK - 1) {
            wait_vmcnt_le<(NSTAGE - 2) * LOADS>();        // this thread's loads of tile kt+1 have landed
            __builtin_amdgcn_s_waitcnt(0xC07F);           // lgkmcnt(0): and its own reads of tile kt have returned
            // ... and everybody's: behind the barrier tile kt+1 is visible and tile kt's stage is free.  A bare
            // barrier: __syncthreads() would add a fence that drains every load in flight.
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            const int nstage = (stage + 1 == NSTAGE) ? 0 : stage + 1;
            issue_part(kt + NSTAGE, stage, 0, KK);        // the refill of the stage just consumed starts here ...
            const T *nsa = smem + nstage * STAGE_ELEMS;
            load_frags(nsa, nsa + BM * BK, 0, na, nb);    // (behind the last tile: read and never used)
        } else {
            // ... and goes on over the next tile's other steps (a wave that has to hand the load unit six loads
            // in a row cannot issue matrix instructions meanwhile)
            issue_part(kt - 1 + NSTAGE, pstage, kk + 1, KK);
            load_frags(sa, sw, kk + 1, na, nb);
        }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int jj = 0; jj < TN; ++jj)
                acc[i][jj] = product(cb[jj], ca[i], acc[i][jj]);   // weights as rows: the tile comes out transposed
        // instruction order asked of the compiler: after each matrix instruction one or two LDS fragment reads and
        // one global->LDS load, instead of all of them in a burst
#pragma unroll
        for (int g = 0; g < TM * TN; ++g) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, (TM + TN + TM * TN - 1) / (TM * TN), 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
    };

    // tile kt lives in stage (kt - kt0) % NSTAGE; the tile being consumed sits in registers, the next one in LDS,
    // NSTAGE-1 more are in flight
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s) issue_tile(kt0 + s, s);
    if constexpr (XT) issue_part(kt0 + NSTAGE - 1, NSTAGE - 1, 0, KK);   // (its other parts: the first tile's steps)
    // (behind the first tile loads, so that the pipeline is already filling while the statistics arrive; these are
    // ordinary loads, younger than the tile loads: once they are back, so are the tiles)
    if constexpr (EPI == EPI_SWIGLU_RS) {
        constexpr int PARTS = (64 * NW >= 2 * BM) ? 2 : 1;   // threads per row (each sums every PARTS-th round of tiles)
        static_assert(64 * NW >= BM, "a thread per row");
        const int r = tid % BM, part = tid / BM;
        float ss = 0.f;
        if (part < PARTS) {
            const int row = min(m0 + r, M - 1);
            for (int t0 = part * RS_MAXT; t0 < rsc.tiles; t0 += PARTS * RS_MAXT) {
                float v[RS_MAXT];
#pragma unroll
                for (int u = 0; u < RS_MAXT; ++u) v[u] = (t0 + u < rsc.tiles) ? rsc.ssq[(int64_t)(t0 + u) * M + row] : 0.f;
#pragma unroll
                for (int u = 0; u < RS_MAXT; ++u) ss += v[u];
            }
        }
        if (PARTS == 2) {
            if (part == 1) s_rs_part[r] = ss;
            __syncthreads();
            if (part == 0) ss += s_rs_part[r];
        }
        if (part == 0) s_rs[r] = 1.0f / sqrtf(ss / (float)rsc.d + rsc.eps);
        __syncthreads();
    }
    frag_t fa[2][TM], fb[2][TN];
    if constexpr (XT) {
        constexpr int PART0 = (LOADS + KK - 1) / KK;       // loads l with l * KK / LOADS == 0
        wait_vmcnt_le<(NSTAGE - 2) * LOADS + PART0>();     // the first tile has landed
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        load_frags(smem, smem + BM * BK, 0, fa[0], fb[0]);
    }
    int stage = 0;
    if constexpr (KK % 2 == 0) {   // an even number of steps per tile: the two fragment sets alternate within a tile
        for (int kt = kt0; kt < kt1; ++kt) {
#pragma unroll
            for (int kk = 0; kk < KK; kk += 2) {
                kstep(fa[0], fb[0], fa[1], fb[1], kt, stage, kk);
                kstep(fa[1], fb[1], fa[0], fb[0], kt, stage, kk + 1);
            }
            stage = (stage + 1 == NSTAGE) ? 0 : stage + 1;
        }
    } else {                       // one step per tile: they alternate from tile to tile
        static_assert(KK == 1 || KK % 2 == 0, "steps per tile");
        int kt = kt0;
        for (; kt + 1 < kt1; kt += 2) {
            kstep(fa[0], fb[0], fa[1], fb[1], kt, stage, 0);
            stage = (stage + 1 == NSTAGE) ? 0 : stage + 1;
            kstep(fa[1], fb[1], fa[0], fb[0], kt + 1, stage, 0);
            stage = (stage + 1 == NSTAGE) ? 0 : stage + 1;
        }
        if (kt < kt1) kstep(fa[0], fb[0], fa[1], fb[1], kt, stage, 0);
    }
    wait_vmcnt_le<0>();   // nothing may still be writing LDS when the block retires

    // ---- epilogue
    // The products take the weights as the row operand, so the accumulators hold the TRANSPOSED tile: a lane owns ONE
    // output row m (m = lane % RT of the tile) and, per tile, runs of four consecutive output columns.  Written out
    // from there, an output row would leave in 2- or 4-byte pieces, one store instruction per value -- hundreds of
    // stores in flight per wave, which the store path takes far longer to retire than the bytes need (measured: a
    // fifth of the decode gate/up kernel).  Instead each wave turns RT output rows at a time into whole rows through
    // a private piece of the now idle LDS ring and stores them 16 bytes per lane, neighbouring lanes on
    // neighbouring addresses.  LDS instructions of one wave execute in order, so the hand-over needs no barrier.
    typedef typename std::conditional<(EPI == EPI_STORE_F32 || EPI == EPI_RESID_F32), float, T>::type OutT;
    constexpr int WCOLS = SWIGLU ? (BN / WN) / 2 : BN / WN;        // output columns of one wave
    constexpr int RB = WCOLS * (int)sizeof(OutT);                 // bytes of one output row of the wave
    constexpr int LPR = RB / 16;                                  // lanes that store one row
    constexpr int ROWS_PER = 64 / LPR;                            // rows one store instruction covers
    constexpr int ITER = RT / ROWS_PER;
    constexpr int PITCH = RB + 16;                                // bytes; the pad spreads the rows over the banks
    constexpr int EPC = 16 / (int)sizeof(OutT);                   // output elements per 16-byte piece
    static_assert(LPR >= 1 && LPR <= 64 && (64 % LPR) == 0 && ROWS_PER <= RT && ITER >= 1, "row pieces per wave");
    static_assert((size_t)NW * RT * PITCH <= (size_t)NSTAGE * STAGE_ELEMS * sizeof(T), "staging fits the ring");
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();   // every wave has consumed its last fragments (they were waited for by the products)
    asm volatile("" ::: "memory");
    unsigned char *stg = smem_raw + (size_t)wave * RT * PITCH;
    const int ml = lane % RT, nq = 4 * (lane / RT);               // the lane's row of a tile; first column of its runs
    const int ldc = SWIGLU ? N / 2 : N;
    const int colbase = SWIGLU ? (n0 + wn * (BN / WN)) / 2 : n0 + wn * (BN / WN);
    OutT *Cbase = (OutT *)Cv + ((EPI == EPI_STORE_F32) ? (int64_t)z * M * N : 0);
    auto put4 = [&](int col, float v0, float v1, float v2, float v3) {   // four consecutive columns of row ml
        unsigned char *dst = stg + ml * PITCH + col * (int)sizeof(OutT);
        if constexpr (sizeof(OutT) == 4) {
            *(f32x4_t *)dst = (f32x4_t){v0, v1, v2, v3};
        } else {
            typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
            *(u32x2 *)dst = (u32x2){pack2_sat<T>(v0, v1, sat), pack2_sat<T>(v2, v3, sat)};
        }
    };
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const float sc = (EPI == EPI_SWIGLU_RS) ? s_rs[wm * (BM / WM) + i * RT + ml] : 1.f;
        if constexpr (SWIGLU) {
            // a 64-wide chunk of weight rows = 32 gate rows, then the 32 matching up rows
            if constexpr (M16) {
#pragma unroll
                for (int p2 = 0; p2 < TN / 4; ++p2)
#pragma unroll
                    for (int q = 0; q < 2; ++q) {
                        const acc_t &ga = acc[i][4 * p2 + q], &ua = acc[i][4 * p2 + 2 + q];
                        put4(32 * p2 + 16 * q + nq, silu_f(ga[0] * sc) * (ua[0] * sc), silu_f(ga[1] * sc) * (ua[1] * sc),
                             silu_f(ga[2] * sc) * (ua[2] * sc), silu_f(ga[3] * sc) * (ua[3] * sc));
                    }
            } else {
#pragma unroll
                for (int p2 = 0; p2 < TN / 2; ++p2)
#pragma unroll
                    for (int vg = 0; vg < 4; ++vg) {
                        const acc_t &ga = acc[i][2 * p2], &ua = acc[i][2 * p2 + 1];
                        put4(32 * p2 + 8 * vg + nq, silu_f(ga[4 * vg] * sc) * (ua[4 * vg] * sc),
                             silu_f(ga[4 * vg + 1] * sc) * (ua[4 * vg + 1] * sc),
                             silu_f(ga[4 * vg + 2] * sc) * (ua[4 * vg + 2] * sc),
                             silu_f(ga[4 * vg + 3] * sc) * (ua[4 * vg + 3] * sc));
                    }
            }
        } else {
#pragma unroll
            for (int jj = 0; jj < TN; ++jj)
#pragma unroll
                for (int vg = 0; vg < AV / 4; ++vg)
                    put4(jj * RT + (M16 ? 0 : 8 * vg) + nq, acc[i][jj][4 * vg], acc[i][jj][4 * vg + 1],
                         acc[i][jj][4 * vg + 2], acc[i][jj][4 * vg + 3]);
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int it = 0; it < ITER; ++it) {
            const int row = it * ROWS_PER + lane / LPR, piece = lane % LPR;
            const u32x4 val = *(const u32x4 *)(stg + row * PITCH + piece * 16);
            const int gm = m0 + wm * (BM / WM) + i * RT + row, col = colbase + piece * EPC;
            if (gm < M && col < ldc) {
                OutT *dst = Cbase + (int64_t)gm * ldc + col;
                if constexpr (EPI == EPI_RESID_F32) {
                    const f32x4_t old = *(const f32x4_t *)dst, add = __builtin_bit_cast(f32x4_t, val);
                    *(f32x4_t *)dst = (f32x4_t){old[0] + add[0], old[1] + add[1], old[2] + add[2], old[3] + add[3]};
                } else {
                    *(u32x4 *)dst = val;
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
}

template <typename T, int BM, int BN, int WM, int WN, int NSTAGE, int BK = 64, bool M16 = false> struct MfmaCfg {
    static constexpr size_t smem = (size_t)NSTAGE * (BM + BN) * BK * sizeof(T);
    static constexpr bool swiglu_ok = ((BN / WN) % 64 == 0);
    template <int E> static void set_attr() {
        (void)hipFuncSetAttribute((const void *)gemm_mfma_kernel<T, BM, BN, WM, WN, NSTAGE, BK, E, M16>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    }
    static void init() {
        set_attr<EPI_STORE_F32>();
        set_attr<EPI_RESID_F32>();
        set_attr<EPI_STORE_T>();
        if constexpr (swiglu_ok) {
            set_attr<EPI_SWIGLU>();
            set_attr<EPI_SWIGLU_RS>();
        }
    }
    // split > 1 only with EPI_STORE_F32, C then being the slice buffer [split][M][N]
    static void run(const void *A, const void *W, void *C, int M, int N, int K, int epi, int split, uint32_t *sat, hipStream_t s,
                    const GemmRowScale *row_scale = nullptr) {
        const GemmRowScale rsc = row_scale ? *row_scale : GemmRowScale{nullptr, 0, 1, 0.f};
        const int mb = (M + BM - 1) / BM, nb = (N + BN - 1) / BN;
        const int units = nb * split;
        const int plain = (split == 1 && mb > 4) ? ((mb % N_XCD == 0) ? 2 : 1) : 0;
        const unsigned grid = plain ? (unsigned)(mb * nb) : (unsigned)((units + N_XCD - 1) / N_XCD * N_XCD * mb);
        const T *a = (const T *)A, *w = (const T *)W;
        switch (epi) {
            case EPI_STORE_F32: gemm_mfma_kernel<T, BM, BN, WM, WN, NSTAGE, BK, EPI_STORE_F32, M16><<<grid, 64 * WM * WN, smem, s>>>(a, w, C, M, N, K, mb, nb, split, plain, sat, rsc); break;
            case EPI_RESID_F32: gemm_mfma_kernel<T, BM, BN, WM, WN, NSTAGE, BK, EPI_RESID_F32, M16><<<grid, 64 * WM * WN, smem, s>>>(a, w, C, M, N, K, mb, nb, 1, plain, sat, rsc); break;
            case EPI_SWIGLU:
                if constexpr (swiglu_ok)
                    gemm_mfma_kernel<T, BM, BN, WM, WN, NSTAGE, BK, EPI_SWIGLU, M16><<<grid, 64 * WM * WN, smem, s>>>(a, w, C, M, N, K, mb, nb, 1, plain, sat, rsc);
                break;
            case EPI_SWIGLU_RS:
                if constexpr (swiglu_ok)
                    gemm_mfma_kernel<T, BM, BN, WM, WN, NSTAGE, BK, EPI_SWIGLU_RS, M16><<<grid, 64 * WM * WN, smem, s>>>(a, w, C, M, N, K, mb, nb, 1, plain, sat, rsc);
                break;
            default: gemm_mfma_kernel<T, BM, BN, WM, WN, NSTAGE, BK, EPI_STORE_T, M16><<<grid, 64 * WM * WN, smem, s>>>(a, w, C, M, N, K, mb, nb, 1, plain, sat, rsc); break;
        }
    }
    // K slices so that the launch has about `want_blocks` blocks, each with >= 4 K tiles
    static int pick_split(int M, int N, int K, size_t slice_cap_floats, int want_blocks) {
        const int64_t tiles = (int64_t)((N + BN - 1) / BN) * ((M + BM - 1) / BM);
        const int KT = K / BK;
        int64_t split = (want_blocks + tiles / 2) / tiles;
        split = std::min<int64_t>(split, KT / 4);
        split = std::min<int64_t>(split, 8);
        split = std::min<int64_t>(split, (int64_t)(slice_cap_floats / ((size_t)M * N)));
        if (split < 2) return 1;
        const int per = (KT + (int)split - 1) / (int)split;
        return (KT + per - 1) / per;   // no empty slice
    }
};

template <typename T> static void gemm_init_t() {
    MfmaCfg<T, 256, 128, 4, 2, 3>::init();
    MfmaCfg<T, 256, 256, 4, 2, 4, 32, true>::init();
    MfmaCfg<T, 256, 128, 4, 2, 3, 64, true>::init();
    MfmaCfg<T, 128, 128, 4, 2, 4>::init();
    MfmaCfg<T, 128, 64, 2, 2, 4>::init();
    MfmaCfg<T, 128, 128, 2, 2, 2>::init();
    MfmaCfg<T, 128, 128, 2, 2, 3, 32>::init();
    MfmaCfg<T, 256, 64, 4, 2, 3>::init();
    MfmaCfg<T, 64, 64, 2, 2, 4>::init();
}
void gemm_init() {
    gemm_init_t<bf16_t>();
    gemm_init_t<f16_t>();
}

template <typename T>
static int gemm_mfma_dispatch(const void *A, const void *W, void *C, int M, int N, int K, int epi, float *slices,
                              size_t slice_cap_floats, uint32_t *sat, hipStream_t s, const GemmRowScale *row_scale);

int launch_gemm(int dtype, int impl, const void *A, const void *W, void *C, int M, int N, int K, int epi,
                float *slices, size_t slice_cap_floats, uint32_t *sat, hipStream_t s, const GemmRowScale *row_scale) {
    if (M <= 0 || N <= 0) return 1;
    if (dtype == KD_F32) {
        gemm_simt<float>(A, W, C, M, N, K, epi, sat, s);
        return 1;
    }
    // (the matrix-core kernel stores whole 16-byte pieces of output rows; the SwiGLU one whole 64-wide chunks)
    if (impl == 0 || (K % 64) != 0 || (N % 16) != 0 || ((epi == EPI_SWIGLU || epi == EPI_SWIGLU_RS) && (N % 64) != 0)) {
        if (dtype == KD_BF16) gemm_simt<bf16_t>(A, W, C, M, N, K, epi, sat, s);
        else gemm_simt<f16_t>(A, W, C, M, N, K, epi, sat, s);
        return 1;
    }
    if (dtype == KD_BF16) return gemm_mfma_dispatch<bf16_t>(A, W, C, M, N, K, epi, slices, slice_cap_floats, sat, s, row_scale);
    return gemm_mfma_dispatch<f16_t>(A, W, C, M, N, K, epi, slices, slice_cap_floats, sat, s, row_scale);
}

template <typename T>
static int gemm_mfma_dispatch(const void *A, const void *W, void *C, int M, int N, int K, int epi, float *slices,
                              size_t slice_cap_floats, uint32_t *sat, hipStream_t s, const GemmRowScale *row_scale) {
    // Configurations picked by measurement on MI355X (M = 256 decode rows / 16384 prefill rows, 1.5B shapes).
    typedef MfmaCfg<T, 256, 128, 4, 2, 3> CfgTall;          // 8 waves, wave tile 64x64, every decode row in one block
    // prefill: 16x16x32 products (measured +3 to +12 % over 32x32x16 at 16384 rows, nothing at decode sizes;
    // the results are bit-identical)
    typedef MfmaCfg<T, 256, 128, 4, 2, 3, 64, true> CfgPrefill;
    typedef MfmaCfg<T, 256, 256, 4, 2, 4, 32, true> CfgWide;   // wave tile 64x128: three fragment reads per four products
    typedef MfmaCfg<T, 128, 128, 4, 2, 4> CfgLarge;         // 8 waves of 32x64: up to 128 rows what counts is loads in flight (22 against 25 us for gate/up with 4 waves of 64x64)
    typedef MfmaCfg<T, 128, 128, 2, 2, 2> CfgLarge2;        // two stages, 64 KB of LDS: two blocks per CU
    typedef MfmaCfg<T, 128, 128, 2, 2, 3, 32> CfgLarge3;    // BK 32, 48 KB of LDS: three blocks per CU
    typedef MfmaCfg<T, 128, 64, 2, 2, 4> CfgMid;            // wave tile 64x32: long-K projections cut into K slices
    typedef MfmaCfg<T, 256, 64, 4, 2, 3> CfgMidTall;        // the same for more than 256 rows
    typedef MfmaCfg<T, 64, 64, 2, 2, 4> CfgSmall;           // wave tile 32x32: many blocks for the small projections
    if (M > 512) {   // prefill: plenty of tiles
        // 256x256 tiles where they still come in several rounds per CU (the wide projections: +10 % measured);
        // the narrow ones (1536 columns: 1.5 rounds of such tiles) keep 256x128
        const int64_t wide_tiles = (int64_t)((M + 255) / 256) * ((N + 255) / 256);
        if (wide_tiles >= 2 * 256) {
            CfgWide::run(A, W, C, M, N, K, epi, 1, sat, s);
            return 1;
        }
        // a large decode batch (a thousand rows) against a narrow projection leaves most CUs without a tile
        // (1024 rows x 1536 columns: 48 tiles of 256x128): cut K into slices, as the small batches do
        const int64_t tiles = (int64_t)((M + 255) / 256) * ((N + 127) / 128);
        if (tiles < 160 && slices && (epi == EPI_STORE_F32 || epi == EPI_RESID_F32)) {
            const int split = CfgPrefill::pick_split(M, N, K, slice_cap_floats, 240);
            if (split > 1) {
                CfgPrefill::run(A, W, slices, M, N, K, EPI_STORE_F32, split, sat, s);
                return split;
            }
        }
        CfgPrefill::run(A, W, C, M, N, K, epi, 1, sat, s);
        return 1;
    }
    // decode: the weights are streamed once; fill the chip with blocks, by K slices where N is small.
    // (Rules from sweeps of every configuration over the projection shapes of the 1.5B, 8B and 14B models at
    // 128, 256 and 400 rows.)
    const bool can_split = slices && (epi == EPI_STORE_F32 || epi == EPI_RESID_F32);
    const int nb128 = (N + 127) / 128;
    // a long reduction amortises a block's fill and drain, and the tile with the most fragment reuse wins at
    // every row count; a short one (the 1.5B model: 24 K tiles) prefers several smaller blocks per CU
    const bool deep = K >= 3072;
    if (epi == EPI_SWIGLU || epi == EPI_SWIGLU_RS || nb128 >= 96) {   // wide outputs: no K slices needed
        // (the vocabulary projection: several rounds of blocks per CU at any tile size, the big tile wins --
        // 240 us against 311 us at 400 rows of the 1.5B shape)
        if (M > 256 && nb128 >= 512 && epi != EPI_SWIGLU && epi != EPI_SWIGLU_RS) CfgPrefill::run(A, W, C, M, N, K, epi, 1, sat, s);
        else if (M > 384 && !deep) CfgLarge3::run(A, W, C, M, N, K, epi, 1, sat, s, row_scale);       // four 128-row blocks, three per CU at a time
        else if (M > 256 && !deep) CfgLarge2::run(A, W, C, M, N, K, epi, 1, sat, s, row_scale);  // three 128-row blocks, not two of 256
        else if (M > 128) CfgTall::run(A, W, C, M, N, K, epi, 1, sat, s, row_scale);    // a weight tile is fetched by exactly one block
        else CfgLarge::run(A, W, C, M, N, K, epi, 1, sat, s, row_scale);
        return 1;
    }
    if ((int64_t)N * K >= (int64_t)8 << 20 && nb128 >= 24) {
        // mid-width outputs with large weights (q/k/v, o and down projections of the 8B / 14B models): 128-column
        // tiles cut into about 240 blocks by K slices (8B down at 256 rows: 33 us against 48 us for 128x64 tiles)
        if (M > 128) {
            const int split = can_split ? CfgTall::pick_split(M, N, K, slice_cap_floats, 240) : 1;
            if (split > 1) {
                CfgTall::run(A, W, slices, M, N, K, EPI_STORE_F32, split, sat, s);
                return split;
            }
            CfgTall::run(A, W, C, M, N, K, epi, 1, sat, s);
            return 1;
        }
        const int split = can_split ? CfgLarge::pick_split(M, N, K, slice_cap_floats, 240) : 1;
        if (split > 1) {
            CfgLarge::run(A, W, slices, M, N, K, EPI_STORE_F32, split, sat, s);
            return split;
        }
        CfgLarge::run(A, W, C, M, N, K, epi, 1, sat, s);
        return 1;
    }
    if ((int64_t)N * K >= (int64_t)8 << 20) {   // narrow output, long K (the 1.5B model's down projection)
        if (M > 256) {
            const int split = can_split ? CfgMidTall::pick_split(M, N, K, slice_cap_floats, 240) : 1;
            if (split > 1) {
                CfgMidTall::run(A, W, slices, M, N, K, EPI_STORE_F32, split, sat, s);
                return split;
            }
            CfgMidTall::run(A, W, C, M, N, K, epi, 1, sat, s);
            return 1;
        }
        const int split = can_split ? CfgMid::pick_split(M, N, K, slice_cap_floats, 240) : 1;
        if (split > 1) {
            CfgMid::run(A, W, slices, M, N, K, EPI_STORE_F32, split, sat, s);
            return split;
        }
        CfgMid::run(A, W, C, M, N, K, epi, 1, sat, s);
        return 1;
    }
    const int split = can_split ? CfgSmall::pick_split(M, N, K, slice_cap_floats, 192) : 1;
    if (split > 1) {
        CfgSmall::run(A, W, slices, M, N, K, EPI_STORE_F32, split, sat, s);
        return split;
    }
    CfgSmall::run(A, W, C, M, N, K, epi, 1, sat, s);
    return 1;
}

}  // namespace pc
