// Index maps shared by kernels and host code (plain integer arithmetic, usable on either side; the host
// build of the tests checks them exhaustively on the CPU).
#pragma once

#if defined(__HIPCC__) || defined(__CUDACC__)
#define PC_HD __host__ __device__
#else
#define PC_HD
#endif

namespace pc {

// ---- KV cache, operand-fragment order (head_dim a multiple of 32, block_size a multiple of 32).
// Element offset of K[token tin][dim d] inside the K half of one (block, kv head) region: tiles of 32 tokens,
// a tile = 2 x (head_dim / 32) fragments [u][kk] of 512 elements; lane (i, g) of fragment (u, kk) holds dims
// 32 kk + 8 g .. + 7 of token 8 (i / 4) + i % 4 + 4 u of the tile, at element (16 g + i) * 8 of the fragment.
PC_HD inline int kv_k_index_frag(int tin, int d, int head_dim) {
    const int tt = tin & 31, u = (tt >> 2) & 1, i = ((tt >> 3) << 2) | (tt & 3);
    const int frag = ((tin >> 5) * 2 + u) * (head_dim >> 5) + (d >> 5);
    return (frag << 9) + (((((d & 31) >> 3) << 4) + i) << 3) + (d & 7);
}
// Element offset of V[token tin][dim d] inside the V half: tiles of 32 tokens, a tile = head_dim / 16 fragments
// [nn]; lane (i, g) of fragment nn holds tokens 8 g .. 8 g + 7 of dim 16 nn + i.
PC_HD inline int kv_v_index_frag(int tin, int d, int head_dim) {
    const int frag = (tin >> 5) * (head_dim >> 4) + (d >> 4);
    return (frag << 9) + (((((tin & 31) >> 3) << 4) + (d & 15)) << 3) + (tin & 7);
}

// ---- GEMM, many row blocks (a multiple of 8): workgroup id -> output tile.  Workgroup i runs on die i % 8.
// Every die owns mb / 8 row blocks and walks all column blocks in groups of 8, patch by patch of `ph` row
// blocks x 8 column blocks (ph = 4 where mb / 8 allows), so that the 32 blocks a die runs at a time share few
// activation and weight slabs.  Returns false for ids past the last tile.
PC_HD inline bool gemm_patch_tile(int id, int mb, int nb, int *bm, int *bn) {
    const int die = id % 8, j = id / 8;
    const int rows_per = mb / 8;
    if (j >= rows_per * nb) return false;
    const int ph = (rows_per % 4 == 0) ? 4 : ((rows_per % 2 == 0) ? 2 : 1);
    const int full = rows_per * 8;                        // tiles of a full group of 8 column blocks
    const int last = (nb - 1) / 8;
    const int cg = (j / full < last) ? j / full : last;
    const int w = (nb - 8 * cg < 8) ? nb - 8 * cg : 8;
    const int jj = j - cg * full;
    const int sg = jj / (ph * w), r = jj % (ph * w);
    *bm = die * rows_per + sg * ph + r % ph;
    *bn = 8 * cg + r / ph;
    return true;
}

}   // namespace pc
