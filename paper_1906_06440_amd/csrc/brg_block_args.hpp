// Arguments shared by the kernels over 64 x 64 x 64 fp32 blocks (brg_block_ring.hpp, brg_block_dma.hpp):
// the shape every block call of the fully connected layers (Algorithm 5 of the paper) and of the
// standalone batch-reduce GEMM benchmark has.
#pragma once

#include "brg_common.hpp"

namespace brg {

struct BlockTileArgs {
    const float *A, *B;
    const float *Amask, *Bmask;  // optional: operand element is taken as 0 where mask <= 0 (ReLU backward)
    float *C;
    const float *bias;           // per row of C (length tiles_m*64) or null
    int act;
    int tiles_m, tiles_n, chain;
    float alpha, beta;
    // element strides (floats): block (tile, c) of A starts at A + tile*a_tile + c*a_chain, its rows are a_ld apart
    int64_t a_tile, a_chain, b_tile, b_chain, c_tile_m, c_tile_n;
    int a_ld, b_ld, c_ld;
    int xcd_patch;  // 1: 16x16 tile grids are dealt to the 8 XCDs as 4x8 patches
    // Address-list form (section 2 of the paper: "two arrays of pointers"): when non-null, block c of the
    // chain is A_ptrs[c] / B_ptrs[c] (plus the tile offset) instead of A + c*a_chain / B + c*b_chain.
    const float *const *A_ptrs, *const *B_ptrs;
};

}  // namespace brg
