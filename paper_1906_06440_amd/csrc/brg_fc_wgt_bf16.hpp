// Weight and bias gradient of a bf16 fully connected layer on 16-wide blocks (Algorithm 5 of the paper run
// on the transposed problem): dWt block (kb, cb) [c][k] = sum over the minibatch of X[n][c] * dY[n][k], fp32.
//
// Both operands of this GEMM have the reduction index (the minibatch row) as their SLOW index in memory:
// X [N/bn][C/16][bn][16 c] and dY [N/bn][K/16][bn][16 k] keep the 16 channels of a row together.  The bf16
// matrix instruction wants 8 consecutive reduction elements per lane, so a 32-row slab of each block is
// staged in LDS as it is stored ([row][16 channels], 32 bytes per row) and read back through the
// transposing LDS read of gfx950 (ds_read_b64_tr_b16): inside a 16-lane group, lane t points at row t/4,
// channel quad t%4, and receives rows 0..3 of channel t.  Two such reads give a lane its 8 rows.
//
//  * One workgroup (4 waves as 2 x 2) owns 2 WT x 2 WT blocks of dWt (WT = 4: 8 channel blocks x 8 feature
//    blocks, 16 MFMAs per 16 LDS reads and wave; WT = 2 when that would start fewer than 128 workgroups)
//    and walks the whole minibatch in steps of 32 rows.
//  * Per step every thread moves WT x 16 bytes global -> registers -> LDS for the step after the one being
//    multiplied (double buffer, one barrier per step).
//  * Bias gradient: the workgroups of the first channel super-block multiply dY by an all-ones operand,
//    which leaves sum_n dY[n][k] in every row of one more accumulator tile per feature block.
#pragma once

#include "brg_common.hpp"

namespace brg {

struct FcWgtBf16Args {
    const bf16_t *X, *dY;
    float *dWt, *db;          // db may be null
    int Nb, Cb, Kb, bn;       // bn a multiple of 32, Cb and Kb multiples of 2 WT
};

template <int WT> __global__ __launch_bounds__(256) void fc_wgt_bf16(FcWgtBf16Args a)
{
    typedef short s4v __attribute__((ext_vector_type(4)));
    typedef short s8v __attribute__((ext_vector_type(8)));
    typedef __attribute__((address_space(3))) s4v *lds_s4p;
    constexpr int SB = 2 * WT;                                         // blocks per side of the super-block
    __shared__ __attribute__((aligned(16))) char slab[2][2 * SB][1024];   // [buffer][chunk: SB of X, SB of dY][32 rows x 32 B]
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int li = lane & 15, kg = lane >> 4;
    const int wy = wave >> 1, wx = wave & 1;                          // channel half, feature half of the super-block
    const int cb0 = blockIdx.x * SB, kb0 = blockIdx.y * SB;
    const int spb = a.bn >> 5;                                        // steps per minibatch block
    const int nsteps = a.Nb * spb;

    // staging: wave w moves chunks WT w .. WT w + WT-1 (chunks 0..SB-1: channel blocks of X, then feature blocks of dY)
    const char *src[WT];
    int64_t blk_stride[WT];                                            // bytes between minibatch blocks
#pragma unroll
    for (int j = 0; j < WT; ++j) {
        const int ch = WT * wave + j;
        if (ch < SB) {
            src[j] = (const char *)a.X + ((int64_t)(cb0 + ch) * a.bn * 16) * 2 + lane * 16;
            blk_stride[j] = (int64_t)a.Cb * a.bn * 32;
        } else {
            src[j] = (const char *)a.dY + ((int64_t)(kb0 + ch - SB) * a.bn * 16) * 2 + lane * 16;
            blk_stride[j] = (int64_t)a.Kb * a.bn * 32;
        }
    }
    bf16x8v stage[WT];
    auto load_step = [&](int s) {
        const int nb = s / spb, r0 = (s - nb * spb) * 32;
#pragma unroll
        for (int j = 0; j < WT; ++j) stage[j] = *(const bf16x8v *)(src[j] + nb * blk_stride[j] + (int64_t)r0 * 32);
    };
    auto store_step = [&](int buf) {
#pragma unroll
        for (int j = 0; j < WT; ++j) *(bf16x8v *)(&slab[buf][WT * wave + j][lane * 16]) = stage[j];
    };

    // transposing reads: rows 8 kg + li/4 (and + 4), channel quad li % 4 of a chunk
    const int tr_off = (8 * kg + (li >> 2)) * 32 + (li & 3) * 8;
    auto frag = [&](int buf, int chunk) {
        const s4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4p)(&slab[buf][chunk][tr_off]));
        const s4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4p)(&slab[buf][chunk][tr_off + 128]));
        return __builtin_bit_cast(bf16x8v, s8v{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]});
    };

    float4v acc[WT][WT], accb[WT];
#pragma unroll
    for (int i = 0; i < WT; ++i) {
        accb[i] = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < WT; ++j) acc[i][j] = float4v{0.f, 0.f, 0.f, 0.f};
    }
    const bool do_db = a.db != nullptr && blockIdx.x == 0 && wy == 0;
    const short one = 0x3F80;                                          // bf16 1.0
    const bf16x8v ones = __builtin_bit_cast(bf16x8v, s8v{one, one, one, one, one, one, one, one});

    load_step(0);
    store_step(0);
    __syncthreads();
    for (int s = 0; s < nsteps; ++s) {
        const int buf = s & 1;
        if (s + 1 < nsteps) load_step(s + 1);
        bf16x8v fa[WT], fb[WT];
#pragma unroll
        for (int i = 0; i < WT; ++i) {
            fa[i] = frag(buf, WT * wy + i);
            fb[i] = frag(buf, SB + WT * wx + i);
        }
#pragma unroll
        for (int i = 0; i < WT; ++i)
#pragma unroll
            for (int j = 0; j < WT; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        if (do_db) {
#pragma unroll
            for (int j = 0; j < WT; ++j) accb[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, fb[j], accb[j], 0, 0, 0);
        }
        if (s + 1 < nsteps) store_step(buf ^ 1);
        __syncthreads();
    }

    // register r of lane l of a tile is row c = 4*(l/16) + r, column k = l%16
#pragma unroll
    for (int i = 0; i < WT; ++i)
#pragma unroll
        for (int j = 0; j < WT; ++j) {
            float *blk = a.dWt + ((int64_t)(kb0 + WT * wx + j) * a.Cb + (cb0 + WT * wy + i)) * 256;
#pragma unroll
            for (int r = 0; r < 4; ++r) blk[(4 * kg + r) * 16 + li] = acc[i][j][r];
        }
    if (do_db && kg == 0) {
#pragma unroll
        for (int j = 0; j < WT; ++j) a.db[(kb0 + WT * wx + j) * 16 + li] = accb[j][0];
    }
}

// dst = src o [mask > 0], eight bf16 per thread (ReLU backward as a pass of its own: the masked gradient
// dZ = dY o [Y > 0] feeds both the by-data and the weight-gradient kernels, and dX o [X > 0] is the
// gradient handed to the producing layer).  dst may alias src.
__global__ __launch_bounds__(256) void fc_mask_bf16(bf16_t *dst, const bf16_t *src, const bf16_t *mask, int64_t n8)
{
    typedef unsigned short us8v __attribute__((ext_vector_type(8)));
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (int64_t)gridDim.x * 256) {
        us8v v = ((const us8v *)src)[i];
        const us8v m = ((const us8v *)mask)[i];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = bf16_to_f32(m[e]) > 0.f ? v[e] : (unsigned short)0;
        ((us8v *)dst)[i] = v;
    }
}

static int launch_fc_mask_bf16(void *dst, const void *src, const void *mask, int64_t n, hipStream_t s, const char *who)
{
    const int64_t n8 = n / 8;                      // (N*K and N*C are multiples of 256 on 16-wide blocks)
    const unsigned grid = (unsigned)((n8 + 255) / 256 < 2048 ? (n8 + 255) / 256 : 2048);
    hipLaunchKernelGGL(fc_mask_bf16, dim3(grid), dim3(256), 0, s, (bf16_t *)dst, (const bf16_t *)src, (const bf16_t *)mask, n8);
    return check_launch(who);
}

static bool fc_wgt_bf16_applies(int Cb, int Kb, int bn)
{
    return Cb % 4 == 0 && Kb % 4 == 0 && bn % 32 == 0 && !knobs().fc_wgt_general.set;
}

static int launch_fc_wgt_bf16(const FcWgtBf16Args &a, hipStream_t s, const char *who)
{
    const bool big = a.Cb % 8 == 0 && a.Kb % 8 == 0 && (a.Cb / 8) * (a.Kb / 8) >= 128;
    if (big) hipLaunchKernelGGL(fc_wgt_bf16<4>, dim3(a.Cb / 8, a.Kb / 8), dim3(256), 0, s, a);
    else hipLaunchKernelGGL(fc_wgt_bf16<2>, dim3(a.Cb / 4, a.Kb / 4), dim3(256), 0, s, a);
    return check_launch(who);
}

}  // namespace brg
