// 1x1 convolutions in bf16 with a long reduction (C >= 256) on few pixels: the batch-reduce GEMM of
// paper section 3.2 / Algorithm 4 (R = S = 1) as a workgroup-tiled GEMM.
//
// The streaming kernel (brg_conv1x1_bf16.hpp) gives every wave its own 64 x 64 (features x pixels) tile and
// loads both operands from global memory per wave.  At 14x14 and 7x7 images with 512..2048 channels the
// weights are megabytes and every wave re-reads its slice of them for only 32..64 pixels: the vector
// memory pipeline of the CU (64 bytes per clock) becomes the bound, at 0.5 - 0.75 KiB per matrix
// instruction.  Here a workgroup of four waves (2 x 2) owns 128 features x 128 pixels and the operands of
// one 32-channel step (8 + 8 KiB) are loaded from global memory ONCE per workgroup, written to LDS and read
// back by the two waves that need each of them: 0.25 KiB per matrix instruction through the memory
// pipeline.
//
//  * Registers are the prefetch buffer (D sets of four 16-byte loads per lane: the loads of a step are
//    issued D-1 steps before they are needed, which is what covers the memory latency with only two
//    workgroups on a CU), LDS only the exchange: two slots of 16 KiB, one __syncthreads per step.  In step
//    u every wave issues the loads of step u+D, writes step u+1 into the slot that was read in step u-1,
//    passes the barrier, reads the fragments of step u+1 and multiplies step u (fragments read a step ago).  The reduction length must be a
//    multiple of D steps (C a multiple of 32 D).
//  * A slab is 1 KiB: one pair of channel blocks of one feature block (weights) or of one 16-pixel group
//    (activations), stored in LDS exactly as the 64 lanes loaded it (lane * 16 bytes).  Activations and
//    reduction-contiguous weights (backward by data) are loaded in matrix-operand order, so a lane reads
//    its operand back with one 16-byte LDS read; forward weights (feature index contiguous inside a block)
//    are loaded linearly and read back with two transposing LDS reads (see conv1x1_bf16, WTR).
//  * Pixel addressing, bias as the accumulators' start value and the epilogue are those of conv1x1_bf16.
#pragma once

#include "brg_conv1x1_bf16.hpp"
#include "brg_conv_tile.hpp"

namespace brg {

// NGW: 16-pixel groups per wave, 4 (workgroup tile 128 x 128) or 2 (128 x 64, for layers that would
// otherwise start fewer workgroups than there are CUs).
template <bool WTR, int D, int NGW> __global__ __launch_bounds__(256) void conv1x1_bf16_lds(Conv1x1Args a)
{
    constexpr int NB = 2 * NGW;                        // pixel slabs of the workgroup
    constexpr int LB = NGW / 2;                        // pixel slabs each wave loads per step
    __shared__ __attribute__((aligned(16))) char lds[2][8 + NB][1024];   // [slot][8 weight slabs, NB pixel slabs][1 KiB]
    const char *__restrict__ I = (const char *)a.I;
    const char *__restrict__ Wt = (const char *)a.Wt;
    char *__restrict__ O = (char *)a.O;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int li = lane & 15, kg = lane >> 4;
    const int wm = wave & 1, wn = wave >> 1;           // this wave multiplies feature blocks 4wm.. x pixel groups 4wn..
    // Workgroups are dealt round-robin to the 8 XCDs: give each XCD a contiguous range of tiles, in
    // feature-major order (its L2 holds few weight slabs, all pixel tiles stream through) or pixel-major
    // order (few pixel slabs, all weights stream through), whichever operand is the smaller one to stream
    const int tile = xcd_tile(blockIdx.x, a.tiles);
    int tx, ty;
    if (a.pixel_major) {
        tx = c1_fdiv(tile, a.tiles_y, a.inv_tiles_y);
        ty = tile - tx * a.tiles_y;
    } else {
        ty = c1_fdiv(tile, a.tiles_x, a.inv_tiles_x);
        tx = tile - ty * a.tiles_x;
    }
    const int kb0 = ty * 8;                            // first feature block of the workgroup
    const int grp0 = tx * NB;                          // first 16-pixel group of the workgroup

    const uint32_t cbs = (uint32_t)(a.Hin * a.Win) * 32u;           // bytes of one channel-block plane
    const uint32_t kbs = (uint32_t)(a.Hout * a.Wout) * 32u;
    const int PQ = a.P * a.Q;
    auto pixel = [&](int grp, uint32_t &in_o, uint32_t &out_o) {    // lane li's pixel of a 16-pixel group
        const int pix = grp * 16 + li;
        const bool ok = pix < a.npix;
        const int p = ok ? pix : a.npix - 1;           // lanes beyond the end load a valid pixel, store nothing
        const int n = c1_fdiv(p, PQ, a.inv_PQ), r = p - n * PQ;
        const int oj = c1_fdiv(r, a.Q, a.inv_Q), oi = r - oj * a.Q;
        in_o = (uint32_t)((n * a.Cb * a.Hin + oj * a.sub) * a.Win + oi * a.sub) * 32u;
        out_o = ok ? (uint32_t)((n * a.Kb * a.Hout + oj * a.osub + a.ooh) * a.Wout + oi * a.osub + a.oow) * 32u + 8u * kg
                   : 0xffffffffu;
    };

    // ---- what this wave LOADS per step: weight slabs 2*wave, 2*wave+1 and pixel slabs LB*wave .. +LB-1
    const uint32_t lane_in = (uint32_t)(kg >> 1) * cbs + 16u * (kg & 1);
    uint32_t in_off[LB], dummy;
#pragma unroll
    for (int j = 0; j < LB; ++j) {
        pixel(grp0 + LB * wave + j, in_off[j], dummy);
        in_off[j] += lane_in;
    }
    const uint32_t w_lane = WTR ? (uint32_t)(lane >> 5) * a.w_ib * 512u + (uint32_t)(lane & 31) * 16u
                                : (uint32_t)((kg >> 1) * a.w_ib * 256 + li * 16 + 8 * (kg & 1)) * 2u;
    const char *wk[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int ob = min(kb0 + 2 * wave + j, a.Kb - 1);
        wk[j] = Wt + ((int64_t)a.wtap + (int64_t)ob * a.w_ob) * 512;
    }
    const uint32_t w_pair = (uint32_t)a.w_ib * 1024u;  // bytes between channel-block pairs

    // ---- what this wave READS from a slot
    const uint32_t rd_b = (uint32_t)lane * 16u;
    const uint32_t rd_a = WTR ? (uint32_t)(kg >> 1) * 512u + (uint32_t)((8 * (kg & 1) + (li >> 2)) * 16 + 4 * (li & 3)) * 2u
                              : (uint32_t)lane * 16u;

    float4v acc[4][NGW];                               // [feature block][pixel group]
#pragma unroll
    for (int f = 0; f < 4; ++f) {
        float4v bv = {0.f, 0.f, 0.f, 0.f};
        if (a.bias) bv = *(const float4v *)((const char *)a.bias + min(kb0 + 4 * wm + f, a.Kb - 1) * 64 + (uint32_t)(16 * kg));
#pragma unroll
        for (int g = 0; g < NGW; ++g) acc[f][g] = bv;
    }

#define L_LOAD(S, U)                                                                                  \
    {                                                                                                 \
        const uint32_t io_ = (uint32_t)(U) * 2u * cbs, wo_ = w_lane + (uint32_t)(U) * w_pair;         \
        S[0] = *(const float4v *)(wk[0] + wo_);                                                       \
        S[1] = *(const float4v *)(wk[1] + wo_);                                                       \
        _Pragma("unroll") for (int j_ = 0; j_ < LB; ++j_) S[2 + j_] = *(const float4v *)(I + (in_off[j_] + io_)); \
        __builtin_amdgcn_sched_barrier(0);                                                            \
    }
#define L_WRITE(S, SLOT)                                                                              \
    {                                                                                                 \
        char *d_ = &lds[SLOT][0][0] + rd_b;                                                           \
        *(float4v *)(d_ + (2 * wave) * 1024) = S[0];                                                  \
        *(float4v *)(d_ + (2 * wave + 1) * 1024) = S[1];                                              \
        _Pragma("unroll") for (int j_ = 0; j_ < LB; ++j_) *(float4v *)(d_ + (8 + LB * wave + j_) * 1024) = S[2 + j_]; \
        __builtin_amdgcn_sched_barrier(0);                                                            \
    }
// operand fragments of one step: four feature blocks, NGW pixel groups
#define L_READ(FA, FB, SLOT)                                                                          \
    {                                                                                                 \
        const char *sa_ = &lds[SLOT][4 * wm][0] + rd_a;                                               \
        const char *sb_ = &lds[SLOT][8 + NGW * wn][0] + rd_b;                                         \
        _Pragma("unroll") for (int f = 0; f < 4; ++f) {                                               \
            if (WTR) {                                                                                \
                typedef short s4v_ __attribute__((ext_vector_type(4)));                               \
                typedef short s8v_ __attribute__((ext_vector_type(8)));                               \
                typedef __attribute__((address_space(3))) s4v_ *lp_;                                  \
                const s4v_ lo_ = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp_)(sa_ + f * 1024));      \
                const s4v_ hi_ = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp_)(sa_ + f * 1024 + 128)); \
                FA[f] = __builtin_bit_cast(bf16x8v, s8v_{lo_[0], lo_[1], lo_[2], lo_[3], hi_[0], hi_[1], hi_[2], hi_[3]}); \
            } else {                                                                                  \
                FA[f] = *(const bf16x8v *)(sa_ + f * 1024);                                           \
            }                                                                                         \
        }                                                                                             \
        _Pragma("unroll") for (int g = 0; g < NGW; ++g) FB[g] = *(const bf16x8v *)(sb_ + g * 1024);   \
        __builtin_amdgcn_sched_barrier(0);                                                            \
    }
#define L_MFMA(FA, FB) L_MFMA_PART(FA, FB, 0, NGW)
// (pixel groups G0 .. G1-1 of a step: the step's matrix instructions are issued in two halves, one on either side
// of the barrier, so that a wave waits there with matrix work queued)
#define L_MFMA_PART(FA, FB, G0, G1)                                                                   \
    {                                                                                                 \
        _Pragma("unroll") for (int g = (G0); g < (G1); ++g) _Pragma("unroll") for (int f = 0; f < 4; ++f) \
            acc[f][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(FA[f], FB[g], acc[f][g], 0, 0, 0);    \
        __builtin_amdgcn_sched_barrier(0);                                                            \
    }

    // D steps per trip, the register sets are named by the step's position in the trip, and no branch
    // surrounds a load: the compiler's wait counts before each LDS write are then exact (a conditional
    // load in the loop would make every step wait for ALL outstanding loads).  The launcher guarantees
    // that the number of steps is a multiple of D; D is even, so the LDS slot and the fragment set of a
    // step are its position's parity.  In step u a wave writes step u+1 to LDS, passes the barrier, issues
    // the fragment reads of step u+1 and only then the matrix instructions of step u, whose fragments were
    // read a step earlier: the LDS latency runs under the matrix pipe instead of in front of it.
    static_assert(D % 2 == 0, "slot parity follows the position in the trip");
    const int units = a.Cb >> 1;                       // steps: channel-block pairs
    float4v S[D][2 + LB];                              // [set][two weight slabs, LB pixel slabs]: 16 bytes per lane each
    bf16x8v fa[2][4], fb[2][NGW];                      // [fragment set][block / group]
#pragma unroll
    for (int j = 0; j < D; ++j) L_LOAD(S[j], j)
    L_WRITE(S[0], 0)
    __syncthreads();
    L_READ(fa[0], fb[0], 0)
    for (int u = 0; u + 2 * D <= units; u += D) {
#pragma unroll
        for (int j = 0; j < D; ++j) {
            L_LOAD(S[j], u + j + D)                    // set j held step u + j, which is in LDS already
            L_WRITE(S[(j + 1) % D], (j + 1) & 1)
            L_MFMA_PART(fa[j & 1], fb[j & 1], 0, NGW / 2)
            __syncthreads();
            L_READ(fa[(j + 1) & 1], fb[(j + 1) & 1], (j + 1) & 1)
            L_MFMA_PART(fa[j & 1], fb[j & 1], NGW / 2, NGW)
        }
    }
#pragma unroll
    for (int j = 0; j < D; ++j) {                      // the last D steps: nothing left to load
        if (j + 1 < D) {
            L_WRITE(S[j + 1], (j + 1) & 1)
            __syncthreads();
            L_READ(fa[(j + 1) & 1], fb[(j + 1) & 1], (j + 1) & 1)
        }
        L_MFMA(fa[j & 1], fb[j & 1])
    }
#undef L_LOAD
#undef L_WRITE
#undef L_READ
#undef L_MFMA
#undef L_MFMA_PART

    // epilogue: register r of lane (li, kg) of tile (f, g) is feature 4kg + r of block kb0 + 4wm + f, pixel li
    // of group grp0 + NGW*wn + g
    uint32_t out_off[NGW];
#pragma unroll
    for (int g = 0; g < NGW; ++g) pixel(grp0 + NGW * wn + g, dummy, out_off[g]);
    act_dispatch(a.act, [&](auto act_c) {
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            const int kb = kb0 + 4 * wm + f;
            if (kb >= a.Kb) break;
            char *ok_ = O + (int64_t)kb * kbs;
#pragma unroll
            for (int g = 0; g < NGW; ++g) {
                if (out_off[g] == 0xffffffffu) continue;
                *(us4v *)(ok_ + out_off[g]) = pack_bf16x4(act4<decltype(act_c)::value>(acc[f][g], a.act));
            }
        }
    });
    if (a.zsib) c1_zero_siblings<4, NGW>(a, O, kbs, kb0 + 4 * wm, grp0 + NGW * wn, li, out_off);
}

}  // namespace brg
