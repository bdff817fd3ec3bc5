// 1x1 convolutions in bf16 as a persistent, ring-staged workgroup GEMM (paper section 3.2 / Algorithm 4 with
// R = S = 1: every output block is one batch-reduce chain over the C/16 channel blocks; backward by data is the
// same pass with the roles of C and K swapped).  For layers with at least 256 channels.
//
// A workgroup of four waves (2 x 2) owns tiles of 128 features x 128 pixels; a wave keeps 64 x 64 of it in sixteen
// accumulator tiles across the whole chain.  What differs from the tiled kernel of brg_conv1x1_lds_bf16.hpp:
//
//  * A stage is FOUR channel blocks (64 reduction elements) of both operands, 32 KiB, and it never passes through
//    registers: every lane fetches, with a direct global -> LDS load, exactly the 16 bytes it will later need as a
//    matrix operand (activations, reduction-contiguous weights) or a linear 16-byte piece of a weight block pair
//    (forward weights, read back through the transposing LDS read).  A slab is 1 KiB = one wave instruction.
//  * Four stage buffers form a ring: while stage s is multiplied, stages s+1 .. s+3 are landing (96 KiB in flight
//    per compute unit).  One workgroup per compute unit, and the workgroups are persistent: the ring runs on
//    across tile boundaries, so the first stages of the next tile land while the last ones of this tile are
//    multiplied and its result is stored.
//  * One barrier per stage, placed between the stage's two groups of sixteen matrix instructions, after the wave
//    has read all its fragments of the stage: the buffer is refilled at once and the first fragments of the next
//    stage are read under the second group.  Fragment reads are inline assembly with explicit waits (the compiler
//    would otherwise wait for all direct loads in flight before any LDS read).
//  * Pixel addressing and the epilogue are those of conv1x1_bf16 (pixels enumerated over the whole batch; strided
//    input sub-sampling and strided output placement per lane).
#pragma once

#include "brg_conv1x1_bf16.hpp"
#include "brg_conv_tile.hpp"

namespace brg {

constexpr int C1R_STAGE_BYTES = 32 * 1024;      // 16 weight slabs + 16 pixel slabs of 1 KiB
constexpr int C1R_NBUF = 4;
constexpr size_t C1R_SMEM = (size_t)C1R_NBUF * C1R_STAGE_BYTES;

__device__ __forceinline__ float4v c1r_read128(unsigned addr)
{
    float4v v;
    asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr));
    return v;
}

typedef float c1r_f2v __attribute__((ext_vector_type(2)));
template <int OFF> __device__ __forceinline__ c1r_f2v c1r_read_tr(unsigned addr)
{
    c1r_f2v v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}

// WTR: forward layout of the weight blocks ([c][k], feature index contiguous) -> transposing reads.
// (launch bounds of two workgroups keep the kernel within 256 registers, so the accumulators stay in VGPRs; the LDS
// it uses admits one workgroup per compute unit)
template <bool WTR> __global__ __launch_bounds__(256, 2) void conv1x1_ring_bf16(Conv1x1Args a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char c1r_smem[];   // the only LDS object
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)c1r_smem;
    const char *__restrict__ I = (const char *)a.I;
    const char *__restrict__ Wt = (const char *)a.Wt;
    char *__restrict__ O = (char *)a.O;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int li = lane & 15, kg = lane >> 4;
    const int wm = wave & 1, wn = wave >> 1;           // this wave multiplies feature blocks 4wm.. x pixel groups 4wn..

    const uint32_t cbs = (uint32_t)(a.Hin * a.Win) * 32u;           // bytes of one channel-block plane
    const uint32_t kbs = (uint32_t)(a.Hout * a.Wout) * 32u;
    const int PQ = a.P * a.Q;
    const int nstage = a.Cb >> 2;                      // stages per tile (the launcher guarantees Cb % 4 == 0, nstage >= 4)
    const int G = gridDim.x;
    const int my_tiles = (a.tiles - (int)blockIdx.x + G - 1) / G;
    const int total = my_tiles * nstage;               // stages of this workgroup's whole stream
    if (total <= 0) return;                            // (uniform)

    auto tile_of = [&](int i, int &kb0, int &grp0) {   // i-th tile of this workgroup
        const int tile = xcd_tile((int)blockIdx.x + i * G, a.tiles);
        int tx, ty;
        if (a.pixel_major) {
            tx = c1_fdiv(tile, a.tiles_y, a.inv_tiles_y);
            ty = tile - tx * a.tiles_y;
        } else {
            ty = c1_fdiv(tile, a.tiles_x, a.inv_tiles_x);
            tx = tile - ty * a.tiles_x;
        }
        kb0 = ty * 8;
        grp0 = tx * 8;
    };
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

    // ---- what this wave LOADS per stage: weight slabs of feature blocks 2 wave, 2 wave + 1 and pixel slabs of
    // groups 2 wave, 2 wave + 1, each for the stage's two channel-block pairs (8 instructions of 1 KiB).
    // LDS: slab (kind, index, pair) at ((kind * 8 + index) * 2 + pair) * 1024, lane L at + 16 L.
    const uint32_t lane_in = (uint32_t)(kg >> 1) * cbs + 16u * (kg & 1);               // operand order
    const uint32_t w_lane = WTR ? (uint32_t)(lane >> 5) * a.w_ib * 512u + (uint32_t)(lane & 31) * 16u      // linear
                                : (uint32_t)((kg >> 1) * a.w_ib * 256 + li * 16 + 8 * (kg & 1)) * 2u;    // operand order
    const uint32_t w_pair = (uint32_t)a.w_ib * 1024u;  // bytes between channel-block pairs
    // issue side of the stream: tile and chain position of the next stage to load
    int ld_tile = 0, ld_step = 0, ld_kb0, ld_grp0;
    uint32_t ld_in[2], dummy;
    const char *ld_w[2];
    auto ld_setup = [&]() {
        tile_of(ld_tile, ld_kb0, ld_grp0);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            pixel(ld_grp0 + 2 * wave + j, ld_in[j], dummy);
            ld_in[j] += lane_in;
            const int ob = min(ld_kb0 + 2 * wave + j, a.Kb - 1);
            ld_w[j] = Wt + ((int64_t)a.wtap + (int64_t)ob * a.w_ob) * 512 + w_lane;
        }
    };
#define C1R_ISSUE(BUF)                                                                                             \
    {                                                                                                              \
        unsigned char *db_ = c1r_smem + (BUF) * C1R_STAGE_BYTES;                                                   \
        _Pragma("unroll") for (int j_ = 0; j_ < 2; ++j_) _Pragma("unroll") for (int p_ = 0; p_ < 2; ++p_)          \
        {                                                                                                          \
            const uint32_t u_ = (uint32_t)(2 * ld_step + p_);                                                      \
            __builtin_amdgcn_global_load_lds((const bf16_t *)(ld_w[j_] + u_ * w_pair),                             \
                                             (bf16_t *)(db_ + ((2 * wave + j_) * 2 + p_) * 1024), 16, 0, 0);        \
            __builtin_amdgcn_global_load_lds((const bf16_t *)(I + (ld_in[j_] + u_ * 2u * cbs)),                    \
                                             (bf16_t *)(db_ + ((8 + 2 * wave + j_) * 2 + p_) * 1024), 16, 0, 0);    \
        }                                                                                                          \
        if (++ld_step == nstage) {                                                                                 \
            ld_step = 0;                                                                                           \
            if (++ld_tile < my_tiles) ld_setup();                                                                  \
        }                                                                                                          \
    }

    // ---- what this wave READS from a stage buffer (byte addresses without the buffer offset)
    const unsigned rd_b = lds0 + (unsigned)((8 + 4 * wn) * 2048) + (unsigned)lane * 16u;
    const unsigned rd_a = lds0 + (unsigned)((4 * wm) * 2048) +
                          (WTR ? (unsigned)(kg >> 1) * 512u + (unsigned)((8 * (kg & 1) + (li >> 2)) * 16 + 4 * (li & 3)) * 2u
                               : (unsigned)lane * 16u);
    float4v fa[2][4], fb[2][4];                        // [fragment set = pair of the stage][feature block / pixel group]
    c1r_f2v ta[2][4][2];
#define C1R_READ(SET, BUF, PAIR)                                                                                   \
    {                                                                                                              \
        const unsigned o_ = (unsigned)((BUF) * C1R_STAGE_BYTES + (PAIR) * 1024);                                   \
        _Pragma("unroll") for (int f = 0; f < 4; ++f)                                                              \
        {                                                                                                          \
            if (WTR) {                                                                                             \
                ta[SET][f][0] = c1r_read_tr<0>(rd_a + o_ + f * 2048);                                              \
                ta[SET][f][1] = c1r_read_tr<128>(rd_a + o_ + f * 2048);                                            \
            } else {                                                                                               \
                fa[SET][f] = c1r_read128(rd_a + o_ + f * 2048);                                                    \
            }                                                                                                      \
            fb[SET][f] = c1r_read128(rd_b + o_ + f * 2048);                                                        \
        }                                                                                                          \
    }
#define C1R_WAIT(SET)                                                                                              \
    {                                                                                                              \
        if (WTR) asm volatile("s_waitcnt lgkmcnt(0)"                                                               \
                              : "+v"(ta[SET][0][0]), "+v"(ta[SET][0][1]), "+v"(ta[SET][1][0]), "+v"(ta[SET][1][1]),  \
                                "+v"(ta[SET][2][0]), "+v"(ta[SET][2][1]), "+v"(ta[SET][3][0]), "+v"(ta[SET][3][1])); \
        else asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(fa[SET][0]), "+v"(fa[SET][1]), "+v"(fa[SET][2]), "+v"(fa[SET][3])); \
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(fb[SET][0]), "+v"(fb[SET][1]), "+v"(fb[SET][2]), "+v"(fb[SET][3])); \
    }
#define C1R_MFMA(SET)                                                                                              \
    {                                                                                                              \
        bf16x8v av_[4], bv_[4];                                                                                    \
        _Pragma("unroll") for (int f = 0; f < 4; ++f)                                                              \
        {                                                                                                          \
            av_[f] = WTR ? __builtin_bit_cast(bf16x8v, float4v{ta[SET][f][0][0], ta[SET][f][0][1], ta[SET][f][1][0], ta[SET][f][1][1]}) \
                         : __builtin_bit_cast(bf16x8v, fa[SET][f]);                                                \
            bv_[f] = __builtin_bit_cast(bf16x8v, fb[SET][f]);                                                      \
        }                                                                                                          \
        _Pragma("unroll") for (int g = 0; g < 4; ++g) _Pragma("unroll") for (int f = 0; f < 4; ++f)                \
            acc[f][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av_[f], bv_[g], acc[f][g], 0, 0, 0);               \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
    }

    float4v acc[4][4];                                 // [feature block][pixel group]
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
        for (int g = 0; g < 4; ++g) acc[f][g] = float4v{0.f, 0.f, 0.f, 0.f};

    // ---- prologue: stage s lives in buffer s % 4; four stages in flight, the first one landed and its first
    // fragments read
    ld_setup();
    int issued = 0;
#pragma unroll
    for (int s = 0; s < 4; ++s)
        if (issued < total) {
            C1R_ISSUE(s)
            ++issued;
        }
    if (total > 3) asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
    else if (total > 2) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    else if (total > 1) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    C1R_READ(0, 0, 0)

    int cs_tile = 0, cs_step = 0, buf = 0;             // compute side of the stream
    for (int it = 0; it < total; ++it) {
        const int nbuf = (buf + 1) & 3;
        C1R_READ(1, buf, 1)
        C1R_WAIT(0)
        __builtin_amdgcn_sched_barrier(0);
        C1R_MFMA(0)
        C1R_WAIT(1)                                    // every LDS read of this stage by this wave is complete
        if (it + 1 < total) {
            // my share of stage it+1 has landed (two later stages may stay in flight; stores of an epilogue that are
            // still on their way only make this wait longer than it has to be) ...
            if (it + 3 < total) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
            else if (it + 2 < total) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();              // ... so has everybody's, and nobody reads this stage's buffer again
            asm volatile("" ::: "memory");
            if (issued < total) {                      // refill it with the stage four steps ahead (it + 4 -> buffer it % 4)
                C1R_ISSUE(buf)
                ++issued;
            }
            C1R_READ(0, nbuf, 0)
            __builtin_amdgcn_sched_barrier(0);
        }
        C1R_MFMA(1)
        buf = nbuf;
        if (++cs_step == nstage) {
            // ---- end of a tile: bias + activation on the accumulators, 8 bytes (4 features of a pixel) per lane
            int kb0, grp0;
            tile_of(cs_tile, kb0, grp0);
            uint32_t out_off[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) pixel(grp0 + 4 * wn + g, dummy, out_off[g]);
            act_dispatch(a.act, [&](auto act_c) {
#pragma unroll
                for (int f = 0; f < 4; ++f) {
                    const int kb = kb0 + 4 * wm + f;
                    if (kb >= a.Kb) break;
                    float4v bv = {0.f, 0.f, 0.f, 0.f};
                    if (a.bias) bv = *(const float4v *)((const char *)a.bias + kb * 64 + 16 * kg);
                    char *ok_ = O + (int64_t)kb * kbs;
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        if (out_off[g] == 0xffffffffu) continue;
                        *(us4v *)(ok_ + out_off[g]) = pack_bf16x4(act4<decltype(act_c)::value>(acc[f][g] + bv, a.act));
                    }
                }
            });
            if (a.zsib) c1_zero_siblings<4, 4>(a, O, kbs, kb0 + 4 * wm, grp0 + 4 * wn, li, out_off);
#pragma unroll
            for (int f = 0; f < 4; ++f)
#pragma unroll
                for (int g = 0; g < 4; ++g) acc[f][g] = float4v{0.f, 0.f, 0.f, 0.f};
            cs_step = 0;
            ++cs_tile;
        }
    }
#undef C1R_ISSUE
#undef C1R_READ
#undef C1R_WAIT
#undef C1R_MFMA
}

}  // namespace brg
