// Batch-reduce GEMM over 64 x 64 x 64 fp32 blocks, one 64 x 64 block of C per workgroup of 8 waves, with a
// ring of four operand stages (forward pass of a fully connected layer, Algorithm 5 of the paper, and any
// strided chain of such blocks that is at least four blocks long).
//
// Every stage holds one A_i / B_i pair (32 KiB, direct global->LDS loads, XOR-swizzled rows as in
// brg_block_dma.hpp).  All 8 waves work on the SAME stage: wave group g (waves 4g .. 4g+3) multiplies the
// k range 32 g .. 32 g + 31 of the pair into its own 32 x 32 accumulators, so the two groups hold partial
// sums of the same C block and are added through LDS at the end.  The schedule is the one of the 128 x 64
// kernel (brg_g128.hpp): the only barrier of a stage sits before the stage's last group of matrix
// instructions, the first fragments of the next stage are read right behind it, and the buffer it frees
// is refilled at once with the stage four steps ahead (three stages, about 6000 matrix-pipe clocks, in
// flight).  Row-fast operands are read with one ds_read_b64 per k step over interleaved MFMA tiles.
//
// PTRS: the address-list form of section 2 of the paper ("two arrays of pointers").  Block i of the chain is
// A_ptrs[i] / B_ptrs[i] (device arrays), read with scalar loads one ring turn ahead of the stage that needs
// them.  Direct loads need 16-byte aligned rows and the arrays cannot be inspected from the host without a
// synchronisation, so every wave first scans the whole list; if any block (or a leading dimension) is less
// aligned, all stages are filled through registers instead (four element loads and one 16-byte LDS store
// per piece, placed exactly where the direct load would have put it).
#pragma once

#include "brg_block_dma.hpp"
#include "brg_g64.hpp"

namespace brg {

constexpr int BR_STAGE = 2 * BD_OPER;                              // floats: A block, B block
constexpr size_t BR_SMEM = 4 * BR_STAGE * sizeof(float);           // 128 KiB: four stages

template <bool AKF, bool BKF, bool PTRS = false> __global__ __launch_bounds__(512) void block_ring_f32(BlockTileArgs a)
{
    extern __shared__ __attribute__((aligned(16))) float br_smem[];   // the only LDS object: starts at byte 0
    const int t = threadIdx.x, lane = t & 63;
    const int wv = __builtin_amdgcn_readfirstlane(t >> 6);          // 0..7
    const int grp = wv >> 2, w4 = wv & 3;
    const int li = lane & 15, kg = lane >> 4;
    const int wm = (w4 & 1) * 32, wn = (w4 >> 1) * 32;

    int tm, tn;
    {
        const int bid = blockIdx.x;
        if (a.xcd_patch) {
            const int x = bid & 7, i = bid >> 3;
            tm = (x & 3) * 4 + (i & 3);
            tn = (x >> 2) * 8 + (i >> 2);
        } else {
            tm = bid % a.tiles_m;
            tn = bid / a.tiles_m;
        }
    }
    const int chain = a.chain;
    const int64_t a_chain = a.a_chain, b_chain = a.b_chain;

    // bias of the rows this wave finishes (group g finishes the row halves h = g, see the epilogue)
    const int m_out = wm + (AKF ? 16 * grp + 4 * kg : 8 * kg + 4 * grp);
    float4v bload;                                                  // (only defined and only used when there is a bias)

    // ---- direct loads: wave wv moves rows 8 wv .. 8 wv + 7 of both blocks, 4 rows per instruction.  Lane L
    // sits at row r = r0 + L/16, piece position L%16, and fetches the logical piece (L%16) ^ (r & 15).
    const int64_t a_toff = tm * a.a_tile, b_toff = tn * a.b_tile;
    const float *gA = PTRS ? nullptr : a.A + a_toff;
    const float *gB = PTRS ? nullptr : a.B + b_toff;
    int ga_off[2], gb_off[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int r = 8 * wv + 4 * j + (lane >> 4);
        const int piece = (lane & 15) ^ (r & 15);
        ga_off[j] = r * a.a_ld + piece * 4;
        gb_off[j] = r * a.b_ld + piece * 4;
    }
    bool direct = true;
    if (PTRS) {
        unsigned bad = (unsigned)((a.a_ld | a.b_ld) & 3) | (unsigned)((a_toff | b_toff) & 3);
        for (int i = lane; i < chain; i += 64)
            bad |= (unsigned)(((uintptr_t)a.A_ptrs[i] | (uintptr_t)a.B_ptrs[i]) & 15u);
        direct = __builtin_amdgcn_ballot_w64(bad != 0u) == 0ull;      // the same answer in every wave
    }
    float *const ldsA = br_smem + 8 * wv * 64;
#define BR_ISSUE(I, BUF)                                                                               \
    {                                                                                                  \
        const float *pa_, *pb_;                                                                        \
        if (PTRS) {                                                                                    \
            pa_ = a.A_ptrs[I] + a_toff;                                                                \
            pb_ = a.B_ptrs[I] + b_toff;                                                                \
        } else {                                                                                       \
            pa_ = gA + (int64_t)(I) * a_chain;                                                         \
            pb_ = gB + (int64_t)(I) * b_chain;                                                         \
        }                                                                                              \
        if (!PTRS || direct) {                                                                         \
            _Pragma("unroll") for (int j = 0; j < 2; ++j)                                              \
            {                                                                                          \
                __builtin_amdgcn_global_load_lds(pa_ + ga_off[j], ldsA + (BUF) * BR_STAGE + j * 256, 16, 0, 0);           \
                __builtin_amdgcn_global_load_lds(pb_ + gb_off[j], ldsA + (BUF) * BR_STAGE + BD_OPER + j * 256, 16, 0, 0); \
            }                                                                                          \
        } else {                                                                                       \
            _Pragma("unroll") for (int j = 0; j < 2; ++j)                                              \
            {                                                                                          \
                float4v va_, vb_;                                                                      \
                _Pragma("unroll") for (int e = 0; e < 4; ++e)                                          \
                {                                                                                      \
                    va_[e] = pa_[ga_off[j] + e];                                                       \
                    vb_[e] = pb_[gb_off[j] + e];                                                       \
                }                                                                                      \
                *(float4v *)(ldsA + (BUF) * BR_STAGE + j * 256 + lane * 4) = va_;                      \
                *(float4v *)(ldsA + (BUF) * BR_STAGE + BD_OPER + j * 256 + lane * 4) = vb_;            \
            }                                                                                          \
        }                                                                                              \
    }

    // ---- fragment addresses (bytes, without the stage offset) of the two 16-deep k slots 2 grp + e of
    // this wave group.  k-fast: fa[x][e], one ds_read_b128 per MFMA tile x; row-fast: fa[0][q] for the k
    // step q, the slot e is an immediate offset of 16 rows, tile x holds rows 2 li + x.
    unsigned fa[2][4], fb[2][4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int k = 4 * kg + s;
        const int slot = 2 * grp + (s & 1);
        if (AKF) {
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                const int m = wm + 16 * x + li;
                fa[x][s] = (m * 64 + (((4 * slot) ^ kg ^ (m & 15)) << 2)) * 4;
            }
        } else {
            const int m = wm + 2 * li;
            fa[0][s] = fa[1][s] = ((32 * grp + k) * 64 + (((m >> 2) ^ (k & 15)) << 2) + (m & 3)) * 4;
        }
        if (BKF) {
#pragma unroll
            for (int y = 0; y < 2; ++y) {
                const int n = wn + 16 * y + li;
                fb[y][s] = (BD_OPER + n * 64 + (((4 * slot) ^ kg ^ (n & 15)) << 2)) * 4;
            }
        } else {
            const int n = wn + 2 * li;
            fb[0][s] = fb[1][s] = (BD_OPER + (32 * grp + k) * 64 + (((n >> 2) ^ (k & 15)) << 2) + (n & 3)) * 4;
        }
    }

    float4v acc[2][2];
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y) acc[x][y] = float4v{0.f, 0.f, 0.f, 0.f};

    // prologue: four stages in flight (the host guarantees chain >= 4), wait for the first
    BR_ISSUE(0, 0)
    BR_ISSUE(1, 1)
    BR_ISSUE(2, 2)
    BR_ISSUE(3, 3)
    // The bias load is issued behind the 16 direct loads (ahead of them its round trip would delay all of them).
    // The counter retires in order, so it only makes the waits below one load more conservative while it is in
    // flight: with 17 loads issued, 13 outstanding means stage 0 (the oldest four) has landed.
    asm volatile("" ::: "memory");                                  // (the bias load stays behind the direct loads)
    if (a.bias) {
        bload = *(const float4v *)(a.bias + tm * 64 + m_out);
        asm volatile("s_waitcnt vmcnt(13)" ::: "memory");
    } else {
        asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
    }
    if (PTRS) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // (register-staged pieces: the LDS stores have landed)
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    // k-fast operand: af[slot][tile] holds the four k steps; row-fast: af2[slot][step] holds the two tiles
    float4v af[2][2], bf[2][2];
    float2v af2[2][4], bf2[2][4];
#define BR_READ_FRAGS(SB, E, SLOT)                                                                 \
    if (AKF) {                                                                                     \
        _Pragma("unroll") for (int x = 0; x < 2; ++x) af[SLOT][x] = g64_read128((SB) + fa[x][E]);  \
    } else {                                                                                       \
        _Pragma("unroll") for (int q = 0; q < 4; ++q)                                              \
            af2[SLOT][q] = g64_read64<(E) * 16 * 256>((SB) + fa[0][q]);                           \
    }                                                                                              \
    if (BKF) {                                                                                     \
        _Pragma("unroll") for (int y = 0; y < 2; ++y) bf[SLOT][y] = g64_read128((SB) + fb[y][E]);  \
    } else {                                                                                       \
        _Pragma("unroll") for (int q = 0; q < 4; ++q)                                              \
            bf2[SLOT][q] = g64_read64<(E) * 16 * 256>((SB) + fb[0][q]);                           \
    }
#define BR_WAIT(SLOT)                                                                              \
    {                                                                                              \
        if (AKF) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(af[SLOT][0]), "+v"(af[SLOT][1]));      \
        else asm volatile("s_waitcnt lgkmcnt(0)"                                                   \
                          : "+v"(af2[SLOT][0]), "+v"(af2[SLOT][1]), "+v"(af2[SLOT][2]), "+v"(af2[SLOT][3])); \
        if (BKF) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(bf[SLOT][0]), "+v"(bf[SLOT][1]));      \
        else asm volatile("s_waitcnt lgkmcnt(0)"                                                   \
                          : "+v"(bf2[SLOT][0]), "+v"(bf2[SLOT][1]), "+v"(bf2[SLOT][2]), "+v"(bf2[SLOT][3])); \
    }
#define BR_MFMA(SLOT)                                                                              \
    _Pragma("unroll") for (int x = 0; x < 2; ++x) _Pragma("unroll") for (int y = 0; y < 2; ++y)    \
    {                                                                                              \
        _Pragma("unroll") for (int q = 0; q < 4; ++q) acc[x][y] = __builtin_amdgcn_mfma_f32_16x16x4f32( \
            AKF ? af[SLOT][x][q] : af2[SLOT][q][x], BKF ? bf[SLOT][y][q] : bf2[SLOT][q][y], acc[x][y], 0, 0, 0); \
        __builtin_amdgcn_sched_barrier(0);                                                         \
    }
    BR_READ_FRAGS(0u, 0, 0)
    int buf = 0;                                   // it % 4
    for (int it = 0; it < chain; ++it) {
        const unsigned sbase = (unsigned)(buf * BR_STAGE) * 4u;
        const int nbuf = (buf + 1) & 3;
        BR_WAIT(0)
        BR_READ_FRAGS(sbase, 1, 1)
        __builtin_amdgcn_sched_barrier(0);
        BR_MFMA(0)
        BR_WAIT(1)                                 // every LDS read of this stage by this wave is complete
        __builtin_amdgcn_sched_barrier(0);
        if (it + 1 < chain) {
            // my share of stage it+1 has landed (the loads of stages it+2 and it+3 may stay in flight) ...
            if (it + 3 < chain) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
            else if (it + 2 < chain) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();          // ... so has everybody's, and nobody reads this stage again
            asm volatile("" ::: "memory");
            if (it + 4 < chain) BR_ISSUE(it + 4, buf)
            const unsigned nbase = (unsigned)(nbuf * BR_STAGE) * 4u;
            BR_READ_FRAGS(nbase, 0, 0)
            __builtin_amdgcn_sched_barrier(0);
        }
        BR_MFMA(1)
        buf = nbuf;
    }
#undef BR_ISSUE
#undef BR_READ_FRAGS
#undef BR_MFMA
#undef BR_WAIT

    // ---- add the two k halves and finish.  Register r of lane l of MFMA tile (x, y) is row 4*(l/16) + r,
    // column l%16 of that tile; a k-fast operand puts tile row/column i at 16 x + i, a row-fast one at
    // 2 i + x, so a lane owns two runs (h = 0, 1) of four consecutive m per column tile y.  Group g hands
    // the runs h = 1 - g to the other group and finishes the runs h = g.  The exchange area is the stage
    // buffer after the last one read: every wave has passed the barrier that retired it.
    float4v run[2][2];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int y = 0; y < 2; ++y)
            run[h][y] = AKF ? acc[h][y]
                            : float4v{acc[0][y][2 * h], acc[1][y][2 * h], acc[0][y][2 * h + 1], acc[1][y][2 * h + 1]};
    float4v *xch = (float4v *)(br_smem + (chain & 3) * BR_STAGE);
    // slot of (group that READS it, wave within group, y, lane)
#pragma unroll
    for (int y = 0; y < 2; ++y) xch[(((1 - grp) * 4 + w4) * 2 + y) * 64 + lane] = grp ? run[0][y] : run[1][y];
    __syncthreads();
    float *Cb = a.C + tm * a.c_tile_m + tn * a.c_tile_n;
#pragma unroll
    for (int y = 0; y < 2; ++y) {
        const int n = wn + (BKF ? 16 * y + li : 2 * li + y);
        float4v v = (grp ? run[1][y] : run[0][y]) + xch[((grp * 4 + w4) * 2 + y) * 64 + lane];
        float *dst = Cb + (int64_t)n * a.c_ld + m_out;
        v = v * a.alpha;
        if (a.beta != 0.f) v += a.beta * *(const float4v *)dst;
        if (a.bias) v += bload;
        v = act_is_slow(a.act) ? apply_act4<true>(v, a.act) : apply_act4<false>(v, a.act);
        *(float4v *)dst = v;
    }
}

// chains shorter than the ring go to the double-buffered kernel
template <bool A_KFAST, bool B_KFAST, bool PTRS = false> static int launch_block_ring(BlockTileArgs &a, hipStream_t s, const char *who)
{
    if (!PTRS && (a.chain < 4 || knobs().no_ring.set)) return launch_block_dma<A_KFAST, B_KFAST>(a, s, who);
    a.xcd_patch = (a.tiles_m == 16 && a.tiles_n == 16) ? 1 : 0;
    auto kern = block_ring_f32<A_KFAST, B_KFAST, PTRS>;
    static thread_local int allowed_on = -1;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess && dev != allowed_on) {
        e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)BR_SMEM);
        if (e == hipSuccess) allowed_on = dev;
    }
    if (e != hipSuccess) return fail(BRG_EHIP, "%s: set-up: %s", who, hipGetErrorString(e));
    hipLaunchKernelGGL(kern, dim3(a.tiles_m * a.tiles_n), dim3(512), BR_SMEM, s, a);
    return check_launch(who);
}

}  // namespace brg
