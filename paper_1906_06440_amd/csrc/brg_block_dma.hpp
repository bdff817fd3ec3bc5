// Batch-reduce GEMM over 64 x 64 x 64 fp32 blocks, variant with direct global->LDS loads.
//
// One workgroup of 8 waves per 64 x 64 block of C, the chain split between two wave groups, a
// 32 x 32 piece of C per wave in four MFMA accumulators.  The block pairs never pass through registers: every wave issues `global_load_lds_dwordx4`
// for its share of the next A_i / B_i pair while the current pair is multiplied.  Lane L of such
// an instruction deposits its 16 bytes at LDS base + 16*L, so a wave instruction fills four rows
// of 64 floats; bank conflicts are avoided by an XOR swizzle instead of row padding: the 16-byte
// piece q of row r is stored at piece position q ^ (r & 15) (the lane simply FETCHES the piece that
// belongs at its position).
//
// The compiler cannot tell which LDS region an in-flight direct load will write and would wait for
// ALL outstanding loads before any LDS read.  The fragment reads are therefore issued as inline
// assembly with explicit s_waitcnt, and every value they produce is passed through the waiting
// statement so that no use can be scheduled ahead of it.
#pragma once

#include "brg_block_args.hpp"

namespace brg {

constexpr int BD_OPER = 64 * 64;           // floats per staged operand block (unpadded)
constexpr int BD_STAGE = 2 * BD_OPER;      // A + B
constexpr size_t BD_SMEM = 2 /*groups*/ * 2 /*buffers*/ * BD_STAGE * sizeof(float);   // 128 KiB

__device__ __forceinline__ float4v bd_read128(unsigned addr)
{
    float4v v;
    asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr));
    return v;
}

template <int OFF> __device__ __forceinline__ float bd_read32(unsigned addr)
{
    float v;
    asm volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}

// wait for every LDS read issued so far; the fragments are operands so that their uses stay behind
__device__ __forceinline__ void bd_wait_lds(float4v (&a)[2], float4v (&b)[2])
{
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a[0]), "+v"(a[1]), "+v"(b[0]), "+v"(b[1]));
}

template <bool A_KFAST, bool B_KFAST>
__global__ __launch_bounds__(512, 1) void block_dma_f32(BlockTileArgs a)
{
    extern __shared__ __attribute__((aligned(16))) float bd_smem[];   // the only LDS object: starts at byte 0
    const int t = threadIdx.x, grp = t >> 8;
    const int lane = t & 63, wv = (t >> 6) & 3;
    const int li = lane & 15, kg = lane >> 4;
    const int wm = (wv & 1) * 32, wn = (wv >> 1) * 32;

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
    const int half = (a.chain + 1) >> 1;
    const int c_begin = grp ? half : 0;
    const int c_count = grp ? a.chain - half : half;
    const int c_skew = 0;   // all tiles walk the chain in the same order: shared blocks stay hot in L2 only briefly

    // ---- direct loads: wave wv moves rows 16*wv .. 16*wv+15 of each block, 4 rows per instruction.
    // Lane L of instruction j sits at row r = 16*wv + 4*j + L/16, piece position L%16, and fetches
    // the logical piece (L%16) ^ (r & 15) of that row.
    const float *gA = a.A + tm * a.a_tile;
    const float *gB = a.B + tn * a.b_tile;
    int ga_off[4], gb_off[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int r = 16 * wv + 4 * j + (lane >> 4);
        const int piece = (lane & 15) ^ (r & 15);
        ga_off[j] = r * a.a_ld + piece * 4;
        gb_off[j] = r * a.b_ld + piece * 4;
    }
    const int stage0 = grp * 2 * BD_STAGE;   // float offset of this group's first stage buffer
    auto issue = [&](int i, int b) {   // i-th pair of this group's half chain
        int c = c_begin + i + c_skew;
        if (c >= a.chain) c -= a.chain;
        const float *pa = gA + (int64_t)c * a.a_chain, *pb = gB + (int64_t)c * a.b_chain;
        float *dA = bd_smem + stage0 + b * BD_STAGE + (16 * wv) * 64;
        float *dB = dA + BD_OPER;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            __builtin_amdgcn_global_load_lds(pa + ga_off[j], dA + j * 256, 16, 0, 0);
            __builtin_amdgcn_global_load_lds(pb + gb_off[j], dB + j * 256, 16, 0, 0);
        }
    };

    // ---- fragment addresses (bytes from LDS base, without the stage offset).
    // k-fast operand (rows = M or N index, 64 contiguous k): lane reads pieces kc/4 + kg of row
    //   m = w? + 16x + li; position = ((kc/4) ^ kg ^ (m & 15)); one address per (x, kc).
    // row-fast operand (rows = k index): lane reads element (k = kc + 4kg + q, m): position of piece
    //   (m>>2) is (m>>2) ^ ((4kg + q) & 15); one address per (x, q), kc is an immediate offset.
    unsigned fa[2][4], fb[2][4];
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            {
                const int m = wm + 16 * x + li;
                if (A_KFAST) fa[x][s] = (m * 64 + (((4 * s) ^ kg ^ (m & 15)) << 2)) * 4;
                else fa[x][s] = ((4 * kg + s) * 64 + (((m >> 2) ^ ((4 * kg + s) & 15)) << 2) + (m & 3)) * 4;
            }
            {
                const int n = wn + 16 * x + li;
                if (B_KFAST) fb[x][s] = (BD_OPER + n * 64 + (((4 * s) ^ kg ^ (n & 15)) << 2)) * 4;
                else fb[x][s] = (BD_OPER + (4 * kg + s) * 64 + (((n >> 2) ^ ((4 * kg + s) & 15)) << 2) + (n & 3)) * 4;
            }
        }

    float4v acc[2][2];
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y) acc[x][y] = float4v{0.f, 0.f, 0.f, 0.f};

    if (c_count > 0) issue(0, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    for (int it = 0; it < half; ++it) {
        const bool work = it < c_count, more = it + 1 < c_count;
        if (more) issue(it + 1, (it + 1) & 1);
        if (work) {
            const unsigned sbase = (unsigned)(stage0 + (it & 1) * BD_STAGE) * 4u;
            float4v af[2][2], bf[2][2];
#define BD_READ_FRAGS(S, SLOT)                                                                        \
    _Pragma("unroll") for (int x = 0; x < 2; ++x)                                                     \
    {                                                                                                 \
        if (A_KFAST) {                                                                                \
            af[SLOT][x] = bd_read128(sbase + fa[x][S]);                                               \
        } else {                                                                                      \
            af[SLOT][x][0] = bd_read32<(S) * 16 * 256>(sbase + fa[x][0]);                             \
            af[SLOT][x][1] = bd_read32<(S) * 16 * 256>(sbase + fa[x][1]);                             \
            af[SLOT][x][2] = bd_read32<(S) * 16 * 256>(sbase + fa[x][2]);                             \
            af[SLOT][x][3] = bd_read32<(S) * 16 * 256>(sbase + fa[x][3]);                             \
        }                                                                                             \
        if (B_KFAST) {                                                                                \
            bf[SLOT][x] = bd_read128(sbase + fb[x][S]);                                               \
        } else {                                                                                      \
            bf[SLOT][x][0] = bd_read32<(S) * 16 * 256>(sbase + fb[x][0]);                             \
            bf[SLOT][x][1] = bd_read32<(S) * 16 * 256>(sbase + fb[x][1]);                             \
            bf[SLOT][x][2] = bd_read32<(S) * 16 * 256>(sbase + fb[x][2]);                             \
            bf[SLOT][x][3] = bd_read32<(S) * 16 * 256>(sbase + fb[x][3]);                             \
        }                                                                                             \
    }
#define BD_MFMA(SLOT)                                                                                 \
    _Pragma("unroll") for (int x = 0; x < 2; ++x) _Pragma("unroll") for (int y = 0; y < 2; ++y)       \
    {                                                                                                 \
        _Pragma("unroll") for (int q = 0; q < 4; ++q) acc[x][y] =                                     \
            __builtin_amdgcn_mfma_f32_16x16x4f32(af[SLOT][x][q], bf[SLOT][y][q], acc[x][y], 0, 0, 0); \
        __builtin_amdgcn_sched_barrier(0);                                                            \
    }
            BD_READ_FRAGS(0, 0)
            bd_wait_lds(af[0], bf[0]);
            BD_READ_FRAGS(1, 1)
            __builtin_amdgcn_sched_barrier(0);
            BD_MFMA(0)
            bd_wait_lds(af[1], bf[1]);
            BD_READ_FRAGS(2, 0)
            __builtin_amdgcn_sched_barrier(0);
            BD_MFMA(1)
            bd_wait_lds(af[0], bf[0]);
            BD_READ_FRAGS(3, 1)
            __builtin_amdgcn_sched_barrier(0);
            BD_MFMA(0)
            bd_wait_lds(af[1], bf[1]);
            __builtin_amdgcn_sched_barrier(0);
            BD_MFMA(1)
#undef BD_READ_FRAGS
#undef BD_MFMA
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // my share of the next pair has landed
        __syncthreads();                                    // ... and so has everybody else's
    }

    // ---- combine the two half-chain partial tiles, epilogue, single store
    float *xch = bd_smem;
    if (grp == 1) {
#pragma unroll
        for (int x = 0; x < 2; ++x)
#pragma unroll
            for (int y = 0; y < 2; ++y)
                *(float4v *)(xch + (wn + 16 * y + li) * 64 + wm + 16 * x + 4 * kg) = acc[x][y];
    }
    __syncthreads();
    if (grp == 0) {
        float *Cb = a.C + tm * a.c_tile_m + tn * a.c_tile_n;
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            const int m = wm + 16 * x + 4 * kg;
            float4v bv = {0.f, 0.f, 0.f, 0.f};
            if (a.bias) bv = *(const float4v *)(a.bias + tm * 64 + m);
#pragma unroll
            for (int y = 0; y < 2; ++y) {
                const int n = wn + 16 * y + li;
                float4v v = acc[x][y] + *(const float4v *)(xch + n * 64 + m);
                float *dst = Cb + (int64_t)n * a.c_ld + m;
                v = v * a.alpha;
                if (a.beta != 0.f) v += a.beta * *(const float4v *)dst;
                v += bv;
                v = act_is_slow(a.act) ? apply_act4<true>(v, a.act) : apply_act4<false>(v, a.act);
                *(float4v *)dst = v;
            }
        }
    }
}

template <bool A_KFAST, bool B_KFAST> static int launch_block_dma(BlockTileArgs &a, hipStream_t s, const char *who)
{
    a.xcd_patch = (a.tiles_m == 16 && a.tiles_n == 16) ? 1 : 0;
    auto kern = block_dma_f32<A_KFAST, B_KFAST>;
    static thread_local int allowed_on = -1;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess && dev != allowed_on) {
        e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)BD_SMEM);
        if (e == hipSuccess) allowed_on = dev;
    }
    if (e != hipSuccess) return fail(BRG_EHIP, "%s: set-up: %s", who, hipGetErrorString(e));
    hipLaunchKernelGGL(kern, dim3(a.tiles_m * a.tiles_n), dim3(512), BD_SMEM, s, a);
    return check_launch(who);
}

}  // namespace brg
