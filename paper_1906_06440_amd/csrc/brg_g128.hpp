// Batch-reduce GEMM over 64 x 64 x 64 fp32 blocks with a 128 x 64 tile per workgroup and a ring of
// three operand stages (fully connected backward pass, Algorithm 5 of the paper run on the
// transposed problems: by-data and weight-gradient GEMM side by side in one launch).
//
// Same job description, block layout in LDS, swizzle and fragment order as the 64 x 64 kernel in
// brg_g64.hpp; what differs is the schedule:
//  * 8 waves own two vertically adjacent C blocks, so every staged B block feeds two A blocks
//    (48 KiB instead of 64 KiB of operands per 128 x 64 x 64 of work) and ONE workgroup fills a CU.
//  * Three stages of 48 KiB.  The only barrier of a stage sits before its LAST group of matrix
//    instructions, after the wave has read all fragments of the stage: every wave crosses it with
//    16 MFMAs still to issue, pre-reads the first fragments of the next stage (which the barrier
//    has just declared complete) behind them, and the matrix pipe never drains.  The buffer that
//    the barrier frees is refilled at once with the stage three steps ahead, so a direct
//    global->LDS load has two full stages (>= 8000 clocks) to land instead of one.
//  * An operand that needs a ReLU mask applied while staging (B of the by-data job, A of the weight
//    job) goes through registers one stage behind the direct loads; the mask of the PRODUCING layer
//    is applied to C in the epilogue.
#pragma once

#include "brg_g64.hpp"

namespace brg {

constexpr int G128_STAGE = 3 * G64_OPER;                          // floats: A block 0, A block 1, B block
constexpr size_t G128_SMEM = 3 * G128_STAGE * sizeof(float);      // 144 KiB: three stages

template <bool AKF, bool BKF, bool MA, bool MB> __device__ __forceinline__ void g128_tile(const G64Job &J, const int bid)
{
    extern __shared__ __attribute__((aligned(16))) float g64_smem[];
    const int t = threadIdx.x, lane = t & 63;
    const int wv = __builtin_amdgcn_readfirstlane(t >> 6);      // 0..7
    const int li = lane & 15, kg = lane >> 4;
    const int wm = (wv & 3) * 32, wn = (wv >> 2) * 32;           // wave tile inside 128 x 64
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) float *)g64_smem;

    const int pairs = J.tiles_m >> 1;
    int tp, tn;
    if (pairs == 8 && J.tiles_n == 16) {
        // 16 x 16 blocks: XCD x (= workgroup % 8) owns block rows 4*(x%4).., columns 8*(x/4)..
        const int x = bid & 7, i = bid >> 3;
        tp = (x & 3) * 2 + (i & 1);
        tn = (x >> 2) * 8 + (i >> 1);
    } else {
        tp = bid % pairs;
        tn = bid / pairs;
    }
    const int chain = J.chain;
    const int64_t a_chain = J.a_chain, b_chain = J.b_chain;

    // ---- direct loads of one stage: 128 A rows (wave wv takes rows 16 wv .. 16 wv + 15, i.e. a quarter
    // of block wv / 4) and 64 B rows (rows 8 wv .. 8 wv + 7).  Lane L of an instruction for rows
    // r0..r0+3 sits at row r = r0 + L/16, position L%16 and fetches logical piece (L%16) ^ (r & 15).
    const float *gA = J.A + (int64_t)(2 * tp + (wv >> 2)) * J.a_tile;
    const float *gB = J.B + (int64_t)tn * J.b_tile;
    int ga_off[4], gb_off[2];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int r = 16 * (wv & 3) + 4 * j + (lane >> 4);
        ga_off[j] = r * J.a_ld + (((lane & 15) ^ (r & 15)) << 2);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int r = 8 * wv + 4 * j + (lane >> 4);
        gb_off[j] = r * J.b_ld + (((lane & 15) ^ (r & 15)) << 2);
    }
    float *const ldsA = g64_smem + (wv >> 2) * G64_OPER + 16 * (wv & 3) * 64;
    float *const ldsB = g64_smem + 2 * G64_OPER + 8 * wv * 64;
    // An operand with a ReLU mask (dZ = dY o [Y > 0]) cannot take the direct path: its share of a stage is
    // loaded into registers together with the mask source one stage after the direct loads of that stage,
    // and written to LDS (same placement) just before the barrier that publishes the stage.
    const float *gAm = MA ? J.Amask + (gA - J.A) : nullptr;
    const float *gBm = MB ? J.Bmask + (gB - J.B) : nullptr;
    float4v ra[4], rma[4], rb[2], rmb[2];
    typedef int int4v __attribute__((ext_vector_type(4)));
#define G128_ISSUE(I, BUF)                                                                             \
    {                                                                                                  \
        const float *pa_ = gA + (int64_t)(I) * a_chain, *pb_ = gB + (int64_t)(I) * b_chain;           \
        if (!MA) {                                                                                     \
            _Pragma("unroll") for (int j = 0; j < 4; ++j) __builtin_amdgcn_global_load_lds(            \
                pa_ + ga_off[j], ldsA + (BUF) * G128_STAGE + 4 * j * 64, 16, 0, 0);                    \
        }                                                                                              \
        if (!MB) {                                                                                     \
            _Pragma("unroll") for (int j = 0; j < 2; ++j) __builtin_amdgcn_global_load_lds(            \
                pb_ + gb_off[j], ldsB + (BUF) * G128_STAGE + 4 * j * 64, 16, 0, 0);                    \
        }                                                                                              \
    }
#define G128_LOAD_MASKED(I)                                                                            \
    {                                                                                                  \
        if (MA) {                                                                                      \
            const float *pa_ = gA + (int64_t)(I) * a_chain, *pm_ = gAm + (int64_t)(I) * a_chain;      \
            _Pragma("unroll") for (int j = 0; j < 4; ++j)                                              \
            {                                                                                          \
                ra[j] = *(const float4v *)(pa_ + ga_off[j]);                                           \
                rma[j] = *(const float4v *)(pm_ + ga_off[j]);                                          \
            }                                                                                          \
        }                                                                                              \
        if (MB) {                                                                                      \
            const float *pb_ = gB + (int64_t)(I) * b_chain, *pm_ = gBm + (int64_t)(I) * b_chain;      \
            _Pragma("unroll") for (int j = 0; j < 2; ++j)                                              \
            {                                                                                          \
                rb[j] = *(const float4v *)(pb_ + gb_off[j]);                                           \
                rmb[j] = *(const float4v *)(pm_ + gb_off[j]);                                          \
            }                                                                                          \
        }                                                                                              \
    }
#define G128_STASH_MASKED(BUF)                                                                         \
    {                                                                                                  \
        if (MA) {                                                                                      \
            _Pragma("unroll") for (int j = 0; j < 4; ++j)                                              \
            {                                                                                          \
                const int4v keep_ = rma[j] > 0.f;                                                      \
                *(float4v *)(ldsA + (BUF) * G128_STAGE + 4 * j * 64 + lane * 4) =                      \
                    __builtin_bit_cast(float4v, __builtin_bit_cast(int4v, ra[j]) & keep_);             \
            }                                                                                          \
        }                                                                                              \
        if (MB) {                                                                                      \
            _Pragma("unroll") for (int j = 0; j < 2; ++j)                                              \
            {                                                                                          \
                const int4v keep_ = rmb[j] > 0.f;                                                      \
                *(float4v *)(ldsB + (BUF) * G128_STAGE + 4 * j * 64 + lane * 4) =                      \
                    __builtin_bit_cast(float4v, __builtin_bit_cast(int4v, rb[j]) & keep_);             \
            }                                                                                          \
        }                                                                                              \
        if (MA || MB) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                               \
    }
    // direct loads per wave and stage that stay in flight across the publishing barrier
    constexpr int NDMA = (MA ? 0 : 4) + (MB ? 0 : 2);

    // ---- fragment addresses (bytes, without the stage offset).  k-fast blocks as in the 64 x 64 kernel:
    // the 16-row MFMA tile x of the wave holds rows 16 x + li, one ds_read_b128 per four k steps.  Row-fast
    // blocks (rows = reduction index) INTERLEAVE the two tiles instead, tile x holding rows 2 li + x, so
    // that one ds_read_b64 at row k fetches the operand of both tiles (8 reads per 16 MFMAs, not 16).
    unsigned fa[2][4], fb[2][4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int k = 4 * kg + s;                  // row of a row-fast block read at step q = s
        if (AKF) {
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                const int m = (wm & 63) + 16 * x + li;
                fa[x][s] = (m * 64 + (((4 * s) ^ kg ^ (m & 15)) << 2)) * 4;
            }
        } else {
            const int m = (wm & 63) + 2 * li;
            fa[0][s] = fa[1][s] = (k * 64 + (((m >> 2) ^ (k & 15)) << 2) + (m & 3)) * 4;
        }
        if (BKF) {
#pragma unroll
            for (int y = 0; y < 2; ++y) {
                const int n = wn + 16 * y + li;
                fb[y][s] = (n * 64 + (((4 * s) ^ kg ^ (n & 15)) << 2)) * 4;
            }
        } else {
            const int n = wn + 2 * li;
            fb[0][s] = fb[1][s] = (k * 64 + (((n >> 2) ^ (k & 15)) << 2) + (n & 3)) * 4;
        }
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            fa[x][s] += lds0 + (wm >> 6) * G64_OPER * 4;
            fb[x][s] += lds0 + 2 * G64_OPER * 4;
        }
    }

    float4v acc[2][2];
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y) acc[x][y] = float4v{0.f, 0.f, 0.f, 0.f};

    // row sums of A (bias gradient) by the tiles of the first tile column.  Thread t owns the 16-byte
    // piece p = t % 32 (four columns m = 4p .. 4p+3 of the two A blocks) in the rows k = r + 16 j,
    // r = t / 32, j = 0..3: these rows share k & 15, hence the swizzled position, so the four reads
    // of a stage differ by a constant offset.
    const bool do_rowsum = J.rowsum != nullptr && tn == 0 && !AKF;
    float4v rs4 = {0.f, 0.f, 0.f, 0.f};
    const int rs_p = t & 31, rs_r = t >> 5;
    const unsigned rs_addr = lds0 + ((rs_p >> 4) * G64_OPER + rs_r * 64) * 4 + (((rs_p & 15) ^ rs_r) << 4);

    // prologue: three stages in flight (the host guarantees chain >= 3), wait for the first
    G128_ISSUE(0, 0)
    G128_ISSUE(1, 1)
    if (MA || MB) {
        G128_LOAD_MASKED(0)
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        G128_STASH_MASKED(0)
        G128_LOAD_MASKED(1)
        asm volatile("" ::: "memory");
        G128_ISSUE(2, 2)
        asm volatile("" ::: "memory");
    } else {
        G128_ISSUE(2, 2)
        asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
    }
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    // k-fast operand: af[slot][tile] holds the four k steps; row-fast: af2[slot][step] holds the two tiles
    float4v af[2][2], bf[2][2];
    float2v af2[2][4], bf2[2][4];
#define G128_READ_FRAGS(SB, S, SLOT)                                                               \
    if (AKF) {                                                                                     \
        _Pragma("unroll") for (int x = 0; x < 2; ++x) af[SLOT][x] = g64_read128((SB) + fa[x][S]);  \
    } else {                                                                                       \
        _Pragma("unroll") for (int q = 0; q < 4; ++q)                                              \
            af2[SLOT][q] = g64_read64<(S) * 16 * 256>((SB) + fa[0][q]);                           \
    }                                                                                              \
    if (BKF) {                                                                                     \
        _Pragma("unroll") for (int y = 0; y < 2; ++y) bf[SLOT][y] = g64_read128((SB) + fb[y][S]);  \
    } else {                                                                                       \
        _Pragma("unroll") for (int q = 0; q < 4; ++q)                                              \
            bf2[SLOT][q] = g64_read64<(S) * 16 * 256>((SB) + fb[0][q]);                           \
    }
#define G128_WAIT(SLOT)                                                                            \
    {                                                                                              \
        if (AKF) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(af[SLOT][0]), "+v"(af[SLOT][1]));      \
        else asm volatile("s_waitcnt lgkmcnt(0)"                                                   \
                          : "+v"(af2[SLOT][0]), "+v"(af2[SLOT][1]), "+v"(af2[SLOT][2]), "+v"(af2[SLOT][3])); \
        if (BKF) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(bf[SLOT][0]), "+v"(bf[SLOT][1]));      \
        else asm volatile("s_waitcnt lgkmcnt(0)"                                                   \
                          : "+v"(bf2[SLOT][0]), "+v"(bf2[SLOT][1]), "+v"(bf2[SLOT][2]), "+v"(bf2[SLOT][3])); \
    }
#define G128_MFMA(SLOT)                                                                            \
    _Pragma("unroll") for (int x = 0; x < 2; ++x) _Pragma("unroll") for (int y = 0; y < 2; ++y)    \
    {                                                                                              \
        _Pragma("unroll") for (int q = 0; q < 4; ++q) acc[x][y] = __builtin_amdgcn_mfma_f32_16x16x4f32( \
            AKF ? af[SLOT][x][q] : af2[SLOT][q][x], BKF ? bf[SLOT][y][q] : bf2[SLOT][q][y], acc[x][y], 0, 0, 0); \
        __builtin_amdgcn_sched_barrier(0);                                                         \
    }
    G128_READ_FRAGS(0u, 0, 0)
    int buf = 0;                                   // it % 3
    for (int it = 0; it < chain; ++it) {
        const unsigned sbase = (unsigned)(buf * G128_STAGE) * 4u;
        int nbuf = buf + 1;
        if (nbuf == 3) nbuf = 0;
        G128_WAIT(0)
        G128_READ_FRAGS(sbase, 1, 1)
        float4v rv[4];
        if (do_rowsum) {   // issued here, consumed one MFMA group later: the wait below is the one the fragments need anyway
            rv[0] = g64_read128o<0>(sbase + rs_addr);
            rv[1] = g64_read128o<16 * 256>(sbase + rs_addr);
            rv[2] = g64_read128o<32 * 256>(sbase + rs_addr);
            rv[3] = g64_read128o<48 * 256>(sbase + rs_addr);
        }
        __builtin_amdgcn_sched_barrier(0);
        G128_MFMA(0)
        G128_WAIT(1)
        if (do_rowsum) {
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(rv[0]), "+v"(rv[1]), "+v"(rv[2]), "+v"(rv[3]));
        }
        G128_READ_FRAGS(sbase, 2, 0)
        if (do_rowsum) {
            rs4 += (rv[0] + rv[1]) + (rv[2] + rv[3]);
        }
        __builtin_amdgcn_sched_barrier(0);
        G128_MFMA(1)
        G128_WAIT(0)
        G128_READ_FRAGS(sbase, 3, 1)
        __builtin_amdgcn_sched_barrier(0);
        G128_MFMA(0)
        G128_WAIT(1)             // every LDS read of this stage by this wave is complete
        __builtin_amdgcn_sched_barrier(0);
        if (it + 1 < chain) {
            // my share of stage it+1 has landed (the loads of stage it+2 may stay in flight) ...
            if (MA || MB) G128_STASH_MASKED(nbuf)  // (masked share of stage it+1: loaded one stage ago)
            if (it + 2 < chain) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NDMA) : "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();          // ... so has everybody's, and nobody reads this stage again
            asm volatile("" ::: "memory");
            if ((MA || MB) && it + 2 < chain) {
                G128_LOAD_MASKED(it + 2)
                asm volatile("" ::: "memory");
            }
            if (it + 3 < chain) G128_ISSUE(it + 3, buf)
            const unsigned nbase = (unsigned)(nbuf * G128_STAGE) * 4u;
            G128_READ_FRAGS(nbase, 0, 0)
            __builtin_amdgcn_sched_barrier(0);
        }
        G128_MFMA(1)
        buf = nbuf;
    }
#undef G128_ISSUE
#undef G128_LOAD_MASKED
#undef G128_STASH_MASKED
#undef G128_READ_FRAGS
#undef G128_MFMA
#undef G128_WAIT

    if (do_rowsum) {   // combine the 16 row groups of every column through LDS (all stages are dead)
        __syncthreads();
        ((float4v *)g64_smem)[rs_r * 32 + rs_p] = rs4;
        __syncthreads();
        if (t < 128) {
            float sum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) sum += g64_smem[r * 128 + t];
            J.rowsum[(2 * tp) * 64 + t] = sum;
        }
    }
    // ---- epilogue on the accumulators.  Register r of lane l of MFMA tile (x, y) is row 4*(l/16) + r,
    // column l%16 of that tile; a k-fast operand puts tile row/column i at 16 x + i, a row-fast one at
    // 2 i + x.  Either way a lane owns runs of four consecutive m (the contiguous index of C).
    float *Cb = J.C + (int64_t)(2 * tp + (wm >> 6)) * J.c_tile_m + (int64_t)tn * J.c_tile_n;
    const float *Cm = J.Cmask ? J.Cmask + (Cb - J.C) : nullptr;
    const int tm = 2 * tp + (wm >> 6);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int m = (wm & 63) + (AKF ? 16 * h + 4 * kg : 8 * kg + 4 * h);
        float4v bv = {0.f, 0.f, 0.f, 0.f};
        if (J.bias) bv = *(const float4v *)(J.bias + tm * 64 + m);
#pragma unroll
        for (int y = 0; y < 2; ++y) {
            const int n = wn + (BKF ? 16 * y + li : 2 * li + y);
            const int64_t off = (int64_t)n * J.c_ld + m;
            float4v v = AKF ? acc[h][y]
                            : float4v{acc[0][y][2 * h], acc[1][y][2 * h], acc[0][y][2 * h + 1], acc[1][y][2 * h + 1]};
            v *= J.alpha;
            if (J.beta != 0.f) v += J.beta * *(const float4v *)(Cb + off);
            v += bv;
            v = act_is_slow(J.act) ? apply_act4<true>(v, J.act) : apply_act4<false>(v, J.act);
            if (Cm) {
                const float4v mk = *(const float4v *)(Cm + off);
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r] = mk[r] > 0.f ? v[r] : 0.f;
            }
            *(float4v *)(Cb + off) = v;
        }
    }
}

// Backward pair: a job with k-fast A is the by-data GEMM (A, B k-fast), any other the weight-gradient
// GEMM (A, B row-fast).
static __global__ __launch_bounds__(512) void g128_kernel(G64Args args)   // (one copy per translation unit)
{
    int ji = 0;
#pragma unroll
    for (int q = 1; q < G64_MAXJOBS; ++q)
        if (q < args.njobs && (int)blockIdx.x >= args.job[q].wg_begin) ji = q;
    const G64Job &J = args.job[ji];
    const int bid = blockIdx.x - J.wg_begin;
    if (J.a_kfast) {
        if (J.Bmask) g128_tile<true, true, false, true>(J, bid);
        else g128_tile<true, true, false, false>(J, bid);
    } else {
        if (J.Amask) g128_tile<false, false, true, false>(J, bid);
        else g128_tile<false, false, false, false>(J, bid);
    }
}

// True when every job of a backward launch can run on the 128 x 64 kernel and the launch fills the chip
// (BRG_FC_G128=0 never, =1 whenever the jobs have the right form).
static bool g128_applies(const G64Args &a)
{
    const bool knob = knobs().fc_g128.set;
    if (knob && knobs().fc_g128.val == 0) return false;
    int wg = 0;
    for (int j = 0; j < a.njobs; ++j) {
        const G64Job &J = a.job[j];
        if (J.kind != G64_GEMM) return false;
        if ((J.tiles_m & 1) || J.chain < 3) return false;
        if (J.a_kfast != J.b_kfast) return false;
        if (J.a_kfast ? J.Amask != nullptr : J.Bmask != nullptr) return false;   // masked: B of the by-data, A of the weight job
        wg += (J.tiles_m >> 1) * J.tiles_n;
    }
    return wg >= 192 || (knob && wg > 0);
}

static int launch_g128(G64Args &a, hipStream_t s, const char *who)
{
    static thread_local int allowed_on = -1;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess && dev != allowed_on) {
        e = hipFuncSetAttribute((const void *)g128_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)G128_SMEM);
        if (e == hipSuccess) allowed_on = dev;
    }
    if (e != hipSuccess) return fail(BRG_EHIP, "%s: set-up: %s", who, hipGetErrorString(e));
    int wg = 0;
    for (int j = 0; j < a.njobs; ++j) {
        a.job[j].wg_begin = wg;
        wg += (a.job[j].tiles_m >> 1) * a.job[j].tiles_n;
    }
    hipLaunchKernelGGL(g128_kernel, dim3(wg), dim3(512), G128_SMEM, s, a);
    return check_launch(who);
}

}  // namespace brg
