// Multi-job batch-reduce GEMM kernel over 64 x 64 x 64 fp32 blocks (fully connected layers,
// Algorithm 5 of the paper, and every chain that has this block shape).
//
// One launch carries up to sixteen independent "jobs" (for example the backward-by-data GEMM, the
// weight-gradient GEMM and the bias gradient of one layer).  A workgroup of 4 waves owns one
// 64 x TN tile of one job's C (TN = 64, or 32 to double the number of tiles of a lone GEMM) and
// walks that tile's whole reduce chain with the accumulators in MFMA registers; two workgroups
// share a CU, so one's prologue, barriers and epilogue hide behind the other's matrix work.
//
//  * Operand blocks go global -> LDS directly (global_load_lds_dwordx4), double buffered, with
//    an XOR swizzle of the 16-byte pieces of each 256-byte row (piece q of row r sits at position
//    q ^ (r & 15)) instead of padding.  The swizzle serves both operand orientations: blocks whose
//    contiguous index is the reduction index are read with one ds_read_b128 per four MFMAs, the
//    others with four ds_read_b32.  The k order fed to the matrix cores is permuted identically
//    for A and B (lane group g takes k = 4g + q at step q), which a sum does not mind.
//  * An operand that needs the ReLU-backward mask (dZ = dY o [Y > 0]) is the one exception: it is
//    loaded into registers together with Y, masked, and written to LDS in the same swizzle.
//  * Fragment reads are inline assembly with explicit waits, because the compiler would otherwise
//    wait for ALL in-flight direct loads before any LDS read.
//  * Epilogue on the accumulators: alpha/beta, bias per row, activation, and optionally the
//    ReLU-backward mask of the PRODUCING layer (C o [Cmask > 0]), then one store.
#pragma once

#include "brg_common.hpp"

namespace brg {

constexpr int G64_OPER = 64 * 64;
constexpr int G64_STAGE = 2 * G64_OPER;                         // floats per stage (A block + B block)
constexpr size_t G64_SMEM = 2 * G64_STAGE * sizeof(float);      // 64 KiB: two stages

enum { G64_GEMM = 0, G64_COLSUM = 1 };

struct G64Job {
    int kind;
    const float *A, *B;          // operand bases
    const float *Amask, *Bmask;  // optional ReLU mask source, indexed like A / B
    float *C;
    const float *bias;           // per row of C, or null
    const float *Cmask;          // optional: C is multiplied by [Cmask > 0] (indexed like C)
    int act;
    int tiles_m, tiles_n, chain;
    float alpha, beta;
    int64_t a_tile, a_chain, b_tile, b_chain, c_tile_m, c_tile_n;   // element strides
    int a_ld, b_ld, c_ld;
    int a_kfast, b_kfast;
    int wg_begin;                // first workgroup of this job
    // Optional by-product of a GEMM whose A blocks are row-fast (rows = reduction index): the tiles
    // of the first tile column also write rowsum[m] = sum over the whole chain of A[m][k] (after the
    // mask), i.e. the bias gradient when A is dZ.
    float *rowsum;
    // G64_COLSUM (stand-alone form of the same sum, used when no GEMM carries it)
    int cs_rows;                 // rows per block (bn)
    // Ragged last tile column (64-wide tiles, B blocks with the reduction index contiguous only): when non-zero, C
    // has n_cols columns in all; the rows of B beyond them are not read (the last valid row is read again instead)
    // and the columns of C beyond them are not written.
    int n_cols;
};

constexpr int G64_MAXJOBS = 16;

struct G64Args {
    G64Job job[G64_MAXJOBS];
    int njobs;
};

__device__ __forceinline__ float4v g64_read128(unsigned addr)
{
    float4v v;
    asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr));
    return v;
}

typedef float float2v __attribute__((ext_vector_type(2)));

template <int OFF> __device__ __forceinline__ float2v g64_read64(unsigned addr)
{
    float2v v;
    asm volatile("ds_read_b64 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}

template <int OFF> __device__ __forceinline__ float4v g64_read128o(unsigned addr)
{
    float4v v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}

// bias gradient: one workgroup per 64 features
__device__ __forceinline__ void g64_colsum(const G64Job &j, int tile)
{
    __shared__ float part[4][64];
    const int kl = threadIdx.x & 63, q = threadIdx.x >> 6;
    const float *base = j.A + tile * j.a_tile + kl;
    const float *mbase = j.Amask ? j.Amask + tile * j.a_tile + kl : nullptr;
    float s = 0.f;
    for (int c = 0; c < j.chain; ++c)
        for (int r = q; r < j.cs_rows; r += 4) {
            const int64_t e = (int64_t)c * j.a_chain + (int64_t)r * j.a_ld;
            float g = base[e];
            if (mbase && !(mbase[e] > 0.f)) g = 0.f;
            s += g;
        }
    part[q][kl] = s;
    __syncthreads();
    if (q == 0) j.C[tile * 64 + kl] = (part[0][kl] + part[1][kl]) + (part[2][kl] + part[3][kl]);
}

// One 64 x TN tile of one GEMM job; AKF / BKF say which operand blocks have the reduction index
// contiguous (compile-time, so that the fragment reads are straight-line code).
template <int TN, bool AKF, bool BKF> __device__ __forceinline__ void g64_tile(const G64Job &J, const int bid)
{
    static_assert(TN == 64 || TN == 32, "tile width");
    constexpr int NB = TN / 32;                // 16-column MFMA tiles per wave along N
    extern __shared__ __attribute__((aligned(16))) float g64_smem[];   // dynamic LDS starts after `part`
    const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
    const int li = lane & 15, kg = lane >> 4;
    const int wm = (wv & 1) * 32, wn = (wv >> 1) * (TN / 2);
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) float *)g64_smem;

    int tm, tn;
    if (J.tiles_m == 16 && J.tiles_n * TN == 1024) {
        // 16 x 16 blocks: XCD x (= workgroup % 8) owns the block patch rows 4*(x%4).., columns 8*(x/4)..
        constexpr int TPB = 64 / TN;           // tiles per block column
        const int x = bid & 7, i = bid >> 3;
        tm = (x & 3) * 4 + (i & 3);
        tn = (x >> 2) * 8 * TPB + (i >> 2);
    } else {
        tm = bid % J.tiles_m;
        tn = bid / J.tiles_m;
    }
    const int chain = J.chain;
    const int64_t a_chain = J.a_chain, b_chain = J.b_chain;   // (locals: keep kernel-argument loads out of the loop)
    // All tiles walk their chains in the same order: tiles that share a panel then ask for the same
    // block at about the same time, so a block only has to live in L2 for a moment (a skewed start
    // would keep whole panels resident and overflow the 4 MiB L2 of an XCD).
    const int c_skew = 0;
    constexpr bool akf = AKF, bkf = BKF;

    // B tile: TN columns.  For TN = 32 the B operand must be k-fast (rows = columns of C).
    const float *gA = J.A + tm * J.a_tile;
    const float *gB = J.B + (TN == 64 ? tn * J.b_tile : (tn >> 1) * J.b_tile + (tn & 1) * 32 * (int64_t)J.b_ld);
    const float *gAm = J.Amask ? J.Amask + (gA - J.A) : nullptr;
    const float *gBm = J.Bmask ? J.Bmask + (gB - J.B) : nullptr;

    // ---- direct loads: A = 64 rows (16 wave instructions of 4 rows), B = TN-or-64 rows.
    // Lane L of an instruction for rows r0..r0+3 sits at row r = r0 + L/16, position L%16 and
    // fetches logical piece (L%16) ^ (r & 15).
    constexpr int B_ROWS = TN;                 // rows of the staged B block (k-fast when TN == 32)
    int ga_off[4], gb_off[4];   // (only the first B_ROWS/16 entries of gb_off are used)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int r = 16 * wv + 4 * j + (lane >> 4);
        ga_off[j] = r * J.a_ld + (((lane & 15) ^ (r & 15)) << 2);
    }
#pragma unroll
    for (int j = 0; j < B_ROWS / 16; ++j) {
        const int r = (B_ROWS / 4) * wv + 4 * j + (lane >> 4);
        int rr = r;
        if (TN == 64 && J.n_cols && tn * 64 + r >= J.n_cols) rr = J.n_cols - 1 - tn * 64;
        gb_off[j] = rr * J.b_ld + (((lane & 15) ^ (r & 15)) << 2);
    }
    float4v ra[4], rm[4];   // register path of a masked operand
#pragma unroll
    for (int j = 0; j < 4; ++j) ra[j] = rm[j] = float4v{0.f, 0.f, 0.f, 0.f};
    typedef int int4v __attribute__((ext_vector_type(4)));
    // (macros rather than lambdas: the loads and the stash of one stage, written out in place)
#define G64_ISSUE(I, BUF)                                                                              \
    {                                                                                                  \
        int c_ = (I) + c_skew;                                                                         \
        if (c_ >= chain) c_ -= chain;                                                                  \
        float *dA_ = g64_smem + (BUF) * G64_STAGE, *dB_ = dA_ + G64_OPER;                              \
        const float *pa_ = gA + (int64_t)c_ * a_chain, *pb_ = gB + (int64_t)c_ * b_chain;          \
        if (gAm) {                                                                                     \
            const float *pm_ = gAm + (int64_t)c_ * a_chain;                                          \
            _Pragma("unroll") for (int j = 0; j < 4; ++j)                                              \
            {                                                                                          \
                ra[j] = *(const float4v *)(pa_ + ga_off[j]);                                           \
                rm[j] = *(const float4v *)(pm_ + ga_off[j]);                                           \
            }                                                                                          \
        } else {                                                                                       \
            _Pragma("unroll") for (int j = 0; j < 4; ++j) __builtin_amdgcn_global_load_lds(            \
                pa_ + ga_off[j], dA_ + (16 * wv + 4 * j) * 64, 16, 0, 0);                              \
        }                                                                                              \
        if (gBm) {                                                                                     \
            const float *pm_ = gBm + (int64_t)c_ * b_chain;                                          \
            _Pragma("unroll") for (int j = 0; j < B_ROWS / 16; ++j)                                    \
            {                                                                                          \
                ra[j] = *(const float4v *)(pb_ + gb_off[j]);                                           \
                rm[j] = *(const float4v *)(pm_ + gb_off[j]);                                           \
            }                                                                                          \
        } else {                                                                                       \
            _Pragma("unroll") for (int j = 0; j < B_ROWS / 16; ++j) __builtin_amdgcn_global_load_lds(  \
                pb_ + gb_off[j], dB_ + ((B_ROWS / 4) * wv + 4 * j) * 64, 16, 0, 0);                    \
        }                                                                                              \
    }
    // masked operand: mask in registers, then the same placement the direct load would have made
#define G64_STASH_MASKED(BUF)                                                                          \
    {                                                                                                  \
        float *dA_ = g64_smem + (BUF) * G64_STAGE, *dB_ = dA_ + G64_OPER;                              \
        if (gAm) {                                                                                     \
            _Pragma("unroll") for (int j = 0; j < 4; ++j)                                              \
            {                                                                                          \
                const int4v keep_ = rm[j] > 0.f;                                                       \
                *(float4v *)(dA_ + (16 * wv + 4 * j) * 64 + lane * 4) =                                \
                    __builtin_bit_cast(float4v, __builtin_bit_cast(int4v, ra[j]) & keep_);             \
            }                                                                                          \
        } else if (gBm) {                                                                              \
            _Pragma("unroll") for (int j = 0; j < B_ROWS / 16; ++j)                                    \
            {                                                                                          \
                const int4v keep_ = rm[j] > 0.f;                                                       \
                *(float4v *)(dB_ + ((B_ROWS / 4) * wv + 4 * j) * 64 + lane * 4) =                      \
                    __builtin_bit_cast(float4v, __builtin_bit_cast(int4v, ra[j]) & keep_);             \
            }                                                                                          \
        }                                                                                              \
    }

    // ---- fragment addresses (bytes, without the stage offset); see the header comment.  A k-fast block
    // puts the 16-row MFMA tile x of the wave at rows 16 x + li (one ds_read_b128 per four k steps); a
    // row-fast block INTERLEAVES the two tiles, tile x holding rows 2 li + x, so that one ds_read_b64 at
    // reduction row k fetches the operand of both tiles.
    static_assert(BKF || NB == 2, "a row-fast B operand needs two column tiles per wave");
    unsigned fa[2][4], fb[NB][4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int k = 4 * kg + s;
        if (akf) {
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                const int m = wm + 16 * x + li;
                fa[x][s] = (m * 64 + (((4 * s) ^ kg ^ (m & 15)) << 2)) * 4 + lds0;
            }
        } else {
            const int m = wm + 2 * li;
            fa[0][s] = fa[1][s] = (k * 64 + (((m >> 2) ^ (k & 15)) << 2) + (m & 3)) * 4 + lds0;
        }
        if (bkf) {
#pragma unroll
            for (int y = 0; y < NB; ++y) {
                const int n = wn + 16 * y + li;
                fb[y][s] = (G64_OPER + n * 64 + (((4 * s) ^ kg ^ (n & 15)) << 2)) * 4 + lds0;
            }
        } else {
            const int n = wn + 2 * li;
#pragma unroll
            for (int y = 0; y < NB; ++y)
                fb[y][s] = (G64_OPER + k * 64 + (((n >> 2) ^ (k & 15)) << 2) + (n & 3)) * 4 + lds0;
        }
    }

    float4v acc[2][NB];
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < NB; ++y) acc[x][y] = float4v{0.f, 0.f, 0.f, 0.f};

    // row sums of A (bias gradient).  Thread t owns the 16-byte piece p = t % 16 (columns m = 4p .. 4p+3)
    // in the rows k = r + 16 j, r = t / 16, j = 0..3: these rows share k & 15, hence the swizzled
    // position, so the four reads of a stage differ by a constant offset.
    const bool do_rowsum = J.rowsum != nullptr && tn == 0 && !akf;
    float4v rs4 = {0.f, 0.f, 0.f, 0.f};
    const int rs_p = t & 15, rs_r = t >> 4;
    const unsigned rs_addr = lds0 + (rs_r * 64) * 4 + ((rs_p ^ rs_r) << 4);

    if (chain > 0) {
        G64_ISSUE(0, 0)
        G64_STASH_MASKED(0)
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    for (int it = 0; it < chain; ++it) {
        const bool more = it + 1 < chain;
        if (more) G64_ISSUE(it + 1, (it + 1) & 1)
        const unsigned sbase = (unsigned)((it & 1) * G64_STAGE) * 4u;
        // k-fast operand: af[slot][tile] holds the four k steps; row-fast: af2[slot][step] holds the two tiles
        float4v af[2][2], bf[2][NB];
        float2v af2[2][4], bf2[2][4];
#define G64_READ_FRAGS(S, SLOT)                                                                    \
    if (akf) {                                                                                     \
        _Pragma("unroll") for (int x = 0; x < 2; ++x) af[SLOT][x] = g64_read128(sbase + fa[x][S]); \
    } else {                                                                                       \
        _Pragma("unroll") for (int q = 0; q < 4; ++q)                                              \
            af2[SLOT][q] = g64_read64<(S) * 16 * 256>(sbase + fa[0][q]);                           \
    }                                                                                              \
    if (bkf) {                                                                                     \
        _Pragma("unroll") for (int y = 0; y < NB; ++y) bf[SLOT][y] = g64_read128(sbase + fb[y][S]); \
    } else {                                                                                       \
        _Pragma("unroll") for (int q = 0; q < 4; ++q)                                              \
            bf2[SLOT][q] = g64_read64<(S) * 16 * 256>(sbase + fb[0][q]);                           \
    }
#define G64_WAIT(SLOT)                                                                             \
    {                                                                                              \
        if (akf) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(af[SLOT][0]), "+v"(af[SLOT][1]));      \
        else asm volatile("s_waitcnt lgkmcnt(0)"                                                   \
                          : "+v"(af2[SLOT][0]), "+v"(af2[SLOT][1]), "+v"(af2[SLOT][2]), "+v"(af2[SLOT][3])); \
        if (bkf && NB == 2) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(bf[SLOT][0]), "+v"(bf[SLOT][NB - 1])); \
        else if (bkf) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(bf[SLOT][0]));                    \
        else asm volatile("s_waitcnt lgkmcnt(0)"                                                   \
                          : "+v"(bf2[SLOT][0]), "+v"(bf2[SLOT][1]), "+v"(bf2[SLOT][2]), "+v"(bf2[SLOT][3])); \
    }
#define G64_MFMA(SLOT)                                                                             \
    _Pragma("unroll") for (int x = 0; x < 2; ++x) _Pragma("unroll") for (int y = 0; y < NB; ++y)   \
    {                                                                                              \
        _Pragma("unroll") for (int q = 0; q < 4; ++q) acc[x][y] = __builtin_amdgcn_mfma_f32_16x16x4f32( \
            akf ? af[SLOT][x][q] : af2[SLOT][q][x], bkf ? bf[SLOT][y][q] : bf2[SLOT][q][y], acc[x][y], 0, 0, 0); \
        __builtin_amdgcn_sched_barrier(0);                                                         \
    }
        G64_READ_FRAGS(0, 0)
        G64_WAIT(0)
        G64_READ_FRAGS(1, 1)
        float4v rv[4];
        if (do_rowsum) {   // issued here, consumed one MFMA group later: the wait below is the one the fragments need anyway
            rv[0] = g64_read128o<0>(sbase + rs_addr);
            rv[1] = g64_read128o<16 * 256>(sbase + rs_addr);
            rv[2] = g64_read128o<32 * 256>(sbase + rs_addr);
            rv[3] = g64_read128o<48 * 256>(sbase + rs_addr);
        }
        __builtin_amdgcn_sched_barrier(0);
        G64_MFMA(0)
        G64_WAIT(1)
        if (do_rowsum) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(rv[0]), "+v"(rv[1]), "+v"(rv[2]), "+v"(rv[3]));
        G64_READ_FRAGS(2, 0)
        if (do_rowsum) rs4 += (rv[0] + rv[1]) + (rv[2] + rv[3]);
        __builtin_amdgcn_sched_barrier(0);
        G64_MFMA(1)
        G64_WAIT(0)
        G64_READ_FRAGS(3, 1)
        __builtin_amdgcn_sched_barrier(0);
        G64_MFMA(0)
        G64_WAIT(1)
        __builtin_amdgcn_sched_barrier(0);
        G64_MFMA(1)
#undef G64_READ_FRAGS
#undef G64_MFMA
#undef G64_WAIT
        if (more) G64_STASH_MASKED((it + 1) & 1)
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");   // my share of the next pair has landed
        __syncthreads();                                               // ... and so has everybody else's
    }

#undef G64_ISSUE
#undef G64_STASH_MASKED
    if (do_rowsum) {   // combine the 16 row groups of every column through LDS (stage buffers are dead)
        ((float4v *)g64_smem)[rs_r * 16 + rs_p] = rs4;
        __syncthreads();
        if (t < 64) {
            float sum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) sum += g64_smem[r * 64 + t];
            J.rowsum[tm * 64 + t] = sum;
        }
    }
    // ---- epilogue on the accumulators.  Register r of lane l of MFMA tile (x, y) is row 4*(l/16) + r,
    // column l%16 of that tile; a k-fast operand puts tile row/column i at 16 x + i, a row-fast one at
    // 2 i + x.  Either way a lane owns runs of four consecutive m (the contiguous index of C).
    float *Cb = J.C + tm * J.c_tile_m + (TN == 64 ? tn * J.c_tile_n : (tn >> 1) * J.c_tile_n + (tn & 1) * 32 * (int64_t)J.c_ld);
    const float *Cm = J.Cmask ? J.Cmask + (Cb - J.C) : nullptr;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int m = wm + (akf ? 16 * h + 4 * kg : 8 * kg + 4 * h);
        float4v bv = {0.f, 0.f, 0.f, 0.f};
        if (J.bias) bv = *(const float4v *)(J.bias + tm * 64 + m);
#pragma unroll
        for (int y = 0; y < NB; ++y) {
            const int n = wn + (bkf ? 16 * y + li : 2 * li + y);
            if (TN == 64 && J.n_cols && tn * 64 + n >= J.n_cols) continue;
            const int64_t off = (int64_t)n * J.c_ld + m;
            float4v v = akf ? acc[h][y]
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

// MODE 0: every job has A row-fast / B k-fast (forward pass, plain BRGEMM).
// MODE 1: backward pair: a job with k-fast A is the by-data GEMM (A, B k-fast), any other the
//         weight-gradient GEMM (A, B row-fast).
template <int TN, int MODE> __global__ __launch_bounds__(256, 2) void g64_kernel(G64Args args)
{
    int ji = 0;
#pragma unroll
    for (int q = 1; q < G64_MAXJOBS; ++q)
        if (q < args.njobs && (int)blockIdx.x >= args.job[q].wg_begin) ji = q;
    const G64Job &J = args.job[ji];
    const int bid = blockIdx.x - J.wg_begin;
    if (J.kind == G64_COLSUM) {
        g64_colsum(J, bid);
        return;
    }
    if (MODE == 0) {
        g64_tile<TN, false, true>(J, bid);
    } else {
        if (J.a_kfast) g64_tile<64, true, true>(J, bid);
        else g64_tile<64, false, false>(J, bid);
    }
}


static int g64_workgroups(G64Args &a, int tn_width)
{
    int wg = 0;
    for (int j = 0; j < a.njobs; ++j) {
        a.job[j].wg_begin = wg;
        wg += a.job[j].kind == G64_COLSUM ? a.job[j].tiles_m : a.job[j].tiles_m * a.job[j].tiles_n * (64 / tn_width);
    }
    return wg;
}

// tn_width 32 is only valid for a single GEMM job whose B operand is k-fast (mode 0).
static int launch_g64(G64Args &a, int tn_width, int mode, hipStream_t s, const char *who)
{
    static thread_local int allowed_on = -1;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess && dev != allowed_on) {
        const void *kerns[3] = {(const void *)g64_kernel<64, 0>, (const void *)g64_kernel<32, 0>,
                                (const void *)g64_kernel<64, 1>};
        for (int i = 0; i < 3 && e == hipSuccess; ++i)
            e = hipFuncSetAttribute(kerns[i], hipFuncAttributeMaxDynamicSharedMemorySize, (int)G64_SMEM);
        if (e == hipSuccess) allowed_on = dev;
    }
    if (e != hipSuccess) return fail(BRG_EHIP, "%s: set-up: %s", who, hipGetErrorString(e));
    if (tn_width == 32 && mode == 0) {
        for (int j = 0; j < a.njobs; ++j)
            if (a.job[j].kind == G64_GEMM) a.job[j].tiles_n *= 2;
        int wg = 0;
        for (int j = 0; j < a.njobs; ++j) {
            a.job[j].wg_begin = wg;
            wg += a.job[j].kind == G64_COLSUM ? a.job[j].tiles_m : a.job[j].tiles_m * a.job[j].tiles_n;
        }
        hipLaunchKernelGGL((g64_kernel<32, 0>), dim3(wg), dim3(256), G64_SMEM, s, a);
    } else {
        const int wg = g64_workgroups(a, 64);
        if (mode == 0) hipLaunchKernelGGL((g64_kernel<64, 0>), dim3(wg), dim3(256), G64_SMEM, s, a);
        else hipLaunchKernelGGL((g64_kernel<64, 1>), dim3(wg), dim3(256), G64_SMEM, s, a);
    }
    return check_launch(who);
}

}  // namespace brg
