// bf16 variant of the tiled convolution kernel (see brg_conv_tile.hpp for the tiling, the halo
// planes in LDS, the virtual-row addressing and the persistent stage stream; all of that is shared).
//
// What differs:
//  * A pixel's 16 channels are two 16-byte chunks of 8 bf16, so a channel block owns two LDS planes.
//  * The matrix instruction is v_mfma_f32_16x16x32_bf16: one MFMA reduces over TWO channel blocks.
//    Lane group g of the MFMA takes channel block (g >> 1) of the pair and channels 8*(g & 1) .. +7
//    from both operands (the k order inside an MFMA is free as long as A and B agree), so the B
//    fragment is one ds_read_b128 from plane (c_b, g & 1) and the A fragment one 16-byte load of
//    eight consecutive reduction elements of weight-block row `lane % 16`.
//  * That A load needs the reduction index contiguous inside a weight block.  The forward layout
//    [c][k] has it strided, so the forward pass reads weights from a transposed copy ([k][c] inside
//    every 16x16 block) that a small pre-pass kernel writes into the caller's workspace; backward by
//    data reduces over k and reads the original layout directly.
//  * Backward by data ("dual convolution") runs through the same kernel: dO is the input, the weight
//    tap of every kernel tap comes from a table (flipped), and for strided layers the input pixels
//    are split into stride x stride parity classes, each a small stride-1 convolution over dO whose
//    results are stored at every stride-th pixel (osub / ooh / oow).
//  * A wave owns KW feature blocks (16*KW output channels): every B fragment read from LDS is used
//    by KW MFMAs, which halves the LDS traffic per flop for KW = 2.
//  * Weights travel through a small register ring, a few units (c_b pair, tap) ahead of their use.
#pragma once

#include "brg_conv_tile.hpp"

namespace brg {

// transposes every 16x16 bf16 block ([c][k] -> [k][c]); src != dst.  A workgroup moves 8 blocks: 16-byte
// loads, a pass through LDS, 16-byte stores (thread t: block t/32, chunk t%32 = row (t%32)/2, half (t%32)%2).
__global__ __launch_bounds__(256) void conv_wt_transpose_bf16(const bf16_t *__restrict__ src, bf16_t *__restrict__ dst,
                                                              int64_t nblocks)
{
    __shared__ bf16_t tile[8][16][18];                  // rows padded to 18 elements: conflict-free column reads
    const int t = threadIdx.x, bl = t >> 5, ch = t & 31, row = ch >> 1, half = ch & 1;
    const int64_t b = (int64_t)blockIdx.x * 8 + bl;
    if (b < nblocks) {
        typedef unsigned short us8 __attribute__((ext_vector_type(8)));
        const us8 v = *(const us8 *)(src + b * 256 + row * 16 + half * 8);   // c = row, k = 8 half .. +7
#pragma unroll
        for (int e = 0; e < 8; ++e) tile[bl][row][half * 8 + e] = v[e];
    }
    __syncthreads();
    if (b < nblocks) {
        typedef unsigned short us8 __attribute__((ext_vector_type(8)));
        us8 v;                                          // k = row, c = 8 half .. +7
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = tile[bl][half * 8 + e][row];
        *(us8 *)(dst + b * 256 + row * 16 + half * 8) = v;
    }
}

// (bx, by): this workgroup's position in a grid of gx persistent workgroups per feature tile
template <int R, int S, int STR, int CG, int NPASS, int KW, bool TP, typename TOut>
__device__ __forceinline__ void conv_tile_bf16_body(const ConvTileArgs &a, int bx, int by, int gx)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const bf16_t *__restrict__ I = (const bf16_t *)a.I;
    const bf16_t *__restrict__ Wt = (const bf16_t *)a.Wt;
    TOut *__restrict__ O = (TOut *)a.O;
    // TP ("tap pair") mode, for layers with a single channel block (the 3-channel stem): the K = 32 of
    // an MFMA is filled with TWO horizontally adjacent taps of the one channel block instead of two
    // channel blocks: lane groups 0-1 take tap s = 2j, groups 2-3 tap s = 2j + 1 (a tap beyond the
    // filter row gets zero weights).
    static_assert(TP || CG % 2 == 0, "channel blocks are consumed in pairs");
    static_assert(!TP || CG == 1, "tap-pair mode handles one channel block");
    constexpr int TAPS = R * S;
    constexpr int SP = (S + 1) / 2;             // tap pairs per filter row
    constexpr int UNITS = TP ? R * SP : (CG / 2) * TAPS;     // MFMA K-steps per stage
    // weight ring: depth divides UNITS so that ring slots are compile-time; WD-1 units of prefetch (five where one
    // feature block per wave leaves the registers for it: measured 6 % on the 7x7 layers, nothing elsewhere)
    constexpr int WD = (UNITS % 6 == 0 && KW == 1) ? 6 : (UNITS % 3 == 0 ? 3 : (UNITS % 4 == 0 ? 4 : 2));
    static_assert(UNITS % WD == 0, "ring depth must divide the units of a stage");

    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);   // uniform: weight addresses below stay scalar
    const int li = lane & 15, kg = lane >> 4;
    const int kb0 = (by * 4 + wave) * KW;                  // first feature block of this wave
    const int nstage = a.Cb / CG;
    const int64_t cb_stride = (int64_t)a.Hin * a.Win * 16;

    int tile_v = bx;
    if (tile_v >= a.ntiles) return;

    {
        const float4v z = {0.f, 0.f, 0.f, 0.f};
        for (int o = t * 16; o < 2 * a.buf_bytes; o += 256 * 16) *(float4v *)(smem + o) = z;
    }

    // halo copy plan of ONE channel block: chunk e = t + 256*i, 2 chunks (of 8 channels) per pixel
    int goff[NPASS], loff[NPASS];
    auto plan = [&](int tile) {
        const int gr0 = tile * a.trg;
        const int rows = min(a.trg, a.total_rows - gr0);
        const int n0 = fdiv(gr0, a.P, a.inv_P);
        const int v_first = n0 * a.Hv + (gr0 - n0 * a.P) * STR;
        const int grl = gr0 + rows - 1;
        const int nl = fdiv(grl, a.P, a.inv_P);
        const int nv = nl * a.Hv + (grl - nl * a.P) * STR + R - v_first;
        const int W2 = a.W * 2, chunks = nv * W2;
#pragma unroll
        for (int i = 0; i < NPASS; ++i) {
            const int e = t + 256 * i;
            const int row = fdiv(e, W2, a.inv_W4), rem = e - row * W2;   // inv_W4 holds 1/(2W) here
            const int v = v_first + row;
            const int n = fdiv(v, a.Hv, a.inv_Hv), ih = v - n * a.Hv - a.ph;
            const bool in_halo = e < chunks;
            const bool real = ih >= 0 && ih < a.H && n < a.N;
            goff[i] = (in_halo && real)
                          ? (((n * a.Cb * a.Hin + ih * a.sub) * a.Win) + (rem >> 1) * a.sub) * 16 + (rem & 1) * 8
                          : -1;
            loff[i] = in_halo ? (rem & 1) * a.plane_bytes + (row * a.Wp + (rem >> 1) + a.pw) * 16 : -1;
        }
    };

    float4v stage[CG][NPASS];   // 16-byte chunks (8 bf16) in flight
    auto load_halo = [&](int sidx) {
#pragma unroll
        for (int c = 0; c < CG; ++c) {
            const bf16_t *src = I + (int64_t)(sidx * CG + c) * cb_stride;
#pragma unroll
            for (int i = 0; i < NPASS; ++i) {
                stage[c][i] = float4v{0.f, 0.f, 0.f, 0.f};
                if (goff[i] >= 0) stage[c][i] = *(const float4v *)(src + goff[i]);
            }
        }
    };
    auto stash_halo = [&](int buf) {
#pragma unroll
        for (int c = 0; c < CG; ++c) {
            unsigned char *dst = smem + buf * a.buf_bytes + c * 2 * a.plane_bytes;
#pragma unroll
            for (int i = 0; i < NPASS; ++i)
                if (loff[i] >= 0) *(float4v *)(dst + loff[i]) = stage[c][i];
        }
    };

    // weights: unit u of stage sidx = (pair p = u / TAPS, tap = u % TAPS); this lane's channel block is
    // ib = sidx*CG + 2p + (kg >> 1); it loads row li, reduction elements 8*(kg&1) .. +7 of the block
    // (ob, ib, tap') for each of its KW feature blocks ob.
    const int64_t wlane = (int64_t)li * 16 + 8 * (kg & 1);
    const uint32_t wlane_b = (uint32_t)((kg >> 1) * a.w_ib * 256 + li * 16 + 8 * (kg & 1)) * 2u;   // bytes, with the pair's second block
    bf16x8v wring[WD][KW];
    // `ulin` counts units from the start of stage sidx and may run into the following stage
    auto load_w = [&](int sidx, int ulin, bf16x8v (&w)[KW]) {
        const int s2 = sidx + ulin / UNITS, u = ulin % UNITS;
        if (TP) {
            const int ts = 2 * (u % SP) + (kg >> 1);           // this lane's tap column
            const int tap = (u / SP) * S + (ts < S ? ts : S - 1);
#pragma unroll
            for (int k = 0; k < KW; ++k) {
                int ob = kb0 + k;
                if (ob >= a.Kb) ob = a.Kb - 1;
                const bf16_t *src = Wt + ((int64_t)ob * a.w_ob + a.wtap[0] + tap) * 256 + wlane;
                w[k] = *(const bf16x8v *)src;
                if (ts >= S) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) w[k][e] = (__bf16)0.0f;
                }
            }
            return;
        }
        // uniform block address (scalar arithmetic) + this lane's 32-bit offset: one load instruction, no
        // vector ALU work per load.  The pair's first block index is even, so the wrap is uniform.
        int ib = s2 * CG + 2 * (u / TAPS);
        if (ib >= a.Cb) ib -= a.Cb;                    // prefetch beyond the tile wraps to its start
        const int tap = u % TAPS;
#pragma unroll
        for (int k = 0; k < KW; ++k) {
            int ob = kb0 + k;
            if (ob >= a.Kb) ob = a.Kb - 1;
            const char *src = (const char *)Wt + ((int64_t)ob * a.w_ob + (int64_t)ib * a.w_ib + a.wtap[tap]) * 512;
            w[k] = *(const bf16x8v *)(src + wlane_b);
        }
    };

    // Pixel p = 16 g + li of a tile is (row p / Q, column p % Q) of the tile's run of output rows whatever the
    // tile: that split is made once (one register per group: invalid flag, row, column).  What changes from tile to
    // tile is where each ROW lives (image, output row, halo row); threads 0 .. trg-1 work that out once per tile
    // into a small LDS table, one tile ahead, and every lane then looks its rows up (two index divisions per
    // lane and group and tile otherwise: more vector instructions than the matrix instructions of a short chain).
    __shared__ int2 rowtab[2][CT_NG * 16];
    int pix[CT_NG];
#pragma unroll
    for (int g = 0; g < CT_NG; ++g) {
        const int p = g * 16 + li;
        const int rr = fdiv(p, a.Q, a.inv_Q), oi = p - rr * a.Q;
        pix[g] = rr < a.trg ? (rr << 8) | oi : (1 << 20);
    }
    auto fill_rowtab = [&](int tile, int tb) {
        if (t < a.trg) {
            const int gr0 = tile * a.trg;
            const int rows = min(a.trg, a.total_rows - gr0);
            const int n0 = fdiv(gr0, a.P, a.inv_P);
            const int v_first = n0 * a.Hv + (gr0 - n0 * a.P) * STR;
            const bool ok = t < rows;
            const int gr = gr0 + (ok ? t : 0);
            const int n = fdiv(gr, a.P, a.inv_P), oj = gr - n * a.P;
            const int lrow = n * a.Hv + oj * STR - v_first;
            rowtab[tb][t] = int2{lrow * a.Wp * 16, ok ? ((n * a.Kb * a.Hout + oj * a.osub + a.ooh) * a.Wout) * 16 : -1};
        }
    };
    const int pcol0 = TP ? (kg & 1) * a.plane_bytes + (kg >> 1) * 16 : kg * a.plane_bytes;
    const int pout0 = (kb0 * a.Hout * a.Wout + a.oow) * 16 + 4 * kg;
    int tb = 0;

    plan(xcd_tile(tile_v, a.ntiles));
    fill_rowtab(xcd_tile(tile_v, a.ntiles), 0);
    load_halo(0);
#pragma unroll
    for (int d = 0; d < WD - 1; ++d) load_w(0, d, wring[d]);
    __syncthreads();
    stash_halo(0);
    __syncthreads();
    int buf = 0;
    while (true) {
        const int tile = xcd_tile(tile_v, a.ntiles);
        const int next_v = tile_v + gx;
        const bool has_next = next_v < a.ntiles;

        int bbase[CT_NG], ooff[CT_NG];
#pragma unroll
        for (int g = 0; g < CT_NG; ++g) {
            const bool dead = pix[g] >> 20;
            const int2 e = rowtab[tb][(pix[g] >> 8) & 255];          // (row 0 for lanes beyond the tile: in bounds)
            const int oi = pix[g] & 255;
            bbase[g] = pcol0 + e.x + oi * (STR * 16);
            ooff[g] = (dead || e.y < 0) ? -1 : e.y + pout0 + oi * a.osub * 16;
        }

        float4v acc[KW][CT_NG];
#pragma unroll
        for (int k = 0; k < KW; ++k)
#pragma unroll
            for (int g = 0; g < CT_NG; ++g) acc[k][g] = float4v{0.f, 0.f, 0.f, 0.f};

        for (int sidx = 0; sidx < nstage; ++sidx) {
            const bool last = sidx + 1 == nstage;
            const bool more = !last || has_next;
            if (last && has_next) {
                plan(xcd_tile(next_v, a.ntiles));
                fill_rowtab(xcd_tile(next_v, a.ntiles), tb ^ 1);
            }
            if (more) load_halo(last ? 0 : sidx + 1);

            const unsigned char *sbuf = smem + buf * a.buf_bytes;
            // B fragments of unit u+1 are fetched during unit u.  With one feature block per wave (unit
            // stride) a second register set holds them.  With two feature blocks per wave the registers do not
            // allow that, and the fragment of pixel group g is re-fetched IN PLACE right after the matrix
            // instructions of unit u on group g have been issued: its LDS latency then runs under the
            // remaining groups of unit u and the first groups of unit u+1, at no register cost.  The strided
            // variant fetches all fragments of a unit right before its matrix instructions.
            constexpr bool BDB = (KW == 1 && STR == 1) || TP;
            bf16x8v bf[BDB ? 2 : 1][CT_NG];
            auto tap_off = [&](int uu) {
                const int p1 = uu / TAPS, t1 = uu % TAPS;
                return TP ? ((uu / SP) * a.Wp + 2 * (uu % SP)) * 16
                          : p1 * 4 * a.plane_bytes + ((t1 / S) * a.Wp + t1 % S) * 16;
            };
            constexpr bool ROLL = !BDB && STR == 1;    // (the strided variant has no register to spare for it)
            if (BDB || ROLL) {
#pragma unroll
                for (int g = 0; g < CT_NG; ++g) bf[0][g] = *(const bf16x8v *)(sbuf + bbase[g]);
            }
#pragma unroll
            for (int u = 0; u < UNITS; ++u) {
                if (!BDB && !ROLL) {
                    const int toff = tap_off(u);
#pragma unroll
                    for (int g = 0; g < CT_NG; ++g) bf[0][g] = *(const bf16x8v *)(sbuf + bbase[g] + toff);
                }
                if (BDB && u + 1 < UNITS) {
                    const int toff = tap_off(u + 1);
#pragma unroll
                    for (int g = 0; g < CT_NG; ++g) bf[(u + 1) & 1][g] = *(const bf16x8v *)(sbuf + bbase[g] + toff);
                }
                // ring: unit u sits in slot u % WD; the slot of unit u-1 is refilled WD-1 units ahead
                bf16x8v wc[KW];
#pragma unroll
                for (int k = 0; k < KW; ++k) wc[k] = wring[u % WD][k];
                load_w(sidx, u + WD - 1, wring[(u + WD - 1) % WD]);
                __builtin_amdgcn_sched_barrier(0);
                if (!ROLL) {
#pragma unroll
                    for (int g = 0; g < CT_NG; ++g) {
#pragma unroll
                        for (int k = 0; k < KW; ++k)
                            acc[k][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wc[k], bf[BDB ? (u & 1) : 0][g], acc[k][g], 0, 0, 0);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                } else {
                    const int toff = u + 1 < UNITS ? tap_off(u + 1) : 0;
#pragma unroll
                    for (int g = 0; g < CT_NG; ++g) {
#pragma unroll
                        for (int k = 0; k < KW; ++k)
                            acc[k][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wc[k], bf[0][g], acc[k][g], 0, 0, 0);
                        if (u + 1 < UNITS) bf[0][g] = *(const bf16x8v *)(sbuf + bbase[g] + toff);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
            if (more) stash_halo(buf ^ 1);
            __syncthreads();
            buf ^= 1;
        }

        // epilogue: bias + activation, then 4 consecutive features of one pixel per lane.  One uniform
        // branch selects a straight-line copy (ACT 0 none, 1 ReLU, 2 sigmoid / tanh).
        auto epilogue = [&](auto act_c) {
            constexpr int ACT = decltype(act_c)::value;
#pragma unroll
            for (int k = 0; k < KW; ++k) {
                if (kb0 + k >= a.Kb) continue;
                float4v bv = {0.f, 0.f, 0.f, 0.f};
                if (a.bias) bv = *(const float4v *)(a.bias + (kb0 + k) * 16 + 4 * kg);
#pragma unroll
                for (int g = 0; g < CT_NG; ++g) {
                    if (ooff[g] < 0) continue;
                    float4v v = acc[k][g] + bv;
                    v = act4<ACT>(v, a.act);
                    TOut *dst = O + ooff[g] + (int64_t)k * a.Hout * a.Wout * 16;
                    if (sizeof(TOut) == 4) *(float4v *)dst = v;
                    else *(us4v *)dst = pack_bf16x4(v);
                }
            }
        };
        act_dispatch(a.act, epilogue);
        if (!has_next) break;
        tile_v = next_v;
        tb ^= 1;
    }
}

template <int R, int S, int STR, int CG, int NPASS, int KW, bool TP, typename TOut>
__global__ __launch_bounds__(256, TP ? 1 : 2) void conv_tile_bf16(ConvTileArgs a)
{
    conv_tile_bf16_body<R, S, STR, CG, NPASS, KW, TP, TOut>(a, blockIdx.x, blockIdx.y, gridDim.x);
}

// Backward by data of a stride-2 3x3 layer: the parity classes with 1x2, 2x1 and 2x2 taps write disjoint
// sub-lattices of dI and are independent, but each alone starts too few workgroups to fill the chip
// (14x14 and 7x7 outputs); blockIdx.z runs the three as ONE grid.  All three use the same tiling
// (unit stride, four channel blocks per stage), so their grids and LDS sizes agree.
struct ConvTileArgs3 {
    ConvTileArgs c[3];
};

template <int KW> __global__ __launch_bounds__(256, 2) void conv_tile_bf16_s2bwd(ConvTileArgs3 a)
{
    if (blockIdx.z == 0) conv_tile_bf16_body<1, 2, 1, 4, 2, KW, false, bf16_t>(a.c[0], blockIdx.x, blockIdx.y, gridDim.x);
    else if (blockIdx.z == 1) conv_tile_bf16_body<2, 1, 1, 4, 2, KW, false, bf16_t>(a.c[1], blockIdx.x, blockIdx.y, gridDim.x);
    else conv_tile_bf16_body<2, 2, 1, 4, 2, KW, false, bf16_t>(a.c[2], blockIdx.x, blockIdx.y, gridDim.x);
}

}  // namespace brg

namespace brg {
// zero fill (16 bytes per thread and step), used where a backward pass leaves pixels untouched
__global__ __launch_bounds__(256) void conv_zero_fill(float4v *dst, int64_t n16)
{
    const float4v z = {0.f, 0.f, 0.f, 0.f};
    for (int64_t i = blockIdx.x * 256ll + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256) dst[i] = z;
}
}  // namespace brg
