// Tiled convolution kernels: Algorithm 4 of the paper mapped onto CDNA4 workgroups.
//
// A workgroup (4 wavefronts) walks over output tiles of 64 feature maps x up to 112 pixels
// (a run of whole output rows, possibly crossing image boundaries).  Wave w owns the
// 16-feature block k_b = 4*blockIdx.y + w and all pixels of the tile, so its C tile is
// 7 MFMA accumulators (16 x 16 each) that stay in registers across the whole reduce chain
// over (c_b, r, s) and are stored once, after bias/activation.
//
// The paper's address lists become address arithmetic:
//  * B operand (input pixels): for each group of CG channel blocks the input rows the tile
//    needs (its "halo") are staged once in LDS, double buffered; every (r, s) tap of the
//    chain is then just a constant byte offset (r*Wp + s)*16 from a per-lane base address.
//    LDS keeps the 16 channels of a pixel as 16-byte chunks in separate planes
//    ([c_b][chunk][row][col]) so that 16 neighbouring pixels are 16 neighbouring 16-byte
//    words: one ds_read_b128 per lane feeds all MFMAs of a tap.
//  * A operand (weights): each wave reads the 16x16 weight blocks of its k_b straight from
//    global memory (L2-resident) into registers, in MFMA operand order, one stage ahead of
//    their use.
//  * Zero padding is logical: border columns of the LDS halo are zeroed once, out-of-image
//    rows are written as zeros when a halo is staged.
//
// Rows are addressed through "virtual rows": image n owns Hv = (P-1)*stride + R rows
// (padding included), output row (n, oj) reads virtual rows n*Hv + oj*stride ... + R-1.
// A tile is a range of global output rows gr = n*P + oj, its halo a contiguous range of
// virtual rows; this also covers tiles that span several small images.
//
// The workgroups are persistent: each walks over tiles blockIdx.x, blockIdx.x + gridDim.x, ...
// and treats (tile, channel group) as one continuous stream of stages, so the first halo of
// the next tile is already in flight while the last stage of the current tile is multiplied
// and its result stored.
//
// The same kernel runs the backward-by-data pass of stride-1 layers (the "dual convolution"):
// dO plays the input, the weight blocks are read transposed and the taps in reverse order.
#pragma once

#include "brg_common.hpp"

namespace brg {

constexpr int CT_NG = 7;          // pixel groups of 16 per tile

struct ConvTileArgs {
    const void *I, *Wt;
    void *O;
    const float *bias;
    int act;
    // "input"/"output" are the roles in THIS pass (for backward by data: input = dO, output = dI).
    // H, W are the dimensions of the input as the kernel sees it: for 1x1 filters with a stride the
    // kernel runs as a stride-1 pass over the sub-sampled image and `sub` is that stride.
    int N, Cb, H, W, Kb, P, Q, ph, pw, sub;
    int Hin, Win;      // physical input dimensions (H*sub, W*sub rounded as stored)
    int Hv, Wp, trg, ntiles, total_rows;
    int plane_bytes;   // bytes of one 16-byte-chunk plane of one halo buffer
    int buf_bytes;     // planes per buffer * plane_bytes
    int w_ob, w_ib;    // weight block index = ob*w_ob + ib*w_ib + tap (in 16x16 blocks)
    float inv_Q, inv_P, inv_Hv, inv_W4;  // reciprocals for the index divisions
    // placement of the logical P x Q output inside the physical Hout x Wout tensor:
    // output pixel (oj, oi) is stored at (oj*osub + ooh, oi*osub + oow); and the weight tap that
    // belongs to kernel tap t (identity forward, flipped / thinned out for backward by data)
    int osub, ooh, oow, Hout, Wout;
    int wtap[16];
};

// Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of
// tiles so that neighbouring tiles (which share halo rows) share an L2.
__device__ __forceinline__ int xcd_tile(int bid, int ntiles)
{
    const int per = ntiles >> 3, rem = ntiles & 7;
    const int x = bid & 7, i = bid >> 3;
    return x * per + (x < rem ? x : rem) + i;   // XCD x owns per + (x < rem) tiles
}

// x / d for 0 <= x < 2^22 via a float reciprocal, with exact fix-up
__device__ __forceinline__ int fdiv(int x, int d, float inv)
{
    int q = (int)((float)x * inv);
    int r = x - q * d;
    if (r < 0) --q;
    if (r >= d) ++q;
    return q;
}

// every 16x16 fp32 block [c][k] -> [k][c] (src != dst)
__global__ __launch_bounds__(256) void conv_wt_transpose_f32(const float *__restrict__ src, float *__restrict__ dst, int64_t nblocks)
{
    const int64_t b = blockIdx.x;
    if (b >= nblocks) return;
    const int t = threadIdx.x;            // t = k*16 + c of the destination
    dst[b * 256 + t] = src[b * 256 + (t & 15) * 16 + (t >> 4)];
}

template <int R, int S, int STR, int CG, int NPASS, int MODE>
__global__ __launch_bounds__(256, 2) void conv_tile_f32(ConvTileArgs a)
{
    // MODE 0: forward, weights as stored; 1: backward by data (taps flipped, roles of c and k swapped);
    // 2: forward with every 16x16 weight block transposed beforehand (reduction index contiguous);
    // 3: backward by data of one parity class of a strided layer (as 1, results placed on every stride-th pixel)
    constexpr bool BWD = MODE == 1 || MODE == 3, WVEC = MODE != 0, PLACE = MODE == 3;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const float *__restrict__ I = (const float *)a.I;
    const float *__restrict__ Wt = (const float *)a.Wt;
    float *__restrict__ O = (float *)a.O;
    constexpr int TAPS = R * S;
    constexpr int UNITS = CG * TAPS;                    // weight blocks consumed per stage

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int li = lane & 15, kg = lane >> 4;
    const int kb_raw = blockIdx.y * 4 + wave;
    const bool kb_ok = kb_raw < a.Kb;
    const int kb = kb_ok ? kb_raw : a.Kb - 1;
    const int nstage = a.Cb / CG;                       // stages per tile
    const int64_t cb_stride = (int64_t)a.Hin * a.Win * 16;

    int tile_v = blockIdx.x;                            // virtual tile index (before the XCD remap)
    if (tile_v >= a.ntiles) return;                     // uniform per workgroup

    // ---- zero both halo buffers once (the padding columns are never written again)
    {
        const float4v z = {0.f, 0.f, 0.f, 0.f};
        for (int o = t * 16; o < 2 * a.buf_bytes; o += 256 * 16) *(float4v *)(smem + o) = z;
    }

    // ---- per-thread halo copy plan of a tile: chunk e = t + 256*i of the halo of ONE c_b
    // (row-major, 4 chunks per pixel); goff < 0 marks a zero row, loff < 0 a chunk beyond the halo
    int goff[NPASS], loff[NPASS];
    auto plan = [&](int tile) {
        const int gr0 = tile * a.trg;
        const int rows = min(a.trg, a.total_rows - gr0);
        const int n0 = fdiv(gr0, a.P, a.inv_P);
        const int v_first = n0 * a.Hv + (gr0 - n0 * a.P) * STR;
        const int grl = gr0 + rows - 1;
        const int nl = fdiv(grl, a.P, a.inv_P);
        const int nv = nl * a.Hv + (grl - nl * a.P) * STR + R - v_first;
        const int W4 = a.W * 4, chunks = nv * W4;
#pragma unroll
        for (int i = 0; i < NPASS; ++i) {
            const int e = t + 256 * i;
            const int row = fdiv(e, W4, a.inv_W4), rem = e - row * W4;
            const int v = v_first + row;
            const int n = fdiv(v, a.Hv, a.inv_Hv), ih = v - n * a.Hv - a.ph;
            const bool in_halo = e < chunks;
            const bool real = ih >= 0 && ih < a.H && n < a.N;
            goff[i] = (in_halo && real)
                          ? (((n * a.Cb * a.Hin + ih * a.sub) * a.Win) + (rem >> 2) * a.sub) * 16 + (rem & 3) * 4
                          : -1;
            loff[i] = in_halo ? (rem & 3) * a.plane_bytes + (row * a.Wp + (rem >> 2) + a.pw) * 16 : -1;
        }
    };

    float4v stage[CG][NPASS];
    auto load_halo = [&](int sidx) {   // channel blocks sidx*CG .. sidx*CG + CG-1 of the planned tile
#pragma unroll
        for (int c = 0; c < CG; ++c) {
            const float *src = I + (int64_t)(sidx * CG + c) * cb_stride;
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
            unsigned char *dst = smem + buf * a.buf_bytes + c * 4 * a.plane_bytes;
#pragma unroll
            for (int i = 0; i < NPASS; ++i)
                if (loff[i] >= 0) *(float4v *)(dst + loff[i]) = stage[c][i];
        }
    };

    // ---- weights: block (ob = kb, ib, tap) at Wt + (kb*w_ob + ib*w_ib + tap')*256, where
    // tap' = tap for the forward pass, TAPS-1-tap (spatially flipped) for backward by data, and wtap[tap] for the
    // parity classes of a strided layer (flipped and thinned out to the taps of the class).
    // Lane (li, kg) needs, for MFMA step q, the element (row li, reduction index 4*kg + q):
    //   forward : block[c = 4kg+q][k = li]  -> four dwords 16 elements apart (one float4 from a transposed copy)
    //   backward: block[c = li][k = 4kg+q]  -> one aligned float4
    const float *wlane = Wt + (int64_t)kb * a.w_ob * 256 + (WVEC ? li * 16 + 4 * kg : 64 * kg + li);
    // All UNITS weight blocks of a stage live in registers (4 per block, MFMA operand order) and the
    // blocks of the NEXT stage are requested at the very start of a stage, BEFORE the halo loads:
    // the memory counter retires in order, so weight loads queued behind HBM-latency halo loads
    // would stall the first MFMAs that need them.
    float wcur[UNITS][4], wnxt[UNITS][4];
    int wt[TAPS];                                       // parity classes: the taps of the class, from the table
#pragma unroll
    for (int tp = 0; tp < TAPS; ++tp) wt[tp] = PLACE ? a.wtap[tp] : (BWD ? TAPS - 1 - tp : tp);
    auto load_w = [&](int sidx, float (&w)[UNITS][4]) {
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
            const int tap = u % TAPS;
            const float *src = wlane + ((int64_t)(sidx * CG + u / TAPS) * a.w_ib + wt[tap]) * 256;
            if (WVEC) {
                const float4v v = *(const float4v *)src;
#pragma unroll
                for (int q = 0; q < 4; ++q) w[u][q] = v[q];
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) w[u][q] = src[q * 16];
            }
        }
    };

    plan(xcd_tile(tile_v, a.ntiles));
    load_w(0, wcur);
    load_halo(0);
    __syncthreads();  // zero fill done
    stash_halo(0);
    __syncthreads();
    int buf = 0;

    while (true) {
        const int tile = xcd_tile(tile_v, a.ntiles);
        const int next_v = tile_v + gridDim.x;
        const bool has_next = next_v < a.ntiles;

        // ---- per-lane pixel addresses of this tile
        int bbase[CT_NG], ooff[CT_NG];
        {
            const int gr0 = tile * a.trg;
            const int rows = min(a.trg, a.total_rows - gr0);
            const int n0 = fdiv(gr0, a.P, a.inv_P);
            const int v_first = n0 * a.Hv + (gr0 - n0 * a.P) * STR;
#pragma unroll
            for (int g = 0; g < CT_NG; ++g) {
                const int p = g * 16 + li;
                const int rr = fdiv(p, a.Q, a.inv_Q), oi = p - rr * a.Q;
                const bool ok = rr < rows;
                const int gr = gr0 + (ok ? rr : 0);
                const int n = fdiv(gr, a.P, a.inv_P), oj = gr - n * a.P;
                const int lrow = n * a.Hv + oj * STR - v_first;
                bbase[g] = kg * a.plane_bytes + (lrow * a.Wp + (ok ? oi : 0) * STR) * 16;
                // (the general placement serves the parity classes of a strided backward pass only: in the other
                // forms it costs registers that the 3x3 kernels do not have)
                if (PLACE)
                    ooff[g] = (ok && kb_ok) ? (((n * a.Kb + kb) * a.Hout + oj * a.osub + a.ooh) * a.Wout + oi * a.osub + a.oow) * 16 + 4 * kg : -1;
                else
                    ooff[g] = (ok && kb_ok) ? (((n * a.Kb + kb) * a.P + oj) * a.Q + oi) * 16 + 4 * kg : -1;
            }
        }

        float4v acc[CT_NG];
#pragma unroll
        for (int g = 0; g < CT_NG; ++g) acc[g] = float4v{0.f, 0.f, 0.f, 0.f};

        for (int sidx = 0; sidx < nstage; ++sidx) {
            // prefetch the next stage of the stream: the next channel group of this tile, or the
            // first one of the next tile
            const bool last = sidx + 1 == nstage;
            const bool more = !last || has_next;
            if (last && has_next) plan(xcd_tile(next_v, a.ntiles));
            if (more) {
                load_w(last ? 0 : sidx + 1, wnxt);
                load_halo(last ? 0 : sidx + 1);
            }

            const unsigned char *sbuf = smem + buf * a.buf_bytes;
            float4v bf[2][CT_NG];
#pragma unroll
            for (int g = 0; g < CT_NG; ++g) bf[0][g] = *(const float4v *)(sbuf + bbase[g]);
#pragma unroll
            for (int u = 0; u < UNITS; ++u) {
                if (u + 1 < UNITS) {   // B fragments of the next unit (c_b, r, s)
                    const int c1 = (u + 1) / TAPS, t1 = (u + 1) % TAPS;
                    const int toff = c1 * 4 * a.plane_bytes + ((t1 / S) * a.Wp + t1 % S) * 16;
#pragma unroll
                    for (int g = 0; g < CT_NG; ++g)
                        bf[(u + 1) & 1][g] = *(const float4v *)(sbuf + bbase[g] + toff);
                }
                __builtin_amdgcn_sched_barrier(0);
                // The four MFMAs of one accumulator are issued back to back: on gfx950 the 16x16
                // MFMAs only reach full rate when consecutive instructions reuse the accumulator.
                // (The scheduling fences keep the compiler from re-interleaving the accumulators.)
#pragma unroll
                for (int g = 0; g < CT_NG; ++g) {
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        acc[g] = __builtin_amdgcn_mfma_f32_16x16x4f32(wcur[u][q], bf[u & 1][g][q], acc[g], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (more) {
                stash_halo(buf ^ 1);
#pragma unroll
                for (int u = 0; u < UNITS; ++u)
#pragma unroll
                    for (int q = 0; q < 4; ++q) wcur[u][q] = wnxt[u][q];
            }
            __syncthreads();
            buf ^= 1;
        }

        // ---- epilogue: bias + activation on the accumulators, one 16-byte store per pixel
        float4v bv = {0.f, 0.f, 0.f, 0.f};
        if (a.bias) bv = *(const float4v *)(a.bias + kb * 16 + 4 * kg);
        act_dispatch(a.act, [&](auto act_c) {
#pragma unroll
            for (int g = 0; g < CT_NG; ++g) {
                if (ooff[g] < 0) continue;
                *(float4v *)(O + ooff[g]) = act4<decltype(act_c)::value>(acc[g] + bv, a.act);
            }
        });
        if (!has_next) break;
        tile_v = next_v;
    }
}

}  // namespace brg
