// The 7x7 stride-2 pad-3 "stem" convolution in bf16 with its 3 input channels stored as ONE channel
// block of 4 (bc = 4: 8 bytes per pixel), forward pass (paper section 3.2, Algorithm 4; the paper's
// Table 2 layer 1).  With a single short channel block the batch-reduce chain of Algorithm 4 (one block
// per filter tap) would fill 4 of the 32 reduction lanes of v_mfma_f32_16x16x32_bf16.  The chain is
// therefore re-blocked BY FILTER ROW: the 7 taps x 4 channels of one filter row are 28 consecutive
// values of the input row (8 bytes per pixel), padded to 32 with an eighth pixel whose weights are
// zero, so one MFMA reduces a whole filter row and an output needs 7 MFMAs instead of 49.
//
//  * B operand (lane = output pixel oi, lane group g): input pixels 2oi - 3 + 2g and + 1 of the row,
//    i.e. 16 contiguous, 16-byte aligned bytes of the halo row in LDS (columns are shifted by the
//    padding, so the address is 16 * (oi + g)): one conflict-free ds_read_b128.
//  * A operand (lane = output feature k, lane group g): taps s = 2g, 2g+1 x 4 channels of filter row r;
//    gathered once per kernel from the [r][s][4c][16k] weight blocks and kept in registers for all
//    tiles (7 rows x KB feature blocks x 4 registers).
//  * A persistent workgroup walks tiles of 4 output rows x all columns x all features; the 13 input rows
//    of a tile go global -> registers -> LDS (zero filled outside the image) one tile ahead.  Each wave
//    takes the pixel groups g = wave, wave + 4 and ALL feature blocks, so a B fragment read from LDS
//    feeds KB MFMAs.
#pragma once

#include "brg_conv1x1_bf16.hpp"

namespace brg {

constexpr int ST_TR = 4;                       // output rows per tile
constexpr int ST_ROWS = 2 * ST_TR + 5;         // input rows per tile
constexpr int ST_NLOAD = 12;                   // 8-byte pixels per thread and tile (>= ST_ROWS * pitch / 256)

struct StemArgs {
    const void *I, *Wt;
    void *O;
    const float *bias;
    int act;
    int N, H, W, Kb, P, Q;
    int ngroups;        // ceil(Q / 16), at most 7
    int pitch;          // pixels per halo row in LDS: 32 * ngroups + 6
    int tiles_per_img;  // ceil(P / ST_TR)
    int ntiles;
};

typedef unsigned short us4s __attribute__((ext_vector_type(4)));

// Pre-pass: filter rows as MFMA A operands, P[kb][r][k][e] with e = 4*s + c (tap s = 0..7, channel c = 0..3;
// tap 7 is zero), so that a lane's eight reduction elements are 16 contiguous bytes.
__global__ __launch_bounds__(256) void conv_stem_pack_weights(const bf16_t *__restrict__ Wt, bf16_t *__restrict__ Pk, int Kb)
{
    const int i = blockIdx.x * 256 + threadIdx.x;      // ((kb*7 + r)*16 + k)*32 + e
    if (i >= Kb * 7 * 16 * 32) return;
    const int e = i & 31, k = (i >> 5) & 15, kr = i >> 9, r = kr % 7, kb = kr / 7;
    const int s = e >> 2, c = e & 3;
    Pk[i] = s < 7 ? Wt[(((int64_t)kb * 49 + r * 7 + s) * 4 + c) * 16 + k] : (bf16_t)0;
}

// PACKED: a.Wt is the pre-packed copy (see above); otherwise the lanes gather their operands from the
// original weight blocks themselves (slower start, no workspace needed).
template <int KB, bool PACKED> __global__ __launch_bounds__(256, 2) void conv_stem_fwd_bf16(StemArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char st_smem[];
    const bf16_t *__restrict__ I = (const bf16_t *)a.I;
    const bf16_t *__restrict__ Wt = (const bf16_t *)a.Wt;
    bf16_t *__restrict__ O = (bf16_t *)a.O;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int li = lane & 15, kg = lane >> 4;
    const int kb0 = blockIdx.y * KB;
    const int buf_bytes = ST_ROWS * a.pitch * 8;

    // ---- weights of filter row r, feature block kb0 + k: elements e = 0..7 of this lane are tap
    // s = 2kg + (e >> 2), channel e & 3, feature li; a tap beyond the filter row is zero
    bf16x8v wa[KB][7];
#pragma unroll
    for (int k = 0; k < KB; ++k) {
        const int kb = kb0 + k < a.Kb ? kb0 + k : a.Kb - 1;
#pragma unroll
        for (int r = 0; r < 7; ++r) {
            if (PACKED) {
                wa[k][r] = *(const bf16x8v *)(Wt + (((int64_t)kb * 7 + r) * 16 + li) * 32 + 8 * kg);
            } else {
                typedef unsigned short us8 __attribute__((ext_vector_type(8)));
                us8 v;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int s = 2 * kg + (e >> 2);
                    const int sc = s < 7 ? s : 6;
                    const unsigned short x = Wt[(((int64_t)kb * 49 + r * 7 + sc) * 4 + (e & 3)) * 16 + li];
                    v[e] = s < 7 ? x : (unsigned short)0;
                }
                wa[k][r] = __builtin_bit_cast(bf16x8v, v);
            }
        }
    }

    // ---- halo copy plan: position e = t + 256 i of the [ST_ROWS][pitch] pixel array (fixed for all tiles)
    int ppos[ST_NLOAD];   // (row << 16) | (column + 3), or -1 beyond the array
    const float inv_pitch = 1.0f / (float)a.pitch;
#pragma unroll
    for (int i = 0; i < ST_NLOAD; ++i) {
        const int e = t + 256 * i;
        const int rr = c1_fdiv(e, a.pitch, inv_pitch);
        ppos[i] = rr < ST_ROWS ? (rr << 16) | (e - rr * a.pitch) : -1;
    }
    us4s stage[ST_NLOAD];
    auto load_halo = [&](int tile) {
        const int n = tile / a.tiles_per_img, oj0 = (tile - n * a.tiles_per_img) * ST_TR;
        const bf16_t *img = I + (int64_t)n * a.H * a.W * 4;
#pragma unroll
        for (int i = 0; i < ST_NLOAD; ++i) {
            const int h = 2 * oj0 - 3 + (ppos[i] >> 16), w = (ppos[i] & 0xffff) - 3;
            stage[i] = us4s{0, 0, 0, 0};
            if (ppos[i] >= 0 && h >= 0 && h < a.H && w >= 0 && w < a.W) stage[i] = *(const us4s *)(img + ((int64_t)h * a.W + w) * 4);
        }
    };
    auto stash_halo = [&](int buf) {
        unsigned char *dst = st_smem + buf * buf_bytes;
#pragma unroll
        for (int i = 0; i < ST_NLOAD; ++i)
            if (ppos[i] >= 0) *(us4s *)(dst + (t + 256 * i) * 8) = stage[i];
    };

    int tile = blockIdx.x;
    if (tile >= a.ntiles) return;
    load_halo(tile);
    stash_halo(0);
    __syncthreads();
    int buf = 0;
    while (true) {
        const int next = tile + gridDim.x;
        const bool has_next = next < a.ntiles;
        if (has_next) load_halo(next);

        const int n = tile / a.tiles_per_img, oj0 = (tile - n * a.tiles_per_img) * ST_TR;
        const unsigned char *sbuf = st_smem + buf * buf_bytes;
#pragma unroll 1
        for (int g = wave; g < a.ngroups; g += 4) {
            const int oi = 16 * g + li;
            const unsigned char *bcol = sbuf + 16 * (oi + kg);     // pixel 2oi - 3 + 2kg sits in column 2oi + 2kg
#pragma unroll 1
            for (int jr = 0; jr < ST_TR; ++jr) {
                const int oj = oj0 + jr;
                if (oj >= a.P) break;                               // uniform per workgroup
                float4v acc[KB];
#pragma unroll
                for (int k = 0; k < KB; ++k) acc[k] = float4v{0.f, 0.f, 0.f, 0.f};
                bf16x8v bf[7];
#pragma unroll
                for (int r = 0; r < 7; ++r) bf[r] = *(const bf16x8v *)(bcol + (2 * jr + r) * a.pitch * 8);
#pragma unroll
                for (int r = 0; r < 7; ++r)
#pragma unroll
                    for (int k = 0; k < KB; ++k)
                        acc[k] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[k][r], bf[r], acc[k], 0, 0, 0);
                // register j of lane (li, kg) is feature 4kg + j of block kb0 + k at pixel (oj, oi)
                if (oi < a.Q) {
                    act_dispatch(a.act, [&](auto act_c) {
#pragma unroll
                        for (int k = 0; k < KB; ++k) {
                            if (kb0 + k >= a.Kb) continue;
                            float4v v = acc[k];
                            if (a.bias) v += *(const float4v *)(a.bias + (kb0 + k) * 16 + 4 * kg);
                            *(us4v *)(O + ((((int64_t)n * a.Kb + kb0 + k) * a.P + oj) * a.Q + oi) * 16 + 4 * kg) =
                                pack_bf16x4(act4<decltype(act_c)::value>(v, a.act));
                        }
                    });
                }
            }
        }
        if (has_next) stash_halo(buf ^ 1);
        __syncthreads();
        if (!has_next) break;
        buf ^= 1;
        tile = next;
    }
}

// ---------------------------------------------------------------------------------------------------
// Backward by data of the same layer (the "dual convolution" of the close of paper section 3.2.2): dI has one channel
// block of 4.  The input pixels (h, w) = (2i + a, 2j + b) of parity class (a, b) receive the filter taps
// r = r0 + 2tr, s = s0 + 2ts (r0 = (a + 1) % 2, 3 or 4 taps per direction) from dO pixel
// (i + drmax - tr, j + dsmax - ts): per class a stride-1 pass over dO, one launch each.
//
//  * The batch-reduce chain runs over (tap, pair of feature blocks); M of the MFMA is the channel block
//    (rows 0..3 real, the other rows have zero weights), N the 16 pixels of a group.  Lane group 0 then
//    holds the four channels of pixel `lane` in its accumulator registers: one 8-byte store per pixel.
//  * dO rows are staged in LDS one feature-block pair at a time as [row][column][2 blocks x 16] = 64 bytes
//    per pixel, the 16-byte chunk q of column c stored at position q ^ ((c >> 2) & 3) so that the B
//    fragments (one ds_read_b128 per tap) are bank-conflict free.
//  * Each wave takes the pixel groups g = wave, wave + 4 of the tile's two class rows; the weights of the
//    current feature-block pair (TR x TS operands) sit in registers.
constexpr int SB_TR = 2;               // class rows per tile
constexpr int SB_ROWS = SB_TR + 3;     // dO rows staged per tile
constexpr int SB_NLOAD = 9;            // 16-byte chunks per thread and stage (>= SB_ROWS * pitch * 4 / 256)

struct StemBwdArgs {
    const void *dO, *Wt;
    void *dI;
    int N, H, W, Kb, P, Q;
    int ca, cb;          // parity class
    int Hc, Wc;          // class pixels per image
    int ngroups;         // ceil(Wc / 16), at most 7
    int pitch;           // staged columns: 16 * ngroups + 3
    int tiles_per_img, ntiles;
};

template <int TR, int TS> __global__ __launch_bounds__(256, 2) void conv_stem_bwd_bf16(StemBwdArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char sb_smem[];
    const bf16_t *__restrict__ dO = (const bf16_t *)a.dO;
    const bf16_t *__restrict__ Wt = (const bf16_t *)a.Wt;
    bf16_t *__restrict__ dI = (bf16_t *)a.dI;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int li = lane & 15, kg = lane >> 4;
    const int r0 = (a.ca + 1) & 1, s0 = (a.cb + 1) & 1;
    constexpr int DRMAX = TR - 2, DSMAX = TS - 2;     // 3 taps: offsets 1, 0, -1; 4 taps: 2, 1, 0, -1
    const int buf_bytes = SB_ROWS * a.pitch * 64;
    const int npairs = (a.Kb + 1) >> 1;

    // ---- staging plan (fixed for all tiles): chunk e = t + 256 i; pixel e >> 2, 16-byte chunk q = t & 3
    const int q = t & 3;
    int ppos[SB_NLOAD], ldst[SB_NLOAD];
    const float inv_pitch = 1.0f / (float)a.pitch;
#pragma unroll
    for (int i = 0; i < SB_NLOAD; ++i) {
        const int pe = (t + 256 * i) >> 2;
        const int hr = c1_fdiv(pe, a.pitch, inv_pitch), c = pe - hr * a.pitch;
        ppos[i] = hr < SB_ROWS ? (hr << 16) | c : -1;
        ldst[i] = pe * 64 + ((q ^ ((c >> 2) & 3)) << 4);
    }
    float4v stage[SB_NLOAD];
    auto load_stage = [&](int tile, int kp) {
        const int n = tile / a.tiles_per_img, i0 = (tile - n * a.tiles_per_img) * SB_TR;
        const int kb = 2 * kp + (q >> 1);
        const bf16_t *src = dO + ((int64_t)n * a.Kb + kb) * a.P * a.Q * 16 + 8 * (q & 1);
#pragma unroll
        for (int i = 0; i < SB_NLOAD; ++i) {
            const int oj = i0 - 1 + (ppos[i] >> 16), oi = (ppos[i] & 0xffff) - 1;
            stage[i] = float4v{0.f, 0.f, 0.f, 0.f};
            if (ppos[i] >= 0 && kb < a.Kb && oj >= 0 && oj < a.P && oi >= 0 && oi < a.Q)
                stage[i] = *(const float4v *)(src + ((int64_t)oj * a.Q + oi) * 16);
        }
    };
    auto stash_stage = [&](int buf) {
        unsigned char *dst = sb_smem + buf * buf_bytes;
#pragma unroll
        for (int i = 0; i < SB_NLOAD; ++i)
            if (ppos[i] >= 0) *(float4v *)(dst + ldst[i]) = stage[i];
    };

    // ---- B fragment addresses: column c = 16g + li + 1 + DSMAX - ts, chunk kg
    int boff[2][TS];
#pragma unroll
    for (int gi = 0; gi < 2; ++gi)
#pragma unroll
        for (int ts = 0; ts < TS; ++ts) {
            const int c = 16 * (wave + 4 * gi) + li + 1 + DSMAX - ts;
            boff[gi][ts] = c * 64 + ((kg ^ ((c >> 2) & 3)) << 4);
        }

    int tile = blockIdx.x;
    if (tile >= a.ntiles) return;
    load_stage(tile, 0);
    stash_stage(0);
    __syncthreads();
    int buf = 0;
    while (true) {
        const int next = tile + gridDim.x;
        const bool has_next = next < a.ntiles;
        float4v acc[2][SB_TR];
#pragma unroll
        for (int gi = 0; gi < 2; ++gi)
#pragma unroll
            for (int jr = 0; jr < SB_TR; ++jr) acc[gi][jr] = float4v{0.f, 0.f, 0.f, 0.f};

        for (int kp = 0; kp < npairs; ++kp) {
            // weights of this feature-block pair: row li = channel (rows >= 4 are zero), 8 features of
            // block 2kp + (kg >> 1)
            bf16x8v wa[TR][TS];
            {
                const int kb = 2 * kp + (kg >> 1);
                const bool live = li < 4 && kb < a.Kb;
                const bf16_t *wp = Wt + (((int64_t)(live ? kb : 0) * 49) * 4 + (live ? li : 0)) * 16 + 8 * (kg & 1);
#pragma unroll
                for (int tr = 0; tr < TR; ++tr)
#pragma unroll
                    for (int ts = 0; ts < TS; ++ts) {
                        bf16x8v v = *(const bf16x8v *)(wp + ((r0 + 2 * tr) * 7 + (s0 + 2 * ts)) * 64);
                        if (!live) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) v[e] = (__bf16)0.0f;
                        }
                        wa[tr][ts] = v;
                    }
            }
            const bool last_kp = kp + 1 == npairs;
            const bool more = !last_kp || has_next;
            if (more) load_stage(last_kp ? next : tile, last_kp ? 0 : kp + 1);

            const unsigned char *sbuf = sb_smem + buf * buf_bytes;
#pragma unroll
            for (int gi = 0; gi < 2; ++gi) {
                if (wave + 4 * gi >= a.ngroups) continue;       // uniform per wave
#pragma unroll
                for (int jr = 0; jr < SB_TR; ++jr)
#pragma unroll
                    for (int tr = 0; tr < TR; ++tr) {
                        const unsigned char *brow = sbuf + (jr + DRMAX - tr + 1) * a.pitch * 64;
#pragma unroll
                        for (int ts = 0; ts < TS; ++ts)
                            acc[gi][jr] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                wa[tr][ts], *(const bf16x8v *)(brow + boff[gi][ts]), acc[gi][jr], 0, 0, 0);
                    }
            }
            if (more) stash_stage(buf ^ 1);
            __syncthreads();
            buf ^= 1;
        }

        // ---- lane group 0: register j = channel j of class pixel (i0 + jr, 16g + li)
        if (kg == 0) {
            const int n = tile / a.tiles_per_img, i0 = (tile - n * a.tiles_per_img) * SB_TR;
#pragma unroll
            for (int gi = 0; gi < 2; ++gi) {
                const int j = 16 * (wave + 4 * gi) + li;
                if (wave + 4 * gi >= a.ngroups || j >= a.Wc) continue;
#pragma unroll
                for (int jr = 0; jr < SB_TR; ++jr) {
                    const int i = i0 + jr;
                    if (i >= a.Hc) continue;
                    const int h = 2 * i + a.ca, w = 2 * j + a.cb;
                    *(us4v *)(dI + (((int64_t)n * a.H + h) * a.W + w) * 4) = pack_bf16x4(acc[gi][jr]);
                }
            }
        }
        if (!has_next) break;
        tile = next;
    }
}

// ---------------------------------------------------------------------------------------------------
// Backward by data of the stem in ONE pass over dO (64 features, H = 2P, W = 2Q).  The four parity
// classes of input pixels share their dO neighbourhood: input pixel (2i + a, 2j + b) collects
// dO(i + d, j + e) for d, e in {-1, 0, 1, 2} through the taps r = 3 - 2d (a = 0; d = 2 has no tap) or
// r = 4 - 2d (a = 1), and s likewise from b and e.  So the 16 rows of a 16 x 16 x 32 matrix instruction
// are filled with 4 classes x 4 channels: for each of the 16 offsets (d, e) and each half of the
// features, A holds W[k][c][r(a, d)][s(b, e)] in row 4(2a + b) + c (zero where a class has no tap) and B
// the dO pixels (i + d, j + e), lane = j.  The result register group of a lane is then the 4 channels of
// input pixel (2i + a, 2j + b), a = kg >> 1, b = kg & 1: one 8-byte store.  Compared with one launch per
// class dO is read once instead of four times, and no matrix row is padding.
//
// A workgroup takes a 16 x 16 tile of (i, j): the 19 x 19 x 64-feature dO halo is staged in LDS as 8
// planes of 8 features (consecutive pixels 16 bytes apart: conflict-free operand reads at any column
// offset); wave w owns rows 4w .. 4w+3, so a B fragment of halo row h serves the up to four output rows
// h - d.  The 32 A fragments stay in registers for all tiles of the (persistent) workgroup.
struct StemBwdFusedArgs {
    const void *dO, *Wt;
    void *dI;
    int N, H, W, P, Q;
    int tiles_r, tiles_c, ntiles;
};

constexpr int SF_T = 16;                              // tile edge in dO positions
constexpr int SF_HW = SF_T + 3;                       // halo edge
constexpr int SF_PLANE = SF_HW * SF_HW * 16;          // bytes of one 8-feature plane
constexpr int SF_CHUNKS = 4 * SF_HW * SF_HW * 2;      // 16-byte chunks of a halo: 4 feature blocks x pixels x 2
constexpr int SF_NLOAD = (SF_CHUNKS + 255) / 256;     // per thread
constexpr int SF_HALF = (SF_NLOAD + 1) / 2;

__global__ __launch_bounds__(256) void conv_stem_bwd_fused_bf16(StemBwdFusedArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[8 * SF_PLANE];
    const char *__restrict__ dO = (const char *)a.dO;
    const bf16_t *__restrict__ Wt = (const bf16_t *)a.Wt;
    char *__restrict__ dI = (char *)a.dI;
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int li = lane & 15, kg = lane >> 4;

    // ---- A fragments: row li = class (a, b) x channel c, 8 features of block 2kh + (kg >> 1)
    bf16x8v wa[4][4][2];                              // [d + 1][e + 1][feature half]
    {
        const int ca = li >> 3, cb = (li >> 2) & 1, c = li & 3;
#pragma unroll
        for (int di = 0; di < 4; ++di)
#pragma unroll
            for (int dj = 0; dj < 4; ++dj) {
                const int r = (ca ? 4 : 3) - 2 * (di - 1), s = (cb ? 4 : 3) - 2 * (dj - 1);
                const bool live = r >= 0 && s >= 0;
#pragma unroll
                for (int kh = 0; kh < 2; ++kh) {
                    const int kb = 2 * kh + (kg >> 1);
                    bf16x8v v = *(const bf16x8v *)(Wt + ((kb * 49 + (live ? r * 7 + s : 0)) * 4 + c) * 16 + 8 * (kg & 1));
                    if (!live) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] = (__bf16)0.0f;
                    }
                    wa[di][dj][kh] = v;
                }
            }
    }

    // ---- halo staging plan (the same for every tile): chunk e = t + 256 i -> (feature block, row, column, half)
    int rel[SF_NLOAD], pos[SF_NLOAD], ldst[SF_NLOAD];
#pragma unroll
    for (int i = 0; i < SF_NLOAD; ++i) {
        const int e = t + 256 * i;
        const int kb = e / (SF_HW * SF_HW * 2), rem = e - kb * (SF_HW * SF_HW * 2);
        const int row = rem / (SF_HW * 2), ch = rem - row * (SF_HW * 2);
        const int col = ch >> 1, half = ch & 1;
        const bool in = e < SF_CHUNKS;
        rel[i] = ((kb * a.P + row) * a.Q + col) * 32 + half * 16;
        pos[i] = in ? (row << 8) | col : -1;
        ldst[i] = (kb * 2 + half) * SF_PLANE + (row * SF_HW + col) * 16;
    }

    const int tiles_img = a.tiles_r * a.tiles_c;
    for (int tile = blockIdx.x; tile < a.ntiles; tile += gridDim.x) {
        const int n = tile / tiles_img, tr = (tile - n * tiles_img) / a.tiles_c, tc = tile - n * tiles_img - tr * a.tiles_c;
        const int i0 = tr * SF_T, j0 = tc * SF_T;
        const char *base = dO + (((int64_t)n * 4 * a.P + (i0 - 1)) * a.Q + (j0 - 1)) * 32;
        // stage the halo through registers, half of the chunks at a time
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            float4v stage[SF_HALF];
#pragma unroll
            for (int ii = 0; ii < SF_HALF; ++ii) {
                const int i = h * SF_HALF + ii;
                if (i >= SF_NLOAD) continue;
                const int gi = i0 - 1 + (pos[i] >> 8), gj = j0 - 1 + (pos[i] & 0xff);
                stage[ii] = float4v{0.f, 0.f, 0.f, 0.f};
                if (pos[i] >= 0 && gi >= 0 && gi < a.P && gj >= 0 && gj < a.Q) stage[ii] = *(const float4v *)(base + rel[i]);
            }
#pragma unroll
            for (int ii = 0; ii < SF_HALF; ++ii) {
                const int i = h * SF_HALF + ii;
                if (i >= SF_NLOAD) continue;
                if (pos[i] >= 0) *(float4v *)(lds + ldst[i]) = stage[ii];
            }
        }
        __syncthreads();

        float4v acc[4];
#pragma unroll
        for (int lr = 0; lr < 4; ++lr) acc[lr] = float4v{0.f, 0.f, 0.f, 0.f};
        const unsigned char *bcol = lds + kg * SF_PLANE + ((4 * wave) * SF_HW + li) * 16;
#pragma unroll
        for (int kh = 0; kh < 2; ++kh)
#pragma unroll
            for (int dj = 0; dj < 4; ++dj)
#pragma unroll
                for (int hr = 0; hr < 7; ++hr) {
                    const bf16x8v b = *(const bf16x8v *)(bcol + kh * 4 * SF_PLANE + (hr * SF_HW + dj) * 16);
#pragma unroll
                    for (int di = 0; di < 4; ++di) {
                        const int lr = hr - di;                     // halo row = output row + (d + 1)
                        if (lr < 0 || lr > 3) continue;
                        acc[lr] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[di][dj][kh], b, acc[lr], 0, 0, 0);
                    }
                }

        // lane (li, kg): the 4 channels of input pixel (2i + (kg >> 1), 2j + (kg & 1)), j = j0 + li
        const int j = j0 + li;
#pragma unroll
        for (int lr = 0; lr < 4; ++lr) {
            const int i = i0 + 4 * wave + lr;
            if (i < a.P && j < a.Q)
                *(us4v *)(dI + (((int64_t)n * a.H + 2 * i + (kg >> 1)) * a.W + 2 * j + (kg & 1)) * 8) = pack_bf16x4(acc[lr]);
        }
        __syncthreads();                                             // the halo is overwritten next
    }
}

}  // namespace brg
