// Weight gradient of convolutions on the blocked layouts (the paper's UPD pass, section 3.2); the bf16 kernels
// come first, their fp32 forms at the end:
//   dWt block (kb, cb, r, s) [c][k] = sum over images and output pixels of I[n][cb][pixel + tap][c] * dO[n][kb][pixel][k]
// for 1x1 filters (stride 1 or 2) and 3x3 filters with padding 1 (stride 1: second kernel, stride 2: third).
//
// The reduction index of this GEMM is the pixel, which both blocked tensors store as the STRIDED index
// (the 16 channels of a pixel are contiguous, 32 bytes).  As in brg_fc_wgt_bf16.hpp, 32-pixel slabs of the
// blocks are staged in LDS as stored and read back through the transposing LDS read of gfx950
// (ds_read_b64_tr_b16: inside a 16-lane group, lane t points at pixel t/4, channel quad t%4, and receives
// pixels 0..3 of channel t), two reads per 8-pixel operand of the 16x16x32 bf16 matrix instruction.
//
//  * A workgroup (4 waves as 2 x 2, wave tile WT x WT accumulator tiles per tap) owns 2 WT channel blocks x
//    2 WT feature blocks for a RANGE of the pixels (grid z); the reduction over N*P*Q pixels is split
//    across workgroups because the blocks of dWt alone are too few to fill the chip.  Partial sums go to
//    the caller's workspace and a second kernel adds the ranges in a fixed order (deterministic).
//  * Steps never cross an image: an image takes ceil(P*Q / 32) steps, the rows past its end are zero.
#pragma once

#include "brg_common.hpp"

namespace brg {

struct ConvWgtArgs {
    const bf16_t *I, *dO;
    float *out;               // dWt (nsplit == 1) or partial sums [split][Kb][Cb][taps][256]
    int N, Cb, Kb, HW;        // HW = output pixels per image
    int HWin, Win, Q, stride; // input pixels per image, input width, output width, stride (1 or 2; no padding)
    int steps_per_img, steps_total, steps_per_split;
};

template <int WT, int PS> __global__ __launch_bounds__(256) void conv_wgt1x1_bf16(ConvWgtArgs a)
{
    typedef short s4v __attribute__((ext_vector_type(4)));
    typedef short s8v __attribute__((ext_vector_type(8)));
    typedef __attribute__((address_space(3))) s4v *lds_s4p;
    constexpr int SB = 2 * WT;
    // a step is PS slabs of 32 pixels: [buffer][chunk: SB of I, SB of dO][slab][32 pixels x 32 B]
    __shared__ __attribute__((aligned(16))) char slab[2][2 * SB][PS][1024];
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int li = lane & 15, kg = lane >> 4;
    const int wy = wave >> 1, wx = wave & 1;
    const int cb0 = blockIdx.x * SB, kb0 = blockIdx.y * SB;
    const int s_begin = blockIdx.z * a.steps_per_split;
    const int s_end = min(a.steps_total, s_begin + a.steps_per_split);

    // staging: wave w moves chunks WT w .. WT w + WT-1; lane L holds half L%2 of pixel row L/2 of each slab
    const int row = lane >> 1;
    const char *src[WT];
    int64_t img_stride[WT];                                            // bytes between images
#pragma unroll
    for (int j = 0; j < WT; ++j) {
        const int ch = WT * wave + j;
        if (ch < SB) {
            src[j] = (const char *)a.I + (int64_t)(cb0 + ch) * a.HWin * 32 + (lane & 1) * 16;
            img_stride[j] = (int64_t)a.Cb * a.HWin * 32;
        } else {
            src[j] = (const char *)a.dO + (int64_t)(kb0 + ch - SB) * a.HW * 32 + (lane & 1) * 16;
            img_stride[j] = (int64_t)a.Kb * a.HW * 32;
        }
    }
    bf16x8v stage[PS][WT];
    auto load_step = [&](int s) {
        const int n = s / a.steps_per_img;
#pragma unroll
        for (int ps = 0; ps < PS; ++ps) {
            const int pix = ((s - n * a.steps_per_img) * PS + ps) * 32 + row;
            const bool ok = pix < a.HW;
            // a strided layer reads input pixel (stride * p, stride * q) for output pixel (p, q)
            int ipix = pix;
            if (a.stride != 1) {
                const int p = pix / a.Q;
                ipix = (p * a.Win + (pix - p * a.Q)) * a.stride;
            }
#pragma unroll
            for (int j = 0; j < WT; ++j) {
                bf16x8v v = {};
                if (ok) v = *(const bf16x8v *)(src[j] + n * img_stride[j] + (int64_t)(WT * wave + j < SB ? ipix : pix) * 32);
                stage[ps][j] = v;
            }
        }
    };
    auto store_step = [&](int buf) {
#pragma unroll
        for (int ps = 0; ps < PS; ++ps)
#pragma unroll
            for (int j = 0; j < WT; ++j) *(bf16x8v *)(&slab[buf][WT * wave + j][ps][lane * 16]) = stage[ps][j];
    };

    // transposing reads: pixels 8 kg + li/4 (and + 4), channel quad li % 4 of a slab
    const int tr_off = (8 * kg + (li >> 2)) * 32 + (li & 3) * 8;
    auto frag = [&](int buf, int chunk, int ps) {
        const s4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4p)(&slab[buf][chunk][ps][tr_off]));
        const s4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4p)(&slab[buf][chunk][ps][tr_off + 128]));
        return __builtin_bit_cast(bf16x8v, s8v{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]});
    };

    float4v acc[WT][WT];
#pragma unroll
    for (int i = 0; i < WT; ++i)
#pragma unroll
        for (int j = 0; j < WT; ++j) acc[i][j] = float4v{0.f, 0.f, 0.f, 0.f};

    if (s_begin < s_end) {
        load_step(s_begin);
        store_step(0);
    }
    __syncthreads();
    for (int s = s_begin; s < s_end; ++s) {
        const int buf = (s - s_begin) & 1;
        if (s + 1 < s_end) load_step(s + 1);
#pragma unroll
        for (int ps = 0; ps < PS; ++ps) {
            bf16x8v fa[WT], fb[WT];
#pragma unroll
            for (int i = 0; i < WT; ++i) {
                fa[i] = frag(buf, WT * wy + i, ps);
                fb[i] = frag(buf, SB + WT * wx + i, ps);
            }
#pragma unroll
            for (int i = 0; i < WT; ++i)
#pragma unroll
                for (int j = 0; j < WT; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (s + 1 < s_end) store_step(buf ^ 1);
        __syncthreads();
    }

    // register r of lane l of a tile is row c = 4*(l/16) + r, column k = l%16
    float *out = a.out + (int64_t)blockIdx.z * a.Kb * a.Cb * 256;
#pragma unroll
    for (int i = 0; i < WT; ++i)
#pragma unroll
        for (int j = 0; j < WT; ++j) {
            float *blk = out + ((int64_t)(kb0 + WT * wx + j) * a.Cb + (cb0 + WT * wy + i)) * 256;
#pragma unroll
            for (int r = 0; r < 4; ++r) blk[(4 * kg + r) * 16 + li] = acc[i][j][r];
        }
}

// 3x3 filters, stride 1, padding 1 (input and output images have the same size H x W).  For the 32 output
// pixels pix0 .. pix0+31 of a step (flattened p*W + q inside an image), tap (r, s) multiplies the input
// pixels at the flattened index + (r-1)*W + (s-1): a WINDOW of 32 + 2W + 2 consecutive input pixels per
// channel block is staged (pixels outside the image as zeros, which also covers the rows above and below
// the image), and a tap is a constant row offset r*W + s into it.  What the window cannot express is the
// left/right border: for s = 0 the outputs with q = 0, for s = 2 those with q = W-1 must not contribute, so
// the I operand of those taps is masked per lane (a lane's 8 pixels are 8 consecutive flattened indices).
// Wave tile 2 x 2 blocks x 9 taps = 36 accumulator tiles.
constexpr int CW3_WINMAX = 160;             // rows of a window: 32 + 2W + 2 with W <= 63

struct ConvWgt3Args {
    const bf16_t *I, *dO;
    float *out;
    int N, Cb, Kb, H, W;
    int steps_per_img, steps_total, steps_per_split;
};

__global__ __launch_bounds__(256) void conv_wgt3x3_bf16(ConvWgt3Args a)
{
    typedef short s4v __attribute__((ext_vector_type(4)));
    typedef short s8v __attribute__((ext_vector_type(8)));
    typedef unsigned u4v __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s4v *lds_s4p;
    __shared__ __attribute__((aligned(16))) char win[2][4][CW3_WINMAX * 32];   // [buffer][channel block][window row x 32 B]
    __shared__ __attribute__((aligned(16))) char slab[2][4][1024];             // [buffer][feature block][32 pixels x 32 B]
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int li = lane & 15, kg = lane >> 4;
    const int wy = wave >> 1, wx = wave & 1;
    const int cb0 = blockIdx.x * 4, kb0 = blockIdx.y * 4;
    const int s_begin = blockIdx.z * a.steps_per_split;
    const int s_end = min(a.steps_total, s_begin + a.steps_per_split);
    const int W = a.W, HW = a.H * a.W;
    const int WIN = 32 + 2 * W + 2;

    // staging of dO: thread t holds 16 bytes of feature block t / 64 (half t%2 of pixel row (t%64)/2)
    const char *dsrc = (const char *)a.dO + (int64_t)(kb0 + wave) * HW * 32 + (lane & 1) * 16;
    const int64_t dimg = (int64_t)a.Kb * HW * 32;
    // staging of the windows: 16-byte pieces e = t, t + 256, ... < 4 * 2 * WIN; piece e is half e%2 of window
    // row (e / 2) % WIN of channel block e / (2 WIN)
    constexpr int NP = (4 * 2 * CW3_WINMAX + 255) / 256;               // 5
    int p_row[NP], p_dst[NP];
    int64_t p_src[NP];
#pragma unroll
    for (int j = 0; j < NP; ++j) {
        const int e = t + 256 * j;
        const int cb = e / (2 * WIN), rem = e - cb * 2 * WIN;
        p_row[j] = cb < 4 ? rem >> 1 : -1000000;                        // (pieces past the last window: never valid)
        p_dst[j] = (cb < 4 ? cb : 0) * (CW3_WINMAX * 32) + (rem >> 1) * 32 + (rem & 1) * 16;
        p_src[j] = (int64_t)(cb0 + (cb < 4 ? cb : 0)) * HW * 32 + (rem & 1) * 16;
    }
    const int64_t iimg = (int64_t)a.Cb * HW * 32;
    bf16x8v dstage, wstage[NP];
    auto load_step = [&](int s) {
        const int n = s / a.steps_per_img;
        const int pix0 = (s - n * a.steps_per_img) * 32;
        {
            const int pix = pix0 + (lane >> 1);
            bf16x8v v = {};
            if (pix < HW) v = *(const bf16x8v *)(dsrc + n * dimg + (int64_t)pix * 32);
            dstage = v;
        }
#pragma unroll
        for (int j = 0; j < NP; ++j) {
            const int idx = pix0 - (W + 1) + p_row[j];                  // flattened input pixel of this window row
            bf16x8v v = {};
            if (idx >= 0 && idx < HW) v = *(const bf16x8v *)((const char *)a.I + n * iimg + p_src[j] + (int64_t)idx * 32);
            wstage[j] = v;
        }
    };
    auto store_step = [&](int buf) {
        *(bf16x8v *)(&slab[buf][wave][lane * 16]) = dstage;
#pragma unroll
        for (int j = 0; j < NP; ++j)
            if (p_row[j] >= 0) *(bf16x8v *)(&win[buf][0][0] + p_dst[j]) = wstage[j];
    };

    // transposing reads: pixels 8 kg + li/4 (and + 4), channel quad li % 4
    const int tr_off = (8 * kg + (li >> 2)) * 32 + (li & 3) * 8;
    auto frag = [&](const char *base) {
        const s4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4p)(base + tr_off));
        const s4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4p)(base + tr_off + 128));
        return __builtin_bit_cast(u4v, s8v{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]});
    };

    float4v acc[9][2][2];
#pragma unroll
    for (int tp = 0; tp < 9; ++tp)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[tp][i][j] = float4v{0.f, 0.f, 0.f, 0.f};

    if (s_begin < s_end) {
        load_step(s_begin);
        store_step(0);
    }
    __syncthreads();
    for (int s = s_begin; s < s_end; ++s) {
        const int buf = (s - s_begin) & 1;
        if (s + 1 < s_end) load_step(s + 1);
        // column masks of this lane's 8 pixels: element j sits in bits 16*(j%2) .. of word j/2
        u4v m_left = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu}, m_right = m_left;
        {
            const int n = s / a.steps_per_img;
            const int p0 = (s - n * a.steps_per_img) * 32 + 8 * kg;
            int q = p0 % W;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const unsigned keep = (j & 1) ? 0x0000FFFFu : 0xFFFF0000u;
                if (q == 0) m_left[j >> 1] &= keep;
                if (q == W - 1) m_right[j >> 1] &= keep;
                q = q + 1 == W ? 0 : q + 1;
            }
        }
        bf16x8v fb[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) fb[j] = __builtin_bit_cast(bf16x8v, frag(&slab[buf][2 * wx + j][0]));
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int sx = 0; sx < 3; ++sx) {
                const int toff = (r * W + sx) * 32;
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    u4v fa = frag(&win[buf][2 * wy + i][0] + toff);
                    if (sx == 0) fa &= m_left;
                    if (sx == 2) fa &= m_right;
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[3 * r + sx][i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8v, fa), fb[j],
                                                                                         acc[3 * r + sx][i][j], 0, 0, 0);
                }
            }
        if (s + 1 < s_end) store_step(buf ^ 1);
        __syncthreads();
    }

    // register r of lane l of a tile is row c = 4*(l/16) + r, column k = l%16; blocks are [kb][cb][tap][c][k]
    float *out = a.out + (int64_t)blockIdx.z * a.Kb * a.Cb * 9 * 256;
#pragma unroll
    for (int tp = 0; tp < 9; ++tp)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                float *blk = out + (((int64_t)(kb0 + 2 * wx + j) * a.Cb + (cb0 + 2 * wy + i)) * 9 + tp) * 256;
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) blk[(4 * kg + rr) * 16 + li] = acc[tp][i][j][rr];
            }
}

// 3x3 filters, stride 2, padding 1: output pixel (p, q) and tap (r, s) meet input pixel (2p + r - 1, 2q + s - 1).
// The input is staged as four PHASE PLANES per channel block, plane (a, b)[y][x] = I[2y + a][2x + b], each
// as wide as the output image; in plane coordinates a tap is again a constant shift: rows r = 0 and 2 read
// plane a = 1 at y = p - 1 and p, row r = 1 plane a = 0 at y = p, and likewise for the columns.  Per plane a
// window of 32 + Q + 1 flattened plane pixels covers the shifts 0, -1, -Q and -Q-1; the taps with a column
// shift of -1 (s = 0) are masked where q = 0; plane pixels outside the image are staged as zeros.
// A workgroup owns 2 channel blocks x 4 feature blocks (wave: 1 x 2 blocks x 9 taps).
constexpr int CW2_WINMAX = 64;              // rows of a plane window: 32 + Q + 1 with Q <= 31

struct ConvWgt2Args {
    const bf16_t *I, *dO;
    float *out;
    int N, Cb, Kb, H, W, P, Q;
    float inv_Q;
    int steps_per_img, steps_total, steps_per_split;
};

__global__ __launch_bounds__(256) void conv_wgt3x3s2_bf16(ConvWgt2Args a)
{
    typedef short s4v __attribute__((ext_vector_type(4)));
    typedef short s8v __attribute__((ext_vector_type(8)));
    typedef unsigned u4v __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s4v *lds_s4p;
    __shared__ __attribute__((aligned(16))) char win[2][2][4][CW2_WINMAX * 32];   // [buffer][channel block][plane 2a+b][row x 32 B]
    __shared__ __attribute__((aligned(16))) char slab[2][4][1024];                // [buffer][feature block][32 pixels x 32 B]
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int li = lane & 15, kg = lane >> 4;
    const int wy = wave >> 1, wx = wave & 1;
    const int cb0 = blockIdx.x * 2, kb0 = blockIdx.y * 4;
    const int s_begin = blockIdx.z * a.steps_per_split;
    const int s_end = min(a.steps_total, s_begin + a.steps_per_split);
    const int H = a.H, W = a.W, Q = a.Q, PQ = a.P * a.Q, HWin = a.H * a.W;
    const int WINS = 32 + Q + 1;

    const char *dsrc = (const char *)a.dO + (int64_t)(kb0 + wave) * PQ * 32 + (lane & 1) * 16;
    const int64_t dimg = (int64_t)a.Kb * PQ * 32;
    // window pieces e = t, t + 256, ... < 2 * 4 * 2 * WINS: half e%2 of row (e/2) % WINS of plane (e / (2 WINS)) % 4 of
    // channel block e / (8 WINS)
    constexpr int NP = (2 * 4 * 2 * CW2_WINMAX + 255) / 256;           // 4
    int p_row[NP], p_dst[NP], p_ab[NP];
    int64_t p_src[NP];
#pragma unroll
    for (int j = 0; j < NP; ++j) {
        const int e = t + 256 * j;
        const int pl = e / (2 * WINS), rem = e - pl * 2 * WINS;         // plane index over both channel blocks
        const bool used = pl < 8;
        p_row[j] = used ? rem >> 1 : -1;
        p_ab[j] = pl & 3;
        p_dst[j] = ((used ? pl : 0) * CW2_WINMAX + (rem >> 1)) * 32 + (rem & 1) * 16;
        p_src[j] = (int64_t)(cb0 + (used ? pl >> 2 : 0)) * HWin * 32 + (rem & 1) * 16;
    }
    const int64_t iimg = (int64_t)a.Cb * HWin * 32;
    bf16x8v dstage, wstage[NP];
    auto load_step = [&](int s) {
        const int n = s / a.steps_per_img;
        const int pix0 = (s - n * a.steps_per_img) * 32;
        {
            const int pix = pix0 + (lane >> 1);
            bf16x8v v = {};
            if (pix < PQ) v = *(const bf16x8v *)(dsrc + n * dimg + (int64_t)pix * 32);
            dstage = v;
        }
#pragma unroll
        for (int j = 0; j < NP; ++j) {
            const int jp = pix0 - (Q + 1) + p_row[j];                   // flattened plane pixel of this window row
            bf16x8v v = {};
            if (p_row[j] >= 0 && jp >= 0) {
                const int y = (int)(((float)jp + 0.5f) * a.inv_Q), x = jp - y * Q;
                const int iy = 2 * y + (p_ab[j] >> 1), ix = 2 * x + (p_ab[j] & 1);
                if (iy < H && ix < W) v = *(const bf16x8v *)((const char *)a.I + n * iimg + p_src[j] + (int64_t)(iy * W + ix) * 32);
            }
            wstage[j] = v;
        }
    };
    auto store_step = [&](int buf) {
        *(bf16x8v *)(&slab[buf][wave][lane * 16]) = dstage;
#pragma unroll
        for (int j = 0; j < NP; ++j)
            if (p_row[j] >= 0) *(bf16x8v *)(&win[buf][0][0][0] + p_dst[j]) = wstage[j];
    };

    const int tr_off = (8 * kg + (li >> 2)) * 32 + (li & 3) * 8;
    auto frag = [&](const char *base) {
        const s4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4p)(base + tr_off));
        const s4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4p)(base + tr_off + 128));
        return __builtin_bit_cast(u4v, s8v{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]});
    };

    float4v acc[9][2];
#pragma unroll
    for (int tp = 0; tp < 9; ++tp)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[tp][j] = float4v{0.f, 0.f, 0.f, 0.f};

    if (s_begin < s_end) {
        load_step(s_begin);
        store_step(0);
    }
    __syncthreads();
    for (int s = s_begin; s < s_end; ++s) {
        const int buf = (s - s_begin) & 1;
        if (s + 1 < s_end) load_step(s + 1);
        // left-border mask of this lane's 8 output pixels: element j sits in bits 16*(j%2) .. of word j/2
        u4v m_left = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu};
        {
            const int n = s / a.steps_per_img;
            const int p0 = (s - n * a.steps_per_img) * 32 + 8 * kg;
            int q = p0 % Q;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (q == 0) m_left[j >> 1] &= (j & 1) ? 0x0000FFFFu : 0xFFFF0000u;
                q = q + 1 == Q ? 0 : q + 1;
            }
        }
        bf16x8v fb[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) fb[j] = __builtin_bit_cast(bf16x8v, frag(&slab[buf][2 * wx + j][0]));
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int sx = 0; sx < 3; ++sx) {
                const int pa = r == 1 ? 0 : 1, pb = sx == 1 ? 0 : 1;              // phase plane
                const int toff = ((r == 0 ? 0 : Q) + (sx == 0 ? 0 : 1)) * 32;    // window row of shift (dy, dx)
                u4v fa = frag(&win[buf][wy][2 * pa + pb][0] + toff);
                if (sx == 0) fa &= m_left;
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[3 * r + sx][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8v, fa), fb[j],
                                                                                  acc[3 * r + sx][j], 0, 0, 0);
            }
        if (s + 1 < s_end) store_step(buf ^ 1);
        __syncthreads();
    }

    float *out = a.out + (int64_t)blockIdx.z * a.Kb * a.Cb * 9 * 256;
#pragma unroll
    for (int tp = 0; tp < 9; ++tp)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            float *blk = out + (((int64_t)(kb0 + 2 * wx + j) * a.Cb + (cb0 + wy)) * 9 + tp) * 256;
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) blk[(4 * kg + rr) * 16 + li] = acc[tp][j][rr];
        }
}

// The 7x7 stride-2 padding-3 stem with ONE channel block of 4 (8 bytes per pixel).  The M side of the GEMM is
// (tap, channel): 49 taps x 4 channels = 196 rows = 13 MFMA tiles; a tile row i is tap 4 mt + i/4, channel i%4.
// With 4-channel pixels a "channel quad" of the transposing read IS a whole pixel, so lane t of a 16-lane
// group points at output pixel t/4 SHIFTED BY TAP t%4 of the tile: one read transposes 4 pixels x 4 taps.
// The input rows a step needs (2p-3 .. 2p+5 for the at most two output rows p, p+1 of its 32 pixels) are
// staged with 4 zero pixels left and right of every row and zero rows outside the image, so a tap is the
// constant offset ((r-3) * pitch + (s-3)) pixels from the lane's pixel and no border masks are needed.
// Wave w owns feature block kb0 + w: 13 accumulator tiles.
constexpr int CWS_PITCH = 232;              // pixels per staged row: 4 + 224 + 4
constexpr int CWS_ROWS = 9;

struct ConvWgtStemArgs {
    const bf16_t *I, *dO;
    float *out;
    int N, Kb, H, W, P, Q;
    float inv_Q;
    int steps_per_img, steps_total, steps_per_split;
};

__global__ __launch_bounds__(256) void conv_wgt_stem_bf16(ConvWgtStemArgs a)
{
    typedef short s4v __attribute__((ext_vector_type(4)));
    typedef short s8v __attribute__((ext_vector_type(8)));
    typedef __attribute__((address_space(3))) s4v *lds_s4p;
    __shared__ __attribute__((aligned(16))) char win[2][CWS_ROWS * CWS_PITCH * 8];   // [buffer][row][pixel x 8 B]
    __shared__ __attribute__((aligned(16))) char slab[2][4][1024];                   // [buffer][feature block][32 pixels x 32 B]
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int li = lane & 15, kg = lane >> 4;
    const int kb0 = blockIdx.y * 4;
    const int s_begin = blockIdx.z * a.steps_per_split;
    const int s_end = min(a.steps_total, s_begin + a.steps_per_split);
    const int H = a.H, W = a.W, Q = a.Q, PQ = a.P * a.Q;

    // the pad pixels are zero for the whole kernel (the staging below never writes them)
    for (int o = t * 16; o < 2 * CWS_ROWS * CWS_PITCH * 8; o += 256 * 16) *(float4v *)(&win[0][0] + o) = float4v{0.f, 0.f, 0.f, 0.f};

    const char *dsrc = (const char *)a.dO + (int64_t)(kb0 + wave) * PQ * 32 + (lane & 1) * 16;
    const int64_t dimg = (int64_t)a.Kb * PQ * 32;
    const int64_t iimg = (int64_t)H * W * 8;
    // window pieces: 16 bytes = 2 pixels; piece e = t, t + 256, ... covers row e / (W/2), pixels 2 (e % (W/2)) ..
    const int ppr = W >> 1;                                            // pieces per input row
    constexpr int NP = (CWS_ROWS * 112 + 255) / 256;                    // 4
    int p_rl[NP], p_px[NP];
#pragma unroll
    for (int j = 0; j < NP; ++j) {
        const int e = t + 256 * j;
        const int rl = e / ppr;
        p_rl[j] = rl < CWS_ROWS ? rl : -1;
        p_px[j] = 2 * (e - rl * ppr);
    }
    bf16x8v dstage, wstage[NP];
    auto load_step = [&](int s) {
        const int n = s / a.steps_per_img;
        const int pix0 = (s - n * a.steps_per_img) * 32;
        {
            const int pix = pix0 + (lane >> 1);
            bf16x8v v = {};
            if (pix < PQ) v = *(const bf16x8v *)(dsrc + n * dimg + (int64_t)pix * 32);
            dstage = v;
        }
        const int p_first = (int)(((float)pix0 + 0.5f) * a.inv_Q);
#pragma unroll
        for (int j = 0; j < NP; ++j) {
            const int iy = 2 * p_first - 3 + p_rl[j];
            bf16x8v v = {};
            if (p_rl[j] >= 0 && iy >= 0 && iy < H) v = *(const bf16x8v *)((const char *)a.I + n * iimg + ((int64_t)iy * W + p_px[j]) * 8);
            wstage[j] = v;
        }
    };
    auto store_step = [&](int buf) {
        *(bf16x8v *)(&slab[buf][wave][lane * 16]) = dstage;
#pragma unroll
        for (int j = 0; j < NP; ++j)
            if (p_rl[j] >= 0) *(bf16x8v *)(&win[buf][(p_rl[j] * CWS_PITCH + 4 + p_px[j]) * 8]) = wstage[j];
    };

    // tap offsets of this lane: in M tile mt it feeds tap 4 mt + li % 4 (tile 12: only tap 48 exists, the
    // other three rows repeat it and are not stored)
    int tapoff[13];
#pragma unroll
    for (int mt = 0; mt < 13; ++mt) {
        int tap = 4 * mt + (li & 3);
        if (tap > 48) tap = 48;
        const int r = tap / 7, sx = tap - 7 * r;
        tapoff[mt] = ((r - 3) * CWS_PITCH + (sx - 3)) * 8;
    }
    const int tr_off = (8 * kg + (li >> 2)) * 32 + (li & 3) * 8;        // dO operand, as in the other kernels

    float4v acc[13];
#pragma unroll
    for (int mt = 0; mt < 13; ++mt) acc[mt] = float4v{0.f, 0.f, 0.f, 0.f};

    __syncthreads();                                                   // zero fill done
    if (s_begin < s_end) {
        load_step(s_begin);
        store_step(0);
    }
    __syncthreads();
    for (int s = s_begin; s < s_end; ++s) {
        const int buf = (s - s_begin) & 1;
        if (s + 1 < s_end) load_step(s + 1);
        // window addresses of this lane's two pixel rows (output pixels 8 kg + li/4 and + 4 of the step)
        int base[2];
        {
            const int n = s / a.steps_per_img;
            const int pix0 = (s - n * a.steps_per_img) * 32;
            const int p_first = (int)(((float)pix0 + 0.5f) * a.inv_Q);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                int pix = pix0 + 8 * kg + (li >> 2) + 4 * h;
                if (pix >= PQ) pix = PQ - 1;                             // (its dO row is zero)
                const int p = (int)(((float)pix + 0.5f) * a.inv_Q), q = pix - p * Q;
                base[h] = ((2 * (p - p_first) + 3) * CWS_PITCH + 4 + 2 * q) * 8;
            }
        }
        bf16x8v fb;
        {
            const s4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4p)(&slab[buf][wave][tr_off]));
            const s4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4p)(&slab[buf][wave][tr_off + 128]));
            fb = __builtin_bit_cast(bf16x8v, s8v{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]});
        }
#pragma unroll
        for (int mt = 0; mt < 13; ++mt) {
            const s4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4p)(&win[buf][base[0] + tapoff[mt]]));
            const s4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4p)(&win[buf][base[1] + tapoff[mt]]));
            const bf16x8v fa = __builtin_bit_cast(bf16x8v, s8v{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]});
            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, acc[mt], 0, 0, 0);
        }
        if (s + 1 < s_end) store_step(buf ^ 1);
        __syncthreads();
    }

    // register rr of lane l of tile mt is row 4*(l/16) + rr = (tap 4 mt + l/16, channel rr), column k = l%16;
    // blocks are [kb][tap][4 c][16 k]
    float *out = a.out + (int64_t)blockIdx.z * a.Kb * 49 * 64;
    const int kb = kb0 + wave;
#pragma unroll
    for (int mt = 0; mt < 13; ++mt) {
        const int tap = 4 * mt + kg;
        if (tap < 49) {
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) out[(((int64_t)kb * 49 + tap) * 4 + rr) * 16 + li] = acc[mt][rr];
        }
    }
}

// ---- fp32 forms.  With fp32 tensors the operand of the 16x16x4 matrix instruction is ONE element per lane
// (row m = lane % 16, reduction index lane / 16), and the 16 channels of a pixel are 16 consecutive floats: a
// lane reads I[pixel 4 j + lane/16][channel lane%16] straight from the staged slab, no transposition.
// 1x1 (stride 1 or 2): a workgroup owns 4 channel blocks x 4 feature blocks, wave tile 2 x 2.
__global__ __launch_bounds__(256) void conv_wgt1x1_f32(ConvWgtArgs a)
{
    __shared__ __attribute__((aligned(16))) float slab[2][8][32 * 16];    // [buffer][chunk: 4 of I, 4 of dO][32 pixels x 16]
    const float *gI = (const float *)a.I, *gO = (const float *)a.dO;
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int li = lane & 15, kg = lane >> 4;
    const int wy = wave >> 1, wx = wave & 1;
    const int cb0 = blockIdx.x * 4, kb0 = blockIdx.y * 4;
    const int s_begin = blockIdx.z * a.steps_per_split;
    const int s_end = min(a.steps_total, s_begin + a.steps_per_split);

    // staging: 16-byte piece e = t + 256 j: chunk e / 128, pixel row (e % 128) / 4, quarter e % 4
    float4v stage[4];
    auto load_step = [&](int s) {
        const int n = s / a.steps_per_img;
        const int pix0 = (s - n * a.steps_per_img) * 32;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int e = t + 256 * j, ch = e >> 7, pix = pix0 + ((e & 127) >> 2), qu = e & 3;
            float4v v = {0.f, 0.f, 0.f, 0.f};
            if (pix < a.HW) {
                if (ch < 4) {
                    int ipix = pix;
                    if (a.stride != 1) {
                        const int p = pix / a.Q;
                        ipix = (p * a.Win + (pix - p * a.Q)) * a.stride;
                    }
                    v = *(const float4v *)(gI + (((int64_t)n * a.Cb + cb0 + ch) * a.HWin + ipix) * 16 + qu * 4);
                } else {
                    v = *(const float4v *)(gO + (((int64_t)n * a.Kb + kb0 + ch - 4) * a.HW + pix) * 16 + qu * 4);
                }
            }
            stage[j] = v;
        }
    };
    auto store_step = [&](int buf) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int e = t + 256 * j;
            *(float4v *)(&slab[buf][e >> 7][(e & 127) * 4]) = stage[j];
        }
    };

    float4v acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = float4v{0.f, 0.f, 0.f, 0.f};

    if (s_begin < s_end) {
        load_step(s_begin);
        store_step(0);
    }
    __syncthreads();
    for (int s = s_begin; s < s_end; ++s) {
        const int buf = (s - s_begin) & 1;
        if (s + 1 < s_end) load_step(s + 1);
#pragma unroll
        for (int j4 = 0; j4 < 8; ++j4) {
            float fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                fa[i] = slab[buf][2 * wy + i][(4 * j4 + kg) * 16 + li];
                fb[i] = slab[buf][4 + 2 * wx + i][(4 * j4 + kg) * 16 + li];
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (s + 1 < s_end) store_step(buf ^ 1);
        __syncthreads();
    }

    float *out = a.out + (int64_t)blockIdx.z * a.Kb * a.Cb * 256;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            float *blk = out + ((int64_t)(kb0 + 2 * wx + j) * a.Cb + (cb0 + 2 * wy + i)) * 256;
#pragma unroll
            for (int r = 0; r < 4; ++r) blk[(4 * kg + r) * 16 + li] = acc[i][j][r];
        }
}

// 3x3, stride 1, padding 1 in fp32: windows as in the bf16 kernel (64 bytes per pixel); a workgroup owns 2 channel
// blocks x 4 feature blocks (wave: 1 x 2 blocks x 9 taps); the border columns are masked per lane and k step.
__global__ __launch_bounds__(256) void conv_wgt3x3_f32(ConvWgt3Args a)
{
    __shared__ __attribute__((aligned(16))) float win[2][2][CW3_WINMAX * 16];   // [buffer][channel block][window row x 16]
    __shared__ __attribute__((aligned(16))) float slab[2][4][32 * 16];          // [buffer][feature block][32 pixels x 16]
    const float *gI = (const float *)a.I, *gO = (const float *)a.dO;
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int li = lane & 15, kg = lane >> 4;
    const int wy = wave >> 1, wx = wave & 1;
    const int cb0 = blockIdx.x * 2, kb0 = blockIdx.y * 4;
    const int s_begin = blockIdx.z * a.steps_per_split;
    const int s_end = min(a.steps_total, s_begin + a.steps_per_split);
    const int W = a.W, HW = a.H * a.W;
    const int WIN = 32 + 2 * W + 2;

    // window pieces e = t + 256 j < 2 * WIN * 4: channel block e / (4 WIN), window row (e / 4) % WIN, quarter e % 4
    constexpr int NP = (2 * CW3_WINMAX * 4 + 255) / 256;               // 5
    int p_row[NP], p_cb[NP];
#pragma unroll
    for (int j = 0; j < NP; ++j) {
        const int e = t + 256 * j;
        const int cb = e / (4 * WIN);
        p_cb[j] = cb;
        p_row[j] = cb < 2 ? (e - cb * 4 * WIN) >> 2 : -1000000;
    }
    float4v dstage[2], wstage[NP];
    auto load_step = [&](int s) {
        const int n = s / a.steps_per_img;
        const int pix0 = (s - n * a.steps_per_img) * 32;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int e = t + 256 * j, kb = e >> 7, pix = pix0 + ((e & 127) >> 2);
            float4v v = {0.f, 0.f, 0.f, 0.f};
            if (pix < HW) v = *(const float4v *)(gO + (((int64_t)n * a.Kb + kb0 + kb) * HW + pix) * 16 + (e & 3) * 4);
            dstage[j] = v;
        }
#pragma unroll
        for (int j = 0; j < NP; ++j) {
            const int idx = pix0 - (W + 1) + p_row[j];
            float4v v = {0.f, 0.f, 0.f, 0.f};
            if (idx >= 0 && idx < HW) v = *(const float4v *)(gI + (((int64_t)n * a.Cb + cb0 + p_cb[j]) * HW + idx) * 16 + (t & 3) * 4);
            wstage[j] = v;
        }
    };
    auto store_step = [&](int buf) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int e = t + 256 * j;
            *(float4v *)(&slab[buf][e >> 7][(e & 127) * 4]) = dstage[j];
        }
#pragma unroll
        for (int j = 0; j < NP; ++j)
            if (p_row[j] >= 0) *(float4v *)(&win[buf][p_cb[j]][p_row[j] * 16 + (t & 3) * 4]) = wstage[j];
    };

    float4v acc[9][2];
#pragma unroll
    for (int tp = 0; tp < 9; ++tp)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[tp][j] = float4v{0.f, 0.f, 0.f, 0.f};

    if (s_begin < s_end) {
        load_step(s_begin);
        store_step(0);
    }
    __syncthreads();
    for (int s = s_begin; s < s_end; ++s) {
        const int buf = (s - s_begin) & 1;
        if (s + 1 < s_end) load_step(s + 1);
        const int n = s / a.steps_per_img;
        int q = ((s - n * a.steps_per_img) * 32 + kg) % W;           // column of this lane's pixel in k step 0
#pragma unroll
        for (int j4 = 0; j4 < 8; ++j4) {
            const int prow = 4 * j4 + kg;
            float fb[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) fb[j] = slab[buf][2 * wx + j][prow * 16 + li];
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
                for (int sx = 0; sx < 3; ++sx) {
                    float fa = win[buf][wy][(prow + r * W + sx) * 16 + li];
                    if (sx == 0 && q == 0) fa = 0.f;
                    if (sx == 2 && q == W - 1) fa = 0.f;
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[3 * r + sx][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(fa, fb[j], acc[3 * r + sx][j], 0, 0, 0);
                }
            q += 4;
            if (q >= W) q -= W;
            if (q >= W) q -= W;
        }
        if (s + 1 < s_end) store_step(buf ^ 1);
        __syncthreads();
    }

    float *out = a.out + (int64_t)blockIdx.z * a.Kb * a.Cb * 9 * 256;
#pragma unroll
    for (int tp = 0; tp < 9; ++tp)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            float *blk = out + (((int64_t)(kb0 + 2 * wx + j) * a.Cb + (cb0 + wy)) * 9 + tp) * 256;
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) blk[(4 * kg + rr) * 16 + li] = acc[tp][j][rr];
        }
}

// 3x3, stride 2, padding 1 in fp32: the four phase planes of conv_wgt3x3s2_bf16 (64 bytes per pixel), windows of
// 32 + Q + 1 plane pixels, no transposition (the operand of 16x16x4 is one element per lane).  A workgroup owns one
// channel block x 4 feature blocks (wave: one feature block x 9 taps); the taps with a column shift of -1 are masked
// where q = 0.
__global__ __launch_bounds__(256) void conv_wgt3x3s2_f32(ConvWgt2Args a)
{
    __shared__ __attribute__((aligned(16))) float win[2][4][CW2_WINMAX * 16];   // [buffer][plane 2a+b][window row x 16]
    __shared__ __attribute__((aligned(16))) float slab[2][4][32 * 16];          // [buffer][feature block][32 pixels x 16]
    const float *gI = (const float *)a.I, *gO = (const float *)a.dO;
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int li = lane & 15, kg = lane >> 4;
    const int cb0 = blockIdx.x, kb0 = blockIdx.y * 4;
    const int s_begin = blockIdx.z * a.steps_per_split;
    const int s_end = min(a.steps_total, s_begin + a.steps_per_split);
    const int H = a.H, W = a.W, Q = a.Q, PQ = a.P * a.Q, HWin = a.H * a.W;
    const int WINS = 32 + Q + 1;

    // window pieces e = t + 256 j < 4 * WINS * 4: plane e / (4 WINS), window row (e / 4) % WINS, quarter e % 4
    constexpr int NP = (4 * CW2_WINMAX * 4 + 255) / 256;                // 4
    int p_row[NP], p_ab[NP];
#pragma unroll
    for (int j = 0; j < NP; ++j) {
        const int e = t + 256 * j;
        const int pl = e / (4 * WINS);
        p_ab[j] = pl & 3;
        p_row[j] = pl < 4 ? (e - pl * 4 * WINS) >> 2 : -1;
    }
    float4v dstage[2], wstage[NP];
    auto load_step = [&](int s) {
        const int n = s / a.steps_per_img;
        const int pix0 = (s - n * a.steps_per_img) * 32;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int e = t + 256 * j, kb = e >> 7, pix = pix0 + ((e & 127) >> 2);
            float4v v = {0.f, 0.f, 0.f, 0.f};
            if (pix < PQ) v = *(const float4v *)(gO + (((int64_t)n * a.Kb + kb0 + kb) * PQ + pix) * 16 + (e & 3) * 4);
            dstage[j] = v;
        }
#pragma unroll
        for (int j = 0; j < NP; ++j) {
            const int jp = pix0 - (Q + 1) + p_row[j];                   // flattened plane pixel of this window row
            float4v v = {0.f, 0.f, 0.f, 0.f};
            if (p_row[j] >= 0 && jp >= 0) {
                const int y = (int)(((float)jp + 0.5f) * a.inv_Q), x = jp - y * Q;
                const int iy = 2 * y + (p_ab[j] >> 1), ix = 2 * x + (p_ab[j] & 1);
                if (iy < H && ix < W) v = *(const float4v *)(gI + (((int64_t)n * a.Cb + cb0) * HWin + iy * W + ix) * 16 + (t & 3) * 4);
            }
            wstage[j] = v;
        }
    };
    auto store_step = [&](int buf) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int e = t + 256 * j;
            *(float4v *)(&slab[buf][e >> 7][(e & 127) * 4]) = dstage[j];
        }
#pragma unroll
        for (int j = 0; j < NP; ++j)
            if (p_row[j] >= 0) *(float4v *)(&win[buf][p_ab[j]][p_row[j] * 16 + (t & 3) * 4]) = wstage[j];
    };

    float4v acc[9];
#pragma unroll
    for (int tp = 0; tp < 9; ++tp) acc[tp] = float4v{0.f, 0.f, 0.f, 0.f};

    if (s_begin < s_end) {
        load_step(s_begin);
        store_step(0);
    }
    __syncthreads();
    for (int s = s_begin; s < s_end; ++s) {
        const int buf = (s - s_begin) & 1;
        if (s + 1 < s_end) load_step(s + 1);
        const int n = s / a.steps_per_img;
        int q = ((s - n * a.steps_per_img) * 32 + kg) % Q;             // column of this lane's output pixel in k step 0
#pragma unroll
        for (int j4 = 0; j4 < 8; ++j4) {
            const int prow = 4 * j4 + kg;
            const float fb = slab[buf][wave][prow * 16 + li];
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
                for (int sx = 0; sx < 3; ++sx) {
                    const int pa = r == 1 ? 0 : 1, pb = sx == 1 ? 0 : 1;             // phase plane
                    const int toff = (r == 0 ? 0 : Q) + (sx == 0 ? 0 : 1);          // window row of shift (dy, dx)
                    float fa = win[buf][2 * pa + pb][(prow + toff) * 16 + li];
                    if (sx == 0 && q == 0) fa = 0.f;
                    acc[3 * r + sx] = __builtin_amdgcn_mfma_f32_16x16x4f32(fa, fb, acc[3 * r + sx], 0, 0, 0);
                }
            q += 4;
            while (q >= Q) q -= Q;
        }
        if (s + 1 < s_end) store_step(buf ^ 1);
        __syncthreads();
    }

    float *out = a.out + (int64_t)blockIdx.z * a.Kb * a.Cb * 9 * 256;
#pragma unroll
    for (int tp = 0; tp < 9; ++tp) {
        float *blk = out + (((int64_t)(kb0 + wave) * a.Cb + cb0) * 9 + tp) * 256;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) blk[(4 * kg + rr) * 16 + li] = acc[tp][rr];
    }
}

// dWt = sum of the partial sums of the ranges.  A workgroup owns 64 consecutive float4 of dWt (n4 is a
// multiple of 64); wave w adds the ranges w, w + 4, ... in order with fully coalesced loads, then the four
// partial sums are added in a fixed order through LDS, so the result does not depend on timing.
__global__ __launch_bounds__(256) void conv_wgt_reduce(const float4v *part, float4v *dWt, int64_t n4, int nsplit)
{
    __shared__ float4v xs[4][64];
    const int il = threadIdx.x & 63, kq = threadIdx.x >> 6;
    const int64_t i = (int64_t)blockIdx.x * 64 + il;
    float4v s0 = {0.f, 0.f, 0.f, 0.f}, s1 = s0;
    int k = kq;
    for (; k + 4 < nsplit; k += 8) {
        s0 += part[i + k * n4];
        s1 += part[i + (k + 4) * n4];
    }
    if (k < nsplit) s0 += part[i + k * n4];
    xs[kq][il] = s0 + s1;
    __syncthreads();
    if (kq == 0) dWt[i] = (xs[0][il] + xs[1][il]) + (xs[2][il] + xs[3][il]);
}

struct ConvWgtPlan {
    bool ok, s2, stem, f32;
    int ps;                   // 32-pixel slabs per step (1x1 kernel)
    int taps, WT, nsplit, steps_per_img, steps_total, steps_per_split;
    int64_t ws_bytes;
};

// 16-wide blocks, block counts that the super-blocks divide, output images of at least 32 pixels;
// 1x1 without padding (stride 1 or 2), or 3x3 with padding 1: stride 1 on images at most 63 pixels wide,
// stride 2 on output images at most 31 pixels wide
static ConvWgtPlan conv_wgt_plan(int64_t N, int64_t C, int64_t H, int64_t W, int64_t K, int64_t R, int64_t S, int64_t sh,
                                 int64_t sw, int64_t ph, int64_t pw, int64_t bc, int64_t bk, bool f32 = false)
{
    ConvWgtPlan p = {};
    p.f32 = f32;
    if (f32 && bc != 16) return p;
    const bool is1 = R == 1 && S == 1 && ph == 0 && pw == 0 && sh == sw && (sh == 1 || sh == 2);
    const bool is3 = R == 3 && S == 3 && ph == 1 && pw == 1 && W >= 3 && W <= 63 && sh == 1 && sw == 1;
    const bool is3s2 = R == 3 && S == 3 && ph == 1 && pw == 1 && sh == 2 && sw == 2 && W >= 3 && (W - 1) / 2 + 1 <= 31;
    if (R == 7 && S == 7 && sh == 2 && sw == 2 && ph == 3 && pw == 3 && bc == 4 && C == 4 && bk == 16) {
        // the stem on one channel block of 4: even widths up to 224, output rows of at least 32 pixels
        const int64_t P = (H - 1) / 2 + 1, Q = (W - 1) / 2 + 1, Kb = K / 16;
        if (W % 2 || W > 224 || Q < 32 || Kb % 4 || N * H * W >= (1ll << 30) || knobs().conv_wgt_general.set) return p;
        p.taps = 49; p.stem = true; p.WT = 2;
        p.steps_per_img = (int)((P * Q + 31) / 32);
        p.steps_total = (int)(N * p.steps_per_img);
        int64_t ns = 512 / (Kb / 4);
        if (ns > p.steps_total / 8) ns = p.steps_total / 8;
        if (ns < 1) ns = 1;
        p.steps_per_split = (int)((p.steps_total + ns - 1) / ns);
        p.nsplit = (p.steps_total + p.steps_per_split - 1) / p.steps_per_split;
        p.ws_bytes = p.nsplit > 1 ? (int64_t)p.nsplit * Kb * 49 * 256 : 0;
        p.ok = true;
        return p;
    }
    if (!(is1 || is3 || is3s2) || bc != 16 || bk != 16) return p;
    const int64_t P = (H - 1) / sh + 1, Q = (W - 1) / sw + 1;     // output size of the layers handled here
    const int64_t Cb = C / 16, Kb = K / 16, HW = P * Q;
    if (N * H * W >= (1ll << 30)) return p;
    if (Cb % 4 || Kb % 4 || HW < 32 || N * HW >= (1ll << 30) || knobs().conv_wgt_general.set) return p;
    p.taps = is1 ? 1 : 9;
    p.s2 = is3s2;
    p.WT = (!f32 && is1 && Cb % 8 == 0 && Kb % 8 == 0 && (Cb / 8) * (Kb / 8) >= 16) ? 4 : 2;
    const int64_t nb = (f32 && is3s2) ? Cb * (Kb / 4) : (is3s2 || (f32 && is3)) ? (Cb / 2) * (Kb / 4) : (Cb / (2 * p.WT)) * (Kb / (2 * p.WT));
    p.ps = 1;
    if (is1 && !f32) {
        p.ps = 2;
        if (knobs().conv_wgt_ps.set) { const int x = knobs().conv_wgt_ps.val; if (x == 1 || x == 2) p.ps = x; }   // tuning knob
    }
    p.steps_per_img = (int)((HW + 32 * p.ps - 1) / (32 * p.ps));
    p.steps_total = (int)(N * p.steps_per_img);
    // workgroups in all: measured best at about 512 (two to three are resident per CU and each waits for its
    // staging loads every step); 1024 where the partial sums then still stay within 16 MB
    int64_t target = 512;
    if (is1 && nb >= 8 && Cb * Kb * 1024 * (1024 / nb) <= (16ll << 20)) target = 1024;
    if (knobs().conv_wgt_target.set) { const int x = knobs().conv_wgt_target.val; if (x > 0) target = x; }   // tuning knob
    int64_t ns = (target + nb - 1) / nb;
    if (ns > (int64_t)p.steps_total * p.ps / 8) ns = (int64_t)p.steps_total * p.ps / 8;   // at least 256 pixels per range
    if (ns < 1) ns = 1;
    p.steps_per_split = (int)((p.steps_total + ns - 1) / ns);
    p.nsplit = (p.steps_total + p.steps_per_split - 1) / p.steps_per_split;
    p.ws_bytes = p.nsplit > 1 ? (int64_t)p.nsplit * Kb * Cb * p.taps * 1024 : 0;
    p.ok = true;
    return p;
}

static int conv_wgt_bf16_launch(const ConvWgtPlan &p, int N, int Cb, int Kb, int H, int W, int stride, const void *I,
                                const void *dO, float *dWt, void *ws, hipStream_t s)
{
    const dim3 grid(Cb / (2 * p.WT), Kb / (2 * p.WT), p.nsplit);
    float *out = p.nsplit > 1 ? (float *)ws : dWt;
    if (p.stem) {
        ConvWgtStemArgs a = {};
        a.I = (const bf16_t *)I; a.dO = (const bf16_t *)dO; a.out = out;
        a.N = N; a.Kb = Kb; a.H = H; a.W = W; a.P = (H - 1) / 2 + 1; a.Q = (W - 1) / 2 + 1;
        a.inv_Q = 1.0f / (float)a.Q;
        a.steps_per_img = p.steps_per_img; a.steps_total = p.steps_total; a.steps_per_split = p.steps_per_split;
        hipLaunchKernelGGL(conv_wgt_stem_bf16, dim3(1, Kb / 4, p.nsplit), dim3(256), 0, s, a);
        int rc = check_launch("brg_conv_bwd_wgt (bf16 stem) launch");
        if (rc || p.nsplit == 1) return rc;
        const int64_t n4s = (int64_t)Kb * 49 * 16;
        hipLaunchKernelGGL(conv_wgt_reduce, dim3((unsigned)(n4s / 64)), dim3(256), 0, s, (const float4v *)ws, (float4v *)dWt, n4s,
                           p.nsplit);
        return check_launch("brg_conv_bwd_wgt (range sum) launch");
    }
    if (p.f32) {
        if (p.taps == 1) {
            ConvWgtArgs a = {};
            a.I = (const bf16_t *)I; a.dO = (const bf16_t *)dO; a.out = out;
            a.N = N; a.Cb = Cb; a.Kb = Kb; a.stride = stride;
            a.Q = (W - 1) / stride + 1; a.HW = ((H - 1) / stride + 1) * a.Q; a.HWin = H * W; a.Win = W;
            a.steps_per_img = p.steps_per_img; a.steps_total = p.steps_total; a.steps_per_split = p.steps_per_split;
            hipLaunchKernelGGL(conv_wgt1x1_f32, dim3(Cb / 4, Kb / 4, p.nsplit), dim3(256), 0, s, a);
        } else if (p.s2) {
            ConvWgt2Args a = {};
            a.I = (const bf16_t *)I; a.dO = (const bf16_t *)dO; a.out = out;
            a.N = N; a.Cb = Cb; a.Kb = Kb; a.H = H; a.W = W; a.P = (H - 1) / 2 + 1; a.Q = (W - 1) / 2 + 1;
            a.inv_Q = 1.0f / (float)a.Q;
            a.steps_per_img = p.steps_per_img; a.steps_total = p.steps_total; a.steps_per_split = p.steps_per_split;
            hipLaunchKernelGGL(conv_wgt3x3s2_f32, dim3(Cb, Kb / 4, p.nsplit), dim3(256), 0, s, a);
        } else {
            ConvWgt3Args a = {};
            a.I = (const bf16_t *)I; a.dO = (const bf16_t *)dO; a.out = out;
            a.N = N; a.Cb = Cb; a.Kb = Kb; a.H = H; a.W = W;
            a.steps_per_img = p.steps_per_img; a.steps_total = p.steps_total; a.steps_per_split = p.steps_per_split;
            hipLaunchKernelGGL(conv_wgt3x3_f32, dim3(Cb / 2, Kb / 4, p.nsplit), dim3(256), 0, s, a);
        }
    } else if (p.s2) {
        ConvWgt2Args a = {};
        a.I = (const bf16_t *)I; a.dO = (const bf16_t *)dO; a.out = out;
        a.N = N; a.Cb = Cb; a.Kb = Kb; a.H = H; a.W = W; a.P = (H - 1) / 2 + 1; a.Q = (W - 1) / 2 + 1;
        a.inv_Q = 1.0f / (float)a.Q;
        a.steps_per_img = p.steps_per_img; a.steps_total = p.steps_total; a.steps_per_split = p.steps_per_split;
        hipLaunchKernelGGL(conv_wgt3x3s2_bf16, dim3(Cb / 2, Kb / 4, p.nsplit), dim3(256), 0, s, a);
    } else if (p.taps == 1) {
        ConvWgtArgs a = {};
        a.I = (const bf16_t *)I; a.dO = (const bf16_t *)dO; a.out = out;
        a.N = N; a.Cb = Cb; a.Kb = Kb; a.stride = stride;
        a.Q = (W - 1) / stride + 1; a.HW = ((H - 1) / stride + 1) * a.Q; a.HWin = H * W; a.Win = W;
        a.steps_per_img = p.steps_per_img; a.steps_total = p.steps_total; a.steps_per_split = p.steps_per_split;
        if (p.WT == 4 && p.ps == 2) hipLaunchKernelGGL((conv_wgt1x1_bf16<4, 2>), grid, dim3(256), 0, s, a);
        else if (p.WT == 4) hipLaunchKernelGGL((conv_wgt1x1_bf16<4, 1>), grid, dim3(256), 0, s, a);
        else if (p.ps == 2) hipLaunchKernelGGL((conv_wgt1x1_bf16<2, 2>), grid, dim3(256), 0, s, a);
        else hipLaunchKernelGGL((conv_wgt1x1_bf16<2, 1>), grid, dim3(256), 0, s, a);
    } else {
        ConvWgt3Args a = {};
        a.I = (const bf16_t *)I; a.dO = (const bf16_t *)dO; a.out = out;
        a.N = N; a.Cb = Cb; a.Kb = Kb; a.H = H; a.W = W;
        a.steps_per_img = p.steps_per_img; a.steps_total = p.steps_total; a.steps_per_split = p.steps_per_split;
        hipLaunchKernelGGL(conv_wgt3x3_bf16, grid, dim3(256), 0, s, a);
    }
    int rc = check_launch("brg_conv_bwd_wgt (bf16) launch");
    if (rc || p.nsplit == 1) return rc;
    const int64_t n4 = (int64_t)Kb * Cb * p.taps * 64;
    hipLaunchKernelGGL(conv_wgt_reduce, dim3((unsigned)(n4 / 64)), dim3(256), 0, s, (const float4v *)ws, (float4v *)dWt, n4,
                       p.nsplit);
    return check_launch("brg_conv_bwd_wgt (range sum) launch");
}

}  // namespace brg
