// Convolutions in bf16 on FEW output pixels (paper section 3.2.2, the paragraph on parallelisation: with a small
// minibatch the work is divided over the feature blocks first; section 4.3, inference at N = 1).  At N = 1 a
// 14x14 or 7x7 layer has 13 or 4 groups of 16 pixels: tiling pixels x feature blocks gives a few dozen workgroups
// that each walk the whole (channel block, r, s) chain, a serial run of up to 288 dependent load-multiply steps on
// a chip with 256 CUs.  This kernel divides the chain as well:
//
//  * One chain unit = one pair of channel blocks at one tap = one v_mfma_f32_16x16x32_bf16 per (feature block,
//    pixel group).  Operands come straight from global memory as in the streaming 1x1 kernel: 16 bytes per lane
//    of the activations (lane = pixel, 8 channels of one block of the pair; the tap shifts the pixel, lanes whose
//    tap falls into the padding load a valid address and multiply zeros) and 16 bytes per lane of the weights.
//  * The four waves of a workgroup own the SAME KW feature blocks x PG pixel groups and take the units
//    w, w+4, w+8, ... of the workgroup's range; blockIdx.z selects one of `gz` ranges of the chain.  The four
//    partial tiles are summed through LDS.  With gz == 1 the result is finished in place (bias, activation,
//    bf16); otherwise it is written as fp32 to `part` and conv_small_reduce adds the gz partial results in a
//    fixed order, so the result does not depend on the schedule.
//  * WTR (forward pass): a weight block is stored with the feature index contiguous; each wave transposes the
//    pair it loaded through a private LDS slot with the transposing LDS read, as the streaming 1x1 kernel does.
#pragma once

#include "brg_conv1x1_bf16.hpp"

namespace brg {

struct ConvSmallArgs {
    const void *I, *Wt;
    void *O;
    float *part;                    // [gz][Kb][npix][16] fp32 when gz > 1
    const float *bias;
    int act;
    int N, Cb, Kb, P, Q;            // logical output pixels P x Q per image
    int Hin, Win, sub, H, W;        // physical input image; logical image H x W = every sub-th pixel of it
    int str, ph, pw, R, S;          // logical input pixel of (oj, oi) at tap (r, s) = (oj*str - ph + r, oi*str - pw + s)
    int Hout, Wout, osub, ooh, oow; // physical output image, output pixel = (oj*osub + ooh, oi*osub + oow)
    int w_ob, w_ib, w_t0, w_dr, w_ds;   // weight block (ob, ib, tap (r, s)) sits at (ob*w_ob + ib*w_ib + w_t0 + r*w_dr + s*w_ds) * 256 elements
    int npix, units, upp, gz;       // N*P*Q; chain units = (Cb / 2) * R * S; units per range; ranges
    int mdiv_taps, mdiv_S;          // ceil(65536 / taps), ceil(65536 / S): x / d == (x * m) >> 16 for x < 4096, d <= 16
    int in_bytes;                   // bytes of the input tensor
    float inv_PQ, inv_Q;
};

// The wave's instruction stream is the bottleneck of a kernel this short (one wave per SIMD, a few dozen
// units), so the per-unit work is kept to a handful of instructions: the unit's (pair, r, s) and the address
// terms that are uniform over the wave are scalar integer arithmetic (divisions by multiply-and-shift, exact
// for the admitted sizes); each lane prepares once, per pixel group, its pixel's offset and a bit mask of the
// taps that fall inside the image; the activations come through buffer loads, whose out-of-range lanes (offset
// beyond the tensor) return zeros, so padding costs one select on the offset and none on the data.
template <int KW, int PG, bool WTR> __global__ __launch_bounds__(256) void conv_small_bf16(ConvSmallArgs a)
{
    constexpr int NB = 16 / (KW + PG);                 // units per batch
    __shared__ float4v part[4][KW * PG][64];           // [wave][tile][lane]
    __shared__ __attribute__((aligned(16))) char wlds[WTR ? 4 * NB * KW * 1024 : 16];
    typedef unsigned u4v_ __attribute__((ext_vector_type(4)));
    const char *__restrict__ Wt = (const char *)a.Wt;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int li = lane & 15, kg = lane >> 4;
    const int kb0 = blockIdx.y * KW;                   // first feature block of this workgroup
    const int taps = a.R * a.S;
    // raw buffer over the input tensor: a lane offset of 0xfffffff0 is out of range and loads zeros
    const __amdgpu_buffer_rsrc_t ibuf = __builtin_amdgcn_make_buffer_rsrc((void *)a.I, 0, a.in_bytes, 0x00020000);

    const uint32_t cbs = (uint32_t)(a.Hin * a.Win) * 32u;           // bytes of one channel-block plane
    const uint32_t kbs = (uint32_t)(a.Hout * a.Wout) * 32u;
    const uint32_t lane_in = (uint32_t)(kg >> 1) * cbs + 16u * (kg & 1);
    uint32_t pix_off[PG], out_off[PG], vmask[PG];
    const int PQ = a.P * a.Q;
#pragma unroll
    for (int g = 0; g < PG; ++g) {
        const int pix = (blockIdx.x * PG + g) * 16 + li;
        const bool ok = pix < a.npix;
        const int p = ok ? pix : a.npix - 1;           // lanes beyond the end compute a valid pixel, store nothing
        const int n = c1_fdiv(p, PQ, a.inv_PQ), r = p - n * PQ;
        const int oj = c1_fdiv(r, a.Q, a.inv_Q), oi = r - oj * a.Q;
        const int hb = oj * a.str - a.ph, wb = oi * a.str - a.pw;
        // (may wrap below zero for a pixel whose first tap is in the padding; the taps inside the image bring it back)
        pix_off[g] = (uint32_t)(n * a.Cb) * cbs + lane_in + (uint32_t)((hb * a.Win + wb) * a.sub) * 32u;
        out_off[g] = ok ? (uint32_t)((n * a.Kb * a.Hout + oj * a.osub + a.ooh) * a.Wout + oi * a.osub + a.oow) * 32u + 8u * kg
                        : 0xffffffffu;
        uint32_t m = 0;
        for (int r2 = 0, t = 0; r2 < a.R; ++r2)
            for (int s2 = 0; s2 < a.S; ++s2, ++t)
                m |= (uint32_t)((unsigned)(hb + r2) < (unsigned)a.H && (unsigned)(wb + s2) < (unsigned)a.W) << t;
        vmask[g] = m;                                  // bit t: tap t of this lane's pixel is inside the image (bits 16.. stay 0)
    }
    const uint32_t w_lane = WTR ? (uint32_t)(lane >> 5) * a.w_ib * 512u + (uint32_t)(lane & 31) * 16u
                                : (uint32_t)((kg >> 1) * a.w_ib * 256 + li * 16 + 8 * (kg & 1)) * 2u;
    char *const wslot = wlds + (WTR ? wave * NB * KW * 1024 : 0);
    const uint32_t tr_off = (uint32_t)(kg >> 1) * 512u + (uint32_t)((8 * (kg & 1) + (li >> 2)) * 16 + 4 * (li & 3)) * 2u;
    const char *wk[KW];
#pragma unroll
    for (int k = 0; k < KW; ++k) {
        const int ob = kb0 + k < a.Kb ? kb0 + k : a.Kb - 1;
        wk[k] = Wt + ((int64_t)a.w_t0 + (int64_t)ob * a.w_ob) * 512;   // (uniform: a scalar base, the lane adds w_lane)
    }
    const int w_pair = a.w_ib * 1024;                  // bytes between channel-block pairs

    float4v acc[KW][PG];
#pragma unroll
    for (int k = 0; k < KW; ++k)
#pragma unroll
        for (int g = 0; g < PG; ++g) acc[k][g] = float4v{0.f, 0.f, 0.f, 0.f};

    // unit u = pair * taps + tap; this wave takes u0 + wave + 4j
    const int u0 = blockIdx.z * a.upp;
    const int u1 = u0 + a.upp < a.units ? u0 + a.upp : a.units;
    const int nw = u0 + wave < u1 ? (u1 - u0 - wave + 3) >> 2 : 0;

    // One batch = NB units with all their loads issued back to back; the loads of the next batch are in flight
    // while one batch is multiplied (two register banks, rotating by name).  No branch separates a load from its
    // use, so the wait counts stay exact: units past the end of the wave's list repeat its last unit with every
    // activation lane out of range (zeros).
#define CS_LOADB(A, B, JB)                                                                             \
    _Pragma("unroll") for (int i = 0; i < NB; ++i) {                                                   \
        const int j_ = (JB) * NB + i;                                                                  \
        const bool live_ = j_ < nw;                                                                    \
        const int u_ = u0 + wave + 4 * (live_ ? j_ : nw - 1);                                          \
        const int cp_ = (u_ * a.mdiv_taps) >> 16;                                                      \
        const int t_ = u_ - cp_ * taps;                                                                \
        const int r_ = (t_ * a.mdiv_S) >> 16;                                                          \
        const int s_ = t_ - r_ * a.S;                                                                  \
        const uint32_t io_ = (uint32_t)cp_ * 2u * cbs + (uint32_t)((r_ * a.Win + s_) * a.sub) * 32u;   \
        const int wo_ = cp_ * w_pair + (r_ * a.w_dr + s_ * a.w_ds) * 512;                              \
        const int bit_ = live_ ? t_ : 31;                                                              \
        _Pragma("unroll") for (int g = 0; g < PG; ++g) {                                               \
            const uint32_t vo_ = (vmask[g] >> bit_) & 1u ? pix_off[g] + io_ : 0xfffffff0u;             \
            B[i][g] = __builtin_bit_cast(bf16x8v, (u4v_)__builtin_amdgcn_raw_buffer_load_b128(ibuf, (int)vo_, 0, 0)); \
        }                                                                                              \
        _Pragma("unroll") for (int k = 0; k < KW; ++k) A[i][k] = *(const bf16x8v *)((wk[k] + wo_) + w_lane); \
    }                                                                                                  \
    __builtin_amdgcn_sched_barrier(0);
// WTR: the blocks of the batch go through the wave's LDS slots (one per unit, so that the round trips overlap)
// and come back transposed, in place
#define CS_COMPB(A, B)                                                                                 \
    if (WTR) {                                                                                         \
        typedef short s4v_ __attribute__((ext_vector_type(4)));                                        \
        typedef short s8v_ __attribute__((ext_vector_type(8)));                                        \
        typedef __attribute__((address_space(3))) s4v_ *lp_;                                           \
        _Pragma("unroll") for (int i = 0; i < NB; ++i)                                                 \
            _Pragma("unroll") for (int k = 0; k < KW; ++k) *(bf16x8v *)(wslot + (i * KW + k) * 1024 + lane * 16) = A[i][k]; \
        _Pragma("unroll") for (int i = 0; i < NB; ++i)                                                 \
            _Pragma("unroll") for (int k = 0; k < KW; ++k) {                                           \
                const s4v_ lo_ = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp_)(wslot + (i * KW + k) * 1024 + tr_off));        \
                const s4v_ hi_ = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp_)(wslot + (i * KW + k) * 1024 + tr_off + 128)); \
                A[i][k] = __builtin_bit_cast(bf16x8v, s8v_{lo_[0], lo_[1], lo_[2], lo_[3], hi_[0], hi_[1], hi_[2], hi_[3]}); \
            }                                                                                          \
    }                                                                                                  \
    _Pragma("unroll") for (int i = 0; i < NB; ++i)                                                     \
        _Pragma("unroll") for (int g = 0; g < PG; ++g)                                                 \
            _Pragma("unroll") for (int k = 0; k < KW; ++k)                                             \
                acc[k][g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[i][k], B[i][g], acc[k][g], 0, 0, 0); \
    __builtin_amdgcn_sched_barrier(0);

    bf16x8v a0[NB][KW], b0[NB][PG], a1[NB][KW], b1[NB][PG];
    if (nw > 0) {
        const int nb = (nw + NB - 1) / NB;
        CS_LOADB(a0, b0, 0)
        if (nb == 1) {
            CS_COMPB(a0, b0)
        } else {
            for (int b = 0; b < nb; b += 2) {
                CS_LOADB(a1, b1, b + 1)
                CS_COMPB(a0, b0)
                CS_LOADB(a0, b0, b + 2)
                CS_COMPB(a1, b1)
            }
        }
    }
#undef CS_LOADB
#undef CS_COMPB

#pragma unroll
    for (int k = 0; k < KW; ++k)
#pragma unroll
        for (int g = 0; g < PG; ++g) part[wave][k * PG + g][lane] = acc[k][g];
    __syncthreads();

    // wave w finishes tiles w, w+4, ...: register r of lane (li, kg) is feature 4kg + r of the block, pixel li
#pragma unroll
    for (int t = 0; t < (KW * PG + 3) / 4; ++t) {
        const int tile = 4 * t + wave;
        if (tile >= KW * PG) break;
        const int k = tile / PG, g = tile - k * PG;
        uint32_t oo = 0xffffffffu;
#pragma unroll
        for (int gg = 0; gg < PG; ++gg) oo = gg == g ? out_off[gg] : oo;
        if (kb0 + k >= a.Kb || oo == 0xffffffffu) continue;
        float4v v = (part[0][tile][lane] + part[1][tile][lane]) + (part[2][tile][lane] + part[3][tile][lane]);
        if (a.gz > 1) {
            const int pix = (blockIdx.x * PG + g) * 16 + li;
            *(float4v *)(a.part + (((int64_t)blockIdx.z * a.Kb + kb0 + k) * a.npix + pix) * 16 + 4 * kg) = v;
        } else {
            if (a.bias) v += *(const float4v *)((const char *)a.bias + (kb0 + k) * 64 + 16 * kg);
            v = act_is_slow(a.act) ? apply_act4<true>(v, a.act) : apply_act4<false>(v, a.act);
            *(us4v *)((char *)a.O + (int64_t)(kb0 + k) * kbs + oo) = pack_bf16x4(v);
        }
    }
}

// Sum of the gz partial results in the order 0, 1, ..., bias, activation, bf16: one thread per (feature block,
// pixel, four features).
__global__ __launch_bounds__(256) void conv_small_reduce(ConvSmallArgs a)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    const int quad = idx & 3, rest = idx >> 2;
    if (rest >= a.Kb * a.npix) return;
    const int kb = c1_fdiv(rest, a.npix, 1.0f / (float)a.npix), pix = rest - kb * a.npix;
    const float *src = a.part + ((int64_t)kb * a.npix + pix) * 16 + 4 * quad;
    const int64_t zs = (int64_t)a.Kb * a.npix * 16;
    float4v v = *(const float4v *)src;
    for (int z = 1; z < a.gz; ++z) v += *(const float4v *)(src + z * zs);
    if (a.bias) v += *(const float4v *)(a.bias + kb * 16 + 4 * quad);
    v = act_is_slow(a.act) ? apply_act4<true>(v, a.act) : apply_act4<false>(v, a.act);
    const int PQ = a.P * a.Q;
    const int n = c1_fdiv(pix, PQ, a.inv_PQ), r = pix - n * PQ;
    const int oj = c1_fdiv(r, a.Q, a.inv_Q), oi = r - oj * a.Q;
    char *o = (char *)a.O + ((int64_t)((n * a.Kb + kb) * a.Hout + oj * a.osub + a.ooh) * a.Wout + oi * a.osub + a.oow) * 32 + 8 * quad;
    *(us4v *)o = pack_bf16x4(v);
}

}  // namespace brg
