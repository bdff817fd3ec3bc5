// Convolutions on blocked NCHWc / KCRSck layouts as batch-reduce chains
// (paper section 3.2, Algorithm 4): the address lists over (c-block, r, s) are
// index arithmetic inside the kernel, padding is logical.
#include <atomic>
#include <cstdlib>

#include "brg_engine.hpp"
#include "brg_conv_tile.hpp"
#include "brg_conv_tile_bf16.hpp"
#include "brg_conv1x1_bf16.hpp"
#include "brg_conv1x1_lds_bf16.hpp"
#include "brg_conv_small_bf16.hpp"
#include "brg_conv_stem_bf16.hpp"
#include "brg_conv_wgt.hpp"

namespace brg {

// Distance (modulo 256 bytes) between the LDS planes that the four 16-lane groups of an operand read address.
// Measured with a read-pattern micro-benchmark and the SQ_LDS_BANK_CONFLICT counter: a 16-byte-per-lane read
// is served without conflicts when the four groups have the SAME offset modulo 256 bytes (any common shift),
// and takes twice the LDS cycles when the groups are 16, 64 or 128 bytes apart.
static int conv_plane_pad()
{
    return knobs().conv_plane_pad.set ? knobs().conv_plane_pad.val : 0;
}


struct ConvDims {
    int N, C, H, W, K, R, S, sh, sw, ph, pw, bc, bk, P, Q, Cb, Kb;
};

// ---- forward.  M = K (output channels), N = flat output pixels (n, oj, oi),
// chain = (c-block, r, s) with depth bc.
template <typename TIn, typename TOut> struct ConvFwdProb {
    static constexpr bool A_KFAST = false, B_KFAST = true;
    ConvDims d;
    const TIn *I, *Wt;
    TOut *O;
    const float *bias;
    int act, tiles_m;
    int64_t npix;
    typedef int64_t RowA;
    struct RowB {
        int64_t base;  // offset of image n, -1 if the column is beyond the last pixel
        int ij0, ii0;
    };
    struct Chain {
        int64_t aoff, boff;
        int r, s;
    };
    __device__ int m0() const { return (blockIdx.x % tiles_m) * ENG_TM; }
    __device__ int64_t n0() const { return (int64_t)(blockIdx.x / tiles_m) * ENG_TN; }
    __device__ int chain_len() const { return d.Cb * d.R * d.S; }
    __device__ int kdepth(int) const { return d.bc; }
    __device__ RowA row_a(int i) const
    {
        int k = m0() + i;
        if (k >= d.K) return -1;
        return (int64_t)(k / d.bk) * d.Cb * d.R * d.S * d.bc * d.bk + k % d.bk;
    }
    __device__ RowB row_b(int j) const
    {
        int64_t px = n0() + j;
        RowB rb;
        if (px >= npix) {
            rb.base = -1; rb.ij0 = 0; rb.ii0 = 0;
            return rb;
        }
        int oi = (int)(px % d.Q);
        int oj = (int)((px / d.Q) % d.P);
        int n = (int)(px / ((int64_t)d.P * d.Q));
        rb.base = (int64_t)n * d.Cb * d.H * d.W * d.bc;
        rb.ij0 = oj * d.sh - d.ph;
        rb.ii0 = oi * d.sw - d.pw;
        return rb;
    }
    __device__ Chain chain(int c) const
    {
        Chain ch;
        int s = c % d.S, r = (c / d.S) % d.R, cb = c / (d.S * d.R);
        ch.r = r; ch.s = s;
        ch.aoff = (((int64_t)cb * d.R + r) * d.S + s) * d.bc * d.bk;
        ch.boff = (int64_t)cb * d.H * d.W * d.bc;
        return ch;
    }
    __device__ float a(const Chain &ch, const RowA &r, int p) const
    {
        return r >= 0 ? to_f32<TIn>(Wt[r + ch.aoff + (int64_t)p * d.bk]) : 0.f;
    }
    __device__ float b(const Chain &ch, const RowB &rb, int p) const
    {
        int ij = rb.ij0 + ch.r, ii = rb.ii0 + ch.s;
        if (rb.base < 0 || ij < 0 || ij >= d.H || ii < 0 || ii >= d.W) return 0.f;
        return to_f32<TIn>(I[rb.base + ch.boff + ((int64_t)ij * d.W + ii) * d.bc + p]);
    }
    __device__ void store4(int i, int j, float4v acc) const
    {
        int64_t px = n0() + j;
        if (px >= npix) return;
        int64_t pq = px % ((int64_t)d.P * d.Q);
        int64_t n = px / ((int64_t)d.P * d.Q);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            int k = m0() + i + r;
            if (k >= d.K) continue;
            float v = acc[r] + (bias ? bias[k] : 0.f);
            O[((n * d.Kb + k / d.bk) * d.P * d.Q + pq) * d.bk + k % d.bk] = from_f32<TOut>(apply_act(v, act));
        }
    }
};

// ---- backward by data (the "dual" convolution, gather form).  M = C (input
// channels), N = flat INPUT pixels (n, h, w), chain = (k-block, r, s) with depth bk:
//   dI[n][c][h][w] = sum_{k,r,s} Wt[k][c][r][s] * dO[n][k][(h+ph-r)/sh][(w+pw-s)/sw]
// over the taps for which both quotients are exact and in range.  The weight
// block is read transposed (c rows, k reduction) straight from the forward layout.
template <typename TIn, typename TOut> struct ConvBwdDataProb {
    static constexpr bool A_KFAST = true, B_KFAST = true;
    ConvDims d;
    const TIn *dO, *Wt;
    TOut *dI;
    int tiles_m;
    int64_t npix;
    typedef int64_t RowA;
    struct RowB {
        int64_t base;
        int h, w;
    };
    struct Chain {
        int64_t aoff, boff;
        int r, s;
    };
    __device__ int m0() const { return (blockIdx.x % tiles_m) * ENG_TM; }
    __device__ int64_t n0() const { return (int64_t)(blockIdx.x / tiles_m) * ENG_TN; }
    __device__ int chain_len() const { return d.Kb * d.R * d.S; }
    __device__ int kdepth(int) const { return d.bk; }
    __device__ RowA row_a(int i) const
    {
        int c = m0() + i;
        if (c >= d.C) return -1;
        return ((int64_t)(c / d.bc) * d.R * d.S * d.bc + c % d.bc) * d.bk;
    }
    __device__ RowB row_b(int j) const
    {
        int64_t px = n0() + j;
        RowB rb;
        if (px >= npix) {
            rb.base = -1; rb.h = 0; rb.w = 0;
            return rb;
        }
        rb.w = (int)(px % d.W);
        rb.h = (int)((px / d.W) % d.H);
        int n = (int)(px / ((int64_t)d.H * d.W));
        rb.base = (int64_t)n * d.Kb * d.P * d.Q * d.bk;
        return rb;
    }
    __device__ Chain chain(int c) const
    {
        Chain ch;
        int s = c % d.S, r = (c / d.S) % d.R, kb = c / (d.S * d.R);
        ch.r = r; ch.s = s;
        ch.aoff = ((int64_t)kb * d.Cb * d.R * d.S + (int64_t)r * d.S + s) * d.bc * d.bk;
        ch.boff = (int64_t)kb * d.P * d.Q * d.bk;
        return ch;
    }
    __device__ float a(const Chain &ch, const RowA &r, int p) const
    {
        return r >= 0 ? to_f32<TIn>(Wt[r + ch.aoff + p]) : 0.f;
    }
    __device__ float b(const Chain &ch, const RowB &rb, int p) const
    {
        if (rb.base < 0) return 0.f;
        int th = rb.h + d.ph - ch.r, tw = rb.w + d.pw - ch.s;
        if (th < 0 || tw < 0) return 0.f;
        int oj = th / d.sh, oi = tw / d.sw;
        if (oj * d.sh != th || oi * d.sw != tw || oj >= d.P || oi >= d.Q) return 0.f;
        return to_f32<TIn>(dO[rb.base + ch.boff + ((int64_t)oj * d.Q + oi) * d.bk + p]);
    }
    __device__ void store4(int i, int j, float4v acc) const
    {
        int64_t px = n0() + j;
        if (px >= npix) return;
        int64_t hw = px % ((int64_t)d.H * d.W);
        int64_t n = px / ((int64_t)d.H * d.W);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            int c = m0() + i + r;
            if (c >= d.C) continue;
            dI[((n * d.Cb + c / d.bc) * d.H * d.W + hw) * d.bc + c % d.bc] = from_f32<TOut>(acc[r]);
        }
    }
};

// ---- weight gradient.  One (r, s) tap per blockIdx.y; M = K, N = C,
// chain = (n, oj) with depth Q (the reduction runs over output pixels):
//   dWt[k][c][r][s] = sum_{n,oj,oi} dO[n][k][oj][oi] * I[n][c][sh*oj+r-ph][sw*oi+s-pw]
template <typename TIn> struct ConvBwdWgtProb {
    static constexpr bool A_KFAST = false, B_KFAST = false;
    ConvDims d;
    const TIn *I, *dO;
    float *dWt;
    int tiles_m;
    typedef int64_t RowA;
    typedef int64_t RowB;
    struct Chain {
        int64_t aoff, boff;
        bool row_ok;
    };
    __device__ int tap_r() const { return blockIdx.y / d.S; }
    __device__ int tap_s() const { return blockIdx.y % d.S; }
    __device__ int m0() const { return (blockIdx.x % tiles_m) * ENG_TM; }
    __device__ int n0() const { return (blockIdx.x / tiles_m) * ENG_TN; }
    __device__ int chain_len() const { return d.N * d.P; }
    __device__ int kdepth(int) const { return d.Q; }
    __device__ RowA row_a(int i) const
    {
        int k = m0() + i;
        if (k >= d.K) return -1;
        return (int64_t)(k / d.bk) * d.P * d.Q * d.bk + k % d.bk;
    }
    __device__ RowB row_b(int j) const
    {
        int c = n0() + j;
        if (c >= d.C) return -1;
        return (int64_t)(c / d.bc) * d.H * d.W * d.bc + c % d.bc;
    }
    __device__ Chain chain(int c) const
    {
        Chain ch;
        int oj = c % d.P, n = c / d.P;
        int ij = oj * d.sh + tap_r() - d.ph;
        ch.row_ok = ij >= 0 && ij < d.H;
        ch.aoff = ((int64_t)n * d.Kb * d.P + oj) * d.Q * d.bk;
        ch.boff = (int64_t)n * d.Cb * d.H * d.W * d.bc + (int64_t)ij * d.W * d.bc;
        return ch;
    }
    __device__ float a(const Chain &ch, const RowA &r, int p) const
    {
        return r >= 0 ? to_f32<TIn>(dO[r + ch.aoff + (int64_t)p * d.bk]) : 0.f;
    }
    __device__ float b(const Chain &ch, const RowB &r, int p) const
    {
        int ii = p * d.sw + tap_s() - d.pw;
        if (r < 0 || !ch.row_ok || ii < 0 || ii >= d.W) return 0.f;
        return to_f32<TIn>(I[r + ch.boff + (int64_t)ii * d.bc]);
    }
    __device__ void store4(int i, int j, float4v acc) const
    {
        int c = n0() + j;
        if (c >= d.C) return;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            int k = m0() + i + r;
            if (k >= d.K) continue;
            dWt[(((((int64_t)(k / d.bk) * d.Cb + c / d.bc) * d.R + tap_r()) * d.S + tap_s()) * d.bc + c % d.bc) * d.bk +
                k % d.bk] = acc[r];
        }
    }
};

static int conv_dims(const brg_conv_desc_t *x, ConvDims *d, const char *who)
{
    BRG_REQUIRE(x != nullptr, BRG_EINVAL, "%s: desc is null", who);
    BRG_REQUIRE(x->N > 0 && x->C > 0 && x->H > 0 && x->W > 0 && x->K > 0 && x->R > 0 && x->S > 0, BRG_EINVAL,
                "%s: sizes must be positive", who);
    BRG_REQUIRE(x->stride_h > 0 && x->stride_w > 0 && x->pad_h >= 0 && x->pad_w >= 0, BRG_EINVAL,
                "%s: bad stride or padding", who);
    BRG_REQUIRE(x->bc > 0 && x->bk > 0 && x->C % x->bc == 0 && x->K % x->bk == 0, BRG_EINVAL,
                "%s: channel blocking (%lld,%lld) does not divide (C,K)=(%lld,%lld)", who, (long long)x->bc,
                (long long)x->bk, (long long)x->C, (long long)x->K);
    BRG_REQUIRE(x->H + 2 * x->pad_h >= x->R && x->W + 2 * x->pad_w >= x->S, BRG_EINVAL,
                "%s: filter larger than the padded image", who);
    BRG_REQUIRE(x->pad_h < x->R && x->pad_w < x->S, BRG_EINVAL, "%s: padding must be smaller than the filter", who);
    BRG_REQUIRE(x->N < (1 << 20) && x->C < (1 << 20) && x->K < (1 << 20) && x->H < (1 << 15) && x->W < (1 << 15) &&
                    x->R < 64 && x->S < 64,
                BRG_EINVAL, "%s: size too large", who);
    // one short channel block (bc = C = 4) is accepted for the bf16 stem kernels only; each entry point checks
    BRG_REQUIRE((x->bc == 16 || (x->bc == 4 && x->C == 4)) && x->bk == 16, BRG_EUNSUPPORTED,
                "%s: only bc = bk = 16 (or one channel block of bc = C = 4) is supported", who);
    d->N = (int)x->N; d->C = (int)x->C; d->H = (int)x->H; d->W = (int)x->W; d->K = (int)x->K;
    d->R = (int)x->R; d->S = (int)x->S; d->sh = (int)x->stride_h; d->sw = (int)x->stride_w;
    d->ph = (int)x->pad_h; d->pw = (int)x->pad_w; d->bc = (int)x->bc; d->bk = (int)x->bk;
    d->P = (d->H + 2 * d->ph - d->R) / d->sh + 1;
    d->Q = (d->W + 2 * d->pw - d->S) / d->sw + 1;
    d->Cb = d->C / d->bc; d->Kb = d->K / d->bk;
    return BRG_OK;
}

// Plan of the tiled kernel for one layer and pass; ok == false means "use the general engine".
struct ConvTilePlan {
    bool ok;
    ConvTileArgs a;
    size_t smem;
    int R, STR, CG, NPASS, KW;
    dim3 grid;
};

// `bwd`: plan the backward-by-data pass (stride 1 only) as a forward pass over dO.
// `bf16`: 2 chunks of 16 bytes per pixel and channel block instead of 4, channel blocks consumed in pairs.
static ConvTilePlan plan_conv_tile(const ConvDims &d, bool bwd, bool bf16 = false)
{
    ConvTilePlan pl;
    pl.ok = false;
    if (d.sh != d.sw || d.sh > 2 || d.R != d.S || !(d.R == 1 || d.R == 3) || d.ph != d.pw) return pl;
    if (bwd && d.sh != 1) return pl;
    if ((int64_t)d.N * d.C * d.H * d.W >= (1ll << 31) || (int64_t)d.N * d.K * d.P * d.Q >= (1ll << 31)) return pl;
    ConvTileArgs &a = pl.a;
    a = ConvTileArgs{};
    int str = d.sh;
    a.N = d.N;
    a.sub = 1;
    if (!bwd) {
        a.Cb = d.Cb; a.Kb = d.Kb; a.H = d.H; a.W = d.W; a.P = d.P; a.Q = d.Q; a.ph = d.ph; a.pw = d.pw;
        a.Hin = d.H; a.Win = d.W;
        a.w_ob = d.Cb * d.R * d.S; a.w_ib = d.R * d.S;
        if (d.R == 1 && str > 1) {   // 1x1 with a stride: a stride-1 pass over the sub-sampled image
            a.sub = str; a.H = d.P; a.W = d.Q; str = 1;
        }
    } else {                        // roles swapped: input = dO (K channels), output = dI (C channels)
        a.Cb = d.Kb; a.Kb = d.Cb; a.H = d.P; a.W = d.Q; a.P = d.H; a.Q = d.W;
        a.ph = d.R - 1 - d.ph; a.pw = d.S - 1 - d.pw;
        a.Hin = d.P; a.Win = d.Q;
        a.w_ob = d.R * d.S; a.w_ib = d.Cb * d.R * d.S;
    }
    if (a.Q > CT_NG * 16) return pl;
    a.Hout = a.P; a.Wout = a.Q; a.osub = 1; a.ooh = 0; a.oow = 0;
    for (int t = 0; t < d.R * d.S; ++t) a.wtap[t] = bwd ? d.R * d.S - 1 - t : t;
    a.Hv = (a.P - 1) * str + d.R;
    int wp = (a.Q - 1) * str + d.S;
    a.Wp = wp > a.W + a.pw ? wp : a.W + a.pw;
    a.trg = (CT_NG * 16) / a.Q;
    a.total_rows = a.N * a.P;
    if (a.total_rows >= (1 << 22) || (int64_t)a.N * a.Hv >= (1 << 22)) return pl;
    a.ntiles = (a.total_rows + a.trg - 1) / a.trg;
    int nv_max = 0;
    for (int tile = 0; tile < a.ntiles; ++tile) {
        int gr0 = tile * a.trg;
        int rows = a.total_rows - gr0 < a.trg ? a.total_rows - gr0 : a.trg;
        int vf = (gr0 / a.P) * a.Hv + (gr0 % a.P) * str;
        int grl = gr0 + rows - 1;
        int nv = (grl / a.P) * a.Hv + (grl % a.P) * str + d.R - vf;
        if (nv > nv_max) nv_max = nv;
    }
    const int cpp = bf16 ? 2 : 4;          // 16-byte chunks per pixel of one channel block
    const int chunks = nv_max * a.W * cpp; // chunks of one channel block's halo
    pl.R = d.R; pl.STR = str; pl.KW = 1;
    if (!bf16) {
        if (d.R == 3) {
            pl.CG = 1;
            pl.NPASS = (str == 1 && chunks <= 1024) ? 4 : 8;
            if (chunks > 256 * pl.NPASS) return pl;
        } else {
            if (a.Cb % 4 == 0 && chunks <= 512) { pl.CG = 4; pl.NPASS = 2; }
            else if (a.Cb % 2 == 0 && chunks <= 1024) { pl.CG = 2; pl.NPASS = 4; }
            else return pl;
        }
    } else {
        if (d.R == 3 && str == 1) {
            if (a.Cb % 4 != 0 || chunks > 512) return pl;
            pl.CG = 4; pl.NPASS = 2;
        } else if (d.R == 3) {
            if (a.Cb % 2 != 0 || chunks > 2048) return pl;
            pl.CG = 2; pl.NPASS = 8;
        } else {
            if (chunks > 256) return pl;
            if (a.Cb % 8 == 0) pl.CG = 8;
            else if (a.Cb % 4 == 0) pl.CG = 4;
            else return pl;
            pl.NPASS = 1;
        }
        pl.KW = a.Kb >= 8 ? 2 : 1;
    }
    int plane = nv_max * a.Wp * 16;
    plane = ((plane + 255) / 256) * 256 + conv_plane_pad();
    a.plane_bytes = plane;
    a.buf_bytes = pl.CG * cpp * plane;
    pl.smem = 2 * (size_t)a.buf_bytes;
    if (pl.smem > 80 * 1024) return pl;         // two workgroups per CU must fit the 160 KiB LDS
    a.inv_Q = 1.0f / a.Q; a.inv_P = 1.0f / a.P; a.inv_Hv = 1.0f / a.Hv; a.inv_W4 = 1.0f / (a.W * cpp);
    // persistent grid: two workgroups per CU over all feature-map tiles, a multiple of 8 per row
    int ktiles = (a.Kb + 4 * pl.KW - 1) / (4 * pl.KW);
    int gx = (512 / ktiles) & ~7;
    if (gx < 8) gx = 8;
    if (gx > a.ntiles) gx = a.ntiles;
    pl.grid = dim3(gx, ktiles);
    pl.ok = true;
    return pl;
}

// dynamic LDS beyond 64 KiB has to be allowed per kernel (and device) before the launch
static int allow_big_lds(const void *kern, size_t smem)
{
    if (smem <= 64 * 1024) return BRG_OK;
    hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return fail(BRG_EHIP, "brg_conv: hipFuncSetAttribute: %s", hipGetErrorString(e));
    return BRG_OK;
}

template <int R, int STR, int CG, int NPASS, int MODE>
static int conv_tile_f32_go(ConvTilePlan &pl, hipStream_t s)
{
    auto kern = conv_tile_f32<R, R, STR, CG, NPASS, MODE>;
    int rc = allow_big_lds((const void *)kern, pl.smem);
    if (rc) return rc;
    hipLaunchKernelGGL(kern, pl.grid, dim3(256), pl.smem, s, pl.a);
    return check_launch("brg_conv (tiled) launch");
}

// MODE: see conv_tile_f32 (0 forward, 1 backward by data, 2 forward with transposed weight blocks)
template <int MODE>
static int conv_tile_f32_launch(ConvTilePlan &pl, const void *I, const void *Wt, void *O, const float *bias,
                                int act, hipStream_t s)
{
    pl.a.I = I; pl.a.Wt = Wt; pl.a.O = O; pl.a.bias = bias; pl.a.act = act;
    const int key = pl.R * 1000 + pl.STR * 100 + pl.CG * 10 + pl.NPASS;
    switch (key) {
    case 3114: return conv_tile_f32_go<3, 1, 1, 4, MODE>(pl, s);
    case 3118: return conv_tile_f32_go<3, 1, 1, 8, MODE>(pl, s);
    case 1142: return conv_tile_f32_go<1, 1, 4, 2, MODE>(pl, s);
    case 1124: return conv_tile_f32_go<1, 1, 2, 4, MODE>(pl, s);
    case 3218:
        if (MODE != 1) return conv_tile_f32_go<3, 2, 1, 8, MODE == 1 ? 0 : MODE>(pl, s);
    }
    return fail(BRG_EUNSUPPORTED, "brg_conv: internal: no tiled kernel for key %d", key);
}

// ---- bf16 tiled kernels: one "view" = one stride-1-or-2 forward-style pass over some input
struct ConvView {
    int N, Cb, Hin, Win, sub, H, W;       // input: physical dims, sub-sampling, dims as the kernel sees them
    int Kb, P, Q, Hout, Wout, osub, ooh, oow;   // output: logical dims and placement in the physical tensor
    int R, S, str, ph, pw;
    int w_ob, w_ib;
    int wtap[16];
};

struct Bf16Plan {
    bool ok;
    ConvTileArgs a;
    size_t smem;
    int key, KW;
    dim3 grid;
};

// fp32: one parity class of a strided backward-by-data pass (a stride-1 pass over dO with the class's taps,
// results placed on every stride-th pixel) on the fp32 tiled kernel in its backward form
static ConvTilePlan plan_view_f32(const ConvView &v)
{
    ConvTilePlan pl;
    pl.ok = false;
    const int taps = v.R * v.S;
    if (v.str != 1 || v.sub != 1 || v.R > 2 || v.S > 2 || v.P <= 0 || v.Q <= 0 || v.Q > CT_NG * 16) return pl;
    if ((int64_t)v.N * v.Cb * v.Hin * v.Win * 16 >= (1ll << 31) || (int64_t)v.N * v.Kb * v.Hout * v.Wout * 16 >= (1ll << 31)) return pl;
    ConvTileArgs &a = pl.a;
    a = ConvTileArgs{};
    a.N = v.N; a.Cb = v.Cb; a.H = v.H; a.W = v.W; a.Kb = v.Kb; a.P = v.P; a.Q = v.Q; a.ph = v.ph; a.pw = v.pw;
    a.sub = 1; a.Hin = v.Hin; a.Win = v.Win; a.w_ob = v.w_ob; a.w_ib = v.w_ib;
    a.osub = v.osub; a.ooh = v.ooh; a.oow = v.oow; a.Hout = v.Hout; a.Wout = v.Wout;
    for (int t = 0; t < 16; ++t) a.wtap[t] = v.wtap[t];
    a.Hv = (a.P - 1) + v.R;
    const int wp = (a.Q - 1) + v.S;
    a.Wp = wp > a.W + a.pw ? wp : a.W + a.pw;
    a.trg = (CT_NG * 16) / a.Q;
    a.total_rows = a.N * a.P;
    if (a.total_rows >= (1 << 22) || (int64_t)a.N * a.Hv >= (1 << 22)) return pl;
    a.ntiles = (a.total_rows + a.trg - 1) / a.trg;
    int nv_max = 0;
    for (int tile = 0; tile < a.ntiles; ++tile) {
        const int gr0 = tile * a.trg;
        const int rows = a.total_rows - gr0 < a.trg ? a.total_rows - gr0 : a.trg;
        const int vf = (gr0 / a.P) * a.Hv + (gr0 % a.P);
        const int grl = gr0 + rows - 1;
        const int nv = (grl / a.P) * a.Hv + (grl % a.P) + v.R - vf;
        if (nv > nv_max) nv_max = nv;
    }
    const int chunks = nv_max * a.W * 4;
    pl.R = v.R; pl.STR = 1; pl.KW = 1;
    if (taps > 1) {
        pl.CG = 1;
        pl.NPASS = chunks <= 1024 ? 4 : 8;
        if (chunks > 256 * pl.NPASS) return pl;
    } else {
        if (a.Cb % 4 == 0 && chunks <= 512) { pl.CG = 4; pl.NPASS = 2; }
        else if (a.Cb % 2 == 0 && chunks <= 1024) { pl.CG = 2; pl.NPASS = 4; }
        else return pl;
    }
    int plane = nv_max * a.Wp * 16;
    plane = ((plane + 255) / 256) * 256 + conv_plane_pad();
    a.plane_bytes = plane;
    a.buf_bytes = pl.CG * 4 * plane;
    pl.smem = 2 * (size_t)a.buf_bytes;
    if (pl.smem > 80 * 1024) return pl;
    a.inv_Q = 1.0f / a.Q; a.inv_P = 1.0f / a.P; a.inv_Hv = 1.0f / a.Hv; a.inv_W4 = 1.0f / (a.W * 4);
    const int ktiles = (a.Kb + 3) / 4;
    int gx = (512 / ktiles) & ~7;
    if (gx < 8) gx = 8;
    if (gx > a.ntiles) gx = a.ntiles;
    pl.grid = dim3(gx, ktiles);
    pl.ok = true;
    return pl;
}

template <int R, int S, int CG, int NPASS> static int conv_tile_f32_view_go(ConvTilePlan &pl, hipStream_t s)
{
    auto kern = conv_tile_f32<R, S, 1, CG, NPASS, 3>;
    int rc = allow_big_lds((const void *)kern, pl.smem);
    if (rc) return rc;
    hipLaunchKernelGGL(kern, pl.grid, dim3(256), pl.smem, s, pl.a);
    return check_launch("brg_conv_bwd_data (tiled, parity class) launch");
}

static int conv_tile_f32_view_launch(ConvTilePlan &pl, int S, const void *dO, const void *Wt, void *dI, hipStream_t s)
{
    pl.a.I = dO; pl.a.Wt = Wt; pl.a.O = dI; pl.a.bias = nullptr; pl.a.act = BRG_ACT_NONE;
    const int key = pl.R * 1000 + S * 100 + pl.CG * 10 + pl.NPASS;
    switch (key) {
    case 1142: return conv_tile_f32_view_go<1, 1, 4, 2>(pl, s);
    case 1124: return conv_tile_f32_view_go<1, 1, 2, 4>(pl, s);
    case 1214: return conv_tile_f32_view_go<1, 2, 1, 4>(pl, s);
    case 1218: return conv_tile_f32_view_go<1, 2, 1, 8>(pl, s);
    case 2114: return conv_tile_f32_view_go<2, 1, 1, 4>(pl, s);
    case 2118: return conv_tile_f32_view_go<2, 1, 1, 8>(pl, s);
    case 2214: return conv_tile_f32_view_go<2, 2, 1, 4>(pl, s);
    case 2218: return conv_tile_f32_view_go<2, 2, 1, 8>(pl, s);
    }
    return fail(BRG_EUNSUPPORTED, "brg_conv_bwd_data: internal: no tiled fp32 kernel for key %d", key);
}

// `grids`: how many such views run as one grid (the fused parity classes of a strided backward pass)
static Bf16Plan plan_view_bf16(const ConvView &v, int grids = 1)
{
    Bf16Plan pl;
    pl.ok = false;
    if (v.Q > CT_NG * 16 || (v.R * v.S > 16 && v.Cb != 1) || v.P <= 0 || v.Q <= 0) return pl;
    ConvTileArgs &a = pl.a;
    a = ConvTileArgs{};
    a.N = v.N; a.Cb = v.Cb; a.H = v.H; a.W = v.W; a.Kb = v.Kb; a.P = v.P; a.Q = v.Q; a.ph = v.ph; a.pw = v.pw;
    a.sub = v.sub; a.Hin = v.Hin; a.Win = v.Win; a.w_ob = v.w_ob; a.w_ib = v.w_ib;
    a.osub = v.osub; a.ooh = v.ooh; a.oow = v.oow; a.Hout = v.Hout; a.Wout = v.Wout;
    for (int t = 0; t < 16; ++t) a.wtap[t] = v.wtap[t];
    a.Hv = (a.P - 1) * v.str + v.R;
    int wp = (a.Q - 1) * v.str + v.S;
    a.Wp = wp > a.W + a.pw ? wp : a.W + a.pw;
    // A group of output pixels may run over the end of an image row; its operand read is then free of bank
    // conflicts only if the next row continues where this one ended.  Full congruence of the halo row pitch with
    // Q (modulo 16 pixels = 256 bytes, measured with a read-pattern micro-benchmark and SQ_LDS_BANK_CONFLICT) was
    // tried on every layer and lost: these kernels are not bound by LDS cycles, and the wider halos cost more than
    // the conflicts (14x14: 22.8 -> 24.9 us, 7x7: 31 -> 38 us).  Kept: congruence modulo 8 pixels for rows of
    // 8..15 pixels, where EVERY 16-lane group crosses a row end (measured: 8 % on the 14x14 layers).
    if (v.str == 1 && v.R * v.S > 1 && a.Cb > 1 && a.Q >= 8 && a.Q < 16 &&
        !(knobs().conv_pitch.set && knobs().conv_pitch.val == 0))
        a.Wp += ((a.Q - a.Wp) % 8 + 8) % 8;
    a.trg = (CT_NG * 16) / a.Q;
    a.total_rows = a.N * a.P;
    if (a.total_rows >= (1 << 22) || (int64_t)a.N * a.Hv >= (1 << 22)) return pl;
    if ((int64_t)a.N * a.Cb * a.Hin * a.Win * 16 >= (1ll << 31) || (int64_t)a.N * a.Kb * a.Hout * a.Wout * 16 >= (1ll << 31))
        return pl;
    a.ntiles = (a.total_rows + a.trg - 1) / a.trg;
    int nv_max = 0;
    for (int tile = 0; tile < a.ntiles; ++tile) {
        int gr0 = tile * a.trg;
        int rows = a.total_rows - gr0 < a.trg ? a.total_rows - gr0 : a.trg;
        int vf = (gr0 / a.P) * a.Hv + (gr0 % a.P) * v.str;
        int grl = gr0 + rows - 1;
        int nv = (grl / a.P) * a.Hv + (grl % a.P) * v.str + v.R - vf;
        if (nv > nv_max) nv_max = nv;
    }
    const int chunks = nv_max * a.W * 2;
    const int taps = v.R * v.S;
    int CG, NPASS;
    bool tp = false;
    if (taps == 1) {
        if (chunks > 256) return pl;
        NPASS = 1;
        if (a.Cb % 8 == 0) CG = 8;
        else if (a.Cb % 4 == 0) CG = 4;
        else return pl;
    } else if (taps == 9 && v.str == 2) {
        if (a.Cb % 2 != 0 || chunks > 2048) return pl;
        CG = 2; NPASS = 8;
    } else if (a.Cb == 1 && taps > 1) {
        // a single channel block (the 3-channel stem): horizontally adjacent taps are paired instead
        if (chunks > 256 * 13) return pl;
        CG = 1; NPASS = 13; tp = true;
        if ((a.Q - 1) * v.str + ((v.S + 1) / 2) * 2 > a.Wp) a.Wp = (a.Q - 1) * v.str + ((v.S + 1) / 2) * 2;
    } else {
        if (v.str != 1 || a.Cb % 2 != 0 || chunks > 1024) return pl;
        NPASS = chunks <= 512 ? 2 : 4;
        // four channel blocks per stage when they fit two workgroups per CU, else two
        const int plane4 = ((nv_max * a.Wp * 16 + 255) / 256) * 256 + conv_plane_pad();
        CG = (a.Cb % 4 == 0 && 2 * 4 * 2 * plane4 <= 80 * 1024) ? 4 : 2;
        if (CG == 2 && NPASS == 2) NPASS = 4;   // (only the deeper copy plan is instantiated for two blocks)
    }
    pl.key = v.R * 10000 + v.S * 1000 + v.str * 100 + CG * 10 + (NPASS % 10);
    // Two feature blocks per wave halve the LDS traffic per flop, but need a grid that still fills the
    // device and a kernel variant that fits the register file (the strided 3x3 variant does not).
    pl.KW = a.Kb >= 8 ? 2 : 1;
    if (pl.KW == 2 && (grids * a.ntiles * ((a.Kb + 7) / 8) < 192 || pl.key == 33228)) pl.KW = 1;
    if (knobs().conv_kw.set) pl.KW = knobs().conv_kw.val == 1 ? 1 : (knobs().conv_kw.val == 2 && a.Kb >= 8 && pl.key != 33228 ? 2 : pl.KW);   // tuning knob
    int plane = nv_max * a.Wp * 16;
    plane = ((plane + 255) / 256) * 256 + conv_plane_pad();
    a.plane_bytes = plane;
    a.buf_bytes = CG * 2 * plane;
    pl.smem = 2 * (size_t)a.buf_bytes;
    if (pl.smem > (tp ? 150 : 80) * 1024) return pl;   // (the tap-pair kernel runs one workgroup per CU)
    a.inv_Q = 1.0f / a.Q; a.inv_P = 1.0f / a.P; a.inv_Hv = 1.0f / a.Hv; a.inv_W4 = 1.0f / (a.W * 2);
    int ktiles = (a.Kb + 4 * pl.KW - 1) / (4 * pl.KW);
    int gx = (512 / ktiles) & ~7;
    if (gx < 8) gx = 8;
    if (gx > a.ntiles) gx = a.ntiles;
    pl.grid = dim3(gx, ktiles);
    pl.ok = true;
    return pl;
}

template <int R, int S, int STR, int CG, int NPASS, int KW, bool TP = false>
static int conv_tile_bf16_go(Bf16Plan &pl, hipStream_t s)
{
    auto kern = conv_tile_bf16<R, S, STR, CG, NPASS, KW, TP, bf16_t>;
    int rc = allow_big_lds((const void *)kern, pl.smem);
    if (rc) return rc;
    hipLaunchKernelGGL(kern, pl.grid, dim3(256), pl.smem, s, pl.a);
    return check_launch("brg_conv (tiled bf16) launch");
}

template <int KW> static int conv_tile_bf16_pick(Bf16Plan &pl, hipStream_t s)
{
    switch (pl.key) {
    case 11181: return conv_tile_bf16_go<1, 1, 1, 8, 1, KW>(pl, s);
    case 11141: return conv_tile_bf16_go<1, 1, 1, 4, 1, KW>(pl, s);
    case 12142: return conv_tile_bf16_go<1, 2, 1, 4, 2, KW>(pl, s);
    case 21142: return conv_tile_bf16_go<2, 1, 1, 4, 2, KW>(pl, s);
    case 22142: return conv_tile_bf16_go<2, 2, 1, 4, 2, KW>(pl, s);
    case 33142: return conv_tile_bf16_go<3, 3, 1, 4, 2, KW>(pl, s);
    case 33228: return conv_tile_bf16_go<3, 3, 2, 2, 8, KW>(pl, s);
    case 33144: return conv_tile_bf16_go<3, 3, 1, 4, 4, KW>(pl, s);
    case 34144: return conv_tile_bf16_go<3, 4, 1, 4, 4, KW>(pl, s);
    case 43144: return conv_tile_bf16_go<4, 3, 1, 4, 4, KW>(pl, s);
    case 44144: return conv_tile_bf16_go<4, 4, 1, 4, 4, KW>(pl, s);
    case 33124: return conv_tile_bf16_go<3, 3, 1, 2, 4, KW>(pl, s);
    case 34124: return conv_tile_bf16_go<3, 4, 1, 2, 4, KW>(pl, s);
    case 43124: return conv_tile_bf16_go<4, 3, 1, 2, 4, KW>(pl, s);
    case 44124: return conv_tile_bf16_go<4, 4, 1, 2, 4, KW>(pl, s);
    case 77213: return conv_tile_bf16_go<7, 7, 2, 1, 13, KW, true>(pl, s);
    }
    return fail(BRG_EUNSUPPORTED, "brg_conv: internal: no tiled bf16 kernel for key %d", pl.key);
}

static int conv_tile_bf16_launch(Bf16Plan &pl, const void *I, const void *Wt, void *O, const float *bias, int act,
                                 hipStream_t s)
{
    pl.a.I = I; pl.a.Wt = Wt; pl.a.O = O; pl.a.bias = bias; pl.a.act = act;
    return pl.KW == 2 ? conv_tile_bf16_pick<2>(pl, s) : conv_tile_bf16_pick<1>(pl, s);
}

static bool bf16_key_known(int key)
{
    return key == 11181 || key == 11141 || key == 12142 || key == 21142 || key == 22142 || key == 33142 || key == 33228 ||
           key == 33144 || key == 34144 || key == 43144 || key == 44144 || key == 77213 || key == 33124 ||
           key == 34124 || key == 43124 || key == 44124;
}

// ---- 1x1 views in bf16: the streaming kernel (no LDS)
template <int KW, int PG> static int conv1x1_go(const Conv1x1Args &a, dim3 grid, bool wtr, hipStream_t s)
{
    if (wtr) hipLaunchKernelGGL((conv1x1_bf16<KW, PG, true>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((conv1x1_bf16<KW, PG, false>), grid, dim3(256), 0, s, a);
    return check_launch("brg_conv (1x1 bf16) launch");
}

static bool conv1x1_bf16_covers(const ConvView &v)
{
    if (v.R != 1 || v.S != 1 || v.str != 1 || v.ph != 0 || v.pw != 0 || (v.Cb & 1) || v.P <= 0 || v.Q <= 0) return false;
    if ((v.P - 1) * v.sub >= v.Hin || (v.Q - 1) * v.sub >= v.Win) return false;
    if ((v.P - 1) * v.osub + v.ooh >= v.Hout || (v.Q - 1) * v.osub + v.oow >= v.Wout) return false;
    const int64_t npix = (int64_t)v.N * v.P * v.Q;
    if (npix >= (1 << 22) || (int64_t)v.N * v.Cb * v.Hin * v.Win * 16 >= (1ll << 31) ||
        (int64_t)v.N * v.Kb * v.Hout * v.Wout * 16 >= (1ll << 31))
        return false;
    return !knobs().conv_no1x1.set;
}

// `wtr`: Wt is in the stored layout of the forward pass (feature index contiguous inside a block) and the
// kernel transposes the blocks itself; otherwise the reduction index is contiguous already (backward by
// data).  The split-reduction variant has no transposing form: with `wtr` it takes a transposed copy that
// a pre-pass writes into `ws`, and is not chosen when there is no workspace.
// `zsib`: (backward by data, output stride 2 at offset 0) the kernel also writes the zero pixels between the
// written ones.
static int conv1x1_bf16_launch(const ConvView &v, const void *I, const void *Wt, void *O, const float *bias, int act,
                               bool wtr, void *ws, hipStream_t s, bool zsib = false)
{
    const int64_t npix = (int64_t)v.N * v.P * v.Q;
    Conv1x1Args a = {};
    a.I = I; a.Wt = Wt; a.O = O; a.bias = bias; a.act = act;
    a.N = v.N; a.Cb = v.Cb; a.Kb = v.Kb; a.P = v.P; a.Q = v.Q;
    a.Hin = v.Hin; a.Win = v.Win; a.sub = v.sub;
    a.Hout = v.Hout; a.Wout = v.Wout; a.osub = v.osub; a.ooh = v.ooh; a.oow = v.oow;
    a.w_ob = v.w_ob; a.w_ib = v.w_ib; a.wtap = v.wtap[0];
    a.npix = (int)npix; a.inv_PQ = 1.0f / (float)(v.P * v.Q); a.inv_Q = 1.0f / (float)v.Q;
    a.zsib = zsib ? 1 : 0;
    // feature blocks per wave / pixel groups per wave: as large as still leaves ~2 waves per SIMD
    int KW = v.Kb >= 16 ? 4 : (v.Kb >= 8 ? 2 : 1), PG = 4;
    auto waves = [&](int kw, int pg) { return ((npix + 16 * pg - 1) / (16 * pg)) * ((v.Kb + kw - 1) / kw); };
    if (waves(KW, PG) < 2048) PG = 2;
    while (KW > 1 && waves(KW, PG) < 2048) KW >>= 1;
    if (knobs().conv_1x1_kw.set) { int x = knobs().conv_1x1_kw.val; if (x == 1 || x == 2 || x == 4) KW = x; }   // tuning knobs
    if (knobs().conv_1x1_pg.set) { int x = knobs().conv_1x1_pg.val; if (x == 2 || x == 4) PG = x; }
    // long reduction on few pixels: the workgroup-tiled kernel (operands shared through LDS), when all its
    // workgroups are resident at once (two per CU); with at most half as many 128 x 128 tiles as CUs, 128 x 64 tiles
    {
        const int units = v.Cb >> 1;
        const int64_t t128 = ((npix + 127) / 128) * ((v.Kb + 7) / 8);
        bool tiled = v.Cb >= 32 && units % 4 == 0 && t128 <= 512;
        // strided layers (sub-sampled input forward, every second output pixel backward) also gain with more
        // tiles than that: the streaming kernel's scattered lines cost it more than the tiled one
        const bool strided = (v.sub == 2 || v.osub == 2) && v.Cb >= 16 && units % 4 == 0;
        tiled = tiled || strided;
        if (knobs().conv_1x1_lds.set) tiled = knobs().conv_1x1_lds.val != 0 && units % 4 == 0;   // tuning knobs
        int ngw = (t128 <= 128 || (v.osub == 2 && t128 > 512)) ? 2 : 4;
        if (knobs().conv_1x1_lds_ngw.set) { int x = knobs().conv_1x1_lds_ngw.val; if (x == 2 || x == 4) ngw = x; }
        if (tiled) {
            a.tiles_x = (int)((npix + 32 * ngw - 1) / (32 * ngw));
            a.tiles_y = (v.Kb + 7) / 8;
            a.tiles = a.tiles_x * a.tiles_y;
            a.inv_tiles_x = 1.0f / (float)a.tiles_x;
            a.inv_tiles_y = 1.0f / (float)a.tiles_y;
            // stream the smaller operand through each XCD's L2 (activation bytes count with the lines that a
            // sub-sampled read wastes)
            a.pixel_major = npix * v.Cb * 32 * v.sub > (int64_t)v.Kb * v.Cb * 512;
            if (knobs().conv_1x1_lds_pm.set) a.pixel_major = knobs().conv_1x1_lds_pm.val != 0;   // tuning knob
            dim3 g3((unsigned)a.tiles);
            if (ngw == 4) {
                if (wtr) hipLaunchKernelGGL((conv1x1_bf16_lds<true, 4, 4>), g3, dim3(256), 0, s, a);
                else hipLaunchKernelGGL((conv1x1_bf16_lds<false, 4, 4>), g3, dim3(256), 0, s, a);
            } else {
                if (wtr) hipLaunchKernelGGL((conv1x1_bf16_lds<true, 4, 2>), g3, dim3(256), 0, s, a);
                else hipLaunchKernelGGL((conv1x1_bf16_lds<false, 4, 2>), g3, dim3(256), 0, s, a);
            }
            return check_launch("brg_conv (1x1 bf16, workgroup-tiled) launch");
        }
    }
    // deep reduction on few pixels: split the channel blocks between the waves of a workgroup
    bool split = v.Cb >= 64 && v.Kb <= 32 && npix <= 16384;
    if (knobs().conv_1x1_split.set) split = knobs().conv_1x1_split.val != 0 && v.Cb >= 8;   // tuning knob
    if ((wtr && !ws) || zsib) split = false;
    if (split) {
        if (wtr) {
            if (!aligned16(ws)) return fail(BRG_EALIGN, "brg_conv_fwd: workspace not 16-byte aligned");
            const int64_t nblk = (int64_t)v.Kb * v.Cb;
            hipLaunchKernelGGL(conv_wt_transpose_bf16, dim3((unsigned)((nblk + 7) / 8)), dim3(256), 0, s, (const bf16_t *)Wt,
                               (bf16_t *)ws, nblk);
            int rc = check_launch("brg_conv_fwd (weight transpose) launch");
            if (rc) return rc;
            a.Wt = ws;
        }
        const int kw = v.Kb >= 4 ? 4 : 2;
        dim3 g2((unsigned)((npix + 31) / 32), (unsigned)((v.Kb + kw - 1) / kw));
        if (kw == 4) hipLaunchKernelGGL((conv1x1_bf16_splitc<4, 2>), g2, dim3(256), 0, s, a);
        else hipLaunchKernelGGL((conv1x1_bf16_splitc<2, 2>), g2, dim3(256), 0, s, a);
        return check_launch("brg_conv (1x1 bf16, split reduction) launch");
    }
    int wf = 4;
    if (knobs().conv_1x1_wf.set) { int x = knobs().conv_1x1_wf.val; if (x == 1 || x == 2 || x == 4) wf = x; }
    a.wf_log2 = wf == 4 ? 2 : (wf == 2 ? 1 : 0);
    const int64_t nchunk = (npix + 16 * PG - 1) / (16 * PG);
    dim3 grid((unsigned)((nchunk + 4 / wf - 1) / (4 / wf)), (unsigned)((v.Kb + wf * KW - 1) / (wf * KW)));
    if (PG == 4) {
        if (KW == 4) return conv1x1_go<4, 4>(a, grid, wtr, s);
        if (KW == 2) return conv1x1_go<2, 4>(a, grid, wtr, s);
        return conv1x1_go<1, 4>(a, grid, wtr, s);
    }
    if (KW == 4) return conv1x1_go<4, 2>(a, grid, wtr, s);
    if (KW == 2) return conv1x1_go<2, 2>(a, grid, wtr, s);
    return conv1x1_go<1, 2>(a, grid, wtr, s);
}

// ---- few output pixels (a small minibatch): feature blocks first, and the chain divided too
struct ConvSmallPlan {
    bool ok;
    int KW, PG, gz, upp;
    int64_t ws_bytes;   // fp32 partial results when gz > 1
};

// `can_split`: a workspace may carry partial results (forward pass).  Chosen when tiling pixels x feature blocks
// alone cannot give every CU a workgroup, or when BRG_CONV_SMALL=1 asks for it on any shape the kernel covers.
static ConvSmallPlan conv_small_plan(const ConvView &v, bool can_split)
{
    ConvSmallPlan pl = {};
    const int taps = v.R * v.S;
    const int64_t npix = (int64_t)v.N * v.P * v.Q;
    if (v.R > 4 || v.S > 4 || taps > 16 || (v.Cb & 1) || v.P <= 0 || v.Q <= 0 || v.str < 1 || v.str > 2 || v.ph < 0 || v.pw < 0) return pl;
    // (the input below 2 GiB: the kernel's out-of-range offset must lie beyond it)
    if (npix * v.Kb >= (1 << 22) || (int64_t)v.N * v.Cb * v.Hin * v.Win * 32 >= (1ll << 31) ||
        (int64_t)v.N * v.Kb * v.Hout * v.Wout * 16 >= (1ll << 31))
        return pl;
    if ((v.P - 1) * v.osub + v.ooh >= v.Hout || (v.Q - 1) * v.osub + v.oow >= v.Wout) return pl;
    if ((v.H - 1) * v.sub >= v.Hin || (v.W - 1) * v.sub >= v.Win) return pl;
    const int dr = v.R > 1 ? v.wtap[v.S] - v.wtap[0] : 0, ds = v.S > 1 ? v.wtap[1] - v.wtap[0] : 0;
    for (int t = 0; t < taps; ++t)   // the kernel steps through the taps with one stride per direction
        if (v.wtap[t] != v.wtap[0] + (t / v.S) * dr + (t % v.S) * ds) return pl;
    if (knobs().conv_small.set && knobs().conv_small.val == 0) return pl;
    const int units = (v.Cb >> 1) * taps;
    if (units >= 4096) return pl;   // (the kernel's multiply-and-shift divisions)
    const int groups = (int)((npix + 15) / 16);
    // operand reuse per wave as long as the grid still covers the device
    int KW = v.Kb >= 2 ? 2 : 1, PG = groups >= 2 ? 2 : 1;
    auto wgs = [&](int kw, int pg) { return (int64_t)((groups + pg - 1) / pg) * ((v.Kb + kw - 1) / kw); };
    if (wgs(KW, PG) < 256) PG = 1;
    if (wgs(KW, PG) < 256) KW = 1;
    const bool forced = knobs().conv_small.on();
    // with enough pixels for the tiled kernels this kernel (no operand sharing between workgroups) loses
    if (!forced && wgs(2, 2) > 512) return pl;
    if (knobs().conv_small_kw.set) { int x = knobs().conv_small_kw.val; if (x == 1 || x == 2) KW = x; }   // tuning knobs
    if (knobs().conv_small_pg.set) { int x = knobs().conv_small_pg.val; if (x == 1 || x == 2) PG = x; }
    // Ranges of the chain.  The second pass costs about as much as 16 chain units of a wave, so only long chains
    // are divided (at most 40 units per wave), or chains of a grid that leaves most CUs without a workgroup.
    int gz = 1;
    if (can_split) {
        gz = (units + 159) / 160;
        const int64_t w = wgs(KW, PG);
        if (w < 64) {
            int fill = (int)(128 / w);
            if (fill > units / 16) fill = units / 16;
            if (fill > gz) gz = fill;
        }
        if (gz > 16) gz = 16;
        if (gz < 1) gz = 1;
        if (knobs().conv_small_gz.set) { int x = knobs().conv_small_gz.val; if (x >= 1 && x <= 16 && x <= units) gz = x; }
    }
    pl.upp = (units + gz - 1) / gz;
    gz = (units + pl.upp - 1) / pl.upp;   // (no empty range)
    pl.KW = KW; pl.PG = PG; pl.gz = gz;
    pl.ws_bytes = gz > 1 ? (int64_t)gz * v.Kb * npix * 64 : 0;
    pl.ok = true;
    return pl;
}

template <int KW, int PG> static void conv_small_go(const ConvSmallArgs &a, dim3 grid, bool wtr, hipStream_t s)
{
    if (wtr) hipLaunchKernelGGL((conv_small_bf16<KW, PG, true>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((conv_small_bf16<KW, PG, false>), grid, dim3(256), 0, s, a);
}

static int conv_small_launch(const ConvView &v, const ConvSmallPlan &pl, const void *I, const void *Wt, void *O,
                             const float *bias, int act, bool wtr, void *ws, hipStream_t s)
{
    const int64_t npix = (int64_t)v.N * v.P * v.Q;
    const int taps = v.R * v.S;
    ConvSmallArgs a = {};
    a.I = I; a.Wt = Wt; a.O = O; a.part = (float *)ws; a.bias = bias; a.act = act;
    a.N = v.N; a.Cb = v.Cb; a.Kb = v.Kb; a.P = v.P; a.Q = v.Q;
    a.Hin = v.Hin; a.Win = v.Win; a.sub = v.sub; a.H = v.H; a.W = v.W;
    a.str = v.str; a.ph = v.ph; a.pw = v.pw; a.R = v.R; a.S = v.S;
    a.Hout = v.Hout; a.Wout = v.Wout; a.osub = v.osub; a.ooh = v.ooh; a.oow = v.oow;
    a.w_ob = v.w_ob; a.w_ib = v.w_ib; a.w_t0 = v.wtap[0]; a.w_dr = v.R > 1 ? v.wtap[v.S] - v.wtap[0] : 0; a.w_ds = v.S > 1 ? v.wtap[1] - v.wtap[0] : 0;
    a.npix = (int)npix; a.units = (v.Cb >> 1) * taps; a.upp = pl.upp; a.gz = pl.gz;
    a.inv_PQ = 1.0f / (float)(v.P * v.Q); a.inv_Q = 1.0f / (float)v.Q;
    a.mdiv_taps = (65536 + taps - 1) / taps; a.mdiv_S = (65536 + v.S - 1) / v.S;
    a.in_bytes = (int)((int64_t)v.N * v.Cb * v.Hin * v.Win * 32);
    if (pl.gz > 1) {
        BRG_REQUIRE(ws != nullptr, BRG_EINVAL, "brg_conv (few pixels): internal: a divided chain without a workspace");
        BRG_REQUIRE(aligned16(ws), BRG_EALIGN, "brg_conv_fwd: workspace not 16-byte aligned");
    }
    const int groups = (int)((npix + 15) / 16);
    dim3 grid((unsigned)((groups + pl.PG - 1) / pl.PG), (unsigned)((v.Kb + pl.KW - 1) / pl.KW), (unsigned)pl.gz);
    if (pl.KW == 2 && pl.PG == 2) conv_small_go<2, 2>(a, grid, wtr, s);
    else if (pl.KW == 2) conv_small_go<2, 1>(a, grid, wtr, s);
    else if (pl.PG == 2) conv_small_go<1, 2>(a, grid, wtr, s);
    else conv_small_go<1, 1>(a, grid, wtr, s);
    int rc = check_launch("brg_conv (few pixels) launch");
    if (rc || pl.gz == 1) return rc;
    const int64_t nthr = npix * v.Kb * 4;
    hipLaunchKernelGGL(conv_small_reduce, dim3((unsigned)((nthr + 255) / 256)), dim3(256), 0, s, a);
    return check_launch("brg_conv (few pixels, sum of the ranges) launch");
}

// ---- the 7x7 stride-2 pad-3 stem with one channel block of 4 (bf16 in and out)
static bool conv_is_stem4(const ConvDims &d)
{
    return d.bc == 4 && d.C == 4 && d.R == 7 && d.S == 7 && d.sh == 2 && d.sw == 2 && d.ph == 3 && d.pw == 3 && d.Q <= 112 &&
           (int64_t)d.N * d.H * d.W * 4 < (1ll << 31) && (int64_t)d.N * d.K * d.P * d.Q < (1ll << 31) &&
           (int64_t)d.N * ((d.P + ST_TR - 1) / ST_TR) < (1 << 22);
}

static int conv_stem_fwd_launch(const ConvDims &d, const void *I, const void *Wt, void *O, const float *bias, int act,
                                void *ws, hipStream_t s)
{
    StemArgs a = {};
    a.I = I; a.Wt = Wt; a.O = O; a.bias = bias; a.act = act;
    if (ws) {   // filter rows re-packed as matrix-core operands (brg_conv_ws_bytes covers the 1 KiB per row and block)
        const int n = d.Kb * 7 * 16 * 32;
        hipLaunchKernelGGL(conv_stem_pack_weights, dim3((n + 255) / 256), dim3(256), 0, s, (const bf16_t *)Wt, (bf16_t *)ws, d.Kb);
        int rc = check_launch("brg_conv_fwd (stem weight packing) launch");
        if (rc) return rc;
        a.Wt = ws;
    }
    a.N = d.N; a.H = d.H; a.W = d.W; a.Kb = d.Kb; a.P = d.P; a.Q = d.Q;
    a.ngroups = (d.Q + 15) / 16;
    a.pitch = 32 * a.ngroups + 6;
    a.tiles_per_img = (d.P + ST_TR - 1) / ST_TR;
    a.ntiles = d.N * a.tiles_per_img;
    const size_t smem = 2 * (size_t)ST_ROWS * a.pitch * 8;
    const int ygroups = (d.Kb + 3) / 4;
    int gx = 512 / ygroups;
    if (gx < 1) gx = 1;
    if (gx > a.ntiles) gx = a.ntiles;
    if (ws) hipLaunchKernelGGL((conv_stem_fwd_bf16<4, true>), dim3(gx, ygroups), dim3(256), smem, s, a);
    else hipLaunchKernelGGL((conv_stem_fwd_bf16<4, false>), dim3(gx, ygroups), dim3(256), smem, s, a);
    return check_launch("brg_conv_fwd (stem) launch");
}

template <int TR, int TS> static int conv_stem_bwd_go(const StemBwdArgs &a, hipStream_t s)
{
    const size_t smem = 2 * (size_t)SB_ROWS * a.pitch * 64;
    auto kern = conv_stem_bwd_bf16<TR, TS>;
    int rc = allow_big_lds((const void *)kern, smem);
    if (rc) return rc;
    int gx = a.ntiles < 512 ? a.ntiles : 512;
    hipLaunchKernelGGL(kern, dim3(gx), dim3(256), smem, s, a);
    return check_launch("brg_conv_bwd_data (stem) launch");
}

// one launch per parity class of the input pixels; every pixel belongs to a class with 3 or 4 taps per direction
static int conv_stem_bwd_launch(const ConvDims &d, const void *dO, const void *Wt, void *dI, hipStream_t s)
{
    // 64 features on an even-sized image: all four parity classes in one pass over dO
    if (d.Kb == 4 && d.H == 2 * d.P && d.W == 2 * d.Q && !knobs().conv_stem_classes.set) {
        StemBwdFusedArgs a = {};
        a.dO = dO; a.Wt = Wt; a.dI = dI;
        a.N = d.N; a.H = d.H; a.W = d.W; a.P = d.P; a.Q = d.Q;
        a.tiles_r = (d.P + SF_T - 1) / SF_T; a.tiles_c = (d.Q + SF_T - 1) / SF_T;
        a.ntiles = d.N * a.tiles_r * a.tiles_c;
        int gx = a.ntiles < 512 ? a.ntiles : 512;
        if (knobs().conv_stem_gx.set) { int x = knobs().conv_stem_gx.val; if (x > 0 && x <= a.ntiles) gx = x; }   // tuning knob
        hipLaunchKernelGGL(conv_stem_bwd_fused_bf16, dim3(gx), dim3(256), 0, s, a);
        return check_launch("brg_conv_bwd_data (stem, fused classes) launch");
    }
    for (int ca = 0; ca < 2; ++ca)
        for (int cb = 0; cb < 2; ++cb) {
            StemBwdArgs a = {};
            a.dO = dO; a.Wt = Wt; a.dI = dI;
            a.N = d.N; a.H = d.H; a.W = d.W; a.Kb = d.Kb; a.P = d.P; a.Q = d.Q;
            a.ca = ca; a.cb = cb;
            a.Hc = (d.H - ca + 1) / 2; a.Wc = (d.W - cb + 1) / 2;
            if (a.Hc <= 0 || a.Wc <= 0) continue;
            a.ngroups = (a.Wc + 15) / 16;
            a.pitch = 16 * a.ngroups + 3;
            a.tiles_per_img = (a.Hc + SB_TR - 1) / SB_TR;
            a.ntiles = d.N * a.tiles_per_img;
            int rc;
            if (ca == 0 && cb == 0) rc = conv_stem_bwd_go<3, 3>(a, s);
            else if (ca == 0) rc = conv_stem_bwd_go<3, 4>(a, s);
            else if (cb == 0) rc = conv_stem_bwd_go<4, 3>(a, s);
            else rc = conv_stem_bwd_go<4, 4>(a, s);
            if (rc) return rc;
        }
    return BRG_OK;
}

// forward view of a layer
static bool conv_fwd_view(const ConvDims &d, ConvView *v)
{
    if (d.sh != d.sw || d.sh > 2) return false;
    *v = ConvView{};
    v->N = d.N; v->Cb = d.Cb; v->Hin = d.H; v->Win = d.W; v->sub = 1; v->H = d.H; v->W = d.W;
    v->Kb = d.Kb; v->P = d.P; v->Q = d.Q; v->Hout = d.P; v->Wout = d.Q; v->osub = 1;
    v->R = d.R; v->S = d.S; v->str = d.sh; v->ph = d.ph; v->pw = d.pw;
    v->w_ob = d.Cb * d.R * d.S; v->w_ib = d.R * d.S;
    if (d.R * d.S > 16 && d.Cb != 1) return false;
    for (int t = 0; t < d.R * d.S && t < 16; ++t) v->wtap[t] = t;
    if (d.R == 1 && d.S == 1 && d.sh > 1) {   // a stride-1 pass over the sub-sampled image
        if (d.ph || d.pw) return false;
        v->sub = d.sh; v->H = d.P; v->W = d.Q; v->str = 1;
    }
    return true;
}

// Backward by data: the input pixels (h, w) with h % stride == a, w % stride == b form parity class
// (a, b).  Within a class, pixel h = stride*i + a receives taps r = r0 + stride*j (r0 = (a + pad) %
// stride) from dO row i + q0 - j (q0 = (a + pad) / stride): a stride-1 forward-style pass over dO with
// R' = #taps rows, top padding R' - 1 - q0 and kernel tap r' = R' - 1 - j.  Returns false when the class
// has no taps (its pixels are zero).
static bool conv_bwd_view(const ConvDims &d, int ca, int cb, ConvView *v)
{
    const int r0 = (ca + d.ph) % d.sh, s0 = (cb + d.pw) % d.sw;
    const int Rc = r0 < d.R ? (d.R - r0 + d.sh - 1) / d.sh : 0, Sc = s0 < d.S ? (d.S - s0 + d.sw - 1) / d.sw : 0;
    const int Hc = ca < d.H ? (d.H - ca + d.sh - 1) / d.sh : 0, Wc = cb < d.W ? (d.W - cb + d.sw - 1) / d.sw : 0;
    if (Rc == 0 || Sc == 0 || Hc == 0 || Wc == 0) return false;
    *v = ConvView{};
    v->N = d.N; v->Cb = d.Kb; v->Hin = d.P; v->Win = d.Q; v->sub = 1; v->H = d.P; v->W = d.Q;
    v->Kb = d.Cb; v->P = Hc; v->Q = Wc; v->Hout = d.H; v->Wout = d.W; v->osub = d.sh; v->ooh = ca; v->oow = cb;
    v->R = Rc; v->S = Sc; v->str = 1;
    v->ph = Rc - 1 - (ca + d.ph) / d.sh; v->pw = Sc - 1 - (cb + d.pw) / d.sw;
    v->w_ob = d.R * d.S; v->w_ib = d.Cb * d.R * d.S;
    if (Rc * Sc > 16 || v->ph < 0 || v->pw < 0) { v->R = 99; return true; }   // not expressible: caller falls back
    for (int rp = 0; rp < Rc; ++rp)
        for (int sp = 0; sp < Sc; ++sp)
            v->wtap[rp * Sc + sp] = (r0 + d.sh * (Rc - 1 - rp)) * d.S + (s0 + d.sw * (Sc - 1 - sp));
    return true;
}

template <typename TIn, typename TOut>
static int conv_fwd_launch(const ConvDims &d, const void *I, const void *Wt, void *O, const float *bias,
                           int act, hipStream_t s)
{
    ConvFwdProb<TIn, TOut> p;
    p.d = d; p.I = (const TIn *)I; p.Wt = (const TIn *)Wt; p.O = (TOut *)O; p.bias = bias; p.act = act;
    p.tiles_m = (d.K + ENG_TM - 1) / ENG_TM;
    p.npix = (int64_t)d.N * d.P * d.Q;
    int64_t tiles_n = (p.npix + ENG_TN - 1) / ENG_TN;
    BRG_REQUIRE(p.tiles_m * tiles_n < (1ll << 31), BRG_EUNSUPPORTED, "brg_conv_fwd: grid too large");
    hipLaunchKernelGGL((engine_kernel<ConvFwdProb<TIn, TOut>>), dim3((unsigned)(p.tiles_m * tiles_n)), dim3(256), 0,
                       s, p);
    return check_launch("brg_conv_fwd launch");
}

template <typename TIn, typename TOut>
static int conv_bwd_data_launch(const ConvDims &d, const void *dO, const void *Wt, void *dI, hipStream_t s)
{
    ConvBwdDataProb<TIn, TOut> p;
    p.d = d; p.dO = (const TIn *)dO; p.Wt = (const TIn *)Wt; p.dI = (TOut *)dI;
    p.tiles_m = (d.C + ENG_TM - 1) / ENG_TM;
    p.npix = (int64_t)d.N * d.H * d.W;
    int64_t tiles_n = (p.npix + ENG_TN - 1) / ENG_TN;
    BRG_REQUIRE(p.tiles_m * tiles_n < (1ll << 31), BRG_EUNSUPPORTED, "brg_conv_bwd_data: grid too large");
    hipLaunchKernelGGL((engine_kernel<ConvBwdDataProb<TIn, TOut>>), dim3((unsigned)(p.tiles_m * tiles_n)), dim3(256),
                       0, s, p);
    return check_launch("brg_conv_bwd_data launch");
}

template <typename TIn>
static int conv_bwd_wgt_launch(const ConvDims &d, const void *I, const void *dO, float *dWt, hipStream_t s)
{
    ConvBwdWgtProb<TIn> p;
    p.d = d; p.I = (const TIn *)I; p.dO = (const TIn *)dO; p.dWt = dWt;
    p.tiles_m = (d.K + ENG_TM - 1) / ENG_TM;
    int tiles_n = (d.C + ENG_TN - 1) / ENG_TN;
    hipLaunchKernelGGL((engine_kernel<ConvBwdWgtProb<TIn>>), dim3(p.tiles_m * tiles_n, d.R * d.S), dim3(256), 0, s,
                       p);
    return check_launch("brg_conv_bwd_wgt launch");
}

}  // namespace brg

extern "C" int brg_conv_fwd(const brg_conv_desc_t *desc, brg_dtype_t dtype, brg_dtype_t out_dtype,
                            const void *I, const void *Wt, void *O, const float *bias, brg_act_t act,
                            void *ws, brg_stream_t stream)
{
    using namespace brg;
    ConvDims d;
    int rc = conv_dims(desc, &d, "brg_conv_fwd");
    if (rc) return rc;
    BRG_REQUIRE(valid_dtype(dtype) && valid_dtype(out_dtype), BRG_EINVAL, "brg_conv_fwd: bad dtype");
    BRG_REQUIRE(valid_act(act), BRG_EINVAL, "brg_conv_fwd: bad activation %d", (int)act);
    BRG_REQUIRE(I && Wt && O, BRG_EINVAL, "brg_conv_fwd: null tensor");
    BRG_REQUIRE(aligned16(I) && aligned16(Wt) && aligned16(O) && aligned16(bias), BRG_EALIGN,
                "brg_conv_fwd: pointer not 16-byte aligned");
    hipStream_t s = (hipStream_t)stream;
    if (d.bc != 16) {
        BRG_REQUIRE(dtype == BRG_BF16 && out_dtype == BRG_BF16 && conv_is_stem4(d), BRG_EUNSUPPORTED,
                    "brg_conv_fwd: a channel block of 4 is only supported for the bf16 7x7 stride-2 pad-3 layer");
        BRG_REQUIRE(aligned16(ws), BRG_EALIGN, "brg_conv_fwd: workspace not 16-byte aligned");
        return conv_stem_fwd_launch(d, I, Wt, O, bias, act, ws, s);
    }
    if (dtype == BRG_F32 && out_dtype == BRG_F32) {
        ConvTilePlan pl = plan_conv_tile(d, false);
        if (pl.ok && !knobs().conv_general.set) {
            if (ws) {
                // weights: every 16x16 block transposed into the workspace: one float4 per matrix-core operand
                BRG_REQUIRE(aligned16(ws), BRG_EALIGN, "brg_conv_fwd: workspace not 16-byte aligned");
                const int64_t nblk = (int64_t)d.Kb * d.Cb * d.R * d.S;
                hipLaunchKernelGGL(conv_wt_transpose_f32, dim3((unsigned)nblk), dim3(256), 0, s, (const float *)Wt, (float *)ws, nblk);
                rc = check_launch("brg_conv_fwd (weight transpose) launch");
                if (rc) return rc;
                return conv_tile_f32_launch<2>(pl, I, ws, O, bias, act, s);
            }
            return conv_tile_f32_launch<0>(pl, I, Wt, O, bias, act, s);
        }
        return conv_fwd_launch<float, float>(d, I, Wt, O, bias, act, s);
    }
    if (dtype == BRG_BF16 && out_dtype == BRG_F32) return conv_fwd_launch<bf16_t, float>(d, I, Wt, O, bias, act, s);
    if (dtype == BRG_BF16 && out_dtype == BRG_BF16) {
        ConvView v;
        Bf16Plan pl;
        pl.ok = false;
        const bool have_view = conv_fwd_view(d, &v);
        if (have_view && !knobs().conv_general.set) {
            // (a workspace sized by brg_conv_ws_bytes holds the partial results of the plan made here)
            const ConvSmallPlan sp = conv_small_plan(v, ws != nullptr);
            if (sp.ok) return conv_small_launch(v, sp, I, Wt, O, bias, act, true, ws, s);
        }
        const bool is1x1 = have_view && conv1x1_bf16_covers(v);
        if (have_view && !is1x1) pl = plan_view_bf16(v);
        if (is1x1 && !knobs().conv_general.set) return conv1x1_bf16_launch(v, I, Wt, O, bias, act, true, ws, s);
        if (pl.ok && bf16_key_known(pl.key) && ws && !knobs().conv_general.set) {
            // weights: every 16x16 block transposed into the workspace, so that the reduction index is
            // contiguous for the matrix-core operand loads
            BRG_REQUIRE(aligned16(ws), BRG_EALIGN, "brg_conv_fwd: workspace not 16-byte aligned");
            const int64_t nblk = (int64_t)d.Kb * d.Cb * d.R * d.S;
            hipLaunchKernelGGL(conv_wt_transpose_bf16, dim3((unsigned)((nblk + 7) / 8)), dim3(256), 0, s, (const bf16_t *)Wt,
                               (bf16_t *)ws, nblk);
            rc = check_launch("brg_conv_fwd (weight transpose) launch");
            if (rc) return rc;
            return conv_tile_bf16_launch(pl, I, ws, O, bias, act, s);
        }
        return conv_fwd_launch<bf16_t, bf16_t>(d, I, Wt, O, bias, act, s);
    }
    return fail(BRG_EUNSUPPORTED, "brg_conv_fwd: fp32 inputs with bf16 output are not supported");
}

extern "C" int brg_conv_bwd_data(const brg_conv_desc_t *desc, brg_dtype_t dtype, brg_dtype_t out_dtype,
                                 const void *dO, const void *Wt, void *dI, void *ws, brg_stream_t stream)
{
    using namespace brg;
    (void)ws;
    ConvDims d;
    int rc = conv_dims(desc, &d, "brg_conv_bwd_data");
    if (rc) return rc;
    BRG_REQUIRE(valid_dtype(dtype) && valid_dtype(out_dtype), BRG_EINVAL, "brg_conv_bwd_data: bad dtype");
    BRG_REQUIRE(dO && Wt && dI, BRG_EINVAL, "brg_conv_bwd_data: null tensor");
    BRG_REQUIRE(aligned16(dO) && aligned16(Wt) && aligned16(dI), BRG_EALIGN,
                "brg_conv_bwd_data: pointer not 16-byte aligned");
    hipStream_t s = (hipStream_t)stream;
    if (d.bc != 16) {
        BRG_REQUIRE(dtype == BRG_BF16 && out_dtype == BRG_BF16 && conv_is_stem4(d) && d.W <= 224, BRG_EUNSUPPORTED,
                    "brg_conv_bwd_data: a channel block of 4 is only supported for the bf16 7x7 stride-2 pad-3 layer");
        return conv_stem_bwd_launch(d, dO, Wt, dI, s);
    }
    if (dtype == BRG_F32 && out_dtype == BRG_F32) {
        ConvTilePlan pl = plan_conv_tile(d, true);
        if (pl.ok && !knobs().conv_general.set)
            return conv_tile_f32_launch<1>(pl, dO, Wt, dI, nullptr, BRG_ACT_NONE, s);
        // stride 2: one tiled pass per parity class of the input pixels; classes without a tap are zero-filled
        if (d.sh == 2 && d.sw == 2 && !knobs().conv_general.set) {
            ConvTilePlan plans[4];
            int svals[4];
            int np = 0;
            bool all_ok = true, holes = false;
            for (int ca = 0; ca < 2 && all_ok; ++ca)
                for (int cb = 0; cb < 2 && all_ok; ++cb) {
                    ConvView v;
                    if (!conv_bwd_view(d, ca, cb, &v)) {
                        if (ca < d.H && cb < d.W) holes = true;
                        continue;
                    }
                    if (v.R == 99) { all_ok = false; break; }
                    plans[np] = plan_view_f32(v);
                    svals[np] = v.S;
                    all_ok = plans[np].ok;
                    ++np;
                }
            if (all_ok && np > 0) {
                if (holes) {
                    const int64_t n16 = (int64_t)d.N * d.C * d.H * d.W * 4 / 16;
                    hipLaunchKernelGGL(conv_zero_fill, dim3(2048), dim3(256), 0, s, (float4v *)dI, n16);
                    rc = check_launch("brg_conv_bwd_data (zero fill) launch");
                    if (rc) return rc;
                }
                for (int i = 0; i < np; ++i) {
                    rc = conv_tile_f32_view_launch(plans[i], svals[i], dO, Wt, dI, s);
                    if (rc) return rc;
                }
                return BRG_OK;
            }
        }
        return conv_bwd_data_launch<float, float>(d, dO, Wt, dI, s);
    }
    if (dtype == BRG_BF16 && out_dtype == BRG_F32) return conv_bwd_data_launch<bf16_t, float>(d, dO, Wt, dI, s);
    if (dtype == BRG_BF16 && out_dtype == BRG_BF16) {
        // one tiled pass per stride x stride parity class of the input pixels
        if (d.sh == d.sw && d.sh <= 2 && !knobs().conv_general.set) {
            Bf16Plan plans[4];
            ConvSmallPlan smalls[4];
            ConvView views[4];
            int np = 0, nclass = d.sh * d.sw;
            bool all_ok = true, holes = false;
            for (int ca = 0; ca < d.sh && all_ok; ++ca)
                for (int cb = 0; cb < d.sw && all_ok; ++cb) {
                    ConvView v;
                    if (!conv_bwd_view(d, ca, cb, &v)) {
                        if (ca < d.H && cb < d.W) holes = true;   // a class without taps: its pixels are zero
                        continue;
                    }
                    if (v.R == 99) { all_ok = false; break; }
                    views[np] = v;
                    smalls[np] = conv_small_plan(v, false);
                    if (smalls[np].ok || conv1x1_bf16_covers(v)) {
                        plans[np].ok = false;
                    } else {
                        // (the 1x2, 2x1 and 2x2-tap classes of a strided 3x3 layer run as one grid)
                        plans[np] = plan_view_bf16(v, d.R == 3 && d.S == 3 && d.sh == 2 ? 3 : 1);
                        all_ok = plans[np].ok && bf16_key_known(plans[np].key);
                    }
                    ++np;
                }
            (void)nclass;
            if (all_ok && np > 0) {
                // 1x1 with stride 2: only class (0, 0) has a tap; its kernel writes the zero pixels itself
                const bool zsib = holes && np == 1 && d.sh == 2 && !smalls[0].ok && conv1x1_bf16_covers(views[0]) && views[0].osub == 2 &&
                                  views[0].ooh == 0 && views[0].oow == 0 && !knobs().conv_zerofill.set;
                if (zsib) return conv1x1_bf16_launch(views[0], dO, Wt, dI, nullptr, BRG_ACT_NONE, false, nullptr, s, true);
                if (holes) {
                    const int64_t n16 = (int64_t)d.N * d.C * d.H * d.W * 2 / 16;
                    hipLaunchKernelGGL(conv_zero_fill, dim3(2048), dim3(256), 0, s, (float4v *)dI, n16);
                    rc = check_launch("brg_conv_bwd_data (zero fill) launch");
                    if (rc) return rc;
                }
                // stride-2 3x3: the 1x2, 2x1 and 2x2 classes as one grid when their plans agree
                int fused[3] = {-1, -1, -1};
                for (int i = 0; i < np; ++i)
                    if (plans[i].ok) {
                        if (plans[i].key == 12142) fused[0] = i;
                        if (plans[i].key == 21142) fused[1] = i;
                        if (plans[i].key == 22142) fused[2] = i;
                    }
                bool fuse = fused[0] >= 0 && fused[1] >= 0 && fused[2] >= 0 && !knobs().conv_nofuse.set;
                for (int j = 1; j < 3 && fuse; ++j) {
                    const Bf16Plan &p0 = plans[fused[0]], &pj = plans[fused[j]];
                    fuse = p0.KW == pj.KW && p0.grid.x == pj.grid.x && p0.grid.y == pj.grid.y;
                }
                if (fuse) {
                    ConvTileArgs3 a3;
                    size_t smem = 0;
                    for (int j = 0; j < 3; ++j) {
                        Bf16Plan &pj = plans[fused[j]];
                        pj.a.I = dO; pj.a.Wt = Wt; pj.a.O = dI; pj.a.bias = nullptr; pj.a.act = BRG_ACT_NONE;
                        a3.c[j] = pj.a;
                        if (pj.smem > smem) smem = pj.smem;
                    }
                    const Bf16Plan &p0 = plans[fused[0]];
                    dim3 g3(p0.grid.x, p0.grid.y, 3);
                    if (p0.KW == 2) {
                        rc = allow_big_lds((const void *)conv_tile_bf16_s2bwd<2>, smem);
                        if (rc) return rc;
                        hipLaunchKernelGGL(conv_tile_bf16_s2bwd<2>, g3, dim3(256), smem, s, a3);
                    } else {
                        rc = allow_big_lds((const void *)conv_tile_bf16_s2bwd<1>, smem);
                        if (rc) return rc;
                        hipLaunchKernelGGL(conv_tile_bf16_s2bwd<1>, g3, dim3(256), smem, s, a3);
                    }
                    rc = check_launch("brg_conv_bwd_data (tiled bf16, three classes) launch");
                    if (rc) return rc;
                }
                for (int i = 0; i < np; ++i) {
                    if (fuse && (i == fused[0] || i == fused[1] || i == fused[2])) continue;
                    if (smalls[i].ok) rc = conv_small_launch(views[i], smalls[i], dO, Wt, dI, nullptr, BRG_ACT_NONE, false, nullptr, s);
                    else
                        rc = conv1x1_bf16_covers(views[i]) ? conv1x1_bf16_launch(views[i], dO, Wt, dI, nullptr, BRG_ACT_NONE, false, nullptr, s)
                                                           : conv_tile_bf16_launch(plans[i], dO, Wt, dI, nullptr, BRG_ACT_NONE, s);
                    if (rc) return rc;
                }
                return BRG_OK;
            }
        }
        return conv_bwd_data_launch<bf16_t, bf16_t>(d, dO, Wt, dI, s);
    }
    return fail(BRG_EUNSUPPORTED, "brg_conv_bwd_data: fp32 inputs with bf16 output are not supported");
}

extern "C" int brg_conv_bwd_wgt(const brg_conv_desc_t *desc, brg_dtype_t dtype, const void *I,
                                const void *dO, float *dWt, void *ws, brg_stream_t stream)
{
    using namespace brg;
    ConvDims d;
    int rc = conv_dims(desc, &d, "brg_conv_bwd_wgt");
    if (rc) return rc;
    BRG_REQUIRE(valid_dtype(dtype), BRG_EINVAL, "brg_conv_bwd_wgt: bad dtype");
    BRG_REQUIRE(I && dO && dWt, BRG_EINVAL, "brg_conv_bwd_wgt: null tensor");
    BRG_REQUIRE(aligned16(I) && aligned16(dO) && aligned16(dWt) && aligned16(ws), BRG_EALIGN,
                "brg_conv_bwd_wgt: pointer not 16-byte aligned");
    hipStream_t s = (hipStream_t)stream;
    const ConvWgtPlan wp = conv_wgt_plan(d.N, d.C, d.H, d.W, d.K, d.R, d.S, d.sh, d.sw, d.ph, d.pw, d.bc, d.bk, dtype == BRG_F32);
    BRG_REQUIRE(d.bc == 16 || (wp.ok && wp.stem && (wp.nsplit == 1 || ws)), BRG_EUNSUPPORTED,
                "brg_conv_bwd_wgt: a channel block of 4 is only supported for the bf16 7x7 stride-2 pad-3 layer with its workspace");
    if (dtype == BRG_F32 && !(wp.ok && (wp.nsplit == 1 || ws))) return conv_bwd_wgt_launch<float>(d, I, dO, dWt, s);
    if (wp.ok && (wp.nsplit == 1 || ws)) return conv_wgt_bf16_launch(wp, d.N, d.Cb, d.Kb, d.H, d.W, d.sh, I, dO, dWt, ws, s);
    return conv_bwd_wgt_launch<bf16_t>(d, I, dO, dWt, s);
}

// ---- the weight gradient for callers that cannot allocate --------------------------------------
// The partial sums of the pixel ranges go to a file-scope device array instead of a caller workspace.
// Every GPU holds its own copy of the array at its own address; that address is asked for once per
// device, with the device current, and kept.
static __device__ __align__(256) unsigned char wgt_scratch[BRG_CONV_BWD_WGT_NOALLOC_MAX_BYTES];

namespace brg {
constexpr int WGT_SCRATCH_MAXDEV = 64;
static std::atomic<void *> wgt_scratch_addr[WGT_SCRATCH_MAXDEV];

static int wgt_scratch_for_current_device(void **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(BRG_EHIP, "brg_conv_bwd_wgt_noalloc: hipGetDevice: %s", hipGetErrorString(e));
    BRG_REQUIRE(dev >= 0 && dev < WGT_SCRATCH_MAXDEV, BRG_EUNSUPPORTED, "brg_conv_bwd_wgt_noalloc: device index %d", dev);
    void *p = wgt_scratch_addr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(wgt_scratch));
        if (e != hipSuccess || !p)
            return fail(BRG_EHIP, "brg_conv_bwd_wgt_noalloc: hipGetSymbolAddress: %s", hipGetErrorString(e));
        wgt_scratch_addr[dev].store(p, std::memory_order_release);   // (two threads racing here store the same address)
    }
    *out = p;
    return BRG_OK;
}
}  // namespace brg

extern "C" int brg_conv_bwd_wgt_noalloc(const brg_conv_desc_t *desc, brg_dtype_t dtype, const void *I,
                                        const void *dO, float *dWt, brg_stream_t stream)
{
    using namespace brg;
    ConvDims d;
    int rc = conv_dims(desc, &d, "brg_conv_bwd_wgt_noalloc");
    if (rc) return rc;
    BRG_REQUIRE(valid_dtype(dtype), BRG_EINVAL, "brg_conv_bwd_wgt_noalloc: bad dtype");
    BRG_REQUIRE(I && dO && dWt, BRG_EINVAL, "brg_conv_bwd_wgt_noalloc: null tensor");
    BRG_REQUIRE(aligned16(I) && aligned16(dO) && aligned16(dWt), BRG_EALIGN,
                "brg_conv_bwd_wgt_noalloc: pointer not 16-byte aligned");
    const int64_t need = brg_conv_bwd_wgt_ws_bytes(desc, dtype);
    BRG_REQUIRE(need <= BRG_CONV_BWD_WGT_NOALLOC_MAX_BYTES, BRG_EUNSUPPORTED,
                "brg_conv_bwd_wgt_noalloc: this layer needs %lld bytes of partial sums, the built-in scratch holds %lld",
                (long long)need, (long long)BRG_CONV_BWD_WGT_NOALLOC_MAX_BYTES);
    void *scratch = nullptr;
    if (need > 0) {
        rc = wgt_scratch_for_current_device(&scratch);
        if (rc) return rc;
    }
    // Same planner and kernels as brg_conv_bwd_wgt.  Every range writes its whole partial result before the
    // range sum reads it, so nothing in the scratch has to start at zero and the previous call's contents
    // are simply overwritten.
    return brg_conv_bwd_wgt(desc, dtype, I, dO, dWt, scratch, stream);
}

extern "C" int64_t brg_conv_bwd_wgt_ws_bytes(const brg_conv_desc_t *desc, brg_dtype_t dtype)
{
    if (!desc || (dtype != BRG_BF16 && dtype != BRG_F32) || desc->N <= 0 || desc->C <= 0 || desc->K <= 0 || desc->H <= 0 || desc->W <= 0) return 0;
    if (desc->bc <= 0 || desc->bk <= 0 || desc->C % desc->bc || desc->K % desc->bk) return 0;
    return brg::conv_wgt_plan(desc->N, desc->C, desc->H, desc->W, desc->K, desc->R, desc->S, desc->stride_h, desc->stride_w,
                              desc->pad_h, desc->pad_w, desc->bc, desc->bk, dtype == BRG_F32).ws_bytes;
}

extern "C" int64_t brg_conv_ws_bytes(const brg_conv_desc_t *desc, brg_dtype_t dtype)
{
    if (!desc || desc->C <= 0 || desc->K <= 0 || desc->R <= 0 || desc->S <= 0) return 0;
    if (dtype == BRG_F32) return desc->C * desc->K * desc->R * desc->S * 4;   // a transposed copy of the fp32 weights
    if (dtype != BRG_BF16) return 0;
    const int64_t copy = desc->C * desc->K * desc->R * desc->S * 2;   // a transposed copy of the bf16 weights
    const int64_t rows = desc->K * desc->R * 64;                        // or filter rows padded to 32 elements
    if (desc->bc == 4) return rows > copy ? rows : copy;
    // or the partial results of a divided chain (few output pixels)
    if (desc->N > 0 && desc->H > 0 && desc->W > 0 && desc->stride_h > 0 && desc->stride_w > 0 && desc->pad_h >= 0 && desc->pad_w >= 0 &&
        desc->bc == 16 && desc->bk == 16 && desc->C % 16 == 0 && desc->K % 16 == 0 && desc->N < (1 << 20) && desc->C < (1 << 20) &&
        desc->K < (1 << 20) && desc->H < (1 << 15) && desc->W < (1 << 15) && desc->R < 64 && desc->S < 64 &&
        desc->H + 2 * desc->pad_h >= desc->R && desc->W + 2 * desc->pad_w >= desc->S) {
        brg::ConvDims d;
        d.N = (int)desc->N; d.C = (int)desc->C; d.H = (int)desc->H; d.W = (int)desc->W; d.K = (int)desc->K;
        d.R = (int)desc->R; d.S = (int)desc->S; d.sh = (int)desc->stride_h; d.sw = (int)desc->stride_w;
        d.ph = (int)desc->pad_h; d.pw = (int)desc->pad_w; d.bc = 16; d.bk = 16;
        d.P = (d.H + 2 * d.ph - d.R) / d.sh + 1; d.Q = (d.W + 2 * d.pw - d.S) / d.sw + 1;
        d.Cb = d.C / 16; d.Kb = d.K / 16;
        brg::ConvView v;
        if (brg::conv_fwd_view(d, &v)) {
            const brg::ConvSmallPlan sp = brg::conv_small_plan(v, true);
            if (sp.ok && sp.ws_bytes > copy) return sp.ws_bytes;
        }
    }
    return copy;
}
