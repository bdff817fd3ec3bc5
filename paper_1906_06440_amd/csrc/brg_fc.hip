// Fully connected layer on blocked layouts (paper section 3.3, Algorithm 5):
// every output block is one batch-reduce chain; bias / ReLU (forward) and the
// ReLU mask (backward) are applied on the fly, never in a separate pass.
#include <cstdlib>

#include "brg_block_dma.hpp"
#include "brg_block_ring.hpp"
#include "brg_g64.hpp"
#include "brg_g128.hpp"
#include "brg_fc_wgt_bf16.hpp"
#include "brg_h64.hpp"
#include "brg_engine.hpp"

namespace brg {

struct FcDims {
    int N, C, K, bn, bc, bk, Nb, Cb, Kb;
};

// ---- forward: Y[n][k] = act(sum_c W[k][c] X[n][c] + b[k]);  M = K, N = batch, chain over C/bc
template <typename TIn, typename TOut> struct FcFwdProb {
    static constexpr bool A_KFAST = false, B_KFAST = true;
    FcDims d;
    const TIn *X, *Wt;
    const float *bias;
    TOut *Y;
    int act, tiles_m;
    typedef int64_t RowA;
    typedef int64_t RowB;
    struct Chain {
        int64_t aoff, boff;
    };
    __device__ int m0() const { return (blockIdx.x % tiles_m) * ENG_TM; }
    __device__ int n0() const { return (blockIdx.x / tiles_m) * ENG_TN; }
    __device__ int chain_len() const { return d.Cb; }
    __device__ int kdepth(int) const { return d.bc; }
    __device__ RowA row_a(int i) const
    {
        int k = m0() + i;
        if (k >= d.K) return -1;
        return (int64_t)(k / d.bk) * d.Cb * d.bc * d.bk + k % d.bk;
    }
    __device__ RowB row_b(int j) const
    {
        int n = n0() + j;
        if (n >= d.N) return -1;
        return ((int64_t)(n / d.bn) * d.Cb * d.bn + n % d.bn) * d.bc;
    }
    __device__ Chain chain(int c) const { return Chain{(int64_t)c * d.bc * d.bk, (int64_t)c * d.bn * d.bc}; }
    __device__ float a(const Chain &ch, const RowA &r, int p) const
    {
        return r >= 0 ? to_f32<TIn>(Wt[r + ch.aoff + (int64_t)p * d.bk]) : 0.f;
    }
    __device__ float b(const Chain &ch, const RowB &r, int p) const
    {
        return r >= 0 ? to_f32<TIn>(X[r + ch.boff + p]) : 0.f;
    }
    __device__ void store4(int i, int j, float4v acc) const
    {
        int n = n0() + j;
        if (n >= d.N) return;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            int k = m0() + i + r;
            if (k >= d.K) continue;
            float v = acc[r] + (bias ? bias[k] : 0.f);
            Y[(((int64_t)(n / d.bn) * d.Kb + k / d.bk) * d.bn + n % d.bn) * d.bk + k % d.bk] =
                from_f32<TOut>(apply_act(v, act));
        }
    }
};

// ---- backward by data: dX[n][c] = sum_k W[k][c] dZ[n][k];  M = C, N = batch, chain over K/bk.
// The weight block is read transposed while it is staged; no transposed copy is made.
template <typename TIn> struct FcBwdDataProb {
    static constexpr bool A_KFAST = true, B_KFAST = true;
    FcDims d;
    const TIn *dY, *Y, *Wt;
    const TIn *Xmask;   // optional: dX is stored as dX o [Xmask > 0] (ReLU backward of the producing layer)
    TIn *dX;
    int relu, tiles_m;
    typedef int64_t RowA;
    typedef int64_t RowB;
    struct Chain {
        int64_t aoff, boff;
    };
    __device__ int m0() const { return (blockIdx.x % tiles_m) * ENG_TM; }
    __device__ int n0() const { return (blockIdx.x / tiles_m) * ENG_TN; }
    __device__ int chain_len() const { return d.Kb; }
    __device__ int kdepth(int) const { return d.bk; }
    __device__ RowA row_a(int i) const
    {
        int c = m0() + i;
        if (c >= d.C) return -1;
        return ((int64_t)(c / d.bc) * d.bc + c % d.bc) * d.bk;
    }
    __device__ RowB row_b(int j) const
    {
        int n = n0() + j;
        if (n >= d.N) return -1;
        return ((int64_t)(n / d.bn) * d.Kb * d.bn + n % d.bn) * d.bk;
    }
    __device__ Chain chain(int c) const
    {
        return Chain{(int64_t)c * d.Cb * d.bc * d.bk, (int64_t)c * d.bn * d.bk};
    }
    __device__ float a(const Chain &ch, const RowA &r, int p) const
    {
        return r >= 0 ? to_f32<TIn>(Wt[r + ch.aoff + p]) : 0.f;
    }
    __device__ float b(const Chain &ch, const RowB &r, int p) const
    {
        if (r < 0) return 0.f;
        int64_t e = r + ch.boff + p;
        if (relu && !(to_f32<TIn>(Y[e]) > 0.f)) return 0.f;
        return to_f32<TIn>(dY[e]);
    }
    __device__ void store4(int i, int j, float4v acc) const
    {
        int n = n0() + j;
        if (n >= d.N) return;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            int c = m0() + i + r;
            if (c >= d.C) continue;
            const int64_t e = (((int64_t)(n / d.bn) * d.Cb + c / d.bc) * d.bn + n % d.bn) * d.bc + c % d.bc;
            float v = acc[r];
            if (Xmask && !(to_f32<TIn>(Xmask[e]) > 0.f)) v = 0.f;
            dX[e] = from_f32<TIn>(v);
        }
    }
};

// ---- weight gradient: dW[k][c] = sum_n dZ[n][k] X[n][c];  M = K, N = C, chain over N/bn
template <typename TIn> struct FcWgtProb {
    static constexpr bool A_KFAST = false, B_KFAST = false;
    FcDims d;
    const TIn *dY, *Y, *X;
    float *dWt;
    int relu, tiles_m;
    typedef int64_t RowA;
    typedef int64_t RowB;
    struct Chain {
        int64_t aoff, boff;
    };
    __device__ int m0() const { return (blockIdx.x % tiles_m) * ENG_TM; }
    __device__ int n0() const { return (blockIdx.x / tiles_m) * ENG_TN; }
    __device__ int chain_len() const { return d.Nb; }
    __device__ int kdepth(int) const { return d.bn; }
    __device__ RowA row_a(int i) const
    {
        int k = m0() + i;
        if (k >= d.K) return -1;
        return (int64_t)(k / d.bk) * d.bn * d.bk + k % d.bk;
    }
    __device__ RowB row_b(int j) const
    {
        int c = n0() + j;
        if (c >= d.C) return -1;
        return (int64_t)(c / d.bc) * d.bn * d.bc + c % d.bc;
    }
    __device__ Chain chain(int c) const
    {
        return Chain{(int64_t)c * d.Kb * d.bn * d.bk, (int64_t)c * d.Cb * d.bn * d.bc};
    }
    __device__ float a(const Chain &ch, const RowA &r, int p) const
    {
        if (r < 0) return 0.f;
        int64_t e = r + ch.aoff + (int64_t)p * d.bk;
        if (relu && !(to_f32<TIn>(Y[e]) > 0.f)) return 0.f;
        return to_f32<TIn>(dY[e]);
    }
    __device__ float b(const Chain &ch, const RowB &r, int p) const
    {
        return r >= 0 ? to_f32<TIn>(X[r + ch.boff + (int64_t)p * d.bc]) : 0.f;
    }
    __device__ void store4(int i, int j, float4v acc) const
    {
        int c = n0() + j;
        if (c >= d.C) return;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            int k = m0() + i + r;
            if (k >= d.K) continue;
            dWt[(((int64_t)(k / d.bk) * d.Cb + c / d.bc) * d.bc + c % d.bc) * d.bk + k % d.bk] = acc[r];
        }
    }
};

// ---- bias gradient: db[k] = sum_n dZ[n][k].  One workgroup per 64 features; 4 batch
// slices per feature are summed in registers and combined through LDS (no atomics, so the
// result is bitwise reproducible).
template <typename TIn>
__global__ __launch_bounds__(256) void fc_dbias_kernel(FcDims d, const TIn *dY, const TIn *Y, int relu,
                                                       float *db)
{
    __shared__ float part[4][64];
    const int kl = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int k = blockIdx.x * 64 + kl;
    float s = 0.f;
    if (k < d.K) {
        const int kb = k / d.bk, kf = k % d.bk;
        for (int n = q; n < d.N; n += 4) {
            int64_t e = (((int64_t)(n / d.bn) * d.Kb + kb) * d.bn + n % d.bn) * d.bk + kf;
            float g = to_f32<TIn>(dY[e]);
            if (relu && !(to_f32<TIn>(Y[e]) > 0.f)) g = 0.f;
            s += g;
        }
    }
    part[q][kl] = s;
    __syncthreads();
    if (q == 0 && k < d.K) db[k] = (part[0][kl] + part[1][kl]) + (part[2][kl] + part[3][kl]);
}

// Bias gradient of a bf16 layer on 64-wide blocks (dZ already masked): db[k] = sum_n dZ[n][k].  One workgroup per
// feature block; thread (row r = t / 8, piece p = t % 8) adds the 8 features of piece p over the rows r and r + 32
// of every batch block (16-byte loads, several in flight), then the 32 row slices are added in a fixed order.
__global__ __launch_bounds__(256) void fc_dbias_bf16_b64(const bf16_t *dZ, float *db, int Nb, int Kb)
{
    typedef unsigned short us8 __attribute__((ext_vector_type(8)));
    __shared__ float part[32][65];
    const int t = threadIdx.x, r = t >> 3, p = t & 7, kb = blockIdx.x;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const bf16_t *src = dZ + (int64_t)kb * 4096 + r * 64 + p * 8;
    const int64_t nstride = (int64_t)Kb * 4096;
#pragma unroll 4
    for (int nb = 0; nb < Nb; ++nb) {
        const us8 v0 = *(const us8 *)(src + nb * nstride), v1 = *(const us8 *)(src + nb * nstride + 32 * 64);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += bf16_to_f32(v0[e]) + bf16_to_f32(v1[e]);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) part[r][p * 8 + e] = acc[e];
    __syncthreads();
    if (t < 64) {
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < 32; ++i) sum += part[i][t];
        db[kb * 64 + t] = sum;
    }
}

static int fc_dims(const brg_fc_desc_t *desc, FcDims *d, const char *who)
{
    BRG_REQUIRE(desc != nullptr, BRG_EINVAL, "%s: desc is null", who);
    BRG_REQUIRE(desc->N > 0 && desc->C > 0 && desc->K > 0 && desc->bn > 0 && desc->bc > 0 && desc->bk > 0,
                BRG_EINVAL, "%s: sizes must be positive", who);
    BRG_REQUIRE(desc->N % desc->bn == 0 && desc->C % desc->bc == 0 && desc->K % desc->bk == 0, BRG_EINVAL,
                "%s: blocking (%lld,%lld,%lld) does not divide (N,C,K)=(%lld,%lld,%lld)", who,
                (long long)desc->bn, (long long)desc->bc, (long long)desc->bk, (long long)desc->N,
                (long long)desc->C, (long long)desc->K);
    BRG_REQUIRE(desc->N < (1 << 24) && desc->C < (1 << 24) && desc->K < (1 << 24), BRG_EINVAL,
                "%s: size too large", who);
    d->N = (int)desc->N; d->C = (int)desc->C; d->K = (int)desc->K;
    d->bn = (int)desc->bn; d->bc = (int)desc->bc; d->bk = (int)desc->bk;
    d->Nb = d->N / d->bn; d->Cb = d->C / d->bc; d->Kb = d->K / d->bk;
    return BRG_OK;
}

// With bc = bk = 16 the blocked layouts of a fully connected layer (Algorithm 5) ARE those of a 1x1
// convolution (Algorithm 4) over N/bn images of bn pixels: X [N/bn][C/16][bn][16] = NCHW16c with H*W = bn,
// W [K/16][C/16][16][16] = KCRS16c16k with R = S = 1, Y likewise.  bf16 layers of that form run on the tuned
// 1x1 convolution kernels (forward with bias and activation, backward by data).
static bool fc_is_conv1x1(const FcDims &d)
{
    return d.bc == 16 && d.bk == 16 && !knobs().fc_general.set;
}

static brg_conv_desc_t fc_as_conv1x1(const FcDims &d)
{
    brg_conv_desc_t c = {d.Nb, d.C, 1, d.bn, d.K, 1, 1, 1, 1, 0, 0, 16, 16};
    return c;
}

static bool fc_blocks_64(const FcDims &d)
{
    return d.bn == 64 && d.bc == 64 && d.bk == 64 && !knobs().fc_general.set;
}

template <typename TIn, typename TOut>
static int fc_fwd_launch(const FcDims &d, const void *X, const void *Wt, const float *bias, int act,
                         void *Y, hipStream_t s)
{
    FcFwdProb<TIn, TOut> p;
    p.d = d; p.X = (const TIn *)X; p.Wt = (const TIn *)Wt; p.bias = bias; p.Y = (TOut *)Y; p.act = act;
    p.tiles_m = (d.K + ENG_TM - 1) / ENG_TM;
    int tiles_n = (d.N + ENG_TN - 1) / ENG_TN;
    hipLaunchKernelGGL((engine_kernel<FcFwdProb<TIn, TOut>>), dim3(p.tiles_m * tiles_n), dim3(256), 0, s, p);
    return check_launch("brg_fc_fwd launch");
}

template <typename TIn>
static int fc_bwd_launch(const FcDims &d, const void *dY, const void *Y, const void *X, const void *Wt,
                         int relu, int relu_in, void *dX, float *dWt, float *dbias, hipStream_t s)
{
    if (dX) {
        FcBwdDataProb<TIn> p;
        p.d = d; p.dY = (const TIn *)dY; p.Y = (const TIn *)Y; p.Wt = (const TIn *)Wt; p.dX = (TIn *)dX;
        p.Xmask = relu_in ? (const TIn *)X : nullptr;
        p.relu = relu;
        p.tiles_m = (d.C + ENG_TM - 1) / ENG_TM;
        int tiles_n = (d.N + ENG_TN - 1) / ENG_TN;
        hipLaunchKernelGGL((engine_kernel<FcBwdDataProb<TIn>>), dim3(p.tiles_m * tiles_n), dim3(256), 0, s, p);
        int rc = check_launch("brg_fc_bwd (data) launch");
        if (rc) return rc;
    }
    if (dWt) {
        FcWgtProb<TIn> p;
        p.d = d; p.dY = (const TIn *)dY; p.Y = (const TIn *)Y; p.X = (const TIn *)X; p.dWt = dWt;
        p.relu = relu;
        p.tiles_m = (d.K + ENG_TM - 1) / ENG_TM;
        int tiles_n = (d.C + ENG_TN - 1) / ENG_TN;
        hipLaunchKernelGGL((engine_kernel<FcWgtProb<TIn>>), dim3(p.tiles_m * tiles_n), dim3(256), 0, s, p);
        int rc = check_launch("brg_fc_bwd (weights) launch");
        if (rc) return rc;
    }
    if (dbias) {
        hipLaunchKernelGGL((fc_dbias_kernel<TIn>), dim3((d.K + 63) / 64), dim3(256), 0, s, d,
                           (const TIn *)dY, (const TIn *)Y, relu, dbias);
        int rc = check_launch("brg_fc_bwd (bias) launch");
        if (rc) return rc;
    }
    return BRG_OK;
}

}  // namespace brg

extern "C" int brg_fc_fwd(const brg_fc_desc_t *desc, brg_dtype_t dtype, brg_dtype_t out_dtype,
                          const void *X, const void *Wt, const float *bias, brg_act_t act, void *Y,
                          brg_stream_t stream)
{
    using namespace brg;
    FcDims d;
    int rc = fc_dims(desc, &d, "brg_fc_fwd");
    if (rc) return rc;
    BRG_REQUIRE(valid_dtype(dtype) && valid_dtype(out_dtype), BRG_EINVAL, "brg_fc_fwd: bad dtype");
    BRG_REQUIRE(valid_act(act), BRG_EINVAL, "brg_fc_fwd: bad activation %d", (int)act);
    BRG_REQUIRE(X && Wt && Y, BRG_EINVAL, "brg_fc_fwd: null tensor");
    BRG_REQUIRE(aligned16(X) && aligned16(Wt) && aligned16(Y) && aligned16(bias), BRG_EALIGN,
                "brg_fc_fwd: pointer not 16-byte aligned");
    hipStream_t s = (hipStream_t)stream;
    if (dtype == BRG_F32 && out_dtype == BRG_F32 && fc_blocks_64(d)) {
        // Y block (nb, kb) [n][k] = sum_cb W(kb, cb) [c][k] * X(nb, cb) [n][c]
        G64Args a = {};
        a.njobs = 1;
        G64Job &j = a.job[0];
        j.kind = G64_GEMM;
        j.A = (const float *)Wt; j.B = (const float *)X; j.C = (float *)Y; j.bias = bias; j.act = act;
        j.tiles_m = d.Kb; j.tiles_n = d.Nb; j.chain = d.Cb; j.alpha = 1.f; j.beta = 0.f;
        j.a_tile = (int64_t)d.Cb * 4096; j.a_chain = 4096; j.b_tile = (int64_t)d.Cb * 4096; j.b_chain = 4096;
        j.c_tile_m = 4096; j.c_tile_n = (int64_t)d.Kb * 4096; j.a_ld = j.b_ld = j.c_ld = 64;
        j.a_kfast = 0; j.b_kfast = 1;
        if (!knobs().fc_g64.set) {
            // a lone GEMM: one 8-wave workgroup per block of Y, the chain split between two wave groups
            BlockTileArgs b = {};
            b.A = j.A; b.B = j.B; b.C = j.C; b.bias = bias; b.act = act;
            b.tiles_m = d.Kb; b.tiles_n = d.Nb; b.chain = d.Cb; b.alpha = 1.f; b.beta = 0.f;
            b.a_tile = j.a_tile; b.a_chain = j.a_chain; b.b_tile = j.b_tile; b.b_chain = j.b_chain;
            b.c_tile_m = j.c_tile_m; b.c_tile_n = j.c_tile_n; b.a_ld = b.b_ld = b.c_ld = 64;
            return launch_block_ring<false, true>(b, s, "brg_fc_fwd launch");
        }
        return launch_g64(a, knobs().fc_g64.val == 32 ? 32 : 64, 0, s, "brg_fc_fwd launch");
    }
    if (dtype == BRG_BF16 && out_dtype == BRG_BF16 && fc_is_conv1x1(d)) {
        const brg_conv_desc_t c = fc_as_conv1x1(d);
        return brg_conv_fwd(&c, dtype, out_dtype, X, Wt, Y, bias, act, nullptr, stream);
    }
    if (dtype == BRG_BF16 && fc_blocks_64(d)) {
        // 64-wide bf16 blocks: the batch-reduce kernel on the bf16 matrix instruction, one workgroup per block of Y;
        // W blocks [c][k] have the reduction index strided (transposing LDS reads), X blocks [n][c] contiguous
        H64Args a = {};
        a.A = (const bf16_t *)Wt; a.B = (const bf16_t *)X; a.C = Y; a.bias = bias; a.act = act;
        a.tiles_m = d.Kb; a.tiles_n = d.Nb; a.chain = d.Cb; a.alpha = 1.f; a.beta = 0.f;
        a.a_tile = (int64_t)d.Cb * 4096; a.a_chain = 4096; a.b_tile = (int64_t)d.Cb * 4096; a.b_chain = 4096;
        a.c_tile_m = 4096; a.c_tile_n = (int64_t)d.Kb * 4096; a.a_ld = a.b_ld = a.c_ld = 64;
        BRG_REQUIRE((int64_t)d.Kb * d.Nb < (1ll << 31), BRG_EUNSUPPORTED, "brg_fc_fwd: grid too large");
        if (out_dtype == BRG_BF16) return launch_h64<false, true, false, bf16_t>(a, s, "brg_fc_fwd (bf16, 64-wide blocks) launch");
        return launch_h64<false, true, false, float>(a, s, "brg_fc_fwd (bf16, 64-wide blocks) launch");
    }
    if (dtype == BRG_F32 && out_dtype == BRG_F32) return fc_fwd_launch<float, float>(d, X, Wt, bias, act, Y, s);
    if (dtype == BRG_BF16 && out_dtype == BRG_F32) return fc_fwd_launch<bf16_t, float>(d, X, Wt, bias, act, Y, s);
    if (dtype == BRG_BF16 && out_dtype == BRG_BF16) return fc_fwd_launch<bf16_t, bf16_t>(d, X, Wt, bias, act, Y, s);
    return fail(BRG_EUNSUPPORTED, "brg_fc_fwd: fp32 inputs with bf16 output are not supported");
}

static int fc_bwd_impl(const brg_fc_desc_t *desc, brg_dtype_t dtype, const void *dY, const void *Y,
                       const void *X, const void *Wt, brg_act_t act, brg_act_t act_in, void *dX, float *dWt,
                       float *dbias, void *ws, brg_stream_t stream)
{
    using namespace brg;
    FcDims d;
    int rc = fc_dims(desc, &d, "brg_fc_bwd");
    if (rc) return rc;
    BRG_REQUIRE(valid_dtype(dtype), BRG_EINVAL, "brg_fc_bwd: bad dtype");
    BRG_REQUIRE(valid_act(act), BRG_EINVAL, "brg_fc_bwd: bad activation %d", (int)act);
    BRG_REQUIRE(act == BRG_ACT_NONE || act == BRG_ACT_RELU, BRG_EUNSUPPORTED,
                "brg_fc_bwd: only NONE and RELU have a backward pass");
    BRG_REQUIRE(dY != nullptr, BRG_EINVAL, "brg_fc_bwd: dY is null");
    BRG_REQUIRE(act != BRG_ACT_RELU || Y != nullptr, BRG_EINVAL, "brg_fc_bwd: RELU needs the forward output Y");
    BRG_REQUIRE(!dX || Wt, BRG_EINVAL, "brg_fc_bwd: dX requested without weights");
    BRG_REQUIRE(!dWt || X, BRG_EINVAL, "brg_fc_bwd: dWt requested without X");
    BRG_REQUIRE(valid_act(act_in), BRG_EINVAL, "brg_fc_bwd_chain: bad act_in %d", (int)act_in);
    BRG_REQUIRE(act_in == BRG_ACT_NONE || act_in == BRG_ACT_RELU, BRG_EUNSUPPORTED,
                "brg_fc_bwd_chain: only NONE and RELU can be fused into the dX epilogue");
    BRG_REQUIRE(act_in == BRG_ACT_NONE || !dX || X, BRG_EINVAL, "brg_fc_bwd_chain: act_in needs X");
    const int relu_in = act_in == BRG_ACT_RELU;
    BRG_REQUIRE(aligned16(dY) && aligned16(Y) && aligned16(X) && aligned16(Wt) && aligned16(dX) &&
                    aligned16(dWt) && aligned16(dbias) && aligned16(ws),
                BRG_EALIGN, "brg_fc_bwd: pointer not 16-byte aligned");
    hipStream_t s = (hipStream_t)stream;
    int relu = act == BRG_ACT_RELU;
    if (dtype == BRG_F32 && fc_blocks_64(d)) {
        // one launch: backward-by-data GEMM, weight-gradient GEMM and bias gradient side by side
        const float *mask = relu ? (const float *)Y : nullptr;
        G64Args a = {};
        int nj = 0;
        if (dX) {   // dX block (nb, cb) [n][c] = sum_kb W(kb, cb)^T [c][k] * dZ(nb, kb) [n][k]
            G64Job &j = a.job[nj++];
            j.kind = G64_GEMM;
            j.A = (const float *)Wt; j.B = (const float *)dY; j.Bmask = mask; j.C = (float *)dX;
            j.Cmask = relu_in ? (const float *)X : nullptr;
            j.tiles_m = d.Cb; j.tiles_n = d.Nb; j.chain = d.Kb; j.alpha = 1.f;
            j.a_tile = 4096; j.a_chain = (int64_t)d.Cb * 4096; j.b_tile = (int64_t)d.Kb * 4096; j.b_chain = 4096;
            j.c_tile_m = 4096; j.c_tile_n = (int64_t)d.Cb * 4096; j.a_ld = j.b_ld = j.c_ld = 64;
            j.a_kfast = 1; j.b_kfast = 1;
        }
        if (dWt) {  // dW block (kb, cb) [c][k] = sum_nb dZ(nb, kb) [n][k] * X(nb, cb) [n][c]
            G64Job &j = a.job[nj++];
            j.kind = G64_GEMM;
            j.A = (const float *)dY; j.Amask = mask; j.B = (const float *)X; j.C = dWt;
            j.tiles_m = d.Kb; j.tiles_n = d.Cb; j.chain = d.Nb; j.alpha = 1.f;
            j.a_tile = 4096; j.a_chain = (int64_t)d.Kb * 4096; j.b_tile = 4096; j.b_chain = (int64_t)d.Cb * 4096;
            j.c_tile_m = (int64_t)d.Cb * 4096; j.c_tile_n = 4096; j.a_ld = j.b_ld = j.c_ld = 64;
            j.a_kfast = 0; j.b_kfast = 0;
        }
        if (dbias && dWt) {
            a.job[nj - 1].rowsum = dbias;   // db[k] = sum_n dZ[n][k]: row sums of the dW job's A operand
        } else if (dbias) {
            G64Job &j = a.job[nj++];
            j.kind = G64_COLSUM;
            j.A = (const float *)dY; j.Amask = mask; j.C = dbias;
            j.tiles_m = d.Kb; j.tiles_n = 1; j.chain = d.Nb;
            j.a_tile = 4096; j.a_chain = (int64_t)d.Kb * 4096; j.a_ld = 64; j.cs_rows = 64;
        }
        a.njobs = nj;
        if (nj == 0) return BRG_OK;
        // unmasked operands and enough tiles: 128 x 64 tiles, one 8-wave workgroup per CU
        if (g128_applies(a)) return launch_g128(a, s, "brg_fc_bwd launch");
        return launch_g64(a, 64, 1, s, "brg_fc_bwd launch");
    }
    if (dtype == BRG_F32) return fc_bwd_launch<float>(d, dY, Y, X, Wt, relu, relu_in, dX, dWt, dbias, s);
    if (fc_blocks_64(d) && (!relu || ws) && (int64_t)d.Kb * d.Cb < (1ll << 31) && (int64_t)d.Nb * d.Cb < (1ll << 31)) {
        // 64-wide bf16 blocks on the bf16 batch-reduce kernel; the ReLU masks are passes of their own, as for
        // 16-wide blocks (dZ = dY o [Y > 0] into the workspace, the producer's mask on dX in place)
        if (relu) {
            rc = launch_fc_mask_bf16(ws, dY, Y, (int64_t)d.N * d.K, s, "brg_fc_bwd (ReLU mask) launch");
            if (rc) return rc;
            dY = ws;
            relu = 0;
        }
        if (dX) {   // dX block (nb, cb) [n][c] = sum_kb W(kb, cb) [c][k] (reduction contiguous) * dZ(nb, kb) [n][k]
            H64Args a = {};
            a.A = (const bf16_t *)Wt; a.B = (const bf16_t *)dY; a.C = dX; a.act = BRG_ACT_NONE;
            a.tiles_m = d.Cb; a.tiles_n = d.Nb; a.chain = d.Kb; a.alpha = 1.f; a.beta = 0.f;
            a.a_tile = 4096; a.a_chain = (int64_t)d.Cb * 4096; a.b_tile = (int64_t)d.Kb * 4096; a.b_chain = 4096;
            a.c_tile_m = 4096; a.c_tile_n = (int64_t)d.Cb * 4096; a.a_ld = a.b_ld = a.c_ld = 64;
            rc = launch_h64<true, true, false, bf16_t>(a, s, "brg_fc_bwd (data, bf16, 64-wide blocks) launch");
            if (rc) return rc;
            if (relu_in) {
                rc = launch_fc_mask_bf16(dX, dX, X, (int64_t)d.N * d.C, s, "brg_fc_bwd (producer mask) launch");
                if (rc) return rc;
            }
        }
        if (dWt) {  // dW block (kb, cb) [c][k] = sum_nb dZ(nb, kb) [n][k] * X(nb, cb) [n][c]: both reductions strided
            H64Args a = {};
            a.A = (const bf16_t *)dY; a.B = (const bf16_t *)X; a.C = dWt; a.act = BRG_ACT_NONE;
            a.tiles_m = d.Kb; a.tiles_n = d.Cb; a.chain = d.Nb; a.alpha = 1.f; a.beta = 0.f;
            a.a_tile = 4096; a.a_chain = (int64_t)d.Kb * 4096; a.b_tile = 4096; a.b_chain = (int64_t)d.Cb * 4096;
            a.c_tile_m = (int64_t)d.Cb * 4096; a.c_tile_n = 4096; a.a_ld = a.b_ld = a.c_ld = 64;
            rc = launch_h64<false, false, false, float>(a, s, "brg_fc_bwd (weights, bf16, 64-wide blocks) launch");
            if (rc) return rc;
        }
        if (dbias) {
            hipLaunchKernelGGL(fc_dbias_bf16_b64, dim3(d.Kb), dim3(256), 0, s, (const bf16_t *)dY, dbias, d.Nb, d.Kb);
            rc = check_launch("brg_fc_bwd (bias) launch");
            if (rc) return rc;
        }
        return BRG_OK;
    }
    if (relu && ws && fc_is_conv1x1(d) && d.bn % 16 == 0) {
        // the masked gradient dZ = dY o [Y > 0] as a pass of its own into the caller's workspace; the tuned
        // kernels below then see an unmasked problem
        rc = launch_fc_mask_bf16(ws, dY, Y, (int64_t)d.N * d.K, s, "brg_fc_bwd (ReLU mask) launch");
        if (rc) return rc;
        dY = ws;
        relu = 0;
    }
    if (dX && !relu && fc_is_conv1x1(d) && (!relu_in || d.bn % 16 == 0)) {
        // backward by data on 16-wide blocks: the dual 1x1 convolution, then the producer's ReLU mask in place
        const brg_conv_desc_t c = fc_as_conv1x1(d);
        rc = brg_conv_bwd_data(&c, dtype, dtype, dY, Wt, dX, nullptr, stream);
        if (rc) return rc;
        if (relu_in) {
            rc = launch_fc_mask_bf16(dX, dX, X, (int64_t)d.N * d.C, s, "brg_fc_bwd (producer mask) launch");
            if (rc) return rc;
        }
        dX = nullptr;
    }
    if (dWt && !relu && fc_is_conv1x1(d) && fc_wgt_bf16_applies(d.Cb, d.Kb, d.bn)) {
        // unmasked weight (and bias) gradient on 16-wide blocks: transposing LDS reads feed the matrix cores
        FcWgtBf16Args w = {(const bf16_t *)X, (const bf16_t *)dY, dWt, dbias, d.Nb, d.Cb, d.Kb, d.bn};
        rc = launch_fc_wgt_bf16(w, s, "brg_fc_bwd (weights, bf16) launch");
        if (rc) return rc;
        dWt = nullptr;
        dbias = nullptr;
    }
    if (!dX && !dWt && !dbias) return BRG_OK;
    return fc_bwd_launch<bf16_t>(d, dY, Y, X, Wt, relu, relu_in, dX, dWt, dbias, s);
}

extern "C" int brg_fc_bwd(const brg_fc_desc_t *desc, brg_dtype_t dtype, const void *dY, const void *Y,
                          const void *X, const void *Wt, brg_act_t act, void *dX, float *dWt,
                          float *dbias, void *ws, brg_stream_t stream)
{
    return fc_bwd_impl(desc, dtype, dY, Y, X, Wt, act, BRG_ACT_NONE, dX, dWt, dbias, ws, stream);
}

extern "C" int brg_fc_bwd_chain(const brg_fc_desc_t *desc, brg_dtype_t dtype, const void *dY, const void *Y,
                                const void *X, const void *Wt, brg_act_t act, brg_act_t act_in, void *dX,
                                float *dWt, float *dbias, void *ws, brg_stream_t stream)
{
    return fc_bwd_impl(desc, dtype, dY, Y, X, Wt, act, act_in, dX, dWt, dbias, ws, stream);
}
