// LSTM layer forward (paper section 3.1, equations (1)-(6), Algorithm 2).
//
// Per time step every workgroup owns a block of hidden units x batch entries and
// runs, for all four gates at once, one batch-reduce chain of C/bc blocks of
// W_g * x_t followed by K/bk blocks of R_g * h_{t-1}.  The rows of the tile are
// ordered (unit, gate) with the gate fastest, so the four pre-activations of one
// (unit, batch) element land in the four accumulator registers of one lane and
// the sigmoid / tanh / cell update run on the accumulators before anything is
// stored.  Time steps are separate launches on the stream (the t -> t+1
// dependency on all of h_t is the kernel boundary).
#include <cstdlib>

#include "brg_engine.hpp"
#include "brg_h64.hpp"
#include "brg_lstm_rec.hpp"

namespace brg {

struct LstmDims {
    int T, N, C, K, bc, bk, Cb, Kb;
};

// T: type of the multiplied tensors (x, W4, R4, h); TS: type of the cell state and the gate values (fp32 for both
// input types: they never enter a matrix product).
template <typename T, typename TS> struct LstmStepProb {
    static constexpr bool A_KFAST = false, B_KFAST = true;
    LstmDims d;
    const T *x_t, *W4, *R4, *h_prev;  // h_prev may be null (zeros)
    const TS *s_prev;                 // may be null (zeros)
    const float *b4;
    T *h_t;
    TS *s_t, *g_t;  // g_t: gate 0 of this step, gate stride = gstride; may be null
    int64_t gstride;
    int tiles_m;

    struct RowA {
        int64_t w, r;  // offsets of this (gate, unit) row inside W4 / R4, -1 if out of range
    };
    typedef int64_t RowB;  // batch row n, -1 if out of range
    struct Chain {
        int64_t aoff, boff;
        bool rec;
    };
    __device__ int m0() const { return (blockIdx.x % tiles_m) * ENG_TM; }
    __device__ int n0() const { return (blockIdx.x / tiles_m) * ENG_TN; }
    __device__ int chain_len() const { return h_prev ? d.Cb + d.Kb : d.Cb; }
    __device__ int kdepth(int c) const { return c < d.Cb ? d.bc : d.bk; }
    __device__ RowA row_a(int i) const
    {
        int row = m0() + i;
        int unit = row >> 2, gate = row & 3;
        RowA ra;
        if (unit >= d.K) {
            ra.w = ra.r = -1;
            return ra;
        }
        int kb = unit / d.bk, kf = unit % d.bk;
        ra.w = (int64_t)gate * d.K * d.C + (int64_t)kb * d.Cb * d.bc * d.bk + kf;
        ra.r = (int64_t)gate * d.K * d.K + (int64_t)kb * d.Kb * d.bk * d.bk + kf;
        return ra;
    }
    __device__ RowB row_b(int j) const
    {
        int n = n0() + j;
        return n < d.N ? (int64_t)n : -1;
    }
    __device__ Chain chain(int c) const
    {
        Chain ch;
        ch.rec = c >= d.Cb;
        if (!ch.rec) {
            ch.aoff = (int64_t)c * d.bc * d.bk;
            ch.boff = (int64_t)c * d.bc;
        } else {
            ch.aoff = (int64_t)(c - d.Cb) * d.bk * d.bk;
            ch.boff = (int64_t)(c - d.Cb) * d.bk;
        }
        return ch;
    }
    __device__ float a(const Chain &ch, const RowA &ra, int p) const
    {
        if (ra.w < 0) return 0.f;
        return ch.rec ? to_f32<T>(R4[ra.r + ch.aoff + (int64_t)p * d.bk])
                      : to_f32<T>(W4[ra.w + ch.aoff + (int64_t)p * d.bk]);
    }
    __device__ float b(const Chain &ch, const RowB &n, int p) const
    {
        if (n < 0) return 0.f;
        return ch.rec ? to_f32<T>(h_prev[n * d.K + ch.boff + p]) : to_f32<T>(x_t[n * d.C + ch.boff + p]);
    }
    // rows i..i+3 are the gates i, c, f, o of one hidden unit
    __device__ void store4(int i, int j, float4v z) const
    {
        int n = n0() + j, unit = (m0() + i) >> 2;
        if (n >= d.N || unit >= d.K) return;
        if (b4) {
            z[0] += b4[unit];
            z[1] += b4[d.K + unit];
            z[2] += b4[2 * d.K + unit];
            z[3] += b4[3 * d.K + unit];
        }
        float it = sigmoidf_(z[0]), ct = tanhf(z[1]), ft = sigmoidf_(z[2]), ot = sigmoidf_(z[3]);
        int64_t e = (int64_t)n * d.K + unit;
        float sp = s_prev ? to_f32<TS>(s_prev[e]) : 0.f;
        float st = ft * sp + it * ct;
        float ht = ot * tanhf(st);
        s_t[e] = from_f32<TS>(st);
        h_t[e] = from_f32<T>(ht);
        if (g_t) {
            g_t[e] = from_f32<TS>(it);
            g_t[gstride + e] = from_f32<TS>(ct);
            g_t[2 * gstride + e] = from_f32<TS>(ft);
            g_t[3 * gstride + e] = from_f32<TS>(ot);
        }
    }
};

// one general launch per time step (any shape)
template <typename T> static int lstm_fwd_steps(const LstmDims &d, const void *x, const void *W4, const void *R4, const float *b4,
                                                const void *h0, const void *s0, void *h, void *s, void *gates, hipStream_t st)
{
    const int64_t NK = (int64_t)d.N * d.K, NC = (int64_t)d.N * d.C;
    for (int t = 0; t < d.T; ++t) {
        LstmStepProb<T, float> p;
        p.d = d;
        p.x_t = (const T *)x + t * NC;
        p.W4 = (const T *)W4; p.R4 = (const T *)R4; p.b4 = b4;
        p.h_prev = t ? (const T *)h + (t - 1) * NK : (const T *)h0;
        p.s_prev = t ? (const float *)s + (t - 1) * NK : (const float *)s0;
        p.h_t = (T *)h + t * NK;
        p.s_t = (float *)s + t * NK;
        p.g_t = gates ? (float *)gates + t * NK : nullptr;
        p.gstride = (int64_t)d.T * NK;
        p.tiles_m = (4 * d.K + ENG_TM - 1) / ENG_TM;
        int tiles_n = (d.N + ENG_TN - 1) / ENG_TN;
        hipLaunchKernelGGL((engine_kernel<LstmStepProb<T, float>>), dim3(p.tiles_m * tiles_n), dim3(256), 0, st, p);
        int rc = check_launch("brg_lstm_fwd launch");
        if (rc) return rc;
    }
    return BRG_OK;
}

// The resident kernel for `np` batch passes and one input type: its address (for the attribute and occupancy
// calls) and its launch.  (Written out per value: inside a template the kernel's name with a dependent argument
// does not convert to an address.)
static const void *lstm_rec_fn(int np, bool bf16)
{
#define BRG_REC_CASE(NPV) \
    case NPV: return bf16 ? (const void *)lstm_rec_bf16_kernel<NPV> : (const void *)lstm_rec_kernel<NPV>;
    switch (np) {
        BRG_REC_CASE(1)
        BRG_REC_CASE(2)
        BRG_REC_CASE(3)
    default:
        BRG_REC_CASE(4)
    }
#undef BRG_REC_CASE
}

static void lstm_rec_launch(int np, bool bf16, int nwg, size_t smem, hipStream_t st, const LstmRecArgs &r)
{
#define BRG_REC_CASE(NPV)                                                                              \
    case NPV:                                                                                          \
        if (bf16) hipLaunchKernelGGL(lstm_rec_bf16_kernel<NPV>, dim3(nwg), dim3(512), smem, st, r);    \
        else hipLaunchKernelGGL(lstm_rec_kernel<NPV>, dim3(nwg), dim3(512), smem, st, r);              \
        return;
    switch (np) {
        BRG_REC_CASE(1)
        BRG_REC_CASE(2)
        BRG_REC_CASE(3)
    default:
        BRG_REC_CASE(4)
    }
#undef BRG_REC_CASE
}

}  // namespace brg

extern "C" int brg_lstm_fwd(const brg_lstm_desc_t *desc, brg_dtype_t dtype, const void *x, const void *W4,
                            const void *R4, const float *b4, const void *h0, const void *s0, void *h,
                            void *s, void *gates, void *ws, brg_stream_t stream)
{
    using namespace brg;
    BRG_REQUIRE(desc != nullptr, BRG_EINVAL, "brg_lstm_fwd: desc is null");
    BRG_REQUIRE(desc->T > 0 && desc->N > 0 && desc->C > 0 && desc->K > 0 && desc->bc > 0 && desc->bk > 0,
                BRG_EINVAL, "brg_lstm_fwd: sizes must be positive");
    BRG_REQUIRE(desc->C % desc->bc == 0 && desc->K % desc->bk == 0, BRG_EINVAL,
                "brg_lstm_fwd: blocking (%lld,%lld) does not divide (C,K)=(%lld,%lld)", (long long)desc->bc,
                (long long)desc->bk, (long long)desc->C, (long long)desc->K);
    BRG_REQUIRE(desc->T < (1 << 20) && desc->N < (1 << 20) && desc->C < (1 << 20) && desc->K < (1 << 20),
                BRG_EINVAL, "brg_lstm_fwd: size too large");
    BRG_REQUIRE(valid_dtype(dtype), BRG_EINVAL, "brg_lstm_fwd: bad dtype");
    BRG_REQUIRE(x && W4 && R4 && h && s, BRG_EINVAL, "brg_lstm_fwd: null tensor");
    BRG_REQUIRE(aligned16(x) && aligned16(W4) && aligned16(R4) && aligned16(b4) && aligned16(h0) &&
                    aligned16(s0) && aligned16(h) && aligned16(s) && aligned16(gates),
                BRG_EALIGN, "brg_lstm_fwd: pointer not 16-byte aligned");

    LstmDims d;
    d.T = (int)desc->T; d.N = (int)desc->N; d.C = (int)desc->C; d.K = (int)desc->K;
    d.bc = (int)desc->bc; d.bk = (int)desc->bk; d.Cb = d.C / d.bc; d.Kb = d.K / d.bk;
    hipStream_t st = (hipStream_t)stream;
    const int64_t NK = (int64_t)d.N * d.K;
    const bool bf16 = dtype == BRG_BF16;
    const int np = (d.N + 63) / 64;                  // batch passes of the resident kernel

    bool fast = d.bc == 64 && d.bk == 64 && np <= 4 && gates && ws && d.K / 4 <= 256 && (int64_t)d.T * NK < (1ll << 30) &&
                (int64_t)d.T * d.N * d.C < (1ll << 31) && !knobs().lstm_general.set;
    if (ws) BRG_REQUIRE(aligned16(ws), BRG_EALIGN, "brg_lstm_fwd: workspace not 16-byte aligned");
    const size_t smem = bf16 ? lr16_smem(d.K) : LR_SMEM;
    const void *rec = lstm_rec_fn(np, bf16);
    if (fast) {
        // All K/4 workgroups of the resident kernel must be on the device together (they wait for each other
        // every time step); the occupancy query says how many fit (asked once per thread, device and kernel).
        // Where they do not fit, the layer runs as one launch per time step instead.
        static thread_local int cap_dev = -1, cap[2][5] = {};
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess && dev != cap_dev) {
            for (int i = 0; i < 2; ++i)
                for (int j = 0; j < 5; ++j) cap[i][j] = 0;
            cap_dev = dev;
        }
        // (the bf16 kernel's LDS size depends on K: its attribute is raised to the largest supported size once)
        if (e == hipSuccess && cap[bf16][np] == 0) {
            int per_cu = 0, ncu = 0;
            const size_t smem_max = bf16 ? lr16_smem(1024) : LR_SMEM;
            e = hipFuncSetAttribute(rec, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_max);
            if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, rec, 512, smem_max);
            if (e == hipSuccess) e = hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev);
            if (e == hipSuccess) cap[bf16][np] = per_cu * ncu > 0 ? per_cu * ncu : -1;
        }
        if (e != hipSuccess) return fail(BRG_EHIP, "brg_lstm_fwd: set-up: %s", hipGetErrorString(e));
        if (cap[bf16][np] < d.K / 4) fast = false;
    }
    if (ws) {   // both words start at zero on either path, so the caller can always read word 1 afterwards
        hipLaunchKernelGGL(lstm_sync_reset, dim3(1), dim3(64), 0, st, (unsigned *)ws);
        int rc = check_launch("brg_lstm_fwd (barrier reset) launch");
        if (rc) return rc;
    }

    // ---- fast path: input projections of all time steps as batch-reduce GEMMs (bias fused) that leave partial
    // pre-activations in `gates`, then ONE resident kernel for the recurrence.
    // Needs: 64-blocking, N <= 256, K/4 workgroups resident together, a gates buffer and a 16-byte workspace
    // for the grid barrier (word 0: arrival counter, word 1: give-up flag).
    if (fast) {
        const int64_t TNK = (int64_t)d.T * NK, TN = (int64_t)d.T * d.N;
        const int tiles_n = (int)((TN + 63) / 64);
        int rc;
        if (!bf16) {
            G64Args a = {};
            a.njobs = 4;
            for (int g = 0; g < 4; ++g) {
                // Zx_g[(t,n)][k] = sum_cb W_g(kb, cb) [c][k] * x[(t,n)][c] + b_g[k]
                G64Job &j = a.job[g];
                j.kind = G64_GEMM;
                j.A = (const float *)W4 + (int64_t)g * d.K * d.C; j.B = (const float *)x;
                j.C = (float *)gates + g * TNK; j.bias = b4 ? b4 + (int64_t)g * d.K : nullptr; j.act = BRG_ACT_NONE;
                j.tiles_m = d.Kb; j.tiles_n = tiles_n; j.chain = d.Cb; j.alpha = 1.f; j.beta = 0.f;
                j.a_tile = (int64_t)d.Cb * 4096; j.a_chain = 4096; j.b_tile = (int64_t)64 * d.C; j.b_chain = 64;
                j.c_tile_m = 64; j.c_tile_n = (int64_t)64 * d.K; j.a_ld = 64; j.b_ld = d.C; j.c_ld = d.K;
                j.a_kfast = 0; j.b_kfast = 1;
                j.n_cols = TN % 64 ? (int)TN : 0;    // T*N need not be a multiple of the tile (the paper's N = 168)
            }
            rc = launch_g64(a, 64, 0, st, "brg_lstm_fwd (input projection) launch");
        } else {
            // the four gate matrices are stored back to back: one launch with 4 K/64 row tiles
            H64Args a = {};
            a.A = (const bf16_t *)W4; a.B = (const bf16_t *)x; a.C = gates; a.bias = b4; a.act = BRG_ACT_NONE;
            a.tiles_m = 4 * d.Kb; a.tiles_n = tiles_n; a.chain = d.Cb; a.alpha = 1.f; a.beta = 0.f;
            a.a_tile = (int64_t)d.Cb * 4096; a.a_chain = 4096; a.b_tile = (int64_t)64 * d.C; a.b_chain = 64;
            a.c_tile_m = 64; a.c_tile_n = (int64_t)64 * d.K; a.a_ld = 64; a.b_ld = d.C; a.c_ld = d.K;
            a.m_inner = d.Kb; a.c_outer = TNK;
            a.n_cols = TN % 64 ? (int)TN : 0;
            rc = launch_h64<false, true, false, float>(a, st, "brg_lstm_fwd (input projection) launch");
        }
        if (rc) return rc;
        LstmRecArgs r;
        r.R4 = R4; r.h0 = h0; r.s0 = (const float *)s0;
        r.h = h; r.s = (float *)s; r.gates = (float *)gates; r.sync = (unsigned *)ws;
        r.T = d.T; r.N = d.N; r.K = d.K; r.spin_limit = 200000u * (unsigned)np;
        // (tests force the give-up path from the host with a limit no wait can meet; every wave still exits normally)
        if (knobs().lstm_spin_limit.set && knobs().lstm_spin_limit.val >= 0) r.spin_limit = (unsigned)knobs().lstm_spin_limit.val;
        // Should other work keep compute units busy for longer than the spin limit, the kernel gives up and
        // reports through sync[1]; the kernel enqueued after it then overwrites h, s and gates with NaN, so
        // that a run that gave up cannot pass for a result.
        lstm_rec_launch(np, bf16, d.K / 4, smem, st, r);
        rc = check_launch("brg_lstm_fwd (recurrence) launch");
        if (rc) return rc;
        hipLaunchKernelGGL(lstm_rec_poison, dim3(256), dim3(256), 0, st, (const unsigned *)ws, h, (int)bf16, (float *)s,
                           (float *)gates, TNK);
        return check_launch("brg_lstm_fwd (give-up check) launch");
    }

    if (bf16) return lstm_fwd_steps<bf16_t>(d, x, W4, R4, b4, h0, s0, h, s, gates, st);
    return lstm_fwd_steps<float>(d, x, W4, R4, b4, h0, s0, h, s, gates, st);
}
