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
#include "brg_lstm_rec.hpp"

namespace brg {

struct LstmDims {
    int T, N, C, K, bc, bk, Cb, Kb;
};

template <typename T> struct LstmStepProb {
    static constexpr bool A_KFAST = false, B_KFAST = true;
    LstmDims d;
    const T *x_t, *W4, *R4, *h_prev, *s_prev;  // h_prev / s_prev may be null (zeros)
    const float *b4;
    T *h_t, *s_t, *g_t;  // g_t: gate 0 of this step, gate stride = gstride; may be null
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
        float sp = s_prev ? to_f32<T>(s_prev[e]) : 0.f;
        float st = ft * sp + it * ct;
        float ht = ot * tanhf(st);
        s_t[e] = from_f32<T>(st);
        h_t[e] = from_f32<T>(ht);
        if (g_t) {
            g_t[e] = from_f32<T>(it);
            g_t[gstride + e] = from_f32<T>(ct);
            g_t[2 * gstride + e] = from_f32<T>(ft);
            g_t[3 * gstride + e] = from_f32<T>(ot);
        }
    }
};

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
    BRG_REQUIRE(dtype == BRG_F32, BRG_EUNSUPPORTED, "brg_lstm_fwd: only fp32 is supported");
    BRG_REQUIRE(x && W4 && R4 && h && s, BRG_EINVAL, "brg_lstm_fwd: null tensor");
    BRG_REQUIRE(aligned16(x) && aligned16(W4) && aligned16(R4) && aligned16(b4) && aligned16(h0) &&
                    aligned16(s0) && aligned16(h) && aligned16(s) && aligned16(gates),
                BRG_EALIGN, "brg_lstm_fwd: pointer not 16-byte aligned");

    LstmDims d;
    d.T = (int)desc->T; d.N = (int)desc->N; d.C = (int)desc->C; d.K = (int)desc->K;
    d.bc = (int)desc->bc; d.bk = (int)desc->bk; d.Cb = d.C / d.bc; d.Kb = d.K / d.bk;
    hipStream_t st = (hipStream_t)stream;
    const int64_t NK = (int64_t)d.N * d.K, NC = (int64_t)d.N * d.C;

    // ---- fast path: input projections of all time steps as four batch-reduce GEMMs (bias fused) that
    // leave partial pre-activations in `gates`, then ONE persistent kernel for the recurrence.
    // Needs: 64-blocking, T*N a multiple of 64, N <= 64, K/4 <= number of CUs, a gates buffer and a
    // 16-byte workspace for the grid barrier (word 0: arrival counter, word 1: give-up flag).
    bool fast = d.bc == 64 && d.bk == 64 && ((int64_t)d.T * d.N) % 64 == 0 && d.N <= 64 && gates && ws &&
                d.K / 4 <= 256 && (int64_t)d.T * NK < (1ll << 30) && !knobs().lstm_general.set;
    if (ws) BRG_REQUIRE(aligned16(ws), BRG_EALIGN, "brg_lstm_fwd: workspace not 16-byte aligned");
    if (fast) {
        // All K/4 workgroups of the resident kernel must be on the device together (they wait for each other
        // every time step).  A workgroup takes more than half of a compute unit's LDS, so that means one per
        // compute unit; the occupancy query confirms it for this device (asked once per thread and device).
        // Where they do not fit, the layer runs as one launch per time step instead.
        static thread_local int cap_dev = -1, cap = 0;
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess && dev != cap_dev) {
            int per_cu = 0, ncu = 0;
            e = hipFuncSetAttribute((const void *)lstm_rec_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)LR_SMEM);
            if (e == hipSuccess)
                e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void *)lstm_rec_kernel, 512, LR_SMEM);
            if (e == hipSuccess) e = hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev);
            if (e == hipSuccess) {
                cap = per_cu * ncu;
                cap_dev = dev;
            }
        }
        if (e != hipSuccess) return fail(BRG_EHIP, "brg_lstm_fwd: set-up: %s", hipGetErrorString(e));
        if (cap < d.K / 4) fast = false;
    }
    if (ws) {   // both words start at zero on either path, so the caller can always read word 1 afterwards
        hipLaunchKernelGGL(lstm_sync_reset, dim3(1), dim3(64), 0, st, (unsigned *)ws);
        int rc = check_launch("brg_lstm_fwd (barrier reset) launch");
        if (rc) return rc;
    }

    // ---- fast path: input projections of all time steps as four batch-reduce GEMMs (bias fused) that
    // leave partial pre-activations in `gates`, then ONE resident kernel for the recurrence.
    // Needs: 64-blocking, T*N a multiple of 64, N <= 64, K/4 workgroups resident together, a gates buffer and a
    // 16-byte workspace for the grid barrier (word 0: arrival counter, word 1: give-up flag).
    if (fast) {
        const int64_t TNK = (int64_t)d.T * NK;
        G64Args a = {};
        a.njobs = 4;
        for (int g = 0; g < 4; ++g) {
            // Zx_g[(t,n)][k] = sum_cb W_g(kb, cb) [c][k] * x[(t,n)][c] + b_g[k]
            G64Job &j = a.job[g];
            j.kind = G64_GEMM;
            j.A = (const float *)W4 + (int64_t)g * d.K * d.C; j.B = (const float *)x;
            j.C = (float *)gates + g * TNK; j.bias = b4 ? b4 + (int64_t)g * d.K : nullptr; j.act = BRG_ACT_NONE;
            j.tiles_m = d.Kb; j.tiles_n = (int)(((int64_t)d.T * d.N) / 64); j.chain = d.Cb; j.alpha = 1.f; j.beta = 0.f;
            j.a_tile = (int64_t)d.Cb * 4096; j.a_chain = 4096; j.b_tile = (int64_t)64 * d.C; j.b_chain = 64;
            j.c_tile_m = 64; j.c_tile_n = (int64_t)64 * d.K; j.a_ld = 64; j.b_ld = d.C; j.c_ld = d.K;
            j.a_kfast = 0; j.b_kfast = 1;
        }
        int rc = launch_g64(a, 64, 0, st, "brg_lstm_fwd (input projection) launch");
        if (rc) return rc;
        LstmRecArgs r;
        r.R4 = (const float *)R4; r.h0 = (const float *)h0; r.s0 = (const float *)s0;
        r.h = (float *)h; r.s = (float *)s; r.gates = (float *)gates; r.sync = (unsigned *)ws;
        r.T = d.T; r.N = d.N; r.K = d.K; r.spin_limit = 200000u;
        // Should other work keep compute units busy for longer than the spin limit, the kernel gives up and
        // reports through sync[1]; the kernel enqueued after it then overwrites h, s and gates with NaN, so
        // that a run that gave up cannot pass for a result.
        hipLaunchKernelGGL(lstm_rec_kernel, dim3(d.K / 4), dim3(512), LR_SMEM, st, r);
        rc = check_launch("brg_lstm_fwd (recurrence) launch");
        if (rc) return rc;
        hipLaunchKernelGGL(lstm_rec_poison, dim3(256), dim3(256), 0, st, (const unsigned *)ws, (float *)h, (float *)s,
                           (float *)gates, TNK);
        return check_launch("brg_lstm_fwd (give-up check) launch");
    }

    for (int t = 0; t < d.T; ++t) {
        LstmStepProb<float> p;
        p.d = d;
        p.x_t = (const float *)x + t * NC;
        p.W4 = (const float *)W4; p.R4 = (const float *)R4; p.b4 = b4;
        p.h_prev = t ? (const float *)h + (t - 1) * NK : (const float *)h0;
        p.s_prev = t ? (const float *)s + (t - 1) * NK : (const float *)s0;
        p.h_t = (float *)h + t * NK;
        p.s_t = (float *)s + t * NK;
        p.g_t = gates ? (float *)gates + t * NK : nullptr;
        p.gstride = (int64_t)d.T * NK;
        p.tiles_m = (4 * d.K + ENG_TM - 1) / ENG_TM;
        int tiles_n = (d.N + ENG_TN - 1) / ENG_TN;
        hipLaunchKernelGGL((engine_kernel<LstmStepProb<float>>), dim3(p.tiles_m * tiles_n), dim3(256), 0, st, p);
        int rc = check_launch("brg_lstm_fwd launch");
        if (rc) return rc;
    }
    return BRG_OK;
}
