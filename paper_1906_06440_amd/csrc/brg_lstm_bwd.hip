// LSTM layer backward pass (paper section 3.1: the backward and weight-update passes are reported there
// without a listing; this is the chain rule on equations (1)-(6), organised the way the forward pass is:
// element-wise gate math plus batch-reduce GEMM chains over the blocked weights).
//
// The gate gradients of all steps live in the workspace as dz [T*N][4 K] (row (t, n), gate g at columns g K ..).
//   for t = T-1 .. 0:   dz_g[t] = gate gradients from dh[t] + dh_rec, ds_next, the stored gates and states
//                       dh_rec  = sum_g R_g^T dz_g[t]            (the only sequential GEMM: 4 K/bk blocks per chain)
//   afterwards, over all time steps at once:
//                       dx = sum_g dz_g W_g,   dW_g = dz_g^T x,   dR_g = dz_g^T h_prev,   db_g = column sums of dz_g
//
// With 64-wide blocks and a minibatch that is a multiple of 64 the GEMMs run on the multi-job kernel for
// 64 x 64 x 64 blocks (brg_g64.hpp): the recurrent one as sixteen jobs (per gate four quarter chains, partial sums added by
// the next step's gate kernel), dx as one chain over (gate, block), dW and dR with the four gates as the
// four jobs of one launch.  Every other shape runs on the general tile engine (brg_engine.hpp) through problem
// functors that read the blocked weights in place.
#include <hip/hip_runtime.h>

#include <cstdlib>

#include "brg_common.hpp"
#include "brg_engine.hpp"
#include "brg_g64.hpp"

namespace brg {

struct LstmBwdDims {
    int T, N, C, K, bc, bk, Cb, Kb;
};

// ---- gate gradients of one time step (element-wise over N x K)
struct LstmBwdStepArgs {
    const float *dh_t, *dh_rec;   // dL/dh_t from outside, and from step t+1 (null at t = T-1)
    int nparts;                   // dh_rec is the sum of this many [N][K] arrays stored back to back
    float *ds;                    // in: dL/ds_t from step t+1 (and ds_last at t = T-1); out: dL/ds_{t-1}
    const float *gates_t;         // i at 0, c at gstride, f at 2 gstride, o at 3 gstride
    const float *s_t, *s_prev;    // s_prev null: zeros
    float *dz_t;                  // this step's rows of dz: [N][4 K], gate g at columns g K ..
    int64_t gstride;              // elements between gates in `gates`
    int n, K;                     // N * K, K
};

__global__ __launch_bounds__(256) void lstm_bwd_step(LstmBwdStepArgs a)
{
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= a.n) return;
    const float i = a.gates_t[e], c = a.gates_t[a.gstride + e], f = a.gates_t[2 * a.gstride + e], o = a.gates_t[3 * a.gstride + e];
    float dht = a.dh_t[e];
    if (a.dh_rec)
        for (int q = 0; q < a.nparts; ++q) dht += a.dh_rec[(int64_t)q * a.n + e];
    const float ts = tanhf(a.s_t[e]);
    const float d_o = dht * ts;
    const float dst = dht * o * (1.f - ts * ts) + a.ds[e];
    const float sp = a.s_prev ? a.s_prev[e] : 0.f;
    a.ds[e] = dst * f;
    const float z0 = dst * c * i * (1.f - i), z1 = dst * i * (1.f - c * c), z2 = dst * sp * f * (1.f - f), z3 = d_o * o * (1.f - o);
    const int row = e / a.K, k = e - row * a.K;
    float *out = a.dz_t + (int64_t)row * 4 * a.K + k;
    out[0] = z0;
    out[a.K] = z1;
    out[2 * a.K] = z2;
    out[3 * a.K] = z3;
}

// ---- GEMMs with the gate index and a weight block as chain: C(m, n) = sum_{g, kb} sum_p A_g,kb(m, p) dz_g(row n, kb*bk + p)
// A is a blocked weight tensor [4][Kb][Mb][bm][bk] read along its contiguous index p:
//   recurrent:  R4, M = K (the h_{t-1} index), rows of dz = the N rows of one time step, output dh_rec [N][K]
//   input:      W4, M = C,                      rows of dz = all T*N rows,               output dx [T*N][C]
struct LstmBwdDataProb {
    static constexpr bool A_KFAST = true, B_KFAST = true;
    const float *Wb, *dz;         // dz [row][4 K] (gate g at columns g K ..), pointing at the first row in question
    float *out;
    int M, Mb, bm, bk, Kb, K, rows, tiles_m;
    typedef int64_t RowA;
    typedef int64_t RowB;
    struct Chain {
        int64_t aoff, boff;
    };
    __device__ int m0() const { return (blockIdx.x % tiles_m) * ENG_TM; }
    __device__ int n0() const { return (blockIdx.x / tiles_m) * ENG_TN; }
    __device__ int chain_len() const { return 4 * Kb; }
    __device__ int kdepth(int) const { return bk; }
    __device__ RowA row_a(int i) const
    {
        const int m = m0() + i;
        return m < M ? (int64_t)m * bk : -1;       // ((m / bm) * bm + m % bm) * bk
    }
    __device__ RowB row_b(int j) const
    {
        const int r = n0() + j;
        return r < rows ? (int64_t)r * 4 * K : -1;
    }
    __device__ Chain chain(int c) const
    {
        const int g = c / Kb, kb = c - g * Kb;
        return Chain{((int64_t)g * Kb + kb) * Mb * bm * bk, (int64_t)g * K + (int64_t)kb * bk};
    }
    __device__ float a(const Chain &ch, const RowA &r, int p) const { return r >= 0 ? Wb[ch.aoff + r + p] : 0.f; }
    __device__ float b(const Chain &ch, const RowB &r, int p) const { return r >= 0 ? dz[ch.boff + r + p] : 0.f; }
    __device__ void store4(int i, int j, float4v acc) const
    {
        const int r = n0() + j;
        if (r >= rows) return;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int m = m0() + i + q;
            if (m < M) out[(int64_t)r * M + m] = acc[q];
        }
    }
};

// ---- weight gradients: dV_g[k][m] = sum over rows (t, n) of dz_g[row][k] * v[row][m], stored blocked
// [K/bk][M/bm][bm][bk]; gate g = blockIdx.y.  v is x (all rows) or h_prev: row (t, n) is h0[n] for t = 0
// (zeros when h0 is null) and h[t-1][n] otherwise.
struct LstmBwdWgtProb {
    static constexpr bool A_KFAST = false, B_KFAST = false;
    const float *dz, *v, *v0;     // v0: the rows of time step 0 when v is shifted by one step (else null and shift = 0)
    float *out;                   // [4][Kb][Mb][bm][bk]
    int K, M, bm, bk, Mb, Kb, rows, N, shift, tiles_m;
    typedef int RowA;
    typedef int RowB;
    struct Chain {
        int row0;
    };
    __device__ int m0() const { return (blockIdx.x % tiles_m) * ENG_TM; }
    __device__ int n0() const { return (blockIdx.x / tiles_m) * ENG_TN; }
    __device__ int chain_len() const { return (rows + 63) / 64; }
    __device__ int kdepth(int c) const { return min(64, rows - 64 * c); }
    __device__ RowA row_a(int i) const { const int k = m0() + i; return k < K ? k : -1; }
    __device__ RowB row_b(int j) const { const int m = n0() + j; return m < M ? m : -1; }
    __device__ Chain chain(int c) const { return Chain{64 * c}; }
    __device__ float a(const Chain &ch, const RowA &k, int p) const
    {
        return k >= 0 ? dz[(int64_t)(ch.row0 + p) * 4 * K + blockIdx.y * K + k] : 0.f;
    }
    __device__ float b(const Chain &ch, const RowB &m, int p) const
    {
        if (m < 0) return 0.f;
        const int row = ch.row0 + p;
        if (!shift) return v[(int64_t)row * M + m];
        if (row < N) return v0 ? v0[(int64_t)row * M + m] : 0.f;
        return v[(int64_t)(row - N) * M + m];
    }
    __device__ void store4(int i, int j, float4v acc) const
    {
        const int m = n0() + j;
        if (m >= M) return;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int k = m0() + i + q;
            if (k < K) out[((((int64_t)blockIdx.y * Kb + k / bk) * Mb + m / bm) * bm + m % bm) * bk + k % bk] = acc[q];
        }
    }
};

// ---- bias gradient: db[g][k] = sum over all rows of dz_g[row][k]; one workgroup per (64 features, gate)
__global__ __launch_bounds__(256) void lstm_bwd_bias(const float *dz, float *db, int rows, int K)
{
    __shared__ float part[4][64];
    const int kl = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int k = blockIdx.x * 64 + kl, g = blockIdx.y;
    float s = 0.f;
    if (k < K) {
        // eight independent partial sums keep eight loads in flight (the order of the additions is fixed)
        const float *col = dz + (int64_t)g * K + k;
        float p8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        int r = q;
        for (; r + 28 < rows; r += 32) {
#pragma unroll
            for (int u = 0; u < 8; ++u) p8[u] += col[(int64_t)(r + 4 * u) * 4 * K];
        }
        for (; r < rows; r += 4) p8[0] += col[(int64_t)r * 4 * K];
        s = ((p8[0] + p8[1]) + (p8[2] + p8[3])) + ((p8[4] + p8[5]) + (p8[6] + p8[7]));
    }
    part[q][kl] = s;
    __syncthreads();
    if (q == 0 && k < K) db[(int64_t)g * K + k] = (part[0][kl] + part[1][kl]) + (part[2][kl] + part[3][kl]);
}

__global__ __launch_bounds__(256) void lstm_bwd_sum(float *dst, const float *parts, int n, int nparts)
{
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= n) return;
    float s = 0.f;
    for (int q = 0; q < nparts; ++q) s += parts[(int64_t)q * n + e];
    dst[e] = s;
}

__global__ __launch_bounds__(256) void lstm_bwd_copy(float *dst, const float *src, int n)   // src null: zeros
{
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e < n) dst[e] = src ? src[e] : 0.f;
}

// bf16 operands of the backward pass are widened (exactly) to fp32 copies in the workspace: four elements per thread
__global__ __launch_bounds__(256) void lstm_bwd_widen(const bf16_t *src, float *dst, int64_t n)
{
    const int64_t e = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (e + 3 < n) {
        const us4v v = *(const us4v *)(src + e);
        *(float4v *)(dst + e) = float4v{to_f32<bf16_t>(v[0]), to_f32<bf16_t>(v[1]), to_f32<bf16_t>(v[2]), to_f32<bf16_t>(v[3])};
    } else {
        for (int64_t i = e; i < n; ++i) dst[i] = to_f32<bf16_t>(src[i]);
    }
}

static int64_t pad16(int64_t bytes) { return (bytes + 15) & ~(int64_t)15; }

}  // namespace brg

extern "C" int64_t brg_lstm_bwd_ws_bytes(const brg_lstm_desc_t *desc)
{
    if (!desc || desc->T <= 0 || desc->N <= 0 || desc->K <= 0) return 0;
    return (4 * desc->T + 17) * desc->N * desc->K * 4;     // dz [T][N][4K], sixteen partial dh_rec [N][K], ds [N][K]
}

extern "C" int64_t brg_lstm_bwd_ws_bytes_dtype(const brg_lstm_desc_t *desc, brg_dtype_t dtype)
{
    const int64_t base = brg_lstm_bwd_ws_bytes(desc);
    if (base == 0 || dtype != BRG_BF16 || desc->C <= 0) return base;
    // + fp32 copies of x, W4, R4, h and h0
    const int64_t T = desc->T, N = desc->N, C = desc->C, K = desc->K;
    return brg::pad16(base) + brg::pad16(T * N * C * 4) + brg::pad16(4 * K * C * 4) + brg::pad16(4 * K * K * 4) + brg::pad16(T * N * K * 4) +
           brg::pad16(N * K * 4);
}

extern "C" int brg_lstm_bwd(const brg_lstm_desc_t *desc, brg_dtype_t dtype, const void *x, const void *W4, const void *R4,
                            const void *h0, const void *s0, const void *h, const void *s, const void *gates,
                            const void *dh, const void *ds_last, void *dx, float *dW4, float *dR4, float *db4, void *dh0,
                            void *ds0, void *ws, brg_stream_t stream)
{
    using namespace brg;
    BRG_REQUIRE(desc != nullptr, BRG_EINVAL, "brg_lstm_bwd: desc is null");
    BRG_REQUIRE(desc->T > 0 && desc->N > 0 && desc->C > 0 && desc->K > 0 && desc->bc > 0 && desc->bk > 0, BRG_EINVAL,
                "brg_lstm_bwd: sizes must be positive");
    BRG_REQUIRE(desc->C % desc->bc == 0 && desc->K % desc->bk == 0, BRG_EINVAL,
                "brg_lstm_bwd: blocking (%lld,%lld) does not divide (C,K)=(%lld,%lld)", (long long)desc->bc, (long long)desc->bk,
                (long long)desc->C, (long long)desc->K);
    BRG_REQUIRE(desc->T < (1 << 20) && desc->N < (1 << 20) && desc->C < (1 << 20) && desc->K < (1 << 20) &&
                    desc->T * desc->N < (1ll << 30) && desc->N * desc->K < (1ll << 30) && desc->N * desc->C < (1ll << 30),
                BRG_EINVAL, "brg_lstm_bwd: size too large");   // (N*K and N*C are 32-bit element counts of the kernels)
    BRG_REQUIRE(valid_dtype(dtype), BRG_EINVAL, "brg_lstm_bwd: bad dtype");
    BRG_REQUIRE(x && W4 && R4 && h && s && gates && dh && ws, BRG_EINVAL,
                "brg_lstm_bwd: null tensor (x, W4, R4, h, s, gates, dh and ws are required)");
    BRG_REQUIRE(aligned16(x) && aligned16(W4) && aligned16(R4) && aligned16(h0) && aligned16(s0) && aligned16(h) && aligned16(s) &&
                    aligned16(gates) && aligned16(dh) && aligned16(ds_last) && aligned16(dx) && aligned16(dW4) && aligned16(dR4) &&
                    aligned16(db4) && aligned16(dh0) && aligned16(ds0) && aligned16(ws),
                BRG_EALIGN, "brg_lstm_bwd: pointer not 16-byte aligned");
    LstmBwdDims d;
    d.T = (int)desc->T; d.N = (int)desc->N; d.C = (int)desc->C; d.K = (int)desc->K;
    d.bc = (int)desc->bc; d.bk = (int)desc->bk; d.Cb = d.C / d.bc; d.Kb = d.K / d.bk;
    hipStream_t st = (hipStream_t)stream;
    const int NK = d.N * d.K;
    const int64_t TNK = (int64_t)d.T * NK;
    float *dz = (float *)ws, *dh_rec = dz + 4 * TNK, *dsb = dh_rec + 16 * (int64_t)NK;   // dh_rec: up to sixteen partial sums
    if (dtype == BRG_BF16) {
        // x, W4, R4, h, h0 arrive in bf16: the pass runs in fp32 on exact fp32 copies of them (no gradient is rounded to
        // bf16 anywhere); the copies follow the fp32 workspace
        char *p = (char *)ws + pad16(brg_lstm_bwd_ws_bytes(desc));
        const void **srcs[5] = {&x, &W4, &R4, &h, &h0};
        const int64_t counts[5] = {(int64_t)d.T * d.N * d.C, (int64_t)4 * d.K * d.C, (int64_t)4 * d.K * d.K, TNK, (int64_t)NK};
        for (int i = 0; i < 5; ++i) {
            if (*srcs[i]) {
                const int64_t nthr = (counts[i] + 3) / 4;
                hipLaunchKernelGGL(lstm_bwd_widen, dim3((unsigned)((nthr + 255) / 256)), dim3(256), 0, st, (const bf16_t *)*srcs[i], (float *)p,
                                   counts[i]);
                int rcw = check_launch("brg_lstm_bwd (bf16 operands to fp32) launch");
                if (rcw) return rcw;
                *srcs[i] = p;
            }
            p += pad16(counts[i] * 4);
        }
    }
    // 64-wide blocks and whole 64-row batch tiles: the GEMMs run on the 64 x 64 x 64 multi-job kernel
    const bool fast = d.bc == 64 && d.bk == 64 && d.N % 64 == 0 && (int64_t)4 * d.K * d.K < (1ll << 31) && !knobs().lstm_general.set;
    const float *hf = (const float *)h, *sf = (const float *)s, *gf = (const float *)gates, *dhf = (const float *)dh;
    const unsigned eg = (unsigned)((NK + 255) / 256);

    hipLaunchKernelGGL(lstm_bwd_copy, dim3(eg), dim3(256), 0, st, dsb, (const float *)ds_last, NK);
    int rc = check_launch("brg_lstm_bwd (state gradient set-up) launch");
    if (rc) return rc;
    const int nsplit_fast = d.Kb >= 4 ? 4 : (d.Kb >= 2 ? 2 : 1);   // pieces of a gate's chain in the recurrent step (fast path)
    const int nparts_fast = 4 * nsplit_fast;                       // ... and the partial sums they leave
    for (int t = d.T - 1; t >= 0; --t) {
        LstmBwdStepArgs a;
        a.dh_t = dhf + (int64_t)t * NK; a.dh_rec = t == d.T - 1 ? nullptr : dh_rec; a.ds = dsb;
        a.gates_t = gf + (int64_t)t * NK; a.s_t = sf + (int64_t)t * NK;
        a.s_prev = t > 0 ? sf + (int64_t)(t - 1) * NK : (const float *)s0;
        a.dz_t = dz + (int64_t)t * 4 * NK; a.gstride = TNK; a.n = NK; a.K = d.K;
        a.nparts = fast ? nparts_fast : 1;
        hipLaunchKernelGGL(lstm_bwd_step, dim3(eg), dim3(256), 0, st, a);
        rc = check_launch("brg_lstm_bwd (gate gradients) launch");
        if (rc) return rc;
        if (t == 0 && !dh0) break;
        // dh_rec[n][k'] = sum_g sum_k dz_g[t][n][k] R_g[k][k']   (for t = 0 this is dL/dh0)
        if (fast) {
            // sixteen jobs: per gate, the four quarters of the chain over the k blocks (chains of K/256 blocks instead of
            // one chain of 4 K/64: sixteen times the workgroups on this latency-bound step); each leaves a partial sum that
            // the next step's gate kernel adds.
            // Job (g, half): C block (n block, k' block) = chain over k blocks of R4_g block [k'][k] x dz_g[t] block [n][k]
            const int nh = nsplit_fast, per = (d.Kb + nh - 1) / nh;
            G64Args ga = {};
            ga.njobs = 4 * nh;
            for (int q = 0; q < 4 * nh; ++q) {
                const int g = q / nh, kb0 = (q % nh) * per, len = kb0 >= d.Kb ? 0 : (kb0 + per <= d.Kb ? per : d.Kb - kb0);   // (0: that job only writes zeros)
                G64Job &j = ga.job[q];
                j.kind = G64_GEMM;
                j.A = (const float *)R4 + ((int64_t)g * d.Kb + (len ? kb0 : 0)) * d.Kb * 4096;
                j.B = dz + (int64_t)t * 4 * NK + (int64_t)g * d.K + (int64_t)(len ? kb0 : 0) * 64;
                j.C = dh_rec + (int64_t)q * NK; j.act = BRG_ACT_NONE;
                j.tiles_m = d.Kb; j.tiles_n = d.N / 64; j.chain = len; j.alpha = 1.f; j.beta = 0.f;
                j.a_tile = 4096; j.a_chain = (int64_t)d.Kb * 4096; j.b_tile = (int64_t)64 * 4 * d.K; j.b_chain = 64;
                j.c_tile_m = 64; j.c_tile_n = (int64_t)64 * d.K; j.a_ld = 64; j.b_ld = 4 * d.K; j.c_ld = d.K;
                j.a_kfast = 1; j.b_kfast = 1;
            }
            rc = launch_g64(ga, 64, 1, st, "brg_lstm_bwd (recurrent) launch");
            if (rc) return rc;
            if (t == 0) {
                hipLaunchKernelGGL(lstm_bwd_sum, dim3(eg), dim3(256), 0, st, (float *)dh0, (const float *)dh_rec, NK, nparts_fast);
                rc = check_launch("brg_lstm_bwd (initial hidden state gradient) launch");
                if (rc) return rc;
            }
            continue;
        }
        LstmBwdDataProb p;
        p.Wb = (const float *)R4; p.dz = dz + (int64_t)t * 4 * NK; p.out = t == 0 ? (float *)dh0 : dh_rec;
        p.M = d.K; p.Mb = d.Kb; p.bm = d.bk; p.bk = d.bk; p.Kb = d.Kb; p.K = d.K; p.rows = d.N;
        p.tiles_m = (d.K + ENG_TM - 1) / ENG_TM;
        hipLaunchKernelGGL((engine_kernel<LstmBwdDataProb>), dim3(p.tiles_m * ((d.N + ENG_TN - 1) / ENG_TN)), dim3(256), 0, st, p);
        rc = check_launch("brg_lstm_bwd (recurrent) launch");
        if (rc) return rc;
    }
    if (ds0) {
        hipLaunchKernelGGL(lstm_bwd_copy, dim3(eg), dim3(256), 0, st, (float *)ds0, (const float *)dsb, NK);
        rc = check_launch("brg_lstm_bwd (state gradient result) launch");
        if (rc) return rc;
    }
    const int rows = d.T * d.N;
    if (fast) {
        if (dx) {   // dx block (row block, c block) = chain over (gate, k block) of W4 block [c][k] x dz block [row][g K + k]
            G64Args ga = {};
            ga.njobs = 1;
            G64Job &j = ga.job[0];
            j.kind = G64_GEMM;
            j.A = (const float *)W4; j.B = dz; j.C = (float *)dx; j.act = BRG_ACT_NONE;
            j.tiles_m = d.Cb; j.tiles_n = rows / 64; j.chain = 4 * d.Kb; j.alpha = 1.f; j.beta = 0.f;
            j.a_tile = 4096; j.a_chain = (int64_t)d.Cb * 4096; j.b_tile = (int64_t)64 * 4 * d.K; j.b_chain = 64;
            j.c_tile_m = 64; j.c_tile_n = (int64_t)64 * d.C; j.a_ld = 64; j.b_ld = 4 * d.K; j.c_ld = d.C;
            j.a_kfast = 1; j.b_kfast = 1;
            rc = launch_g64(ga, 64, 1, st, "brg_lstm_bwd (input gradient) launch");
            if (rc) return rc;
        }
        // weight gradients: the four gates are four jobs of one launch; block (k block, m block) [m][k] = chain over
        // 64-row blocks of dz_g block [row][k] (rows = reduction) x v block [row][m]
        auto wgt = [&](float *out, const float *v, int M, int Mb, int row_first, int nblk, float beta) {
            G64Args ga = {};
            ga.njobs = 4;
            for (int g = 0; g < 4; ++g) {
                G64Job &j = ga.job[g];
                j.kind = G64_GEMM;
                j.A = dz + (int64_t)row_first * 4 * d.K + (int64_t)g * d.K; j.B = v; j.C = out + (int64_t)g * d.Kb * Mb * 4096; j.act = BRG_ACT_NONE;
                j.tiles_m = d.Kb; j.tiles_n = Mb; j.chain = nblk; j.alpha = 1.f; j.beta = beta;
                j.a_tile = 64; j.a_chain = (int64_t)64 * 4 * d.K; j.b_tile = 64; j.b_chain = (int64_t)64 * M;
                j.c_tile_m = (int64_t)Mb * 4096; j.c_tile_n = 4096; j.a_ld = 4 * d.K; j.b_ld = M; j.c_ld = 64;
                j.a_kfast = 0; j.b_kfast = 0;
            }
            return launch_g64(ga, 64, 1, st, "brg_lstm_bwd (weight gradient) launch");
        };
        if (dW4) {
            rc = wgt(dW4, (const float *)x, d.C, d.Cb, 0, rows / 64, 0.f);
            if (rc) return rc;
        }
        if (dR4) {
            // h_prev of row (t, n) is h[t-1][n]: the rows of time steps 1.. pair with h from its start; those of
            // step 0 with h0 (nothing to add when h0 is null)
            if (d.T > 1) {
                rc = wgt(dR4, hf, d.K, d.Kb, d.N, (rows - d.N) / 64, 0.f);
                if (rc) return rc;
            } else {
                hipLaunchKernelGGL(lstm_bwd_copy, dim3((unsigned)((4 * (int64_t)d.K * d.K + 255) / 256)), dim3(256), 0, st, dR4,
                                   (const float *)nullptr, 4 * d.K * d.K);
                rc = check_launch("brg_lstm_bwd (weight gradient clear) launch");
                if (rc) return rc;
            }
            if (h0) {
                rc = wgt(dR4, (const float *)h0, d.K, d.Kb, 0, d.N / 64, 1.f);
                if (rc) return rc;
            }
        }
        if (db4) {
            hipLaunchKernelGGL(lstm_bwd_bias, dim3((d.K + 63) / 64, 4), dim3(256), 0, st, (const float *)dz, db4, rows, d.K);
            rc = check_launch("brg_lstm_bwd (bias gradient) launch");
            if (rc) return rc;
        }
        return BRG_OK;
    }
    if (dx) {
        LstmBwdDataProb p;
        p.Wb = (const float *)W4; p.dz = dz; p.out = (float *)dx;
        p.M = d.C; p.Mb = d.Cb; p.bm = d.bc; p.bk = d.bk; p.Kb = d.Kb; p.K = d.K; p.rows = rows;
        p.tiles_m = (d.C + ENG_TM - 1) / ENG_TM;
        hipLaunchKernelGGL((engine_kernel<LstmBwdDataProb>), dim3(p.tiles_m * ((rows + ENG_TN - 1) / ENG_TN)), dim3(256), 0, st, p);
        rc = check_launch("brg_lstm_bwd (input gradient) launch");
        if (rc) return rc;
    }
    for (int which = 0; which < 2; ++which) {
        float *out = which ? dR4 : dW4;
        if (!out) continue;
        LstmBwdWgtProb p;
        p.dz = dz; p.out = out; p.K = d.K; p.bk = d.bk; p.Kb = d.Kb; p.rows = rows; p.N = d.N;
        if (which) { p.v = hf; p.v0 = (const float *)h0; p.shift = 1; p.M = d.K; p.bm = d.bk; p.Mb = d.Kb; }
        else { p.v = (const float *)x; p.v0 = nullptr; p.shift = 0; p.M = d.C; p.bm = d.bc; p.Mb = d.Cb; }
        p.tiles_m = (d.K + ENG_TM - 1) / ENG_TM;
        hipLaunchKernelGGL((engine_kernel<LstmBwdWgtProb>), dim3(p.tiles_m * ((p.M + ENG_TN - 1) / ENG_TN), 4), dim3(256), 0, st, p);
        rc = check_launch("brg_lstm_bwd (weight gradient) launch");
        if (rc) return rc;
    }
    if (db4) {
        hipLaunchKernelGGL(lstm_bwd_bias, dim3((d.K + 63) / 64, 4), dim3(256), 0, st, (const float *)dz, db4, rows, d.K);
        rc = check_launch("brg_lstm_bwd (bias gradient) launch");
        if (rc) return rc;
    }
    return BRG_OK;
}
