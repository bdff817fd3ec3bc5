// brg_gemm / brg_gemm_strided: the batch-reduce GEMM of section 2 of the paper,
//   C = act(beta*C + alpha * sum_i A_i*B_i + bias),
// for arbitrary m, n, k and leading dimensions.  Chains of 64-deep blocks with m and n multiples of 64 --
// the shape of config 1 and of every block call of the fully connected and LSTM layers -- run on the staged
// kernels: fp32 on the four-stage ring (brg_block_ring.hpp), bf16 on the bf16 matrix instruction
// (brg_h64.hpp), in the strided AND in the address-list form.  Everything else takes the general tile engine.
#include <cstdlib>

#include "brg_block_dma.hpp"
#include "brg_block_ring.hpp"
#include "brg_engine.hpp"
#include "brg_h64.hpp"

namespace brg {

template <typename TIn, typename TOut, bool PTRS> struct GemmProb {
    static constexpr bool A_KFAST = false;  // column-major m x k: rows contiguous
    static constexpr bool B_KFAST = true;   // column-major k x n: reduction index contiguous
    int m, n, k, count;
    int64_t lda, ldb, ldc;
    const void *const *A_ptrs, *const *B_ptrs;
    const TIn *A, *B;
    int64_t strideA, strideB;
    TOut *C;
    float alpha, beta;
    const float *bias;
    int act;
    int tiles_m;

    typedef int64_t RowA;  // row index or -1
    typedef int64_t RowB;  // column offset j*ldb or -1
    struct Chain {
        const TIn *a, *b;
    };

    __device__ int tile_m0() const { return (blockIdx.x % tiles_m) * ENG_TM; }
    __device__ int tile_n0() const { return (blockIdx.x / tiles_m) * ENG_TN; }
    __device__ int chain_len() const { return count; }
    __device__ int kdepth(int) const { return k; }
    __device__ RowA row_a(int i) const
    {
        int r = tile_m0() + i;
        return r < m ? (int64_t)r : -1;
    }
    __device__ RowB row_b(int j) const
    {
        int c = tile_n0() + j;
        return c < n ? (int64_t)c * ldb : -1;
    }
    __device__ Chain chain(int c) const
    {
        Chain ch;
        if (PTRS) {
            ch.a = (const TIn *)A_ptrs[c];
            ch.b = (const TIn *)B_ptrs[c];
        } else {
            ch.a = A + (int64_t)c * strideA;
            ch.b = B + (int64_t)c * strideB;
        }
        return ch;
    }
    __device__ float a(const Chain &ch, const RowA &r, int p) const
    {
        return r >= 0 ? to_f32<TIn>(ch.a[r + (int64_t)p * lda]) : 0.f;
    }
    __device__ float b(const Chain &ch, const RowB &r, int p) const
    {
        return r >= 0 ? to_f32<TIn>(ch.b[r + p]) : 0.f;
    }
    __device__ void store4(int i, int j, float4v acc) const
    {
        int col = tile_n0() + j;
        if (col >= n) return;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            int row = tile_m0() + i + r;
            if (row >= m) continue;
            TOut *dst = C + row + (int64_t)col * ldc;
            float v = alpha * acc[r];
            if (beta != 0.f) v += beta * to_f32<TOut>(*dst);
            if (bias) v += bias[row];
            *dst = from_f32<TOut>(apply_act(v, act));
        }
    }
};

template <typename TIn, typename TOut, bool PTRS>
static int launch_gemm(int64_t m, int64_t n, int64_t k, int64_t lda, int64_t ldb, int64_t ldc,
                       const void *const *A_ptrs, const void *const *B_ptrs, const void *A,
                       int64_t strideA, const void *B, int64_t strideB, void *C, int64_t count,
                       float alpha, float beta, const float *bias, int act, hipStream_t stream)
{
    GemmProb<TIn, TOut, PTRS> p;
    p.m = (int)m; p.n = (int)n; p.k = (int)k; p.count = (int)count;
    p.lda = lda; p.ldb = ldb; p.ldc = ldc;
    p.A_ptrs = A_ptrs; p.B_ptrs = B_ptrs;
    p.A = (const TIn *)A; p.B = (const TIn *)B;
    p.strideA = strideA; p.strideB = strideB;
    p.C = (TOut *)C;
    p.alpha = alpha; p.beta = beta; p.bias = bias; p.act = act;
    p.tiles_m = (int)((m + ENG_TM - 1) / ENG_TM);
    const int64_t tiles_n = (n + ENG_TN - 1) / ENG_TN;
    BRG_REQUIRE((int64_t)p.tiles_m * tiles_n < (1ll << 31), BRG_EINVAL, "brg_gemm: %lld x %lld tiles exceed the grid limit",
                (long long)p.tiles_m, (long long)tiles_n);
    dim3 grid((unsigned)((int64_t)p.tiles_m * tiles_n));
    hipLaunchKernelGGL((engine_kernel<GemmProb<TIn, TOut, PTRS>>), grid, dim3(256), 0, stream, p);
    return check_launch("brg_gemm launch");
}

static int gemm_common(int dtype, int out_dtype, int64_t m, int64_t n, int64_t k, int64_t lda,
                       int64_t ldb, int64_t ldc, bool ptrs, const void *const *A_ptrs,
                       const void *const *B_ptrs, const void *A, int64_t strideA, const void *B,
                       int64_t strideB, void *C, int64_t count, float alpha, float beta,
                       const float *bias, int act, brg_stream_t stream)
{
    BRG_REQUIRE(valid_dtype(dtype) && valid_dtype(out_dtype), BRG_EINVAL, "brg_gemm: bad dtype");
    BRG_REQUIRE(valid_act(act), BRG_EINVAL, "brg_gemm: bad activation %d", act);
    BRG_REQUIRE(m >= 0 && n >= 0 && k >= 0 && count >= 0, BRG_EINVAL, "brg_gemm: negative size");
    BRG_REQUIRE(m < (1 << 30) && n < (1 << 30) && k < (1 << 30) && count < (1 << 30), BRG_EINVAL,
                "brg_gemm: size too large");
    BRG_REQUIRE(lda >= (m > 1 ? m : 1) && ldb >= (k > 1 ? k : 1) && ldc >= (m > 1 ? m : 1), BRG_EINVAL,
                "brg_gemm: leading dimension smaller than the block (lda=%lld ldb=%lld ldc=%lld)",
                (long long)lda, (long long)ldb, (long long)ldc);
    BRG_REQUIRE(C != nullptr, BRG_EINVAL, "brg_gemm: C is null");
    if (count > 0 && k > 0) {
        if (ptrs) BRG_REQUIRE(A_ptrs && B_ptrs, BRG_EINVAL, "brg_gemm: null pointer array");
        else BRG_REQUIRE(A && B, BRG_EINVAL, "brg_gemm: null A or B");
    }
    if (!ptrs) BRG_REQUIRE(strideA >= 0 && strideB >= 0, BRG_EINVAL, "brg_gemm_strided: negative stride");
    BRG_REQUIRE(aligned16(C) && aligned16(bias) && aligned16(A_ptrs) && aligned16(B_ptrs) &&
                    aligned16(A) && aligned16(B),
                BRG_EALIGN, "brg_gemm: pointer not 16-byte aligned");
    if (m == 0 || n == 0) return BRG_OK;
    if (count == 0 || k == 0) count = 0;
    hipStream_t s = (hipStream_t)stream;
    const bool blocks64 = count > 0 && k == 64 && m % 64 == 0 && n % 64 == 0 && ldc % 4 == 0 && lda < (1 << 24) &&
                          ldb < (1 << 24) && ldc < (1 << 24) && (m / 64) * (n / 64) < (1ll << 31) && !knobs().gemm_general.set;
    // 64 x 64 x 64 fp32 blocks: the ring kernel.  Strided form: rows must be 16-byte aligned (decided here);
    // address-list form: chains of at least four blocks, alignment decided inside the kernel.
    if (blocks64 && dtype == BRG_F32 && out_dtype == BRG_F32 &&
        (ptrs ? count >= 4 : (lda % 4 == 0 && ldb % 4 == 0 && strideA % 4 == 0 && strideB % 4 == 0))) {
        BlockTileArgs a = {};
        a.A = (const float *)A; a.B = (const float *)B; a.C = (float *)C; a.bias = bias; a.act = act;
        a.A_ptrs = (const float *const *)A_ptrs; a.B_ptrs = (const float *const *)B_ptrs;
        a.tiles_m = (int)(m / 64); a.tiles_n = (int)(n / 64); a.chain = (int)count; a.alpha = alpha; a.beta = beta;
        a.a_tile = 64; a.a_chain = strideA; a.b_tile = 64 * ldb; a.b_chain = strideB;
        a.c_tile_m = 64; a.c_tile_n = 64 * ldc; a.a_ld = (int)lda; a.b_ld = (int)ldb; a.c_ld = (int)ldc;
        if (ptrs) return launch_block_ring<false, true, true>(a, s, "brg_gemm launch");
        return launch_block_ring<false, true>(a, s, "brg_gemm_strided launch");
    }
    // 64 x 64 x 64 bf16 blocks: the bf16 matrix-instruction kernel (A blocks through the transposing LDS read)
    if (blocks64 && dtype == BRG_BF16 &&
        (ptrs || (lda % 8 == 0 && ldb % 8 == 0 && strideA % 8 == 0 && strideB % 8 == 0))) {
        H64Args a = {};
        a.A = (const bf16_t *)A; a.B = (const bf16_t *)B; a.C = C; a.bias = bias; a.act = act;
        a.A_ptrs = (const bf16_t *const *)A_ptrs; a.B_ptrs = (const bf16_t *const *)B_ptrs;
        a.tiles_m = (int)(m / 64); a.tiles_n = (int)(n / 64); a.chain = (int)count; a.alpha = alpha; a.beta = beta;
        a.a_tile = 64; a.a_chain = strideA; a.b_tile = 64 * ldb; a.b_chain = strideB;
        a.c_tile_m = 64; a.c_tile_n = 64 * ldc; a.a_ld = (int)lda; a.b_ld = (int)ldb; a.c_ld = (int)ldc;
        const char *who = ptrs ? "brg_gemm (bf16) launch" : "brg_gemm_strided (bf16) launch";
        if (out_dtype == BRG_F32) return ptrs ? launch_h64<false, true, true, float>(a, s, who) : launch_h64<false, true, false, float>(a, s, who);
        return ptrs ? launch_h64<false, true, true, bf16_t>(a, s, who) : launch_h64<false, true, false, bf16_t>(a, s, who);
    }
#define BRG_GEMM_GO(TI, TO)                                                                         \
    return ptrs ? launch_gemm<TI, TO, true>(m, n, k, lda, ldb, ldc, A_ptrs, B_ptrs, A, strideA, B,  \
                                            strideB, C, count, alpha, beta, bias, act, s)           \
                : launch_gemm<TI, TO, false>(m, n, k, lda, ldb, ldc, A_ptrs, B_ptrs, A, strideA, B, \
                                             strideB, C, count, alpha, beta, bias, act, s)
    if (dtype == BRG_F32 && out_dtype == BRG_F32) { BRG_GEMM_GO(float, float); }
    if (dtype == BRG_BF16 && out_dtype == BRG_F32) { BRG_GEMM_GO(bf16_t, float); }
    if (dtype == BRG_BF16 && out_dtype == BRG_BF16) { BRG_GEMM_GO(bf16_t, bf16_t); }
#undef BRG_GEMM_GO
    return fail(BRG_EUNSUPPORTED, "brg_gemm: fp32 inputs with bf16 output are not supported");
}

}  // namespace brg

extern "C" int brg_gemm(brg_dtype_t dtype, brg_dtype_t out_dtype, int64_t m, int64_t n, int64_t k,
                        int64_t lda, int64_t ldb, int64_t ldc, const void *const *A_ptrs,
                        const void *const *B_ptrs, void *C, int64_t count, float alpha, float beta,
                        const float *bias, brg_act_t act, brg_stream_t stream)
{
    return brg::gemm_common(dtype, out_dtype, m, n, k, lda, ldb, ldc, true, A_ptrs, B_ptrs, nullptr, 0,
                            nullptr, 0, C, count, alpha, beta, bias, act, stream);
}

extern "C" int brg_gemm_strided(brg_dtype_t dtype, brg_dtype_t out_dtype, int64_t m, int64_t n,
                                int64_t k, int64_t lda, int64_t ldb, int64_t ldc, const void *A,
                                int64_t strideA, const void *B, int64_t strideB, void *C,
                                int64_t count, float alpha, float beta, const float *bias,
                                brg_act_t act, brg_stream_t stream)
{
    return brg::gemm_common(dtype, out_dtype, m, n, k, lda, ldb, ldc, false, nullptr, nullptr, A,
                            strideA, B, strideB, C, count, alpha, beta, bias, act, stream);
}
