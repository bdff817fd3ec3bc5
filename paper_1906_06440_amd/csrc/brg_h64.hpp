// Batch-reduce GEMM over 64 x 64 x 64 bf16 blocks on the bf16 matrix instruction (section 2 of the paper:
// the kernel "agnostic of the compute precision"; Algorithm 1), strided or address-list form.
//
// One workgroup of 4 waves (2 x 2) owns one 64 x 64 block of C; every wave keeps a 32 x 32 piece of it in
// four 16x16 accumulator tiles (fp32) across the whole chain and stores it once.  Two workgroups share a
// compute unit, so one's barriers and epilogue hide behind the other's matrix work.
//
//  * A stage is one (A_i, B_i) pair: two blocks of 64 rows x 128 bytes, moved global -> LDS directly
//    (16 bytes per lane, 8 rows per wave instruction) into a ring of three stages, so the loads of two
//    pairs are in flight while one is multiplied; one barrier per stage.  Rows are not padded: the
//    16-byte piece p of row r sits at position p ^ (r & 7) (the lane fetches the piece that belongs
//    at its position), which makes both kinds of fragment read conflict-free.
//  * v_mfma_f32_16x16x32_bf16 wants 8 consecutive reduction elements per lane.  An operand block whose
//    reduction index is contiguous in memory (B of the plain form: column-major k x n) gives them with
//    one ds_read_b128.  A block whose reduction index is the strided one (A of the plain form:
//    column-major m x k) is read through the transposing LDS read of gfx950 (ds_read_b64_tr_b16: inside
//    a 16-lane group lane t points at row t/4, 8-byte quad t%4 of a 16-column strip and receives rows
//    0..3 of column t); two such reads give a lane its 8 reduction elements.  Which operand is which is
//    a template parameter, so transposed blocks (backward passes) need no copy.
//  * Address-list form: the two pointer arrays are read with scalar loads one stage ahead.  Direct
//    loads need 16-byte aligned rows; the arrays live in device memory, so the kernel itself looks at
//    every listed pointer first (each wave scans the list) and, when any block is less aligned, stages
//    all blocks through registers instead (element loads, then one 16-byte LDS store per piece).
#pragma once

#include "brg_common.hpp"

namespace brg {

constexpr int H64_OPER_BYTES = 64 * 128;              // one 64 x 64 bf16 block
constexpr int H64_STAGE_BYTES = 2 * H64_OPER_BYTES;   // A block, B block
constexpr int H64_STAGES = 3;
constexpr size_t H64_SMEM = H64_STAGES * H64_STAGE_BYTES;   // 48 KiB

struct H64Args {
    const bf16_t *A, *B;                            // strided form: block c of tile t at A + t*a_tile + c*a_chain
    const bf16_t *const *A_ptrs, *const *B_ptrs;    // address-list form (DEVICE arrays), used by the PTRS kernels
    void *C;                                        // fp32 or bf16
    const float *bias;                              // per row of C, or null
    int act;
    int tiles_m, tiles_n, chain;
    float alpha, beta;
    int64_t a_tile, a_chain, b_tile, b_chain, c_tile_m, c_tile_n;   // element strides
    int a_ld, b_ld, c_ld;                           // row pitch of the staged blocks / of C, in elements
    // Optional: several stacked problems in one launch.  With m_inner > 0 the row tile tm stands for (tm / m_inner,
    // tm % m_inner) and the C block starts at (tm / m_inner) * c_outer + (tm % m_inner) * c_tile_m; A and bias are
    // indexed by tm as a whole (the four gate matrices of an LSTM, stored back to back).
    int m_inner;
    int64_t c_outer;
    // Ragged last tile column (B blocks with the reduction index contiguous only): when non-zero, C has n_cols
    // columns in all; rows of B beyond them are not read (the last valid row is read again) and not written in C.
    int n_cols;
};

typedef float h64_f2v __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float4v h64_read128(unsigned addr)
{
    float4v v;
    asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr));
    return v;
}

template <int OFF> __device__ __forceinline__ h64_f2v h64_read_tr(unsigned addr)
{
    h64_f2v v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}

// AKF / BKF: the reduction index is the contiguous one in the A / B blocks.
template <bool AKF, bool BKF, bool PTRS, typename TOut> __global__ __launch_bounds__(256, 2) void h64_kernel(H64Args a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char h64_smem[];   // the only LDS object
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)h64_smem;
    const int t = threadIdx.x, lane = t & 63;
    const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
    const int li = lane & 15, kg = lane >> 4;
    const int wm = (wv & 1) * 32, wn = (wv >> 1) * 32;
    const int tm = blockIdx.x % a.tiles_m, tn = blockIdx.x / a.tiles_m;
    const int chain = a.chain;
    const int64_t a_toff = (int64_t)tm * a.a_tile, b_toff = (int64_t)tn * a.b_tile;
    const int64_t a_chain = a.a_chain, b_chain = a.b_chain;

    // ---- staging: wave wv moves rows 16 wv .. 16 wv + 15 of both blocks, 8 rows per instruction.  Lane L sits
    // at row r = r0 + L/8, piece position L%8, and fetches the logical piece (L%8) ^ (r & 7).
    int ga_off[2], gb_off[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int r = 16 * wv + 8 * j + (lane >> 3);
        const int piece = (lane & 7) ^ (r & 7);
        int rb = r;
        if (BKF && a.n_cols && tn * 64 + r >= a.n_cols) rb = a.n_cols - 1 - tn * 64;
        ga_off[j] = r * a.a_ld + piece * 8;
        gb_off[j] = rb * a.b_ld + piece * 8;
    }
    bool direct = true;
    if (PTRS) {
        unsigned bad = (unsigned)((a.a_ld | a.b_ld) & 7) | (unsigned)((a_toff | b_toff) & 7);
        for (int i = lane; i < chain; i += 64)
            bad |= (unsigned)(((uintptr_t)a.A_ptrs[i] | (uintptr_t)a.B_ptrs[i]) & 15u);
        direct = __builtin_amdgcn_ballot_w64(bad != 0u) == 0ull;      // the same answer in every wave
    }
    typedef unsigned short h64_us8 __attribute__((ext_vector_type(8)));
#define H64_ISSUE(I, BUF)                                                                              \
    {                                                                                                  \
        const bf16_t *pa_, *pb_;                                                                       \
        if (PTRS) {                                                                                    \
            pa_ = a.A_ptrs[I] + a_toff;                                                                \
            pb_ = a.B_ptrs[I] + b_toff;                                                                \
        } else {                                                                                       \
            pa_ = a.A + a_toff + (int64_t)(I) * a_chain;                                               \
            pb_ = a.B + b_toff + (int64_t)(I) * b_chain;                                               \
        }                                                                                              \
        unsigned char *dA_ = h64_smem + (BUF) * H64_STAGE_BYTES + (16 * wv) * 128;                     \
        unsigned char *dB_ = dA_ + H64_OPER_BYTES;                                                     \
        if (!PTRS || direct) {                                                                         \
            _Pragma("unroll") for (int j = 0; j < 2; ++j)                                              \
            {                                                                                          \
                __builtin_amdgcn_global_load_lds(pa_ + ga_off[j], (bf16_t *)(dA_ + j * 1024), 16, 0, 0); \
                __builtin_amdgcn_global_load_lds(pb_ + gb_off[j], (bf16_t *)(dB_ + j * 1024), 16, 0, 0); \
            }                                                                                          \
        } else {                                                                                       \
            _Pragma("unroll") for (int j = 0; j < 2; ++j)                                              \
            {                                                                                          \
                h64_us8 va_, vb_;                                                                      \
                _Pragma("unroll") for (int e = 0; e < 8; ++e)                                          \
                {                                                                                      \
                    va_[e] = pa_[ga_off[j] + e];                                                       \
                    vb_[e] = pb_[gb_off[j] + e];                                                       \
                }                                                                                      \
                *(h64_us8 *)(dA_ + j * 1024 + lane * 16) = va_;                                        \
                *(h64_us8 *)(dB_ + j * 1024 + lane * 16) = vb_;                                        \
            }                                                                                          \
        }                                                                                              \
    }

    // ---- fragment addresses (bytes from the start of a stage).
    // reduction-contiguous block: row i = w? + 16 x + li, k sub-step s: logical piece 4 s + kg, one ds_read_b128.
    // reduction-strided block: strip of 16 columns at w? + 16 x; the lane points at row 32 s + 8 kg + li/4 (+ 4 for
    //   the second read), 8-byte quad li % 4 of the strip; s is an immediate offset of 32 rows.
    unsigned fa[2][2], fb[2][2];
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            if (AKF) {
                const int i = wm + 16 * x + li;
                fa[x][h] = lds0 + i * 128 + (((4 * h + kg) ^ (i & 7)) << 4);
            } else {
                const int col = wm + 16 * x + 4 * (li & 3), row = 8 * kg + (li >> 2) + 4 * h;
                fa[x][h] = lds0 + row * 128 + (((col >> 3) ^ (row & 7)) << 4) + ((col >> 2) & 1) * 8;
            }
            if (BKF) {
                const int i = wn + 16 * x + li;
                fb[x][h] = lds0 + H64_OPER_BYTES + i * 128 + (((4 * h + kg) ^ (i & 7)) << 4);
            } else {
                const int col = wn + 16 * x + 4 * (li & 3), row = 8 * kg + (li >> 2) + 4 * h;
                fb[x][h] = lds0 + H64_OPER_BYTES + row * 128 + (((col >> 3) ^ (row & 7)) << 4) + ((col >> 2) & 1) * 8;
            }
        }

    float4v acc[2][2];
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y) acc[x][y] = float4v{0.f, 0.f, 0.f, 0.f};

    if (chain > 0) H64_ISSUE(0, 0)
    if (chain > 1) H64_ISSUE(1, 1)

    int buf = 0;
    for (int it = 0; it < chain; ++it) {
        // my share of stage `it` has landed (the four loads of stage it+1 may stay in flight) ...
        if (it + 1 < chain) asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();   // ... so has everybody's, and nobody still reads the stage before it
        asm volatile("" ::: "memory");
        if (it + 2 < chain) {
            const int nb = buf == 0 ? 2 : buf - 1;           // (it + 2) % 3
            H64_ISSUE(it + 2, nb)
        }
        const unsigned sb = (unsigned)(buf * H64_STAGE_BYTES);
        // fragments of both k sub-steps: reduction-contiguous operands f?[x][s], strided ones two 8-byte halves
        float4v af[2][2], bf[2][2];
        h64_f2v at[2][2][2], bt[2][2][2];
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            if (AKF) {
                af[x][0] = h64_read128(sb + fa[x][0]);
                af[x][1] = h64_read128(sb + fa[x][1]);
            } else {
                at[x][0][0] = h64_read_tr<0>(sb + fa[x][0]);
                at[x][0][1] = h64_read_tr<0>(sb + fa[x][1]);
                at[x][1][0] = h64_read_tr<32 * 128>(sb + fa[x][0]);
                at[x][1][1] = h64_read_tr<32 * 128>(sb + fa[x][1]);
            }
            if (BKF) {
                bf[x][0] = h64_read128(sb + fb[x][0]);
                bf[x][1] = h64_read128(sb + fb[x][1]);
            } else {
                bt[x][0][0] = h64_read_tr<0>(sb + fb[x][0]);
                bt[x][0][1] = h64_read_tr<0>(sb + fb[x][1]);
                bt[x][1][0] = h64_read_tr<32 * 128>(sb + fb[x][0]);
                bt[x][1][1] = h64_read_tr<32 * 128>(sb + fb[x][1]);
            }
        }
        if (AKF) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(af[0][0]), "+v"(af[0][1]), "+v"(af[1][0]), "+v"(af[1][1]));
        else asm volatile("s_waitcnt lgkmcnt(0)"
                          : "+v"(at[0][0][0]), "+v"(at[0][0][1]), "+v"(at[0][1][0]), "+v"(at[0][1][1]), "+v"(at[1][0][0]),
                            "+v"(at[1][0][1]), "+v"(at[1][1][0]), "+v"(at[1][1][1]));
        if (BKF) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(bf[0][0]), "+v"(bf[0][1]), "+v"(bf[1][0]), "+v"(bf[1][1]));
        else asm volatile("s_waitcnt lgkmcnt(0)"
                          : "+v"(bt[0][0][0]), "+v"(bt[0][0][1]), "+v"(bt[0][1][0]), "+v"(bt[0][1][1]), "+v"(bt[1][0][0]),
                            "+v"(bt[1][0][1]), "+v"(bt[1][1][0]), "+v"(bt[1][1][1]));
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            bf16x8v av[2], bv[2];
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                av[x] = AKF ? __builtin_bit_cast(bf16x8v, af[x][s])
                            : __builtin_bit_cast(bf16x8v, float4v{at[x][s][0][0], at[x][s][0][1], at[x][s][1][0], at[x][s][1][1]});
                bv[x] = BKF ? __builtin_bit_cast(bf16x8v, bf[x][s])
                            : __builtin_bit_cast(bf16x8v, float4v{bt[x][s][0][0], bt[x][s][0][1], bt[x][s][1][0], bt[x][s][1][1]});
            }
#pragma unroll
            for (int x = 0; x < 2; ++x)
#pragma unroll
                for (int y = 0; y < 2; ++y) acc[x][y] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[x], bv[y], acc[x][y], 0, 0, 0);
        }
        buf = buf == 2 ? 0 : buf + 1;
    }
#undef H64_ISSUE

    // ---- epilogue: register r of lane l of tile (x, y) is row m = 16 x + 4 (l / 16) + r, column n = 16 y + l % 16
    // of the wave's piece; a lane owns runs of four consecutive m, the contiguous index of C.
    TOut *Cb = (TOut *)a.C + tn * a.c_tile_n +
               (a.m_inner > 0 ? (tm / a.m_inner) * a.c_outer + (tm % a.m_inner) * a.c_tile_m : tm * a.c_tile_m);
#pragma unroll
    for (int x = 0; x < 2; ++x) {
        const int m = wm + 16 * x + 4 * kg;
        float4v bv = {0.f, 0.f, 0.f, 0.f};
        if (a.bias) bv = *(const float4v *)(a.bias + tm * 64 + m);
#pragma unroll
        for (int y = 0; y < 2; ++y) {
            const int n = wn + 16 * y + li;
            if (a.n_cols && tn * 64 + n >= a.n_cols) continue;
            TOut *dst = Cb + (int64_t)n * a.c_ld + m;
            float4v v = acc[x][y] * a.alpha;
            if (a.beta != 0.f) {
                if (std::is_same<TOut, float>::value) {
                    v += a.beta * *(const float4v *)dst;
                } else {
                    const us4v old = *(const us4v *)dst;
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] += a.beta * bf16_to_f32(old[r]);
                }
            }
            v += bv;
            v = act_is_slow(a.act) ? apply_act4<true>(v, a.act) : apply_act4<false>(v, a.act);
            if (std::is_same<TOut, float>::value) *(float4v *)dst = v;
            else *(us4v *)dst = pack_bf16x4(v);
        }
    }
}

template <bool AKF, bool BKF, bool PTRS, typename TOut> static int launch_h64(const H64Args &a, hipStream_t s, const char *who)
{
    hipLaunchKernelGGL((h64_kernel<AKF, BKF, PTRS, TOut>), dim3((unsigned)(a.tiles_m * a.tiles_n)), dim3(256), H64_SMEM, s, a);
    return check_launch(who);
}

}  // namespace brg
