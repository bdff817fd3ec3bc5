// Persistent recurrent kernel of the LSTM forward pass (paper section 3.1, Algorithm 2).
//
// Algorithm 2 runs, per time step and output block, one reduce chain over the C/bc blocks of
// W_g * x_t followed by the K/bk blocks of R_g * h_{t-1}.  The first half does not depend on the
// recurrence, so it is computed for ALL time steps up front as four batch-reduce GEMMs (one per
// gate, bias fused) that leave the partial pre-activations in the `gates` buffer.  This kernel
// continues every chain with the recurrent half and applies the gate non-linearities and the state
// update on the accumulators, overwriting the partial sums in place with the gate values.
//
//  * One workgroup per CU for the WHOLE sequence; workgroup c owns hidden units 4c .. 4c+3 with all
//    four gates = 16 rows of the stacked recurrent matrix, i.e. one 16-row MFMA tile whose rows are
//    ordered (unit, gate): the four pre-activations of a (unit, batch) element land in the four
//    accumulator registers of one lane, so sigma / tanh / cell update need no data exchange.
//  * Its 16 x K slice of R (64 KiB for K = 1024) is loaded into LDS once and stays there for all T
//    steps (the "weights reused from cache" of the paper, made explicit).
//  * Per step every workgroup streams h_{t-1} (N x K) through wave-private rings of direct global->LDS
//    loads in chunks of 64 reduction elements.  8 waves: wave w multiplies batch rows 16 (w % 4) ..
//    + 15 with the chunks of parity w / 4, so every SIMD holds two waves with independent loads,
//    fragment reads and matrix instructions (one wave's load issue and LDS round trip hide behind
//    the other's MFMAs); the two partial sums of a batch tile are added through LDS before the gate math.
//  * The dependency "all of h_t before step t+1" is a grid barrier: a release/acquire counter in
//    device memory.  The spin is bounded; on expiry every workgroup sets an error flag and leaves.
#pragma once

#include "brg_common.hpp"
#include "brg_g64.hpp"

namespace brg {

constexpr int LR_LD = 1028;                       // padded row length of the R slice in LDS (floats)
constexpr int LR_RS_BYTES = 16 * LR_LD * 4;       // 65792
constexpr int LR_SLOT_BYTES = 16 * 64 * 4;        // one wave's share of an h chunk: 16 batch rows x 64 reduction elements
constexpr int LR_WAVES = 8;
constexpr int LR_RING = 2;                        // slots per wave
constexpr size_t LR_SMEM = LR_RS_BYTES + LR_WAVES * LR_RING * LR_SLOT_BYTES;   // 131328 bytes

struct LstmRecArgs {
    const void *R4;        // [4][Kb][Kb][64][64] blocked recurrent weights (fp32, or bf16 for the bf16 kernel)
    const void *h0;        // [N][K] or null (fp32 / bf16)
    const float *s0;       // [N][K] or null
    void *h;               // [T][N][K] (fp32 / bf16)
    float *s;              // [T][N][K]
    float *gates;          // [4][T][N][K]: in = W x + b, out = gate values
    unsigned *sync;        // sync[0] = barrier counter, sync[1] = error flag (both zero at launch)
    int T, N, K;
    unsigned spin_limit;
};

// Grid barrier of one time step: every workgroup has stored its part of h[ts-1] (`target` arrivals).  Returns
// true when the wait gave up (the same value for the whole workgroup).
__device__ __forceinline__ bool lr_step_barrier(unsigned *sync, unsigned target, unsigned spin_limit, int *bail, int t)
{
    if (t == 0) {
        unsigned spins = 0, bad = 0;
        while (__hip_atomic_load(sync, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            ++spins;
            if ((spins & 63u) == 0 && __hip_atomic_load(sync + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) bad = 1;
            if (spins > spin_limit) bad = 1;
            if (bad) break;
        }
        if (bad) __hip_atomic_store(sync + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *bail = (int)bad;
    }
    __syncthreads();
    return *bail != 0;
    // ASSUMPTION (outside what the memory model promises, checked by the parity tests on every run):
    // no acquire follows the barrier.  h[ts-1] was written through to memory (device-scope stores) before
    // the counter moved, and the step relies on no cache on the reading side holding an older copy of
    // those addresses: every launch starts with clean caches, h[ts-1] is read by nobody before this
    // point, and the L2 of an XCD whose own workgroups wrote 16-byte (bf16: 8-byte) pieces of a 128-byte
    // line of h[ts-1] must not serve the other pieces of that line from a copy fetched before their
    // writers stored them (it does not: write-through stores of part of a line do not make the L2 fetch
    // and keep the rest of it).  It breaks if anything reads h[ts-1] before the barrier (a prefetch, a
    // wider store that reads the line first) or if a later part allocates whole lines on partial
    // write-through stores.  The fence that would make it formal was measured: an agent-scope acquire
    // here (L2 invalidate on all 8 XCDs) takes the fp32 step from 12.6 to 28 us, acquire plus a release
    // before the arrival to 75 us.
}

// NP = number of 64-row batch passes per time step (N <= 64 NP): the workgroup streams the rows of one pass at
// a time through the same rings, so larger minibatches (the paper's N = 168) stay on the resident kernel.
template <int NP> __global__ __launch_bounds__(512, 1) void lstm_rec_kernel(LstmRecArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lr_smem[];
    __shared__ int lr_bail;
    __shared__ float4v lr_xch[2][4][64];           // partial sums of the odd-chunk waves (two passes in flight)
    float *Rs = (float *)lr_smem;
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lr_smem;
    const int t = threadIdx.x, lane = t & 63;
    const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
    const int bt = wv & 3, hf = wv >> 2;           // batch tile, chunk parity
    const int li = lane & 15, kg = lane >> 4;
    const int cu = blockIdx.x, nwg = gridDim.x;
    const int K = a.K, Kb = K >> 6;
    const int64_t NK = (int64_t)a.N * K, TNK = (int64_t)a.T * NK;
    const float *R4 = (const float *)a.R4, *h0 = (const float *)a.h0;
    float *hout = (float *)a.h;

    // ---- recurrent weights of units 4cu .. 4cu+3, all gates -> LDS rows 4u + g, k contiguous.
    // Element R_g[k_out][k_in] sits at R4[g][k_out/64][k_in/64][k_in%64][k_out%64]: one float4 holds
    // the four units of this workgroup for one (g, k_in).
    {
        const int kb_out = (4 * cu) >> 6, kf = (4 * cu) & 63;
        for (int e = t; e < 4 * K; e += 512) {
            const int g = e / K, kin = e - g * K;
            const float4v v = *(const float4v *)(R4 + ((((int64_t)g * Kb + kb_out) * Kb + (kin >> 6)) * 64 + (kin & 63)) * 64 + kf);
#pragma unroll
            for (int u = 0; u < 4; ++u) Rs[(4 * u + g) * LR_LD + kin] = v[u];
        }
    }
    if (t == 0) lr_bail = 0;
    __syncthreads();

    // fragment addresses: A = R slice row li, B = row li of this wave's slot, piece (4s + kg) ^ li
    const unsigned a_addr = lds0 + (li * LR_LD + 4 * kg) * 4;
    const unsigned ring0 = LR_RS_BYTES + wv * LR_RING * LR_SLOT_BYTES;
    unsigned b_addr[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) b_addr[s] = lds0 + ring0 + li * 256 + (((4 * s + kg) ^ li) << 4);

    // direct loads of one chunk: in pass p the wave moves its batch rows 64 p + 16 bt .. + 15, 4 rows per instruction
    int g_off[4][4];   // (first NP rows used; a bound that depends on NP keeps the host pass from emitting the kernel)
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int rl = 4 * j + (lane >> 4);              // row inside the slot
            int r = 64 * p + 16 * bt + rl;
            const int piece = (lane & 15) ^ rl;
            if (r >= a.N) r = a.N - 1;                       // rows beyond the batch: harmless duplicates
            g_off[p][j] = r * K + piece * 4;
        }

    const int nchunk = K >> 6;
    const int unit = 4 * cu + kg;
    // the cell state of (n, unit) is produced and consumed by this lane only: it lives in a register
    float s_reg[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int n = 64 * p + 16 * bt + li;
        s_reg[p] = (n < a.N && hf == 0 && a.s0) ? a.s0[(int64_t)n * K + unit] : 0.f;
    }

    for (int ts = 0; ts < a.T; ++ts) {
        const float *hprev = ts ? hout + (int64_t)(ts - 1) * NK : h0;
        // partial pre-activations W x + b of this step: independent of the recurrence, so the loads are
        // in flight while the workgroup waits at the barrier
        float zx[NP][4];
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int n = 64 * p + 16 * bt + li;
            const int64_t e = (int64_t)ts * NK + (int64_t)n * K + unit;
#pragma unroll
            for (int g = 0; g < 4; ++g) zx[p][g] = 0.f;
            if (n < a.N && hf == 0) {
#pragma unroll
                for (int g = 0; g < 4; ++g) zx[p][g] = a.gates[g * TNK + e];
            }
        }
        // ---- grid barrier: every workgroup has stored its part of h[ts-1]
        if (ts > 0 && lr_step_barrier(a.sync, (unsigned)ts * (unsigned)nwg, a.spin_limit, &lr_bail, t)) return;

#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int n = 64 * p + 16 * bt + li;
            const bool row_ok = n < a.N && hf == 0;        // the even-chunk waves finish the step
            const int64_t e = (int64_t)ts * NK + (int64_t)n * K + unit;
            float4v acc = {0.f, 0.f, 0.f, 0.f}, acc2 = {0.f, 0.f, 0.f, 0.f};
            if (hprev) {
                // A wave moves and consumes its own rows and chunks only, so its ring needs no workgroup
                // barrier: it waits for its own loads.
#define LR_ISSUE(C, SLOT)                                                                                        \
    {                                                                                                            \
        float *dst_ = (float *)(lr_smem + ring0 + (SLOT) * LR_SLOT_BYTES);                                       \
        const float *src_ = hprev + (C) * 64;                                                                    \
        _Pragma("unroll") for (int j = 0; j < 4; ++j)                                                            \
            __builtin_amdgcn_global_load_lds(src_ + g_off[p][j], dst_ + j * 256, 16, 0, 0);                      \
    }
                // every load and store issued before this pass is older than its chunk loads, so the counts
                // below cover them
                const int nmy = (nchunk - hf + 1) >> 1;      // chunks hf, hf + 2, ...
                if (nmy > 0) LR_ISSUE(hf, 0)
                if (nmy > 1) LR_ISSUE(hf + 2, 1)
                for (int i = 0; i < nmy; ++i) {
                    const int c = hf + 2 * i;
                    // chunk c has landed when at most the loads of the next one are outstanding
                    if (i + 1 < nmy) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
                    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                    const unsigned sb = (unsigned)((i & 1) * LR_SLOT_BYTES);
                    const unsigned sa = (unsigned)(c * 64 * 4);
                    float4v af[4], bf[4];
#pragma unroll
                    for (int s = 0; s < 4; ++s) {
                        af[s] = g64_read128(a_addr + sa + s * 64);
                        bf[s] = g64_read128(b_addr[s] + sb);
                    }
                    asm volatile("s_waitcnt lgkmcnt(0)"
                                 : "+v"(af[0]), "+v"(af[1]), "+v"(af[2]), "+v"(af[3]), "+v"(bf[0]), "+v"(bf[1]), "+v"(bf[2]),
                                   "+v"(bf[3]));
                    // the slot's fragments are in registers: refill it with the chunk after the next
                    if (i + 2 < nmy) LR_ISSUE(c + 4, i & 1)
                    // two accumulators take turns: a single dependent chain of 16x16x4 MFMAs issues at only
                    // two thirds of the matrix-pipe rate
#pragma unroll
                    for (int s = 0; s < 4; ++s)
#pragma unroll
                        for (int q = 0; q < 4; q += 2) {
                            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(af[s][q], bf[s][q], acc, 0, 0, 0);
                            acc2 = __builtin_amdgcn_mfma_f32_16x16x4f32(af[s][q + 1], bf[s][q + 1], acc2, 0, 0, 0);
                        }
                }
            }
#undef LR_ISSUE
            // ---- the odd-chunk waves hand their partial sums to the even-chunk waves of the same batch tile
            if (hf == 1) lr_xch[p & 1][bt][lane] = acc + acc2;
            __syncthreads();
            if (hf == 0) acc += lr_xch[p & 1][bt][lane];

            // ---- gates and state update on the accumulators (register r = gate r of unit kg, batch row n)
            if (row_ok) {
                float z[4];
#pragma unroll
                for (int g = 0; g < 4; ++g) z[g] = (acc[g] + acc2[g]) + zx[p][g];
                const float it = sigmoidf_(z[0]), ct = tanhf(z[1]), ft = sigmoidf_(z[2]), ot = sigmoidf_(z[3]);
                s_reg[p] = ft * s_reg[p] + it * ct;
                const float ht = ot * tanhf(s_reg[p]);
                // h is what the other workgroups wait for: written through to memory (device scope)
                __hip_atomic_store(hout + e, ht, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                a.s[e] = s_reg[p];
                a.gates[e] = it;
                a.gates[TNK + e] = ct;
                a.gates[2 * TNK + e] = ft;
                a.gates[3 * TNK + e] = ot;
            }
        }
        // ---- arrive: all stores of this workgroup have completed before the counter moves
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (t == 0) __hip_atomic_fetch_add(a.sync, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// ---- the same recurrence with bf16 operands (section 2 of the paper: the kernel is agnostic of the compute
// precision): R and h are bf16, the products go through v_mfma_f32_16x16x32_bf16 (fp32 accumulation), the cell
// state, the gate values and the partial pre-activations stay fp32.  h_t is rounded to bf16 once, when it is
// stored, and that stored value is what step t+1 multiplies.  The R slice (16 rows x K bf16, rows padded by
// 16 bytes) and the rings (16 batch rows x 64 reduction elements = 2 KiB per slot) take half the LDS of the
// fp32 form; the four units of a batch row are gathered into one lane so that h leaves as 8-byte stores.
constexpr int LR16_SLOT_BYTES = 16 * 128;
__host__ __device__ constexpr int lr16_ld(int K) { return K + 8; }                 // bf16 elements per LDS row of the R slice
__host__ __device__ constexpr size_t lr16_smem(int K) { return (size_t)16 * lr16_ld(K) * 2 + LR_WAVES * LR_RING * LR16_SLOT_BYTES; }

template <int NP> __global__ __launch_bounds__(512, 1) void lstm_rec_bf16_kernel(LstmRecArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lr_smem[];
    __shared__ int lr_bail;
    __shared__ float4v lr_xch[2][4][64];
    bf16_t *Rs = (bf16_t *)lr_smem;
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lr_smem;
    const int t = threadIdx.x, lane = t & 63;
    const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
    const int bt = wv & 3, hf = wv >> 2;
    const int li = lane & 15, kg = lane >> 4;
    const int cu = blockIdx.x, nwg = gridDim.x;
    const int K = a.K, Kb = K >> 6, LD = lr16_ld(K);
    const int64_t NK = (int64_t)a.N * K, TNK = (int64_t)a.T * NK;
    const bf16_t *R4 = (const bf16_t *)a.R4, *h0 = (const bf16_t *)a.h0;
    bf16_t *hout = (bf16_t *)a.h;

    {   // R slice: rows 4u + g, k contiguous; four consecutive bf16 in memory are the four units of one (g, k_in)
        const int kb_out = (4 * cu) >> 6, kf = (4 * cu) & 63;
        for (int e = t; e < 4 * K; e += 512) {
            const int g = e / K, kin = e - g * K;
            const us4v v = *(const us4v *)(R4 + ((((int64_t)g * Kb + kb_out) * Kb + (kin >> 6)) * 64 + (kin & 63)) * 64 + kf);
#pragma unroll
            for (int u = 0; u < 4; ++u) Rs[(4 * u + g) * LD + kin] = v[u];
        }
    }
    if (t == 0) lr_bail = 0;
    __syncthreads();

    // fragments: A = 8 consecutive k of R slice row li, B = piece (4s + kg) of row li of this wave's slot
    const unsigned rs_bytes = (unsigned)(16 * LD * 2);
    const unsigned a_addr = lds0 + (li * LD + 8 * kg) * 2;
    const unsigned ring0 = rs_bytes + wv * LR_RING * LR16_SLOT_BYTES;
    unsigned b_addr[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) b_addr[s] = lds0 + ring0 + li * 128 + (((4 * s + kg) ^ (li & 7)) << 4);

    // direct loads of one chunk: 16 batch rows x 128 bytes, 8 rows per instruction
    int g_off[4][2];   // (first NP rows used)
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int rl = 8 * j + (lane >> 3);
            int r = 64 * p + 16 * bt + rl;
            const int piece = (lane & 7) ^ (rl & 7);
            if (r >= a.N) r = a.N - 1;
            g_off[p][j] = r * K + piece * 8;
        }

    const int nchunk = K >> 6;
    const int unit = 4 * cu + kg;
    float s_reg[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int n = 64 * p + 16 * bt + li;
        s_reg[p] = (n < a.N && hf == 0 && a.s0) ? a.s0[(int64_t)n * K + unit] : 0.f;
    }

    for (int ts = 0; ts < a.T; ++ts) {
        const bf16_t *hprev = ts ? hout + (int64_t)(ts - 1) * NK : h0;
        float zx[NP][4];
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int n = 64 * p + 16 * bt + li;
            const int64_t e = (int64_t)ts * NK + (int64_t)n * K + unit;
#pragma unroll
            for (int g = 0; g < 4; ++g) zx[p][g] = 0.f;
            if (n < a.N && hf == 0) {
#pragma unroll
                for (int g = 0; g < 4; ++g) zx[p][g] = a.gates[g * TNK + e];
            }
        }
        if (ts > 0 && lr_step_barrier(a.sync, (unsigned)ts * (unsigned)nwg, a.spin_limit, &lr_bail, t)) return;

#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int n = 64 * p + 16 * bt + li;
            const bool row_ok = n < a.N && hf == 0;
            const int64_t e = (int64_t)ts * NK + (int64_t)n * K + unit;
            float4v acc = {0.f, 0.f, 0.f, 0.f}, acc2 = {0.f, 0.f, 0.f, 0.f};
            if (hprev) {
#define LR_ISSUE(C, SLOT)                                                                                        \
    {                                                                                                            \
        bf16_t *dst_ = (bf16_t *)(lr_smem + ring0 + (SLOT) * LR16_SLOT_BYTES);                                   \
        const bf16_t *src_ = hprev + (C) * 64;                                                                   \
        _Pragma("unroll") for (int j = 0; j < 2; ++j)                                                            \
            __builtin_amdgcn_global_load_lds(src_ + g_off[p][j], dst_ + j * 512, 16, 0, 0);                      \
    }
                const int nmy = (nchunk - hf + 1) >> 1;
                if (nmy > 0) LR_ISSUE(hf, 0)
                if (nmy > 1) LR_ISSUE(hf + 2, 1)
                for (int i = 0; i < nmy; ++i) {
                    const int c = hf + 2 * i;
                    if (i + 1 < nmy) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
                    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                    const unsigned sb = (unsigned)((i & 1) * LR16_SLOT_BYTES);
                    const unsigned sa = (unsigned)(c * 128);
                    float4v af[2], bf[2];
#pragma unroll
                    for (int s = 0; s < 2; ++s) {
                        af[s] = g64_read128(a_addr + sa + s * 64);
                        bf[s] = g64_read128(b_addr[s] + sb);
                    }
                    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(af[0]), "+v"(af[1]), "+v"(bf[0]), "+v"(bf[1]));
                    if (i + 2 < nmy) LR_ISSUE(c + 4, i & 1)
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8v, af[0]), __builtin_bit_cast(bf16x8v, bf[0]),
                                                                 acc, 0, 0, 0);
                    acc2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8v, af[1]), __builtin_bit_cast(bf16x8v, bf[1]),
                                                                  acc2, 0, 0, 0);
                }
            }
#undef LR_ISSUE
            if (hf == 1) lr_xch[p & 1][bt][lane] = acc + acc2;
            __syncthreads();
            if (hf == 0) acc += lr_xch[p & 1][bt][lane];

            float ht = 0.f;
            if (row_ok) {
                float z[4];
#pragma unroll
                for (int g = 0; g < 4; ++g) z[g] = (acc[g] + acc2[g]) + zx[p][g];
                const float it = sigmoidf_(z[0]), ct = tanhf(z[1]), ft = sigmoidf_(z[2]), ot = sigmoidf_(z[3]);
                s_reg[p] = ft * s_reg[p] + it * ct;
                ht = ot * tanhf(s_reg[p]);
                a.s[e] = s_reg[p];
                a.gates[e] = it;
                a.gates[TNK + e] = ct;
                a.gates[2 * TNK + e] = ft;
                a.gates[3 * TNK + e] = ot;
            }
            if (hf == 0) {   // (wave-uniform) the units 4cu .. 4cu+3 of batch row n sit in lanes li, li+16, li+32, li+48
                const unsigned hb = (unsigned)f32_to_bf16(ht);
                const unsigned h1 = (unsigned)__shfl((int)hb, li + 16), h2 = (unsigned)__shfl((int)hb, li + 32),
                               h3 = (unsigned)__shfl((int)hb, li + 48);
                if (row_ok && kg == 0) {
                    const unsigned long long packed = (unsigned long long)(hb | (h1 << 16)) | ((unsigned long long)(h2 | (h3 << 16)) << 32);
                    // h is what the other workgroups wait for: written through to memory (device scope)
                    __hip_atomic_store((unsigned long long *)(hout + e), packed, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (t == 0) __hip_atomic_fetch_add(a.sync, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

__global__ void lstm_sync_reset(unsigned *sync)
{
    if (threadIdx.x < 2) sync[threadIdx.x] = 0u;
}

// Runs after lstm_rec_kernel on the same stream: if that kernel gave up waiting (sync[1] != 0), every
// element of h (fp32 or bf16), s [tnk] and gates [4 tnk] becomes NaN.  Returns at once otherwise.
__global__ __launch_bounds__(256) void lstm_rec_poison(const unsigned *sync, void *h, int h_bf16, float *s, float *gates, int64_t tnk)
{
    if (__hip_atomic_load(sync + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) return;
    const float nan = __uint_as_float(0x7FC00000u);
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < tnk; i += (int64_t)gridDim.x * 256) {
        if (h_bf16) ((bf16_t *)h)[i] = (bf16_t)0x7FC0u;
        else ((float *)h)[i] = nan;
        s[i] = nan;
#pragma unroll
        for (int g = 0; g < 4; ++g) gates[g * tnk + i] = nan;
    }
}

}  // namespace brg
