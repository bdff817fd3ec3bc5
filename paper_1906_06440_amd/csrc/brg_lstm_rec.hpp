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
    const float *R4;       // [4][Kb][Kb][64][64] blocked recurrent weights
    const float *h0, *s0;  // [N][K] or null
    float *h, *s;          // [T][N][K]
    float *gates;          // [4][T][N][K]: in = W x + b, out = gate values
    unsigned *sync;        // sync[0] = barrier counter, sync[1] = error flag (both zero at launch)
    int T, N, K;
    unsigned spin_limit;
};

__global__ __launch_bounds__(512, 1) void lstm_rec_kernel(LstmRecArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lr_smem[];
    __shared__ int lr_bail;
    __shared__ float4v lr_xch[4][64];              // partial sums of the odd-chunk waves
    float *Rs = (float *)lr_smem;
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lr_smem;
    const int t = threadIdx.x, lane = t & 63;
    const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
    const int bt = wv & 3, hf = wv >> 2;           // batch tile, chunk parity
    const int li = lane & 15, kg = lane >> 4;
    const int cu = blockIdx.x, nwg = gridDim.x;
    const int K = a.K, Kb = K >> 6;
    const int64_t NK = (int64_t)a.N * K, TNK = (int64_t)a.T * NK;

    // ---- recurrent weights of units 4cu .. 4cu+3, all gates -> LDS rows 4u + g, k contiguous.
    // Element R_g[k_out][k_in] sits at R4[g][k_out/64][k_in/64][k_in%64][k_out%64]: one float4 holds
    // the four units of this workgroup for one (g, k_in).
    {
        const int kb_out = (4 * cu) >> 6, kf = (4 * cu) & 63;
        for (int e = t; e < 4 * K; e += 512) {
            const int g = e / K, kin = e - g * K;
            const float4v v = *(const float4v *)(a.R4 + ((((int64_t)g * Kb + kb_out) * Kb + (kin >> 6)) * 64 + (kin & 63)) * 64 + kf);
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

    // direct loads of one chunk: the wave moves its batch rows 16 bt .. 16 bt + 15, 4 rows per instruction
    int g_off[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int rl = 4 * j + (lane >> 4);              // row inside the slot
        int r = 16 * bt + rl;
        const int piece = (lane & 15) ^ rl;
        if (r >= a.N) r = a.N - 1;                       // rows beyond the batch: harmless duplicates
        g_off[j] = r * K + piece * 4;
    }

    const int nchunk = K >> 6;
    const int n = 16 * bt + li, unit = 4 * cu + kg;
    const bool row_ok = n < a.N && hf == 0;        // the even-chunk waves finish the step
    // the cell state of (n, unit) is produced and consumed by this lane only: it lives in a register
    float s_reg = (row_ok && a.s0) ? a.s0[(int64_t)n * K + unit] : 0.f;

    for (int ts = 0; ts < a.T; ++ts) {
        const float *hprev = ts ? a.h + (int64_t)(ts - 1) * NK : a.h0;
        const int64_t e = (int64_t)ts * NK + (int64_t)n * K + unit;
        // partial pre-activations W x + b of this step: independent of the recurrence, so the loads are
        // in flight while the workgroup waits at the barrier
        float zx[4] = {0.f, 0.f, 0.f, 0.f};
        if (row_ok) {
#pragma unroll
            for (int g = 0; g < 4; ++g) zx[g] = a.gates[g * TNK + e];
        }
        // ---- grid barrier: every workgroup has stored its part of h[ts-1]
        if (ts > 0) {
            if (t == 0) {
                const unsigned target = (unsigned)ts * (unsigned)nwg;
                unsigned spins = 0, bad = 0;
                while (__hip_atomic_load(a.sync, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
                    ++spins;
                    if ((spins & 63u) == 0 && __hip_atomic_load(a.sync + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) bad = 1;
                    if (spins > a.spin_limit) bad = 1;
                    if (bad) break;
                }
                if (bad) __hip_atomic_store(a.sync + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                lr_bail = (int)bad;
            }
            __syncthreads();
            if (lr_bail) return;                            // the same value for the whole workgroup
            // ASSUMPTION (outside what the memory model promises, checked by the parity tests on every run):
            // no acquire follows the barrier.  h[ts-1] was written through to memory (device-scope stores,
            // see below) before the counter moved, and the step relies on no cache on the reading side
            // holding an older copy of those addresses: every launch starts with clean caches, h[ts-1] is
            // read by nobody before this point, and the L2 of an XCD whose own workgroups wrote 16-byte
            // pieces of a 128-byte line of h[ts-1] must not serve the other pieces of that line from a
            // copy fetched before their writers stored them (it does not: write-through stores of part of
            // a line do not make the L2 fetch and keep the rest of it).  It breaks if anything here reads
            // h[ts-1] before the barrier (a prefetch, a wider store that reads the line first) or if a
            // later part allocates whole lines on partial write-through stores.  The fence that would make
            // it formal was measured: an agent-scope acquire here (L2 invalidate on all 8 XCDs) takes the
            // step from 12.6 to 28 us, acquire plus a release before the arrival to 75 us.
        }

        float4v acc = {0.f, 0.f, 0.f, 0.f}, acc2 = {0.f, 0.f, 0.f, 0.f};
        if (hprev) {
            // A wave moves and consumes its own rows and chunks only, so its ring needs no workgroup
            // barrier: it waits for its own loads.
            auto issue = [&](int c, int slot) {
                float *dst = (float *)(lr_smem + ring0 + slot * LR_SLOT_BYTES);
                const float *src = hprev + c * 64;
#pragma unroll
                for (int j = 0; j < 4; ++j) __builtin_amdgcn_global_load_lds(src + g_off[j], dst + j * 256, 16, 0, 0);
            };
            // the four zx loads above are older than every chunk load, so the counts below cover them
            const int nmy = (nchunk - hf + 1) >> 1;      // chunks hf, hf + 2, ...
            if (nmy > 0) issue(hf, 0);
            if (nmy > 1) issue(hf + 2, 1);
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
                if (i + 2 < nmy) issue(c + 4, i & 1);
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
        // ---- the odd-chunk waves hand their partial sums to the even-chunk waves of the same batch tile
        if (hf == 1) lr_xch[bt][lane] = acc + acc2;
        __syncthreads();
        if (hf == 0) acc += lr_xch[bt][lane];

        // ---- gates and state update on the accumulators (register r = gate r of unit kg, batch row n)
        if (row_ok) {
            float z[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) z[g] = (acc[g] + acc2[g]) + zx[g];
            const float it = sigmoidf_(z[0]), ct = tanhf(z[1]), ft = sigmoidf_(z[2]), ot = sigmoidf_(z[3]);
            s_reg = ft * s_reg + it * ct;
            const float ht = ot * tanhf(s_reg);
            // h is what the other workgroups wait for: written through to memory (device scope)
            __hip_atomic_store(a.h + e, ht, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            a.s[e] = s_reg;
            a.gates[e] = it;
            a.gates[TNK + e] = ct;
            a.gates[2 * TNK + e] = ft;
            a.gates[3 * TNK + e] = ot;
        }
        // ---- arrive: all stores of this workgroup have completed before the counter moves
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
// element of h, s [tnk] and gates [4 tnk] becomes NaN.  Returns at once otherwise.
__global__ __launch_bounds__(256) void lstm_rec_poison(const unsigned *sync, float *h, float *s, float *gates, int64_t tnk)
{
    if (__hip_atomic_load(sync + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) return;
    const float nan = __uint_as_float(0x7FC00000u);
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < tnk; i += (int64_t)gridDim.x * 256) {
        h[i] = nan;
        s[i] = nan;
#pragma unroll
        for (int g = 0; g < 4; ++g) gates[g * tnk + i] = nan;
    }
}

}  // namespace brg
