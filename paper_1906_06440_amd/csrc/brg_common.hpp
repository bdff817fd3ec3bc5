// Shared host/device helpers of the batch-reduce GEMM library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cstdarg>
#include <cstdio>
#include <type_traits>

#include "brg.h"
#include "brg_knobs.hpp"

namespace brg {

// ---------------------------------------------------------------- errors ----
char *last_error_buf();  // thread-local, 512 bytes (defined in brg_host.cpp)

inline int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(last_error_buf(), 512, fmt, ap);
    va_end(ap);
    return code;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline bool valid_dtype(int d) { return d == BRG_F32 || d == BRG_BF16; }
inline bool valid_act(int a) { return a >= BRG_ACT_NONE && a <= BRG_ACT_TANH; }
inline size_t dtype_size(int d) { return d == BRG_BF16 ? 2 : 4; }

// Check the launch that was just enqueued.
inline int check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(BRG_EHIP, "%s: %s", what, hipGetErrorString(e));
    return BRG_OK;
}

#define BRG_REQUIRE(cond, code, ...)                  \
    do {                                              \
        if (!(cond)) return ::brg::fail(code, __VA_ARGS__); \
    } while (0)

// ---------------------------------------------------------------- device ----
typedef uint16_t bf16_t;  // raw bfloat16 bits

typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8v __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round to nearest even; NaN stays a (quiet) NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return bf16_to_f32(v); }

template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return f32_to_bf16(v); }

// Activations applied on the accumulators (fp32).  The logistic and tanh use the
// full-range expf so that the result stays within a few ulp of the double definition.
__device__ __forceinline__ float sigmoidf_(float z) { return 1.0f / (1.0f + expf(-z)); }

__device__ __forceinline__ float apply_act(float z, int act)
{
    switch (act) {
    case BRG_ACT_RELU: return z > 0.0f ? z : 0.0f;
    case BRG_ACT_SIGMOID: return sigmoidf_(z);
    case BRG_ACT_TANH: return tanhf(z);
    default: return z;
    }
}

typedef unsigned short us4v __attribute__((ext_vector_type(4)));

// four fp32 -> four bf16, round to nearest even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ us4v pack_bf16x4(float4v v)
{
    typedef float f2v __attribute__((ext_vector_type(2)));
    typedef __bf16 b2v __attribute__((ext_vector_type(2)));
    typedef unsigned short us2v __attribute__((ext_vector_type(2)));
    const us2v lo = __builtin_bit_cast(us2v, __builtin_convertvector(f2v{v[0], v[1]}, b2v));
    const us2v hi = __builtin_bit_cast(us2v, __builtin_convertvector(f2v{v[2], v[3]}, b2v));
    return us4v{lo[0], lo[1], hi[0], hi[1]};
}

// Epilogue activation of one accumulator register group.  Kernels unroll their epilogue over many
// tiles; with expf/tanhf bodies inlined per tile behind run-time branches the common NONE/ReLU case has
// to jump over them tile after tile, and every taken branch costs an instruction-fetch bubble (measured:
// a third of the run time of the short-lived waves of the 1x1 convolution).  So a kernel takes ONE
// uniform branch on act_is_slow() around two copies of its epilogue: TRANS = false handles NONE and ReLU
// with a select per element, TRANS = true the transcendental activations.
__device__ __forceinline__ bool act_is_slow(int act) { return act > BRG_ACT_RELU; }

template <bool TRANS> __device__ __forceinline__ float4v apply_act4(float4v v, int act)
{
    if (TRANS) {
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = act == BRG_ACT_SIGMOID ? sigmoidf_(v[r]) : tanhf(v[r]);
    } else {
        const bool relu = act == BRG_ACT_RELU;
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = (relu && !(v[r] > 0.0f)) ? 0.0f : v[r];
    }
    return v;
}

// The same with the activation class as a compile-time constant (0 none, 1 ReLU, 2 sigmoid / tanh), for
// epilogues that are instantiated once per class behind a single uniform branch:
//     act_dispatch(act, [&](auto act_c) { ... act4<decltype(act_c)::value>(v, act) ... });
template <int ACT> __device__ __forceinline__ float4v act4(float4v v, int act)
{
    if (ACT == 1) {
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = __builtin_fmaxf(v[r], 0.0f);   // NaN -> 0, like z > 0 ? z : 0
    } else if (ACT == 2) {
        v = apply_act4<true>(v, act);
    }
    return v;
}

template <class F> __device__ __forceinline__ void act_dispatch(int act, F &&f)
{
    if (act == BRG_ACT_NONE) f(std::integral_constant<int, 0>{});
    else if (act == BRG_ACT_RELU) f(std::integral_constant<int, 1>{});
    else f(std::integral_constant<int, 2>{});
}

}  // namespace brg
