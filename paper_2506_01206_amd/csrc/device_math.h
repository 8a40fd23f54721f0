// Device-side helpers shared by the gfx950 kernels: I/O element access for float32 and
// bfloat16 storage, and the float32 evaluation of softplus and SiLU used by the layer
// (delta = softplus(dt + dt_bias); gate = silu(z)).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mamba {

typedef uint16_t bf16_t;  // bfloat16 bit pattern in memory

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float bf16_to_f32(uint32_t bits) { return __uint_as_float(bits << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t pair) { return __uint_as_float(pair & 0xffff0000u); }

// float32 -> bfloat16, round to nearest even (one rounding, at the store).
__device__ __forceinline__ uint32_t f32_to_bf16(float f)
{
    return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)f);
}
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi)
{
    typedef float f2 __attribute__((ext_vector_type(2)));
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    f2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, b2));
}

__device__ __forceinline__ float ld_io(const float *p, int64_t i) { return p[i]; }
__device__ __forceinline__ float ld_io(const bf16_t *p, int64_t i) { return bf16_to_f32(p[i]); }
__device__ __forceinline__ void st_io(float *p, int64_t i, float v) { p[i] = v; }
__device__ __forceinline__ void st_io(bf16_t *p, int64_t i, float v) { p[i] = (bf16_t)f32_to_bf16(v); }

// 2^v and log2(v) on the hardware transcendental unit (v_exp_f32 / v_log_f32, ~1 ulp).
__device__ __forceinline__ float exp2_hw(float v) { return __builtin_amdgcn_exp2f(v); }
__device__ __forceinline__ float log2_hw(float v) { return __builtin_amdgcn_logf(v); }
__device__ __forceinline__ float rcp_hw(float v) { return __builtin_amdgcn_rcpf(v); }

// softplus(v) = log(1 + e^v) = max(v, 0) + log1p(w), w = e^-|v| <= 1, to ~1e-7 relative (plus the
// rounding of the exp2 argument for large |v|).  The sum s = 1 + w drops w's low bits; they are
// recovered exactly as r = w - (s - 1) and added back: log1p(w) = log(s) + log1p(r / s), which is
// log(s) + r to first order (s is in [1, 2] and |r| <= 2^-24, so r and r / s differ by < 2^-25).
// No threshold and no overflow: w never exceeds 1.
__device__ __forceinline__ float softplus_f32(float v)
{
    const float w = exp2_hw(-fabsf(v) * kLog2e);
    const float s = 1.0f + w;
    const float r = w - (s - 1.0f);
    return fmaxf(v, 0.0f) + fmaf(log2_hw(s), kLn2, r);
}

// silu(v) = v / (1 + e^-v)
__device__ __forceinline__ float silu_f32(float v)
{
    return v * rcp_hw(1.0f + exp2_hw(-v * kLog2e));
}

}  // namespace mamba
