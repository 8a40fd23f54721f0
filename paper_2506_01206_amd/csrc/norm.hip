// RMSNorm in front of the block's input projection (the Mamba-130M drafter of the paper, Sec. 3.1,
// normalizes the residual stream before every mixer):  y[m, :] = x[m, :] * rsqrt(mean(x[m, :]^2) + eps) * w
// HBM-bound: one wavefront per token row, 16-byte loads, the row kept in registers between the
// reduction and the scaling so that it is read once.
#include "device_math.h"
#include "launch.h"

namespace mamba {
namespace {

constexpr int kWave = 64;
constexpr int kRowsPerBlock = 4;
constexpr int kMaxVecs = 8;  // 8 vectors of 8 bf16 per lane: rows up to 4096 features stay in registers

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// C % 8 == 0 and C <= 64 * 8 * kMaxVecs
__global__ void __launch_bounds__(kWave * kRowsPerBlock)
rmsnorm_kernel(const bf16_t *__restrict__ x, const float *__restrict__ w, bf16_t *__restrict__ y, int64_t M,
               int64_t C, float eps)
{
    const int lane = threadIdx.x & 63;
    const int64_t m = (int64_t)blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
    if (m >= M) return;                                  // whole wavefronts leave together
    const int64_t vecs = C / 8;
    const uint4 *xr = reinterpret_cast<const uint4 *>(x + m * C);
    uint4 raw[kMaxVecs];
    float ss = 0.0f;
#pragma unroll
    for (int i = 0; i < kMaxVecs; ++i) {
        const int64_t v = lane + (int64_t)i * kWave;
        raw[i] = v < vecs ? xr[v] : make_uint4(0, 0, 0, 0);
        const uint32_t u[4] = {raw[i].x, raw[i].y, raw[i].z, raw[i].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float a = bf16_lo(u[j]), b = bf16_hi(u[j]);
            ss = fmaf(a, a, ss);
            ss = fmaf(b, b, ss);
        }
    }
    ss = wave_sum(ss);
    const float scale = __builtin_amdgcn_rsqf(ss / (float)C + eps);
    uint4 *yr = reinterpret_cast<uint4 *>(y + m * C);
#pragma unroll
    for (int i = 0; i < kMaxVecs; ++i) {
        const int64_t v = lane + (int64_t)i * kWave;
        if (v >= vecs) continue;
        const float4 w0 = reinterpret_cast<const float4 *>(w)[2 * v], w1 = reinterpret_cast<const float4 *>(w)[2 * v + 1];
        uint4 o;
        o.x = f32x2_to_bf16x2(bf16_lo(raw[i].x) * scale * w0.x, bf16_hi(raw[i].x) * scale * w0.y);
        o.y = f32x2_to_bf16x2(bf16_lo(raw[i].y) * scale * w0.z, bf16_hi(raw[i].y) * scale * w0.w);
        o.z = f32x2_to_bf16x2(bf16_lo(raw[i].z) * scale * w1.x, bf16_hi(raw[i].z) * scale * w1.y);
        o.w = f32x2_to_bf16x2(bf16_lo(raw[i].w) * scale * w1.z, bf16_hi(raw[i].w) * scale * w1.w);
        yr[v] = o;
    }
}

}  // namespace

hipError_t launch_rmsnorm(const NormArgs &a, hipStream_t stream)
{
    const unsigned blocks = (unsigned)((a.M + kRowsPerBlock - 1) / kRowsPerBlock);
    rmsnorm_kernel<<<blocks, kWave * kRowsPerBlock, 0, stream>>>(static_cast<const bf16_t *>(a.x), a.w,
                                                               static_cast<bf16_t *>(a.y), a.M, a.C, a.eps);
    return hipGetLastError();
}

}  // namespace mamba
