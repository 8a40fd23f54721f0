// One selective-state update for every live branch of a draft tree (Sec. 4.1 of the paper:
// tree drafting is batch generation, and a child continues from its parent's state), gfx950.
//
//   p = parent[j];  h_out[j] = exp(delta_j A) h_in[p] + delta_j B_j x_j
//   out[j] = (C_j . h_out[j] + D x_j) silu(z_j)
//
// The step moves 2 * D * N * 4 bytes of state per branch for D * N state updates: it is bound
// by HBM.  The state row of a branch is walked as float4s, one per lane, consecutive lanes on
// consecutive float4s, so every wavefront load and store is one contiguous 1 KiB run.  A lane
// therefore owns 4 of the N states of a channel; the N/4 lanes of a channel sum their partial
// C.h with DPP lane exchanges inside a quad (and a half-row mirror for N = 32).  With a parent
// index the gather is fused into the load of h_in, which makes a separate state copy unnecessary.
#include "device_math.h"
#include "launch.h"

namespace mamba {
namespace {

constexpr int kBlock = 256;

template <int CTRL> __device__ __forceinline__ float dpp_add(float v)
{
    const int o = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false);
    return v + __int_as_float(o);
}

// sum over the Q = N/4 adjacent lanes that share a channel; every one of them gets the total
template <int Q> __device__ __forceinline__ float channel_sum(float v)
{
    if constexpr (Q >= 2) v = dpp_add<0xB1>(v);   // quad_perm [1,0,3,2]
    if constexpr (Q >= 4) v = dpp_add<0x4E>(v);   // quad_perm [2,3,0,1]
    if constexpr (Q >= 8) v = dpp_add<0x141>(v);  // row_half_mirror: lane i <-> 7 - i of each 8
    return v;
}

template <int N> __device__ __forceinline__ float4 ld4_io(const float *p) { return *reinterpret_cast<const float4 *>(p); }
template <int N> __device__ __forceinline__ float4 ld4_io(const bf16_t *p)
{
    const uint2 r = *reinterpret_cast<const uint2 *>(p);
    return make_float4(bf16_lo(r.x), bf16_hi(r.x), bf16_lo(r.y), bf16_hi(r.y));
}

// grid: (ceil(D * N / 4 / 256), n_out); lane <-> one float4 of the branch's (D, N) state
template <typename T, int N, bool HAS_Z, bool SOFTPLUS>
__global__ void __launch_bounds__(kBlock)
state_step_kernel(float *h_out, const float *h_in, const int32_t *__restrict__ parent,
                  const T *__restrict__ x, const T *__restrict__ dt, const float *__restrict__ A,
                  const T *__restrict__ Bm, const T *__restrict__ Cm,
                  const float *__restrict__ Dskip, const T *__restrict__ z,
                  const float *__restrict__ dt_bias, T *__restrict__ out, int64_t n_in, int64_t D)
{
    constexpr int Q = N / 4;
    const int64_t j = blockIdx.y;
    const int64_t row4 = D * Q;  // float4s per branch
    const int64_t f_raw = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const bool live = f_raw < row4;
    const int64_t f = live ? f_raw : row4 - 1;
    const int64_t d = f / Q;
    const int q = (int)(f - d * Q);

    const int64_t p = parent ? (int64_t)parent[j] : j;
    const bool p_ok = p >= 0 && p < n_in;

    float4 h = make_float4(0.f, 0.f, 0.f, 0.f);
    if (p_ok) h = reinterpret_cast<const float4 *>(h_in)[p * row4 + f];
    const float4 a = reinterpret_cast<const float4 *>(A)[f];
    const float4 bv = ld4_io<N>(Bm + j * N + 4 * q);
    const float4 cv = ld4_io<N>(Cm + j * N + 4 * q);
    const float xv = ld_io(x, j * D + d);
    const float v = ld_io(dt, j * D + d) + (dt_bias ? dt_bias[d] : 0.0f);
    const float delta = SOFTPLUS ? softplus_f32(v) : v;
    const float u = delta * xv;
    const float dl = delta * kLog2e;

    h.x = fmaf(exp2_hw(dl * a.x), h.x, u * bv.x);
    h.y = fmaf(exp2_hw(dl * a.y), h.y, u * bv.y);
    h.z = fmaf(exp2_hw(dl * a.z), h.z, u * bv.z);
    h.w = fmaf(exp2_hw(dl * a.w), h.w, u * bv.w);
    float y = h.x * cv.x;
    y = fmaf(h.y, cv.y, y);
    y = fmaf(h.z, cv.z, y);
    y = fmaf(h.w, cv.w, y);
    y = channel_sum<Q>(y);

    if (!p_ok) {
        const float nan = __int_as_float(0x7fc00000);
        h = make_float4(nan, nan, nan, nan);
        y = nan;
    }
    if (live) {
        reinterpret_cast<float4 *>(h_out)[j * row4 + f] = h;
        if (q == 0) {
            if (Dskip) y = fmaf(Dskip[d], xv, y);
            if constexpr (HAS_Z) y *= silu_f32(ld_io(z, j * D + d));
            st_io(out, j * D + d, y);
        }
    }
}

template <typename T, int N> hipError_t launch_step_n(const StepArgs &a, hipStream_t stream)
{
    const int64_t row4 = a.D * (N / 4);
    dim3 grid((unsigned)((row4 + kBlock - 1) / kBlock), (unsigned)a.n_out);
#define MAMBA_STEP(HZ, SP)                                                                        \
    state_step_kernel<T, N, HZ, SP><<<grid, kBlock, 0, stream>>>(                                 \
        a.h_out, a.h_in, a.parent, static_cast<const T *>(a.x), static_cast<const T *>(a.dt), a.A, \
        static_cast<const T *>(a.Bm), static_cast<const T *>(a.Cm), a.Dskip,                      \
        static_cast<const T *>(a.z), a.dt_bias, static_cast<T *>(a.out), a.n_in, a.D)
    if (a.z) {
        if (a.dt_softplus) MAMBA_STEP(true, true);
        else MAMBA_STEP(true, false);
    } else {
        if (a.dt_softplus) MAMBA_STEP(false, true);
        else MAMBA_STEP(false, false);
    }
#undef MAMBA_STEP
    return hipGetLastError();
}

template <typename T> hipError_t launch_step_io(const StepArgs &a, hipStream_t stream)
{
    switch (a.N) {
    case 4: return launch_step_n<T, 4>(a, stream);
    case 8: return launch_step_n<T, 8>(a, stream);
    case 16: return launch_step_n<T, 16>(a, stream);
    case 32: return launch_step_n<T, 32>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_step(const StepArgs &a, hipStream_t stream)
{
    if (a.io == kIoBf16) return launch_step_io<bf16_t>(a, stream);
    return launch_step_io<float>(a, stream);
}

}  // namespace mamba
