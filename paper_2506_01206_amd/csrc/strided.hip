// Conv1d and selective scan for token tensors that are not contiguous time-major: element (b, t, d) of a
// tensor lies at b * stride[0] + t * stride[1] + d * stride[2] elements from its base.  This is what makes a
// channel-major (batch, D, L) caller, or a view into a wider row (x | z packed side by side), expressible at
// the boundary.  Same arithmetic as conv1d.hip and scan.hip, in their order of operations:
//
//   conv   y[b,t,d] = act(bias[d] + sum_k w[d,k] xpad[b,t+k,d])
//   scan   delta = softplus(dt + dt_bias);  h_t = exp(delta_t A) h_{t-1} + delta_t B_t x_t
//          y_t = C_t . h_t + D x_t;  out_t = y_t silu(z_t)
//
// These kernels are the plain form: a lane owns one channel and walks time, no time chunks, no vector
// accesses, nothing tuned.  The tuned kernels need contiguous rows; api.cpp sends every call whose strides
// describe that layout to them and only the rest here.
#include "device_math.h"
#include "launch.h"

namespace mamba {
namespace {

constexpr int kWave = 64;
constexpr int kConvSeg = 128;   // tokens per workgroup of the conv kernel
constexpr int kMaxK = 4;        // longest conv the library takes

struct Strides {
    int64_t b, l, d;
};

// grid: (ceil(D / 64), ceil(L / kConvSeg), batch); block: 64
template <typename T>
__global__ void __launch_bounds__(kWave)
conv1d_strided_kernel(const T *x, Strides xs, const float *__restrict__ w, const float *__restrict__ bias,
                      const T *state_in, T *y, Strides ys, T *state_out, int64_t L, int64_t D, int K, int apply_silu)
{
    const int64_t d = (int64_t)blockIdx.x * kWave + threadIdx.x;
    if (d >= D) return;
    const int64_t b = blockIdx.z;
    const int64_t t0 = (int64_t)blockIdx.y * kConvSeg;
    const int64_t t1 = t0 + kConvSeg < L ? t0 + kConvSeg : L;
    float wk[kMaxK];
    for (int k = 0; k < K; ++k) wk[k] = w[d * K + k];
    const float bv = bias ? bias[d] : 0.0f;
    // padded input at time t (t may be negative: the carried window, oldest first, or zero)
    auto xpad = [&](int64_t t) -> float {
        if (t >= 0) return ld_io(x, b * xs.b + t * xs.l + d * xs.d);
        return state_in ? ld_io(state_in, (b * D + d) * (K - 1) + (K - 1 + t)) : 0.0f;
    };
    float win[kMaxK - 1];
    for (int k = 0; k < K - 1; ++k) win[k] = xpad(t0 - (K - 1) + k);
    for (int64_t t = t0; t < t1; ++t) {
        const float xt = xpad(t);
        float acc = bv;
        for (int k = 0; k < K - 1; ++k) acc = fmaf(wk[k], win[k], acc);
        acc = fmaf(wk[K - 1], xt, acc);
        st_io(y, b * ys.b + t * ys.l + d * ys.d, apply_silu ? silu_f32(acc) : acc);
        for (int k = 0; k + 1 < K - 1; ++k) win[k] = win[k + 1];
        win[K - 2] = xt;
    }
    // the workgroup that reaches the end of the sequence leaves the last K - 1 padded inputs
    if (state_out && t1 == L && (t0 < L || (L == 0 && blockIdx.y == 0))) {
        for (int k = 0; k < K - 1; ++k) st_io(state_out, (b * D + d) * (K - 1) + k, xpad(L - (K - 1) + k));
    }
}

// grid: (ceil(D / 64), batch); block: 64
template <typename T, int N>
__global__ void __launch_bounds__(kWave)
scan_strided_kernel(const T *x, Strides xs, const T *dt, Strides ds, const float *__restrict__ A, const T *Bm,
                    const T *Cm, const float *__restrict__ Dskip, const T *z, Strides zs,
                    const float *__restrict__ dt_bias, const float *h0, T *out, Strides os, float *h_final,
                    int64_t L, int64_t D, int dt_softplus)
{
    const int64_t d = (int64_t)blockIdx.x * kWave + threadIdx.x;
    if (d >= D) return;
    const int64_t b = blockIdx.y;
    float h[N], a2[N];
#pragma unroll
    for (int n = 0; n < N; ++n) {
        a2[n] = A[d * N + n] * kLog2e;
        h[n] = h0 ? h0[(b * D + d) * N + n] : 0.0f;
    }
    const float bias = dt_bias ? dt_bias[d] : 0.0f;
    const float dsk = Dskip ? Dskip[d] : 0.0f;
    for (int64_t t = 0; t < L; ++t) {
        const float xv = ld_io(x, b * xs.b + t * xs.l + d * xs.d);
        const float v = ld_io(dt, b * ds.b + t * ds.l + d * ds.d) + bias;
        const float delta = dt_softplus ? softplus_f32(v) : v;
        const float u = delta * xv;
        float y = dsk * xv;
        const T *bt = Bm + (b * L + t) * N, *ct = Cm + (b * L + t) * N;   // the same address in every lane
#pragma unroll
        for (int n = 0; n < N; ++n) {
            const float a = exp2_hw(delta * a2[n]);
            h[n] = fmaf(a, h[n], u * ld_io(bt, n));
            y = fmaf(h[n], ld_io(ct, n), y);
        }
        if (z) y *= silu_f32(ld_io(z, b * zs.b + t * zs.l + d * zs.d));
        st_io(out, b * os.b + t * os.l + d * os.d, y);
    }
    if (h_final) {
#pragma unroll
        for (int n = 0; n < N; ++n) h_final[(b * D + d) * N + n] = h[n];
    }
}

template <typename T>
hipError_t launch_conv_strided_io(const ConvStridedArgs &a, hipStream_t stream)
{
    const int64_t segs = a.L > 0 ? (a.L + kConvSeg - 1) / kConvSeg : 1;
    const dim3 grid((unsigned)((a.D + kWave - 1) / kWave), (unsigned)segs, (unsigned)a.batch);
    conv1d_strided_kernel<T><<<grid, kWave, 0, stream>>>(
        static_cast<const T *>(a.x), Strides{a.xs[0], a.xs[1], a.xs[2]}, a.w, a.bias,
        static_cast<const T *>(a.state_in), static_cast<T *>(a.y), Strides{a.ys[0], a.ys[1], a.ys[2]},
        static_cast<T *>(a.state_out), a.L, a.D, a.K, a.apply_silu);
    return hipGetLastError();
}

template <typename T, int N>
hipError_t launch_scan_strided_n(const ScanStridedArgs &a, hipStream_t stream)
{
    const dim3 grid((unsigned)((a.D + kWave - 1) / kWave), (unsigned)a.batch);
    scan_strided_kernel<T, N><<<grid, kWave, 0, stream>>>(
        static_cast<const T *>(a.x), Strides{a.xs[0], a.xs[1], a.xs[2]}, static_cast<const T *>(a.dt),
        Strides{a.ds[0], a.ds[1], a.ds[2]}, a.A, static_cast<const T *>(a.Bm), static_cast<const T *>(a.Cm),
        a.Dskip, static_cast<const T *>(a.z), Strides{a.zs[0], a.zs[1], a.zs[2]}, a.dt_bias, a.h0,
        static_cast<T *>(a.out), Strides{a.os[0], a.os[1], a.os[2]}, a.h_final, a.L, a.D, a.dt_softplus);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_scan_strided_io(const ScanStridedArgs &a, hipStream_t stream)
{
    switch (a.N) {
    case 4: return launch_scan_strided_n<T, 4>(a, stream);
    case 8: return launch_scan_strided_n<T, 8>(a, stream);
    case 16: return launch_scan_strided_n<T, 16>(a, stream);
    case 32: return launch_scan_strided_n<T, 32>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_conv1d_strided(const ConvStridedArgs &a, hipStream_t stream)
{
    if (a.io == kIoBf16) return launch_conv_strided_io<bf16_t>(a, stream);
    return launch_conv_strided_io<float>(a, stream);
}

hipError_t launch_scan_strided(const ScanStridedArgs &a, hipStream_t stream)
{
    if (a.io == kIoBf16) return launch_scan_strided_io<bf16_t>(a, stream);
    return launch_scan_strided_io<float>(a, stream);
}

}  // namespace mamba
