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

// The state is read once and written once per step: streaming (non-temporal) accesses keep it from displacing the
// weights and token rows in the caches (measured cold in a replayed graph: 64 branches x 4096 channels 9.9 -> 9.2 us,
// 32 x 1536 3.5 -> 2.9 us).
typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 ld_stream(const float4 *p)
{
    const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
    return make_float4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ void st_stream(float4 *p, float4 v)
{
    f32x4 t;
    t.x = v.x; t.y = v.y; t.z = v.z; t.w = v.w;
    __builtin_nontemporal_store(t, reinterpret_cast<f32x4 *>(p));
}

constexpr int kStepUnroll = 4;

// grid: (ceil(D * N / 4 / (256 * U)), n_out).  A lane owns U float4s of the branch's (D, N) state,
// 256 float4s apart, so every wavefront load or store is still one contiguous 1 KiB run; all
// loads of the U pieces are issued before the first one is used, which keeps several KiB per
// wavefront in flight (the step is a single pass over the state and lives on memory latency).
template <typename T, int N, int U, bool HAS_Z, bool SOFTPLUS>
__global__ void __launch_bounds__(kBlock)
state_step_kernel(float *h_out, const float *h_in, const int32_t *__restrict__ parent,
                  const T *__restrict__ x, const T *__restrict__ dt, const float *__restrict__ A,
                  const T *__restrict__ Bm, const T *__restrict__ Cm,
                  const float *__restrict__ Dskip, const T *__restrict__ z,
                  const float *__restrict__ dt_bias, T *__restrict__ out, int64_t n_in, int64_t D,
                  const bf16_t *__restrict__ dt_w, int64_t dt_rank)
{
    constexpr int Q = N / 4;
    const int64_t j = blockIdx.y;
    const int64_t row4 = D * Q;  // float4s per branch
    const float4 *a4 = reinterpret_cast<const float4 *>(A);

    int64_t f[U], d[U];
    bool live[U];
    float4 h[U], a[U], bv[U], cv[U];
    float xv[U], dv[U], zv[U], bias[U], dsk[U];
#pragma unroll
    for (int i = 0; i < U; ++i) {
        const int64_t f_raw = ((int64_t)blockIdx.x * U + i) * kBlock + threadIdx.x;
        live[i] = f_raw < row4;
        f[i] = live[i] ? f_raw : row4 - 1;
        d[i] = f[i] / Q;
        const int q = (int)(f[i] - d[i] * Q);
        a[i] = a4[f[i]];
        bv[i] = ld4_io<N>(Bm + j * N + 4 * q);
        cv[i] = ld4_io<N>(Cm + j * N + 4 * q);
        xv[i] = ld_io(x, j * D + d[i]);
        if (sizeof(T) == 2 && dt_w) {
            // dt projection fused in: the Q lanes of a channel share the dt_rank products (4 at a time)
            const uint2 *wrow = reinterpret_cast<const uint2 *>(dt_w + d[i] * dt_rank);
            const uint2 *lrow = reinterpret_cast<const uint2 *>(reinterpret_cast<const bf16_t *>(dt) + j * dt_rank);
            float acc = 0.0f;
#pragma unroll 4
            for (int64_t c = q; c < dt_rank / 4; c += Q) {
                const uint2 a2 = wrow[c], b2 = lrow[c];
                acc = fmaf(bf16_lo(a2.x), bf16_lo(b2.x), acc);
                acc = fmaf(bf16_hi(a2.x), bf16_hi(b2.x), acc);
                acc = fmaf(bf16_lo(a2.y), bf16_lo(b2.y), acc);
                acc = fmaf(bf16_hi(a2.y), bf16_hi(b2.y), acc);
            }
            dv[i] = bf16_to_f32(f32_to_bf16(channel_sum<Q>(acc)));     // rounded like the stored tensor it replaces
        } else {
            dv[i] = ld_io(dt, j * D + d[i]);
        }
        zv[i] = HAS_Z ? ld_io(z, j * D + d[i]) : 0.0f;
        bias[i] = dt_bias ? dt_bias[d[i]] : 0.0f;
        dsk[i] = Dskip ? Dskip[d[i]] : 0.0f;
    }
    // the state row is the only load that has to wait for the parent index
    const int64_t p = parent ? (int64_t)parent[j] : j;
    const bool p_ok = p >= 0 && p < n_in;
    const float4 *hin4 = reinterpret_cast<const float4 *>(h_in) + (p_ok ? p : 0) * row4;
#pragma unroll
    for (int i = 0; i < U; ++i) h[i] = ld_stream(hin4 + f[i]);
#pragma unroll
    for (int i = 0; i < U; ++i) {
        const float v = dv[i] + bias[i];
        const float delta = SOFTPLUS ? softplus_f32(v) : v;
        const float u = delta * xv[i];
        const float dl = delta * kLog2e;
        float4 hh = h[i];
        hh.x = fmaf(exp2_hw(dl * a[i].x), hh.x, u * bv[i].x);
        hh.y = fmaf(exp2_hw(dl * a[i].y), hh.y, u * bv[i].y);
        hh.z = fmaf(exp2_hw(dl * a[i].z), hh.z, u * bv[i].z);
        hh.w = fmaf(exp2_hw(dl * a[i].w), hh.w, u * bv[i].w);
        float y = hh.x * cv[i].x;
        y = fmaf(hh.y, cv[i].y, y);
        y = fmaf(hh.z, cv[i].z, y);
        y = fmaf(hh.w, cv[i].w, y);
        y = channel_sum<Q>(y);
        if (!p_ok) {
            const float nan = __int_as_float(0x7fc00000);
            hh = make_float4(nan, nan, nan, nan);
            y = nan;
        }
        if (live[i]) {
            st_stream(reinterpret_cast<float4 *>(h_out) + j * row4 + f[i], hh);
            if (f[i] - d[i] * Q == 0) {
                y = fmaf(dsk[i], xv[i], y);
                if constexpr (HAS_Z) y *= silu_f32(zv[i]);
                st_io(out, j * D + d[i], y);
            }
        }
    }
}

// The same step with what a channel's lanes have in common formed once per channel: with several float4s per lane
// (many branches: the launch moves tens of MB and lives on bandwidth) a workgroup covers 64 U channels, one per
// thread, and every lane of the plain kernel above would fetch x, dt, z, dt_bias and D of each of its U channels for
// itself: five small loads per piece, each a full trip through the address unit for 2 or 4 bytes a lane, and softplus
// and SiLU four times per channel.  Here the state rows are requested first, each thread then does one channel's
// token-side work (same operations in the same order, so the results are bit for bit the plain kernel's) and leaves
// delta * log2(e), delta * x, x, D and silu(z) in LDS for the lanes that own the channel's states.
// grid: (ceil(D * N / 4 / (256 * U)), n_out)
template <typename T, int N, int U, bool HAS_Z, bool SOFTPLUS>
__global__ void __launch_bounds__(kBlock)
state_step_shared_kernel(float *h_out, const float *h_in, const int32_t *__restrict__ parent,
                         const T *__restrict__ x, const T *__restrict__ dt, const float *__restrict__ A,
                         const T *__restrict__ Bm, const T *__restrict__ Cm,
                         const float *__restrict__ Dskip, const T *__restrict__ z,
                         const float *__restrict__ dt_bias, T *__restrict__ out, int64_t n_in, int64_t D)
{
    constexpr int Q = N / 4;
    constexpr int kChannels = kBlock * U / Q;                     // channels whose states this workgroup owns
    __shared__ __attribute__((aligned(16))) float4 ch4[kChannels];   // delta * log2(e), delta * x, x, D
    __shared__ float chg[kChannels];                                  // silu(z)
    const int64_t j = blockIdx.y;
    const int64_t row4 = D * Q;  // float4s per branch
    const int64_t d_lo = (int64_t)blockIdx.x * kChannels;
    const float4 *a4 = reinterpret_cast<const float4 *>(A);

    // the state rows are the bytes that count: the parent index and their requests go out first
    const int64_t p = parent ? (int64_t)parent[j] : j;
    const bool p_ok = p >= 0 && p < n_in;
    const float4 *hin4 = reinterpret_cast<const float4 *>(h_in) + (p_ok ? p : 0) * row4;
    int64_t f[U];
    bool live[U];
    float4 h[U], a[U];
#pragma unroll
    for (int i = 0; i < U; ++i) {
        const int64_t f_raw = ((int64_t)blockIdx.x * U + i) * kBlock + threadIdx.x;
        live[i] = f_raw < row4;
        f[i] = live[i] ? f_raw : row4 - 1;
        h[i] = ld_stream(hin4 + f[i]);
    }
#pragma unroll
    for (int i = 0; i < U; ++i) a[i] = a4[f[i]];
    const int q = (int)(threadIdx.x % Q);                         // 256 i is a multiple of Q: the same for all pieces
    const float4 bv = ld4_io<N>(Bm + j * N + 4 * q), cv = ld4_io<N>(Cm + j * N + 4 * q);

    for (int c = threadIdx.x; c < kChannels; c += kBlock) {
        const int64_t dc = d_lo + c;
        if (dc >= D) break;
        const float xv = ld_io(x, j * D + dc);
        const float v = ld_io(dt, j * D + dc) + (dt_bias ? dt_bias[dc] : 0.0f);
        const float zv = HAS_Z ? ld_io(z, j * D + dc) : 0.0f;
        const float delta = SOFTPLUS ? softplus_f32(v) : v;
        ch4[c] = make_float4(delta * kLog2e, delta * xv, xv, Dskip ? Dskip[dc] : 0.0f);
        if constexpr (HAS_Z) chg[c] = silu_f32(zv);
    }
    __syncthreads();

#pragma unroll
    for (int i = 0; i < U; ++i) {
        const int64_t d = f[i] / Q;
        const int ci = (int)(d - d_lo);
        const float4 t = ch4[ci];
        const float dl = t.x, u = t.y;
        float4 hh = h[i];
        hh.x = fmaf(exp2_hw(dl * a[i].x), hh.x, u * bv.x);
        hh.y = fmaf(exp2_hw(dl * a[i].y), hh.y, u * bv.y);
        hh.z = fmaf(exp2_hw(dl * a[i].z), hh.z, u * bv.z);
        hh.w = fmaf(exp2_hw(dl * a[i].w), hh.w, u * bv.w);
        float y = hh.x * cv.x;
        y = fmaf(hh.y, cv.y, y);
        y = fmaf(hh.z, cv.z, y);
        y = fmaf(hh.w, cv.w, y);
        y = channel_sum<Q>(y);
        if (!p_ok) {
            const float nan = __int_as_float(0x7fc00000);
            hh = make_float4(nan, nan, nan, nan);
            y = nan;
        }
        if (live[i]) {
            st_stream(reinterpret_cast<float4 *>(h_out) + j * row4 + f[i], hh);
            if (f[i] - d * Q == 0) {
                y = fmaf(t.w, t.z, y);
                if constexpr (HAS_Z) y *= chg[ci];
                st_io(out, j * D + d, y);
            }
        }
    }
}

// Fork, conv step and state update of one layer in a single launch (Sec. 4.1: a child continues from its parent's
// states; the draft loop of a tree is this, once per layer and position).  x is the input *before* the conv:
//   win = conv_src[p, d, :];  a = conv_bias[d] + sum_k w[d,k] win[k] + w[d,K-1] x[j,d];  x_c = silu(a)
//   conv_dst[j, d, :] = (win[1..], x[j,d]);  then the step above on x_c rounded to the I/O type
// in the arithmetic order of the conv kernel and of the step kernel, so that the result is bit for bit what
// mamba_conv1d_fwd (L = 1, on the window gathered by parent) followed by mamba_state_step gives.
// The workgroup's channels (256 U / (N/4) of them) are convolved first, one channel per thread: window, taps,
// bias and input are loaded once per channel, not once per lane (with the conv evaluated by every lane of a channel
// the wide step was bound by the issue of its many small loads: 17.7 us against 13.1 us for two launches); x_c goes
// through LDS to the lanes that own the channel's states, whose state rows are already on their way by then.
// (Forming the step's token-side values per channel in the same loop, as state_step_shared_kernel does, helped one
// shape and cost three -- 64 x 4096: 9.4 -> 8.7 us, 32 x 1536: 3.7 -> 4.0, 128 x 4096: 17.9 -> 19.8 -- and is not done.)
// grid: (ceil(D * N / 4 / (256 * U)), n_out)
template <typename T, int N, int U, bool HAS_Z, bool SOFTPLUS>
__global__ void __launch_bounds__(kBlock)
state_step_conv_kernel(float *h_out, const float *h_in, const int32_t *__restrict__ parent,
                       const T *__restrict__ x, const T *__restrict__ dt, const float *__restrict__ A,
                       const T *__restrict__ Bm, const T *__restrict__ Cm,
                       const float *__restrict__ Dskip, const T *__restrict__ z,
                       const float *__restrict__ dt_bias, T *__restrict__ out, int64_t n_in, int64_t D,
                       const float *__restrict__ conv_w, const float *__restrict__ conv_bias, const T *conv_src,
                       T *conv_dst, T *__restrict__ xc_out, int conv_k, int conv_silu)
{
    constexpr int Q = N / 4;
    constexpr int kChannels = kBlock * U / Q;                     // channels whose states this workgroup owns
    __shared__ float xs[kChannels];
    const int H = conv_k - 1;                                     // 1 .. 3 carried inputs per channel
    const int64_t j = blockIdx.y;
    const int64_t row4 = D * Q;  // float4s per branch
    const int64_t d_lo = (int64_t)blockIdx.x * kChannels;
    const float4 *a4 = reinterpret_cast<const float4 *>(A);

    int64_t f[U], d[U];
    bool live[U];
    float4 h[U], a[U], bv[U], cv[U];
    float dv[U], zv[U], bias[U], dsk[U];
#pragma unroll
    for (int i = 0; i < U; ++i) {
        const int64_t f_raw = ((int64_t)blockIdx.x * U + i) * kBlock + threadIdx.x;
        live[i] = f_raw < row4;
        f[i] = live[i] ? f_raw : row4 - 1;
        d[i] = f[i] / Q;
        const int q = (int)(f[i] - d[i] * Q);
        a[i] = a4[f[i]];
        bv[i] = ld4_io<N>(Bm + j * N + 4 * q);
        cv[i] = ld4_io<N>(Cm + j * N + 4 * q);
        dv[i] = ld_io(dt, j * D + d[i]);
        zv[i] = HAS_Z ? ld_io(z, j * D + d[i]) : 0.0f;
        bias[i] = dt_bias ? dt_bias[d[i]] : 0.0f;
        dsk[i] = Dskip ? Dskip[d[i]] : 0.0f;
    }
    // the state row and the window are the loads that have to wait for the parent index
    const int64_t p = parent ? (int64_t)parent[j] : j;
    const bool p_ok = p >= 0 && p < n_in;
    const float4 *hin4 = reinterpret_cast<const float4 *>(h_in) + (p_ok ? p : 0) * row4;
#pragma unroll
    for (int i = 0; i < U; ++i) h[i] = ld_stream(hin4 + f[i]);

    // conv step, one channel per thread, same order of operations as the conv kernel: bias, taps oldest to newest,
    // then the new input
    const float nan = __int_as_float(0x7fc00000);
    for (int c = threadIdx.x; c < kChannels; c += kBlock) {
        const int64_t dc = d_lo + c;
        if (dc >= D) break;
        // With one float4 per lane (few branches: the launch lives on latency) every fetch is unconditional, a tap
        // the window does not have re-reads its last one and is dropped afterwards: a load under a condition is
        // waited for inside its branch, one memory latency after the other.  With several float4s per lane (many
        // branches: the launch lives on bandwidth) the conditional form measured faster (64 x 4096: 9.4 against
        // 10.7 us), so it stays there.
        float wk[4], carried[3];
        const T *win = conv_src + ((p_ok ? p : 0) * D + dc) * H;
        if constexpr (U == 1) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float v = conv_w[dc * conv_k + (k <= H ? k : H)];
                wk[k] = k <= H ? v : 0.0f;
            }
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                const float v = ld_io(win, k < H ? k : H - 1);
                carried[k] = k < H ? v : 0.0f;
            }
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) wk[k] = k <= H ? conv_w[dc * conv_k + k] : 0.0f;
#pragma unroll
            for (int k = 0; k < 3; ++k) carried[k] = k < H ? ld_io(win, k) : 0.0f;
        }
        const float xpre = ld_io(x, j * D + dc);
        float acc = conv_bias ? conv_bias[dc] : 0.0f;
#pragma unroll
        for (int k = 0; k < 3; ++k)
            if (k < H) acc = fmaf(wk[k], carried[k], acc);
        float wlast = wk[0];
#pragma unroll
        for (int k = 1; k < 4; ++k)
            if (k == H) wlast = wk[k];
        acc = fmaf(wlast, xpre, acc);
        const float xc = conv_silu ? silu_f32(acc) : acc;
        // the stored tensor the step would read
        xs[c] = sizeof(T) == 2 ? bf16_to_f32(f32_to_bf16(xc)) : xc;
        // new window: the carried inputs move up, the new input comes last (NaN in front where the parent was bad)
        T *nwin = conv_dst + (j * D + dc) * H;
#pragma unroll
        for (int k = 0; k < 2; ++k)
            if (k + 1 < H) st_io(nwin, k, p_ok ? carried[k + 1] : nan);
        st_io(nwin, H - 1, xpre);
        if (xc_out) st_io(xc_out, j * D + dc, p_ok ? xc : nan);
    }
    __syncthreads();

#pragma unroll
    for (int i = 0; i < U; ++i) {
        const float xv = xs[d[i] - d_lo];
        const float v = dv[i] + bias[i];
        const float delta = SOFTPLUS ? softplus_f32(v) : v;
        const float u = delta * xv;
        const float dl = delta * kLog2e;
        float4 hh = h[i];
        hh.x = fmaf(exp2_hw(dl * a[i].x), hh.x, u * bv[i].x);
        hh.y = fmaf(exp2_hw(dl * a[i].y), hh.y, u * bv[i].y);
        hh.z = fmaf(exp2_hw(dl * a[i].z), hh.z, u * bv[i].z);
        hh.w = fmaf(exp2_hw(dl * a[i].w), hh.w, u * bv[i].w);
        float y = hh.x * cv[i].x;
        y = fmaf(hh.y, cv[i].y, y);
        y = fmaf(hh.z, cv[i].z, y);
        y = fmaf(hh.w, cv[i].w, y);
        y = channel_sum<Q>(y);
        if (!p_ok) {
            hh = make_float4(nan, nan, nan, nan);
            y = nan;
        }
        if (live[i]) {
            st_stream(reinterpret_cast<float4 *>(h_out) + j * row4 + f[i], hh);
            if (f[i] - d[i] * Q == 0) {
                y = fmaf(dsk[i], xv, y);
                if constexpr (HAS_Z) y *= silu_f32(zv[i]);
                st_io(out, j * D + d[i], y);
            }
        }
    }
}

// The same step for a draft position of the whole block, where the x projection arrives as partial sums (see
// StepArgs::xpart): what does not depend on it (the state row above all) is requested first, then the parts are
// added up, and dt (through the fused dt projection), B and C come out of LDS.  Kept apart from the plain kernel,
// which stays as lean as it was.
// grid: (ceil(D * N / 4 / (256 * U)), n_out).  A lane owns U float4s of the branch's (D, N) state,
// 256 float4s apart, so every wavefront load or store is still one contiguous 1 KiB run; all
// loads of the U pieces are issued before the first one is used, which keeps several KiB per
// wavefront in flight (the step is a single pass over the state and lives on memory latency).
template <typename T, int N, int U, bool HAS_Z, bool SOFTPLUS>
__global__ void __launch_bounds__(kBlock)
state_step_xproj_kernel(float *h_out, const float *h_in, const int32_t *__restrict__ parent,
                  const T *__restrict__ x, const T *__restrict__ dt, const float *__restrict__ A,
                  const T *__restrict__ Bm, const T *__restrict__ Cm,
                  const float *__restrict__ Dskip, const T *__restrict__ z,
                  const float *__restrict__ dt_bias, T *__restrict__ out, int64_t n_in, int64_t D,
                  const bf16_t *__restrict__ dt_w, int64_t dt_rank, const float *__restrict__ xpart, int n_parts)
{
    constexpr int Q = N / 4;
    constexpr int CW = 4;                                         // dt_w pieces a lane can hold ahead of the x projection sums
    const int64_t j = blockIdx.y;
    const int64_t row4 = D * Q;  // float4s per branch
    const float4 *a4 = reinterpret_cast<const float4 *>(A);
    __shared__ __attribute__((aligned(16))) float xs[256];
    const bool hold_w = dt_rank / 4 <= CW * Q;

    int64_t f[U], d[U];
    int q[U];
    bool live[U];
    float4 h[U], a[U], bv[U], cv[U];
    float xv[U], dv[U], zv[U], bias[U], dsk[U];
    uint2 wq[U][CW];
    // everything that does not depend on the x projection is requested first
#pragma unroll
    for (int i = 0; i < U; ++i) {
        const int64_t f_raw = ((int64_t)blockIdx.x * U + i) * kBlock + threadIdx.x;
        live[i] = f_raw < row4;
        f[i] = live[i] ? f_raw : row4 - 1;
        d[i] = f[i] / Q;
        q[i] = (int)(f[i] - d[i] * Q);
        a[i] = a4[f[i]];
        xv[i] = ld_io(x, j * D + d[i]);
        zv[i] = HAS_Z ? ld_io(z, j * D + d[i]) : 0.0f;
        bias[i] = dt_bias ? dt_bias[d[i]] : 0.0f;
        dsk[i] = Dskip ? Dskip[d[i]] : 0.0f;
#pragma unroll
        for (int c = 0; c < CW; ++c) wq[i][c] = make_uint2(0, 0);
        if (hold_w) {
            const uint2 *wrow = reinterpret_cast<const uint2 *>(dt_w + d[i] * dt_rank);
#pragma unroll
            for (int c = 0; c < CW; ++c)
                if (q[i] + c * Q < dt_rank / 4) wq[i][c] = wrow[q[i] + c * Q];
        }
    }
    // the state row is the only load that has to wait for the parent index
    const int64_t p = parent ? (int64_t)parent[j] : j;
    const bool p_ok = p >= 0 && p < n_in;
    const float4 *hin4 = reinterpret_cast<const float4 *>(h_in) + (p_ok ? p : 0) * row4;
#pragma unroll
    for (int i = 0; i < U; ++i) h[i] = ld_stream(hin4 + f[i]);
    // The branch's row of the x projection (dt low rank | B | C) arrives as n_parts partial sums: they are added
    // up in order and rounded to bf16, as the stored tensors they replace would have been.
    {
        const int xn = (int)dt_rank + 2 * N;
        for (int k = threadIdx.x; k < xn; k += kBlock) {
            // the parts of one sum lie side by side (n_parts % 4 == 0): four 16-byte loads in flight at a time
            const float4 *pr = reinterpret_cast<const float4 *>(xpart + (j * xn + k) * n_parts);
            float sum = 0.0f;
            for (int c = 0; c < n_parts / 4; c += 4) {
                float4 v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) v[u] = pr[min(c + u, n_parts / 4 - 1)];
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (c + u < n_parts / 4) sum = (((sum + v[u].x) + v[u].y) + v[u].z) + v[u].w;
            }
            xs[k] = bf16_to_f32(f32_to_bf16(sum));
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < U; ++i) {
            bv[i] = *reinterpret_cast<const float4 *>(&xs[dt_rank + 4 * q[i]]);
            cv[i] = *reinterpret_cast<const float4 *>(&xs[dt_rank + N + 4 * q[i]]);
            float acc = 0.0f;
            if (hold_w) {
#pragma unroll
                for (int c = 0; c < CW; ++c) {
                    const int cc = q[i] + c * Q;
                    if (cc < dt_rank / 4) {
                        const float4 b4 = *reinterpret_cast<const float4 *>(&xs[4 * cc]);
                        acc = fmaf(bf16_lo(wq[i][c].x), b4.x, acc);
                        acc = fmaf(bf16_hi(wq[i][c].x), b4.y, acc);
                        acc = fmaf(bf16_lo(wq[i][c].y), b4.z, acc);
                        acc = fmaf(bf16_hi(wq[i][c].y), b4.w, acc);
                    }
                }
            } else {
                const uint2 *wrow = reinterpret_cast<const uint2 *>(dt_w + d[i] * dt_rank);
                for (int64_t c = q[i]; c < dt_rank / 4; c += Q) {
                    const uint2 a2 = wrow[c];
                    const float4 b4 = *reinterpret_cast<const float4 *>(&xs[4 * c]);
                    acc = fmaf(bf16_lo(a2.x), b4.x, acc);
                    acc = fmaf(bf16_hi(a2.x), b4.y, acc);
                    acc = fmaf(bf16_lo(a2.y), b4.z, acc);
                    acc = fmaf(bf16_hi(a2.y), b4.w, acc);
                }
            }
            dv[i] = bf16_to_f32(f32_to_bf16(channel_sum<Q>(acc)));
        }
    }
#pragma unroll
    for (int i = 0; i < U; ++i) {
        const float v = dv[i] + bias[i];
        const float delta = SOFTPLUS ? softplus_f32(v) : v;
        const float u = delta * xv[i];
        const float dl = delta * kLog2e;
        float4 hh = h[i];
        hh.x = fmaf(exp2_hw(dl * a[i].x), hh.x, u * bv[i].x);
        hh.y = fmaf(exp2_hw(dl * a[i].y), hh.y, u * bv[i].y);
        hh.z = fmaf(exp2_hw(dl * a[i].z), hh.z, u * bv[i].z);
        hh.w = fmaf(exp2_hw(dl * a[i].w), hh.w, u * bv[i].w);
        float y = hh.x * cv[i].x;
        y = fmaf(hh.y, cv[i].y, y);
        y = fmaf(hh.z, cv[i].z, y);
        y = fmaf(hh.w, cv[i].w, y);
        y = channel_sum<Q>(y);
        if (!p_ok) {
            const float nan = __int_as_float(0x7fc00000);
            hh = make_float4(nan, nan, nan, nan);
            y = nan;
        }
        if (live[i]) {
            st_stream(reinterpret_cast<float4 *>(h_out) + j * row4 + f[i], hh);
            if (q[i] == 0) {
                y = fmaf(dsk[i], xv[i], y);
                if constexpr (HAS_Z) y *= silu_f32(zv[i]);
                st_io(out, j * D + d[i], y);
            }
        }
    }
}

template <typename T, int N, int U> hipError_t launch_step_u(const StepArgs &a, hipStream_t stream)
{
    const int64_t row4 = a.D * (N / 4);
    const int64_t per_block = (int64_t)kBlock * U;
    dim3 grid((unsigned)((row4 + per_block - 1) / per_block), (unsigned)a.n_out);
    if (U > 1 && !a.dt_w && !a.conv_w) {
#define MAMBA_STEP_S(HZ, SP)                                                                      \
    state_step_shared_kernel<T, N, U, HZ, SP><<<grid, kBlock, 0, stream>>>(                       \
        a.h_out, a.h_in, a.parent, static_cast<const T *>(a.x), static_cast<const T *>(a.dt), a.A, \
        static_cast<const T *>(a.Bm), static_cast<const T *>(a.Cm), a.Dskip,                      \
        static_cast<const T *>(a.z), a.dt_bias, static_cast<T *>(a.out), a.n_in, a.D)
        if (a.z) {
            if (a.dt_softplus) MAMBA_STEP_S(true, true);
            else MAMBA_STEP_S(true, false);
        } else {
            if (a.dt_softplus) MAMBA_STEP_S(false, true);
            else MAMBA_STEP_S(false, false);
        }
#undef MAMBA_STEP_S
        return hipGetLastError();
    }
    if constexpr (U <= kStepUnroll) {
#define MAMBA_STEP(HZ, SP)                                                                        \
    state_step_kernel<T, N, U, HZ, SP><<<grid, kBlock, 0, stream>>>(                              \
        a.h_out, a.h_in, a.parent, static_cast<const T *>(a.x), static_cast<const T *>(a.dt), a.A, \
        static_cast<const T *>(a.Bm), static_cast<const T *>(a.Cm), a.Dskip,                      \
        static_cast<const T *>(a.z), a.dt_bias, static_cast<T *>(a.out), a.n_in, a.D,                \
        static_cast<const bf16_t *>(a.dt_w), a.dt_rank)
#define MAMBA_STEP_X(HZ, SP)                                                                      \
    state_step_xproj_kernel<T, N, U, HZ, SP><<<grid, kBlock, 0, stream>>>(                        \
        a.h_out, a.h_in, a.parent, static_cast<const T *>(a.x), static_cast<const T *>(a.dt), a.A, \
        static_cast<const T *>(a.Bm), static_cast<const T *>(a.Cm), a.Dskip,                      \
        static_cast<const T *>(a.z), a.dt_bias, static_cast<T *>(a.out), a.n_in, a.D,                \
        static_cast<const bf16_t *>(a.dt_w), a.dt_rank, a.xpart, a.n_parts)
    if (a.conv_w) {
        if constexpr (U == 2) {
            return hipErrorInvalidValue;                          // the conv variant is built for U = 1 and 4 only (see launch_step_n)
        } else {
#define MAMBA_STEP_C(HZ, SP)                                                                      \
    state_step_conv_kernel<T, N, U, HZ, SP><<<grid, kBlock, 0, stream>>>(                         \
        a.h_out, a.h_in, a.parent, static_cast<const T *>(a.x), static_cast<const T *>(a.dt), a.A, \
        static_cast<const T *>(a.Bm), static_cast<const T *>(a.Cm), a.Dskip,                      \
        static_cast<const T *>(a.z), a.dt_bias, static_cast<T *>(a.out), a.n_in, a.D, a.conv_w,   \
        a.conv_bias, static_cast<const T *>(a.conv_src), static_cast<T *>(a.conv_dst),             \
        static_cast<T *>(a.xc_out), a.conv_k, a.conv_silu)
            if (a.z) {
                if (a.dt_softplus) MAMBA_STEP_C(true, true);
                else MAMBA_STEP_C(true, false);
            } else {
                if (a.dt_softplus) MAMBA_STEP_C(false, true);
                else MAMBA_STEP_C(false, false);
            }
#undef MAMBA_STEP_C
            return hipGetLastError();
        }
    }
    if (a.xpart && a.dt_w) {
        if (a.z) {
            if (a.dt_softplus) MAMBA_STEP_X(true, true);
            else MAMBA_STEP_X(true, false);
        } else {
            if (a.dt_softplus) MAMBA_STEP_X(false, true);
            else MAMBA_STEP_X(false, false);
        }
        return hipGetLastError();
    }
    if (a.z) {
        if (a.dt_softplus) MAMBA_STEP(true, true);
        else MAMBA_STEP(true, false);
    } else {
        if (a.dt_softplus) MAMBA_STEP(false, true);
        else MAMBA_STEP(false, false);
    }
#undef MAMBA_STEP
#undef MAMBA_STEP_X
    return hipGetLastError();
    } else {
        return hipErrorInvalidValue;   // eight float4s per lane exist for the plain step only
    }
}

template <typename T, int N> hipError_t launch_step_n(const StepArgs &a, hipStream_t stream)
{
    // several float4s per lane as long as that still leaves about three workgroups per CU
    const int64_t row4 = a.D * (N / 4);
    auto blocks = [&](int u) { return a.n_out * ((row4 + kBlock * u - 1) / (kBlock * u)); };
    // the plain step with eight per lane while that gives between 1.5 and 4 workgroups per CU: 64 branches x 4096
    // channels 8.7 -> 7.6 us, the time of a bare copy of the same state rows; 128 branches are better off with four
    if (!a.conv_w && !a.dt_w && blocks(8) >= 384 && blocks(8) < 1024) return launch_step_u<T, N, 8>(a, stream);
    if (blocks(kStepUnroll) >= 768) return launch_step_u<T, N, kStepUnroll>(a, stream);
    if (kStepUnroll > 2 && blocks(2) >= 768 && !a.conv_w) return launch_step_u<T, N, 2>(a, stream);
    return launch_step_u<T, N, 1>(a, stream);
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
