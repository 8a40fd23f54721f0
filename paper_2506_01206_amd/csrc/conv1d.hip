// Causal depthwise conv1d over time with optional SiLU (first stage of the selective-SSM layer,
// run over the context when the drafter encodes it and over one token per branch while it
// drafts), gfx950.
//
//   y[b,t,d] = act(bias[d] + sum_k w[d,k] xpad[b,t+k,d]),  xpad = [carried K-1 rows or zeros ; x]
//   conv_state_out[b,d,:] = last K-1 rows of xpad
//
// HBM-bound: 2 elements moved per output.  A lane owns VEC adjacent channels (16 bytes of a token
// row), walks a tile of consecutive tokens and keeps the K-1 previous rows in registers, so every
// input element is read once (plus K-1 halo rows per tile) and every wavefront access is a
// contiguous run.  Loads of the next group of rows are issued before the current group is used.
// In tree drafting (Sec. 4.1) a branch starts from the window of its parent: the carried rows can be
// read through a parent index, which replaces a separate copy of the window.
#include "device_math.h"
#include "launch.h"

namespace mamba {
namespace {

constexpr int kBlock = 64;
constexpr int kRows = 8;       // rows loaded together, one group ahead

template <typename T, int VEC> struct RowVec;
template <> struct RowVec<float, 4> { typedef float4 type; };
template <> struct RowVec<float, 1> { typedef float type; };
template <> struct RowVec<bf16_t, 8> { typedef uint4 type; };
template <> struct RowVec<bf16_t, 1> { typedef uint16_t type; };

__device__ __forceinline__ void unpack_row(float4 r, float *v) { v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w; }
__device__ __forceinline__ void unpack_row(float r, float *v) { v[0] = r; }
__device__ __forceinline__ void unpack_row(uint16_t r, float *v) { v[0] = bf16_to_f32(r); }
__device__ __forceinline__ void unpack_row(uint4 r, float *v)
{
    v[0] = bf16_lo(r.x); v[1] = bf16_hi(r.x); v[2] = bf16_lo(r.y); v[3] = bf16_hi(r.y);
    v[4] = bf16_lo(r.z); v[5] = bf16_hi(r.z); v[6] = bf16_lo(r.w); v[7] = bf16_hi(r.w);
}
__device__ __forceinline__ void pack_row(const float *v, float4 &r) { r = make_float4(v[0], v[1], v[2], v[3]); }
__device__ __forceinline__ void pack_row(const float *v, float &r) { r = v[0]; }
__device__ __forceinline__ void pack_row(const float *v, uint16_t &r) { r = (uint16_t)f32_to_bf16(v[0]); }
__device__ __forceinline__ void pack_row(const float *v, uint4 &r)
{
    r = make_uint4(f32x2_to_bf16x2(v[0], v[1]), f32x2_to_bf16x2(v[2], v[3]),
                   f32x2_to_bf16x2(v[4], v[5]), f32x2_to_bf16x2(v[6], v[7]));
}

// COUNT contiguous elements, COUNT * sizeof(T) a multiple of 16 bytes and p 16-byte aligned:
// moved as 16-byte vectors (the per-lane blocks of weights and of carried state are such blocks).
template <int COUNT> __device__ __forceinline__ void ld_block(const float *p, float *f)
{
    const float4 *q = reinterpret_cast<const float4 *>(p);
#pragma unroll
    for (int v = 0; v < COUNT / 4; ++v) unpack_row(q[v], f + 4 * v);
}
template <int COUNT> __device__ __forceinline__ void ld_block(const bf16_t *p, float *f)
{
    const uint4 *q = reinterpret_cast<const uint4 *>(p);
#pragma unroll
    for (int v = 0; v < COUNT / 8; ++v) unpack_row(q[v], f + 8 * v);
}
template <int COUNT> __device__ __forceinline__ void st_block(float *p, const float *f)
{
    float4 *q = reinterpret_cast<float4 *>(p);
#pragma unroll
    for (int v = 0; v < COUNT / 4; ++v) pack_row(f + 4 * v, q[v]);
}
template <int COUNT> __device__ __forceinline__ void st_block(bf16_t *p, const float *f)
{
    uint4 *q = reinterpret_cast<uint4 *>(p);
#pragma unroll
    for (int v = 0; v < COUNT / 8; ++v) pack_row(f + 8 * v, q[v]);
}

// grid: (channel-vector groups, time tiles, batch)
template <typename T, int VEC, int K, bool SILU>
__global__ void __launch_bounds__(kBlock)
conv1d_kernel(const T *__restrict__ x, const float *__restrict__ w, const float *__restrict__ bias,
              const T *state_in, T *__restrict__ y, T *state_out, int64_t L, int64_t D,
              int64_t tile_len, const int32_t *__restrict__ parent, int64_t n_in)
{
    typedef typename RowVec<T, VEC>::type row_t;
    constexpr int H = K - 1;
    const int64_t b = blockIdx.z;
    const int64_t dv = (int64_t)blockIdx.x * kBlock + threadIdx.x;  // channel-vector index
    if (dv * VEC >= D) return;                                      // no cross-lane work below
    const int64_t d0 = dv * VEC;
    const int64_t t0 = (int64_t)blockIdx.y * tile_len;
    const int64_t t1 = (t0 + tile_len < L) ? t0 + tile_len : L;

    float wr[VEC][K], br[VEC];
    if constexpr (VEC > 1) {
        ld_block<VEC * K>(w + d0 * K, &wr[0][0]);
    } else {
#pragma unroll
        for (int k = 0; k < K; ++k) wr[0][k] = w[d0 * K + k];
    }
#pragma unroll
    for (int c = 0; c < VEC; ++c) br[c] = bias ? bias[d0 + c] : 0.0f;

    const T *xb = x + b * L * D + d0;
    T *yb = y + b * L * D + d0;
    auto ld_row = [&](int64_t t) { return *reinterpret_cast<const row_t *>(xb + t * D); };

    // window: the H rows before t0 in padded time; win[H-1] is the newest.  Rows before token 0
    // come from the carried state, whose (VEC, H) block of this lane is one contiguous run.
    float win[H > 0 ? H : 1][VEC];
    float carried[VEC * (H > 0 ? H : 1)];
    if (t0 < H) {
        // a draft branch continues from its parent's window (the copy is fused into this load)
        const int64_t pb = parent ? (int64_t)parent[b] : b;
        const bool p_ok = !parent || (pb >= 0 && pb < n_in);
        if (!state_in) {
#pragma unroll
            for (int i = 0; i < VEC * H; ++i) carried[i] = 0.0f;
        } else if (!p_ok) {
#pragma unroll
            for (int i = 0; i < VEC * H; ++i) carried[i] = __int_as_float(0x7fc00000);
        } else if constexpr (VEC > 1) {
            ld_block<VEC * H>(state_in + (pb * D + d0) * H, carried);
        } else {
#pragma unroll
            for (int k = 0; k < H; ++k) carried[k] = ld_io(state_in, (pb * D + d0) * H + k);
        }
    }
#pragma unroll
    for (int i = 0; i < H; ++i) {
        const int64_t t = t0 - H + i;  // token index of this window row, negative => carried state
        if (t >= 0) {
            unpack_row(ld_row(t), win[i]);
        } else {
#pragma unroll
            for (int c = 0; c < VEC; ++c) {
                float v = 0.0f;
#pragma unroll
                for (int k = 0; k < H; ++k)
                    if (k == H + t) v = carried[c * H + k];
                win[i][c] = v;
            }
        }
    }

    auto emit = [&](int64_t t, row_t raw) {
        float cur[VEC], o[VEC];
        unpack_row(raw, cur);
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            float acc = br[c];
#pragma unroll
            for (int k = 0; k < H; ++k) acc = fmaf(wr[c][k], win[k][c], acc);
            acc = fmaf(wr[c][K - 1], cur[c], acc);
            o[c] = SILU ? silu_f32(acc) : acc;
        }
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
#pragma unroll
            for (int k = 0; k + 1 < H; ++k) win[k][c] = win[k + 1][c];
            if (H > 0) win[H - 1][c] = cur[c];
        }
        row_t packed;
        pack_row(o, packed);
        *reinterpret_cast<row_t *>(yb + t * D) = packed;
    };

    int64_t t = t0;
    row_t cur[kRows];
    if (t + kRows <= t1) {
#pragma unroll
        for (int i = 0; i < kRows; ++i) cur[i] = ld_row(t + i);
    }
    for (; t + kRows <= t1; t += kRows) {
        row_t nxt[kRows];
        const bool more = t + 2 * kRows <= t1;
        if (more) {
#pragma unroll
            for (int i = 0; i < kRows; ++i) nxt[i] = ld_row(t + kRows + i);
        }
#pragma unroll
        for (int i = 0; i < kRows; ++i) emit(t + i, cur[i]);
        if (more) {
#pragma unroll
            for (int i = 0; i < kRows; ++i) cur[i] = nxt[i];
        }
    }
    for (; t < t1; ++t) emit(t, ld_row(t));

    if (state_out && t1 == L) {
        float last[VEC * (H > 0 ? H : 1)];
#pragma unroll
        for (int c = 0; c < VEC; ++c)
#pragma unroll
            for (int k = 0; k < H; ++k) last[c * H + k] = win[k][c];
        if constexpr (VEC > 1) {
            st_block<VEC * H>(state_out + (b * D + d0) * H, last);
        } else {
#pragma unroll
            for (int k = 0; k < H; ++k) st_io(state_out, (b * D + d0) * H + k, last[k]);
        }
    }
}

template <typename T, int VEC, int K> hipError_t launch_conv_k(const ConvArgs &a, hipStream_t stream)
{
    const int64_t vecs = (a.D + VEC - 1) / VEC;
    const unsigned gx = (unsigned)((vecs + kBlock - 1) / kBlock);
    // Time tiles: enough workgroups to fill the chip, long enough to amortize the K-1 halo rows.
    // An in-place state update keeps one tile so that a thread reads the state before it writes it.
    // Short inputs get shorter tiles (down to one group of rows) until there are about two wavefronts per SIMD.
    int64_t tile_len = 32;
    while (tile_len > kRows && (int64_t)gx * ((a.L + tile_len - 1) / tile_len) * a.batch < 2048) tile_len /= 2;
    if (a.state_out && a.state_in == a.state_out) tile_len = a.L;
    if ((a.L + tile_len - 1) / tile_len > 65535) tile_len = (a.L + 65534) / 65535;
    if (tile_len < 1) tile_len = 1;
    int64_t tiles = (a.L + tile_len - 1) / tile_len;
    if (tiles < 1) tiles = 1;  // L == 0: one tile that only passes the carried state on
    dim3 grid(gx, (unsigned)tiles, (unsigned)a.batch);
    const T *x = static_cast<const T *>(a.x);
    const T *si = static_cast<const T *>(a.state_in);
    T *y = static_cast<T *>(a.y);
    T *so = static_cast<T *>(a.state_out);
    if (a.apply_silu)
        conv1d_kernel<T, VEC, K, true><<<grid, kBlock, 0, stream>>>(x, a.w, a.bias, si, y, so, a.L, a.D, tile_len, a.parent, a.n_in);
    else
        conv1d_kernel<T, VEC, K, false><<<grid, kBlock, 0, stream>>>(x, a.w, a.bias, si, y, so, a.L, a.D, tile_len, a.parent, a.n_in);
    return hipGetLastError();
}

template <typename T, int VEC> hipError_t launch_conv_v(const ConvArgs &a, hipStream_t stream)
{
    switch (a.K) {
    case 2: return launch_conv_k<T, VEC, 2>(a, stream);
    case 3: return launch_conv_k<T, VEC, 3>(a, stream);
    case 4: return launch_conv_k<T, VEC, 4>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_conv1d(const ConvArgs &a, hipStream_t stream)
{
    // 16-byte channel vectors need every token row to start on a 16-byte boundary
    if (a.io == kIoBf16) {
        if (a.D % 8 == 0) return launch_conv_v<bf16_t, 8>(a, stream);
        return launch_conv_v<bf16_t, 1>(a, stream);
    }
    if (a.D % 4 == 0) return launch_conv_v<float, 4>(a, stream);
    return launch_conv_v<float, 1>(a, stream);
}

}  // namespace mamba
