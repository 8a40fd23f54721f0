// Selective scan in a single pass for shapes with many independent channels (batch x D large enough to
// fill the chip without cutting time), gfx950.  Same arithmetic as scan.hip:
//
//   delta = softplus(dt + dt_bias);  h_t = exp(delta_t A) h_{t-1} + delta_t B_t x_t
//   y_t = C_t . h_t + D x_t;  out_t = y_t silu(z_t)
//
// No time chunks: every token is walked once, nothing but the operands goes through memory.
//
// A workgroup of four wavefronts owns 64 adjacent channels of one batch row and walks the sequence in
// tiles of 64 steps.  It works in two lane layouts that hand over through LDS:
//   * token layout (loads, per-token arithmetic, stores): a thread owns 8 adjacent channels of two steps of
//     the tile, so a wavefront touches 8 rows x 128 bytes per access; it forms delta and delta * x for
//     its 8 tokens (softplus once per token and channel, not once per state lane) and leaves them in LDS,
//     and after the recurrence picks up y for the same tokens, adds the skip term, gates and stores;
//   * state layout (the recurrence): a lane owns N / 4 states of one channel, the four lanes of a channel
//     sit in one quad and add their partial C . h with DPP exchanges (four steps at a time).  States and A * log2(e) stay in
//     registers for the whole sequence; delta, delta * x (8 bytes per channel and step) and B_t, C_t come
//     from LDS.  Per state update: mul, exp2, mul, fma, fma.
// With N / 4 states per lane a layer of 4096 channels x 8 rows gives 2048 wavefronts, two per SIMD.
// The next tile's rows are requested before the recurrence of the current tile starts and are consumed
// after it; barriers order LDS only, so stores and prefetches stay in flight across them.
#include "device_math.h"
#include "launch.h"

namespace mamba {
namespace {

// sched_barrier mask: scalar, memory and LDS instructions may still be moved across; vector ALU ones stay put
constexpr int kSchedMemoryOnly = 0x4 | 0x10 | 0x20 | 0x40 | 0x80 | 0x100 | 0x200;
constexpr int kThreads = 256;
constexpr int kChannels = 64;   // channels per workgroup
constexpr int kTile = 64;       // steps per tile (a multiple of 32)
constexpr int kYStride = 80;    // floats per row of the y tile: 16-byte aligned rows, 16 banks apart, so that the four
                                // rows a wavefront writes at a time fall two lanes to a bank, the least possible

__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// eight adjacent channels of one token row, as they lie in memory
template <typename T> struct Row8;
template <> struct Row8<bf16_t> {
    uint4 v;
    __device__ __forceinline__ void load(const bf16_t *p) { v = *reinterpret_cast<const uint4 *>(p); }
    __device__ __forceinline__ void unpack(float *f) const
    {
        f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x); f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
        f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z); f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
    }
};
template <> struct Row8<float> {
    float4 a, b;
    __device__ __forceinline__ void load(const float *p)
    {
        a = reinterpret_cast<const float4 *>(p)[0];
        b = reinterpret_cast<const float4 *>(p)[1];
    }
    __device__ __forceinline__ void unpack(float *f) const
    {
        f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
    }
};
__device__ __forceinline__ void store_row8(bf16_t *p, const float *f)
{
    *reinterpret_cast<uint4 *>(p) = make_uint4(f32x2_to_bf16x2(f[0], f[1]), f32x2_to_bf16x2(f[2], f[3]),
                                               f32x2_to_bf16x2(f[4], f[5]), f32x2_to_bf16x2(f[6], f[7]));
}
__device__ __forceinline__ void store_row8(float *p, const float *f)
{
    reinterpret_cast<float4 *>(p)[0] = make_float4(f[0], f[1], f[2], f[3]);
    reinterpret_cast<float4 *>(p)[1] = make_float4(f[4], f[5], f[6], f[7]);
}

// four adjacent elements of a B or C row
__device__ __forceinline__ float4 load4(const bf16_t *p)
{
    const uint2 r = *reinterpret_cast<const uint2 *>(p);
    return make_float4(bf16_lo(r.x), bf16_hi(r.x), bf16_lo(r.y), bf16_hi(r.y));
}
__device__ __forceinline__ float4 load4(const float *p) { return *reinterpret_cast<const float4 *>(p); }

template <int CTRL> __device__ __forceinline__ float dpp_take(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
// Four values per lane, summed over the four lanes of a quad, lane q keeping the total of value q.  The lanes
// swap what they do not keep twice (pairs, then pairs of pairs): 3 additions and 6 selects, against 8 additions
// and 4 selects for four full sums of which each lane would keep one.
__device__ __forceinline__ float quad_sum_scatter(const float (&p)[4], int q)
{
    const bool odd = q & 1, high = q & 2;
    const float keep0 = odd ? p[1] : p[0], send0 = odd ? p[0] : p[1];
    const float keep1 = odd ? p[3] : p[2], send1 = odd ? p[2] : p[3];
    const float r0 = keep0 + dpp_take<0xB1>(send0);      // quad_perm [1,0,3,2]: values 0 / 1 over the pair
    const float r1 = keep1 + dpp_take<0xB1>(send1);      // values 2 / 3 over the pair
    const float keep = high ? r1 : r0, send = high ? r0 : r1;
    return keep + dpp_take<0x4E>(send);                  // quad_perm [2,3,0,1]
}

// grid: (ceil(D / 64), batch); block: 256.  D % 8 == 0, N % 4 == 0.
// (The tiles in LDS allow two workgroups to a compute unit, two wavefronts to a SIMD; stating that, and unrolling
// the tile loop fully, lets the compiler's scheduler keep more LDS operands in flight: 8192 tokens x 8 x 4096
// channels 1.25 -> 1.18 ms.  With 32 states the same two hints make it spill, so that variant keeps the defaults.)
template <typename T, int N, bool HAS_Z, bool SOFTPLUS>
__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(N > 16 ? 1 : 2, N > 16 ? 8 : 2)))
scan_direct_kernel(const T *x, const T *dt, const float *__restrict__ A, const T *Bm, const T *Cm,
                   const float *__restrict__ Dskip, const T *z, const float *__restrict__ dt_bias,
                   const float *h0 /* may alias h_final */, T *out, float *h_final, int64_t L, int64_t D)
{
    constexpr int SPL = N / 4;                       // states per lane
    constexpr int kBcGroups = 2 * kTile * N / 4;     // groups of four B or C values in a tile
    constexpr int kBcIters = (kBcGroups + kThreads - 1) / kThreads;
    constexpr int kRows = kTile / 32;                // token rows per thread and tile
    constexpr int kGroupUnroll = N > 16 ? 8 : kTile / 4;   // groups of four steps unrolled in the tile loop
    __shared__ __attribute__((aligned(16))) float2 lds_du[kTile][kChannels];   // delta, delta * x
    __shared__ __attribute__((aligned(16))) float lds_bc[kTile][2 * N];        // B_t | C_t
    __shared__ __attribute__((aligned(16))) float lds_y[kTile][kYStride];      // C . h per token

    const int tid = threadIdx.x;
    const int64_t b = blockIdx.y;
    const int64_t c_block = (int64_t)blockIdx.x * kChannels;
    const int64_t row0 = b * L;

    // ---- token layout: row lr of the tile, channels lc .. lc + 7
    const int lr = tid >> 3, lcg = tid & 7;
    const int64_t lc_raw = c_block + 8 * lcg;
    const bool l_live = lc_raw < D;
    const int64_t lc = l_live ? lc_raw : D - 8;      // dead threads shadow the last channels and store nothing
    float bias8[8], dsk8[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        bias8[i] = dt_bias ? dt_bias[lc + i] : 0.0f;
        dsk8[i] = Dskip ? Dskip[lc + i] : 0.0f;
    }

    // ---- state layout: channel cc of the block, states q * SPL .. q * SPL + SPL - 1
    const int lane = tid & 63;
    const int cc = (tid >> 6) * 16 + (lane >> 2), q = lane & 3;
    // where the token layout put this channel's (delta, delta * x) within its row (see publish)
    const int cc_slot = (cc & ~7) + 2 * ((((cc & 7) >> 1) + (cc >> 4)) & 3) + (cc & 1);
    const int64_t c_raw = c_block + cc;
    const bool c_live = c_raw < D;
    const int64_t c = c_live ? c_raw : D - 1;
    float a2[SPL], h[SPL];
#pragma unroll
    for (int j = 0; j < SPL; ++j) {
        a2[j] = A[c * N + q * SPL + j] * kLog2e;
        h[j] = h0 ? h0[(b * D + c) * N + q * SPL + j] : 0.0f;
    }

    // rows of a tile as fetched: kept raw until the tile's turn (x and z again for the gate and skip term)
    struct Rows {
        Row8<T> x[kRows], dt[kRows], z[kRows];
        float4 bc[kBcIters];
    };
    Rows nxt;
    Row8<T> x_cur[kRows], z_cur[kRows];

    // requests the rows of the tile that starts at step t_base (rows past the end re-read the last row)
    auto fetch = [&](Rows &r, int64_t t_base) {
#pragma unroll
        for (int i = 0; i < kRows; ++i) {
            int64_t t = t_base + lr + 32 * i;
            t = t < L ? t : L - 1;
            const int64_t o = (row0 + t) * D + lc;
            r.x[i].load(x + o);
            r.dt[i].load(dt + o);
            if constexpr (HAS_Z) r.z[i].load(z + o);
        }
#pragma unroll
        for (int it = 0; it < kBcIters; ++it) {
            const int g = tid + it * kThreads;                 // group index: (array, step, four values)
            if (kBcGroups % kThreads == 0 || g < kBcGroups) {
                const int arr = g / (kTile * N / 4), rem = g % (kTile * N / 4);
                const int s = rem / (N / 4), n4 = rem % (N / 4);
                int64_t ts = t_base + s;
                ts = ts < L ? ts : L - 1;
                r.bc[it] = load4((arr ? Cm : Bm) + (row0 + ts) * N + 4 * n4);
            }
        }
    };
    // per-token arithmetic of fetched rows into LDS; they become the current rows
    auto publish = [&](const Rows &r, int64_t t_base) {
        const bool tail = t_base + kTile > L;                // uniform: only the last tile can be ragged
#pragma unroll
        for (int i = 0; i < kRows; ++i) {
            const bool valid = t_base + lr + 32 * i < L;
            float xv[8], dv[8];
            r.x[i].unpack(xv);
            r.dt[i].unpack(dv);
            // a thread's four 16-byte pieces go to slots rotated by lcg / 2: the eight threads of a row then
            // write eight different groups of four banks at a time (unrotated, four of them share a group)
            float4 *dst = reinterpret_cast<float4 *>(&lds_du[lr + 32 * i][8 * lcg]);
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                float d[2];
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    const float v = dv[e + k] + bias8[e + k];
                    d[k] = SOFTPLUS ? softplus_f32(v) : v;
                    if (tail) d[k] = valid ? d[k] : 0.0f;    // steps past the end leave the state as it is
                }
                dst[(e / 2 + (lcg >> 1)) & 3] = make_float4(d[0], d[0] * xv[e], d[1], d[1] * xv[e + 1]);
            }
            x_cur[i] = r.x[i];
            if constexpr (HAS_Z) z_cur[i] = r.z[i];
        }
#pragma unroll
        for (int it = 0; it < kBcIters; ++it) {
            const int g = tid + it * kThreads;
            if (kBcGroups % kThreads == 0 || g < kBcGroups) {
                const int arr = g / (kTile * N / 4), rem = g % (kTile * N / 4);
                const int s = rem / (N / 4), n4 = rem % (N / 4);
                const bool ok = t_base + s < L;
                *reinterpret_cast<float4 *>(&lds_bc[s][arr * N + 4 * n4]) = ok ? r.bc[it] : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
    };
    // skip term, gate and store of the current tile
    auto epilogue = [&](int64_t t_base) {
#pragma unroll
        for (int i = 0; i < kRows; ++i) {
            float xv[8], yv[8], ov[8], zv[8];
            x_cur[i].unpack(xv);
            const float4 y0 = *reinterpret_cast<const float4 *>(&lds_y[lr + 32 * i][8 * lcg]);
            const float4 y1 = *reinterpret_cast<const float4 *>(&lds_y[lr + 32 * i][8 * lcg + 4]);
            yv[0] = y0.x; yv[1] = y0.y; yv[2] = y0.z; yv[3] = y0.w; yv[4] = y1.x; yv[5] = y1.y; yv[6] = y1.z; yv[7] = y1.w;
            if constexpr (HAS_Z) z_cur[i].unpack(zv);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float y = fmaf(dsk8[e], xv[e], yv[e]);
                ov[e] = HAS_Z ? y * silu_f32(zv[e]) : y;
            }
            const int64_t t = t_base + lr + 32 * i;
            if (l_live && t < L) store_row8(out + (row0 + t) * D + lc, ov);
        }
    };

    struct Group {
        float2 du[4];
        float bv[4][SPL], cv[4][SPL];
    };
    auto read_group = [&](Group &g, int s4) {
#pragma unroll
        for (int j4 = 0; j4 < 4; ++j4) {
            const int s = s4 + j4;
            g.du[j4] = lds_du[s][cc_slot];
            if constexpr (SPL % 4 == 0) {
#pragma unroll
                for (int j = 0; j < SPL; j += 4) {
                    const float4 b4 = *reinterpret_cast<const float4 *>(&lds_bc[s][q * SPL + j]);
                    const float4 c4 = *reinterpret_cast<const float4 *>(&lds_bc[s][N + q * SPL + j]);
                    g.bv[j4][j] = b4.x; g.bv[j4][j + 1] = b4.y; g.bv[j4][j + 2] = b4.z; g.bv[j4][j + 3] = b4.w;
                    g.cv[j4][j] = c4.x; g.cv[j4][j + 1] = c4.y; g.cv[j4][j + 2] = c4.z; g.cv[j4][j + 3] = c4.w;
                }
            } else {
#pragma unroll
                for (int j = 0; j < SPL; ++j) {
                    g.bv[j4][j] = lds_bc[s][q * SPL + j];
                    g.cv[j4][j] = lds_bc[s][N + q * SPL + j];
                }
            }
        }
    };

    const int64_t n_tiles = (L + kTile - 1) / kTile;
    fetch(nxt, 0);
    publish(nxt, 0);
    lds_barrier();

    for (int64_t k = 0; k < n_tiles; ++k) {
        const int64_t t_base = k * kTile;
        const bool more = k + 1 < n_tiles;
        if (more) fetch(nxt, t_base + kTile);

        // the recurrence over the tile, four steps at a time; after four steps lane q holds y of step s4 + q.
        // The LDS operands of a group of four steps are requested one group ahead.
        Group cur;
        read_group(cur, 0);
#pragma unroll kGroupUnroll
        for (int s4 = 0; s4 < kTile; s4 += 4) {
            Group ahead;
            read_group(ahead, (s4 + 4) & (kTile - 1));       // the last group re-reads the first, unused
            // the exponentials of the four steps as one run (exp2 next to exp2 issues at its own rate, scattered
            // among multiplies it slows its neighbours), then the updates
            float a[4][SPL], yp[4];
#pragma unroll
            for (int j4 = 0; j4 < 4; ++j4)
#pragma unroll
                for (int j = 0; j < SPL; ++j) a[j4][j] = cur.du[j4].x * a2[j];
            __builtin_amdgcn_sched_barrier(kSchedMemoryOnly);
#pragma unroll
            for (int j4 = 0; j4 < 4; ++j4)
#pragma unroll
                for (int j = 0; j < SPL; ++j) a[j4][j] = exp2_hw(a[j4][j]);
            __builtin_amdgcn_sched_barrier(kSchedMemoryOnly);
#pragma unroll
            for (int j4 = 0; j4 < 4; ++j4) {
                yp[j4] = 0.0f;
#pragma unroll
                for (int j = 0; j < SPL; ++j) {
                    h[j] = fmaf(a[j4][j], h[j], cur.du[j4].y * cur.bv[j4][j]);
                    yp[j4] = fmaf(h[j], cur.cv[j4][j], yp[j4]);
                }
            }
            lds_y[s4 + q][cc] = quad_sum_scatter(yp, q);
            cur = ahead;
        }
        lds_barrier();   // y of the tile is complete; delta, delta * x, B and C of the tile are used up
        epilogue(t_base);
        if (more) publish(nxt, t_base + kTile);
        lds_barrier();   // the next tile is in LDS; y has been read
    }

    if (h_final && c_live) {
#pragma unroll
        for (int j = 0; j < SPL; ++j) h_final[(b * D + c) * N + q * SPL + j] = h[j];
    }
}

template <typename T, int N>
hipError_t launch_direct_n(const ScanArgs &a, hipStream_t stream)
{
    const dim3 grid((unsigned)((a.D + kChannels - 1) / kChannels), (unsigned)a.batch);
    const T *x = static_cast<const T *>(a.x), *dt = static_cast<const T *>(a.dt);
    const T *Bm = static_cast<const T *>(a.Bm), *Cm = static_cast<const T *>(a.Cm);
    const T *z = static_cast<const T *>(a.z);
    T *out = static_cast<T *>(a.out);
#define MAMBA_LAUNCH_DIRECT(HZ, SP)                                                                   \
    scan_direct_kernel<T, N, HZ, SP><<<grid, kThreads, 0, stream>>>(x, dt, a.A, Bm, Cm, a.Dskip, z, a.dt_bias, \
                                                                    a.h0, out, a.h_final, a.L, a.D)
    if (z) {
        if (a.dt_softplus) MAMBA_LAUNCH_DIRECT(true, true);
        else MAMBA_LAUNCH_DIRECT(true, false);
    } else {
        if (a.dt_softplus) MAMBA_LAUNCH_DIRECT(false, true);
        else MAMBA_LAUNCH_DIRECT(false, false);
    }
#undef MAMBA_LAUNCH_DIRECT
    return hipGetLastError();
}

template <typename T> hipError_t launch_direct_io(const ScanArgs &a, hipStream_t stream)
{
    switch (a.N) {
    case 4: return launch_direct_n<T, 4>(a, stream);
    case 8: return launch_direct_n<T, 8>(a, stream);
    case 16: return launch_direct_n<T, 16>(a, stream);
    case 32: return launch_direct_n<T, 32>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

// The single-pass kernel serves a shape when its token rows can be read in 16-byte pieces and there are enough
// 64-channel blocks to give nearly every compute unit a workgroup: then walking every token once beats cutting
// time, which walks every token twice.  A lone workgroup takes the same time per step whatever the grid, so the
// crossover is where the two-pass kernels stop fitting their work into that time (measured on 2048 tokens:
// 192 blocks 185 us against 174 us in two passes, 256 blocks 194 against 234, 512 blocks 25 % ahead).
bool scan_direct_applies(int64_t batch, int64_t L, int64_t D, int64_t N)
{
    if (L < 1 || D % 8 != 0 || N % 4 != 0 || batch > 65535) return false;
    const int64_t blocks = batch * ((D + kChannels - 1) / kChannels);
    return blocks >= 224;
}

hipError_t launch_scan_direct(const ScanArgs &a, hipStream_t stream)
{
    if (a.io == kIoBf16) return launch_direct_io<bf16_t>(a, stream);
    return launch_direct_io<float>(a, stream);
}

}  // namespace mamba
