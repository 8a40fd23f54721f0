// Selective scan for gfx950 (context encoding; Sec. 3.1 of the paper: the drafter encodes
// the prefix once, with memory that does not grow with its length).
//
//   delta = softplus(dt + dt_bias);  h_t = exp(delta_t A) h_{t-1} + delta_t B_t x_t
//   y_t = C_t . h_t + D x_t;  out_t = y_t silu(z_t)
//
// Mapping.  One wavefront per workgroup; a lane owns CPL adjacent channels and keeps their
// CPL x N float32 states (and A * log2 e) in VGPRs for the whole time range it walks.  B_t and
// C_t are the same for all channels of a batch row: they are staged through LDS as float32 and
// read back with wave-uniform (broadcast) loads.  The recurrence is elementwise: 4 VALU
// operations and one hardware exp2 per state update, no matrix product anywhere, and it is this
// instruction stream (the exp2 issues at half the FMA rate), not HBM, that bounds it.
//
// Time chunking.  A batch row offers only D / (64 CPL) wavefronts, far fewer than the 1024
// SIMDs of the chip, so long sequences are cut into n_chunks time chunks that run in parallel:
//   pass 1 (scan_chunk_state): every chunk but the last integrates from a zero state and
//       writes its local end state H_c and the sum of its deltas S_c;
//   carry (scan_carry): h_in[0] = h0, h_in[c+1] = exp(A S_c) h_in[c] + H_c, a short serial
//       loop per (d, n) (the decay over a whole chunk needs only S_c, not a product per step);
//   pass 2 (scan_chunk_out): every chunk runs the full recurrence from its true h_in[c].
// With one chunk only pass 2 runs, straight from h0.
#include <mutex>

#include "../../include/mamba_hip.h"
#include "device_math.h"
#include "launch.h"

// Chunk states of the allocation-free entry point (mamba_scan_fwd_static): device memory that comes with the code
// object, one copy per GPU at its own address, held until the process ends.
static __device__ __align__(256) unsigned char scratch[MAMBA_SCAN_STATIC_BYTES];

namespace mamba {
namespace {

constexpr int kWave = 64;
constexpr int kTile = 4;  // time steps whose token loads are issued together, one tile ahead

template <typename T, int CPL> struct RawT;
template <> struct RawT<float, 1> { typedef float type; };
template <> struct RawT<float, 2> { typedef float2 type; };
template <> struct RawT<bf16_t, 1> { typedef uint16_t type; };
template <> struct RawT<bf16_t, 2> { typedef uint32_t type; };

template <typename T, int CPL>
__device__ __forceinline__ typename RawT<T, CPL>::type ld_raw(const T *p)
{
    return *reinterpret_cast<const typename RawT<T, CPL>::type *>(p);
}

__device__ __forceinline__ void unpack(float r, float *v) { v[0] = r; }
__device__ __forceinline__ void unpack(float2 r, float *v) { v[0] = r.x; v[1] = r.y; }
__device__ __forceinline__ void unpack(uint16_t r, float *v) { v[0] = bf16_to_f32(r); }
__device__ __forceinline__ void unpack(uint32_t r, float *v) { v[0] = bf16_lo(r); v[1] = bf16_hi(r); }

template <int CPL> __device__ __forceinline__ void st_pack(float *p, const float *v)
{
    if constexpr (CPL == 1) p[0] = v[0];
    else *reinterpret_cast<float2 *>(p) = make_float2(v[0], v[1]);
}
template <int CPL> __device__ __forceinline__ void st_pack(bf16_t *p, const float *v)
{
    if constexpr (CPL == 1) p[0] = (bf16_t)f32_to_bf16(v[0]);
    else *reinterpret_cast<uint32_t *>(p) = f32x2_to_bf16x2(v[0], v[1]);
}

// B_t and C_t staged through LDS as float32: a tile of kBcTile time steps is fetched with
// coalesced vector loads one tile ahead, widened once, and written to one of two LDS buffers;
// every step then reads its N values with wave-uniform (broadcast) 16-byte LDS reads into
// VGPRs.  Compared with scalar loads this keeps SGPR operands (which issue slower) and the
// bf16 unpacking out of the inner loop.  NARR = 1 stages B only, 2 stages B and C.
// sched_barrier mask: scalar, memory and LDS instructions may still be moved across; vector ALU ones stay put
constexpr int kSchedMemoryOnly = 0x4 | 0x10 | 0x20 | 0x40 | 0x80 | 0x100 | 0x200;
constexpr int kBcTile = 16;
static_assert(kBcTile % kTile == 0, "B/C tiles must start on a token-tile boundary");

template <typename T, int N, int NARR> struct BcStage {
    static constexpr int kPerTile = kBcTile * N;                 // elements per array per tile
    static constexpr int kPerLane = (kPerTile + kWave - 1) / kWave;
    static constexpr int kBufFloats = NARR * kPerTile;
    float *lds;            // [2][NARR][kBcTile][N]
    const T *src[NARR];    // row base of this batch row
    int64_t last;          // index of the last valid element, t1 * N - 1
    float raw[NARR][kPerLane];

    __device__ __forceinline__ void issue(int64_t tile_t0)
    {
#pragma unroll
        for (int a = 0; a < NARR; ++a)
#pragma unroll
            for (int j = 0; j < kPerLane; ++j) {
                int64_t i = tile_t0 * N + (int)threadIdx.x + kWave * j;
                i = i < last ? i : last;   // steps past the chunk end are never used
                raw[a][j] = ld_io(src[a], i);
            }
    }
    __device__ __forceinline__ void commit(int buf)
    {
#pragma unroll
        for (int a = 0; a < NARR; ++a)
#pragma unroll
            for (int j = 0; j < kPerLane; ++j) {
                const int e = (int)threadIdx.x + kWave * j;
                if (kPerTile % kWave == 0 || e < kPerTile) lds[buf * kBufFloats + a * kPerTile + e] = raw[a][j];
            }
        __syncthreads();
    }
    // N values of array a for step s of buffer buf
    __device__ __forceinline__ void read(int buf, int a, int s, float *f) const
    {
        const float4 *p = reinterpret_cast<const float4 *>(lds + buf * kBufFloats + a * kPerTile + s * N);
#pragma unroll
        for (int q = 0; q < N / 4; ++q) {
            const float4 v = p[q];
            f[4 * q] = v.x; f[4 * q + 1] = v.y; f[4 * q + 2] = v.z; f[4 * q + 3] = v.w;
        }
    }
};

template <int N, int CPL> struct LaneState {
    float h[CPL][N];
    float a2[CPL][N];  // A * log2(e)
    float bias[CPL];
    float dskip[CPL];
};

template <int N, int CPL>
__device__ __forceinline__ void load_lane_params(LaneState<N, CPL> &s, const float *__restrict__ A,
                                                 const float *__restrict__ Dskip,
                                                 const float *__restrict__ dt_bias, int64_t d0)
{
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        const float4 *ap = reinterpret_cast<const float4 *>(A + (d0 + c) * N);
#pragma unroll
        for (int q = 0; q < N / 4; ++q) {
            const float4 v = ap[q];
            s.a2[c][4 * q + 0] = v.x * kLog2e;
            s.a2[c][4 * q + 1] = v.y * kLog2e;
            s.a2[c][4 * q + 2] = v.z * kLog2e;
            s.a2[c][4 * q + 3] = v.w * kLog2e;
        }
        s.bias[c] = dt_bias ? dt_bias[d0 + c] : 0.0f;
        s.dskip[c] = Dskip ? Dskip[d0 + c] : 0.0f;
    }
}

template <int N, int CPL>
__device__ __forceinline__ void load_state(float (&h)[CPL][N], const float *p /* (d0, 0) */)
{
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        const float4 *hp = reinterpret_cast<const float4 *>(p + c * N);
#pragma unroll
        for (int q = 0; q < N / 4; ++q) {
            const float4 v = hp[q];
            h[c][4 * q + 0] = v.x;
            h[c][4 * q + 1] = v.y;
            h[c][4 * q + 2] = v.z;
            h[c][4 * q + 3] = v.w;
        }
    }
}

template <int N, int CPL>
__device__ __forceinline__ void store_state(const float (&h)[CPL][N], float *p)
{
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        float4 *hp = reinterpret_cast<float4 *>(p + c * N);
#pragma unroll
        for (int q = 0; q < N / 4; ++q)
            hp[q] = make_float4(h[c][4 * q], h[c][4 * q + 1], h[c][4 * q + 2], h[c][4 * q + 3]);
    }
}

// ---------------------------------------------------------------------------------------
// pass 2 (and the only pass when n_chunks == 1): full recurrence with outputs
// grid: (channel groups, n_chunks, batch), block: one wavefront
template <typename T, int N, int CPL, bool HAS_Z, bool SOFTPLUS>
__global__ void __launch_bounds__(kWave)
scan_chunk_out(const T *__restrict__ x, const T *__restrict__ dt, const float *__restrict__ A,
               const T *__restrict__ Bm, const T *__restrict__ Cm, const float *__restrict__ Dskip,
               const T *__restrict__ z, const float *__restrict__ dt_bias,
               const float *h_start /* h0 (may be null, may alias h_final) or chunk states */,
               int h_start_chunked, T *__restrict__ out, float *h_final, int64_t L, int64_t D,
               int64_t chunk_len, int n_chunks)
{
    typedef typename RawT<T, CPL>::type raw_t;
    const int lane = threadIdx.x;
    const int64_t b = blockIdx.z;
    const int chunk = blockIdx.y;
    const int64_t d_lane = ((int64_t)blockIdx.x * kWave + lane) * CPL;
    const bool live = d_lane < D;                 // CPL == 2 only runs with D even
    const int64_t d0 = live ? d_lane : D - CPL;   // dead lanes shadow the last channels, store nothing
    const int64_t t0 = (int64_t)chunk * chunk_len;
    const int64_t t1 = (t0 + chunk_len < L) ? t0 + chunk_len : L;

    LaneState<N, CPL> s;
    load_lane_params<N, CPL>(s, A, Dskip, dt_bias, d0);
    if (h_start_chunked) {
        load_state<N, CPL>(s.h, h_start + (((int64_t)b * n_chunks + chunk) * D + d0) * N);
    } else if (h_start) {
        load_state<N, CPL>(s.h, h_start + (b * D + d0) * N);
    } else {
#pragma unroll
        for (int c = 0; c < CPL; ++c)
#pragma unroll
            for (int n = 0; n < N; ++n) s.h[c][n] = 0.0f;
    }

    const int64_t row0 = b * L;
    __shared__ __attribute__((aligned(16))) float lds_bc[2 * BcStage<T, N, 2>::kBufFloats];
    BcStage<T, N, 2> bc;
    bc.lds = lds_bc;
    bc.src[0] = Bm + row0 * N;
    bc.src[1] = Cm + row0 * N;
    bc.last = t1 * N - 1;
    bc.issue(t0);
    bc.commit(0);
    if (t0 + kBcTile < t1) bc.issue(t0 + kBcTile);
    // at the first step of every later B/C tile: publish the prefetched tile, fetch the one after
    auto bc_advance = [&](int64_t t) {
        const int rel = (int)(t - t0);
        if ((rel & (kBcTile - 1)) == 0 && rel != 0) {
            bc.commit((rel / kBcTile) & 1);
            if (t + kBcTile < t1) bc.issue(t + kBcTile);
        }
    };
    auto step = [&](int64_t t, raw_t xr, raw_t dr, raw_t zr) {
        const int rel = (int)(t - t0);
        const int buf = (rel / kBcTile) & 1, sidx = rel & (kBcTile - 1);
        float bf[N], cf[N];
        bc.read(buf, 0, sidx, bf);
        bc.read(buf, 1, sidx, cf);
        float xv[CPL], dv[CPL], zv[CPL], ov[CPL];
        unpack(xr, xv);
        unpack(dr, dv);
        if constexpr (HAS_Z) unpack(zr, zv);
#pragma unroll
        for (int c = 0; c < CPL; ++c) {
            const float v = dv[c] + s.bias[c];
            const float delta = SOFTPLUS ? softplus_f32(v) : v;
            const float u = delta * xv[c];
            float y = s.dskip[c] * xv[c];
            // The exponentials of a channel's states are issued as one run, the plain instructions around them
            // as runs of their own: exp2 next to exp2 issues at its own rate, exp2 scattered among multiplies
            // costs every neighbour extra (a bare loop of this update: 22 cycles per update in runs of 16, 25 to
            // 28 interleaved, which is what the compiler's scheduler produces when left alone).
            float a[N];
#pragma unroll
            for (int n = 0; n < N; ++n) a[n] = delta * s.a2[c][n];
            __builtin_amdgcn_sched_barrier(kSchedMemoryOnly);
#pragma unroll
            for (int n = 0; n < N; ++n) a[n] = exp2_hw(a[n]);
            __builtin_amdgcn_sched_barrier(kSchedMemoryOnly);
#pragma unroll
            for (int n = 0; n < N; ++n) {
                s.h[c][n] = fmaf(a[n], s.h[c][n], u * bf[n]);
                y = fmaf(s.h[c][n], cf[n], y);
            }
            ov[c] = HAS_Z ? y * silu_f32(zv[c]) : y;
        }
        if (live) st_pack<CPL>(out + (row0 + t) * D + d0, ov);
    };

    raw_t xc[kTile], dc[kTile], zc[kTile];
    auto load_tile = [&](int64_t t, raw_t *xa, raw_t *da, raw_t *za) {
#pragma unroll
        for (int i = 0; i < kTile; ++i) {
            const int64_t o = (row0 + t + i) * D + d0;
            xa[i] = ld_raw<T, CPL>(x + o);
            da[i] = ld_raw<T, CPL>(dt + o);
            if constexpr (HAS_Z) za[i] = ld_raw<T, CPL>(z + o);
        }
    };
    int64_t t = t0;
    if (t + kTile <= t1) load_tile(t, xc, dc, zc);
#pragma nounroll
    for (; t + kTile <= t1; t += kTile) {
        raw_t xn[kTile], dn[kTile], zn[kTile];
        const bool more = t + 2 * kTile <= t1;
        if (more) load_tile(t + kTile, xn, dn, zn);
        bc_advance(t);
#pragma unroll
        for (int i = 0; i < kTile; ++i) step(t + i, xc[i], dc[i], zc[i]);
        if (more) {
#pragma unroll
            for (int i = 0; i < kTile; ++i) {
                xc[i] = xn[i];
                dc[i] = dn[i];
                if constexpr (HAS_Z) zc[i] = zn[i];
            }
        }
    }
#pragma nounroll
    for (; t < t1; ++t) {
        const int64_t o = (row0 + t) * D + d0;
        raw_t zr = raw_t();
        if constexpr (HAS_Z) zr = ld_raw<T, CPL>(z + o);
        bc_advance(t);
        step(t, ld_raw<T, CPL>(x + o), ld_raw<T, CPL>(dt + o), zr);
    }

    if (h_final && chunk == n_chunks - 1 && live) store_state<N, CPL>(s.h, h_final + (b * D + d0) * N);
}

// ---------------------------------------------------------------------------------------
// pass 1: local end state of a chunk from a zero state, and the sum of its deltas
// grid: (channel groups, n_chunks - 1, batch); chunk c writes slot c + 1 of ws_state
template <typename T, int N, int CPL, bool SOFTPLUS>
__global__ void __launch_bounds__(kWave)
scan_chunk_state(const T *__restrict__ x, const T *__restrict__ dt, const float *__restrict__ A,
                 const T *__restrict__ Bm, const float *__restrict__ dt_bias,
                 float *__restrict__ ws_state, float *__restrict__ ws_sumdt, int64_t L, int64_t D,
                 int64_t chunk_len, int n_chunks)
{
    typedef typename RawT<T, CPL>::type raw_t;
    const int lane = threadIdx.x;
    const int64_t b = blockIdx.z;
    const int chunk = blockIdx.y;
    const int64_t d_lane = ((int64_t)blockIdx.x * kWave + lane) * CPL;
    const bool live = d_lane < D;
    const int64_t d0 = live ? d_lane : D - CPL;
    const int64_t t0 = (int64_t)chunk * chunk_len;
    const int64_t t1 = t0 + chunk_len;  // never the last chunk, so t1 <= L

    LaneState<N, CPL> s;
    load_lane_params<N, CPL>(s, A, nullptr, dt_bias, d0);
    float sum[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        sum[c] = 0.0f;
#pragma unroll
        for (int n = 0; n < N; ++n) s.h[c][n] = 0.0f;
    }

    const int64_t row0 = b * L;
    __shared__ __attribute__((aligned(16))) float lds_bc[2 * BcStage<T, N, 1>::kBufFloats];
    BcStage<T, N, 1> bc;
    bc.lds = lds_bc;
    bc.src[0] = Bm + row0 * N;
    bc.last = t1 * N - 1;
    bc.issue(t0);
    bc.commit(0);
    if (t0 + kBcTile < t1) bc.issue(t0 + kBcTile);
    auto bc_advance = [&](int64_t t) {
        const int rel = (int)(t - t0);
        if ((rel & (kBcTile - 1)) == 0 && rel != 0) {
            bc.commit((rel / kBcTile) & 1);
            if (t + kBcTile < t1) bc.issue(t + kBcTile);
        }
    };
    auto step = [&](int64_t t, raw_t xr, raw_t dr) {
        const int rel = (int)(t - t0);
        float bf[N];
        bc.read((rel / kBcTile) & 1, 0, rel & (kBcTile - 1), bf);
        float xv[CPL], dv[CPL];
        unpack(xr, xv);
        unpack(dr, dv);
#pragma unroll
        for (int c = 0; c < CPL; ++c) {
            const float v = dv[c] + s.bias[c];
            const float delta = SOFTPLUS ? softplus_f32(v) : v;
            const float u = delta * xv[c];
            sum[c] += delta;
            // exponentials as one run per channel (see pass 2)
            float a[N];
#pragma unroll
            for (int n = 0; n < N; ++n) a[n] = delta * s.a2[c][n];
            __builtin_amdgcn_sched_barrier(kSchedMemoryOnly);
#pragma unroll
            for (int n = 0; n < N; ++n) a[n] = exp2_hw(a[n]);
            __builtin_amdgcn_sched_barrier(kSchedMemoryOnly);
#pragma unroll
            for (int n = 0; n < N; ++n) s.h[c][n] = fmaf(a[n], s.h[c][n], u * bf[n]);
        }
    };

    raw_t xc[kTile], dc[kTile];
    auto load_tile = [&](int64_t t, raw_t *xa, raw_t *da) {
#pragma unroll
        for (int i = 0; i < kTile; ++i) {
            const int64_t o = (row0 + t + i) * D + d0;
            xa[i] = ld_raw<T, CPL>(x + o);
            da[i] = ld_raw<T, CPL>(dt + o);
        }
    };
    int64_t t = t0;
    if (t + kTile <= t1) load_tile(t, xc, dc);
#pragma nounroll
    for (; t + kTile <= t1; t += kTile) {
        raw_t xn[kTile], dn[kTile];
        const bool more = t + 2 * kTile <= t1;
        if (more) load_tile(t + kTile, xn, dn);
        bc_advance(t);
#pragma unroll
        for (int i = 0; i < kTile; ++i) step(t + i, xc[i], dc[i]);
        if (more) {
#pragma unroll
            for (int i = 0; i < kTile; ++i) {
                xc[i] = xn[i];
                dc[i] = dn[i];
            }
        }
    }
#pragma nounroll
    for (; t < t1; ++t) {
        const int64_t o = (row0 + t) * D + d0;
        bc_advance(t);
        step(t, ld_raw<T, CPL>(x + o), ld_raw<T, CPL>(dt + o));
    }

    if (live) {
        const int64_t slot = (int64_t)b * n_chunks + chunk;
        store_state<N, CPL>(s.h, ws_state + ((slot + 1) * D + d0) * N);
#pragma unroll
        for (int c = 0; c < CPL; ++c) ws_sumdt[slot * D + d0 + c] = sum[c];
    }
}

// ---------------------------------------------------------------------------------------
// carry: slot 0 <- h0; slot c <- exp(A S_{c-1}) slot_{c-1} + slot_c for c = 1 .. n_chunks - 1.
// The chain over chunks is serial per (b, d, n) and each link waits on a load, so it is cut into
// kCarrySegs segments that run side by side in one workgroup: every segment first folds its own
// chunks from a zero state (composite decay exp(A * sum S) and offset), the composites are
// exchanged through LDS, each segment derives its incoming state from the segments before it,
// and then walks its chunks again writing the true states.  block: (64 lanes over (b,d,n), segs)
constexpr int kCarrySegs = 8;
constexpr int kCarryBatch = 8;  // loads issued together

template <bool WRITE>
__device__ __forceinline__ float carry_walk(float h, float a2, float *st, const float *sd, int c0, int c1,
                                            int64_t DN, int64_t D)
{
    int c = c0;
    for (; c + kCarryBatch <= c1; c += kCarryBatch) {
        float loc[kCarryBatch], sm[kCarryBatch];
#pragma unroll
        for (int i = 0; i < kCarryBatch; ++i) {
            loc[i] = st[(int64_t)(c + i) * DN];
            sm[i] = sd[(int64_t)(c + i - 1) * D];
        }
#pragma unroll
        for (int i = 0; i < kCarryBatch; ++i) {
            h = fmaf(exp2_hw(a2 * sm[i]), h, loc[i]);
            if (WRITE) st[(int64_t)(c + i) * DN] = h;
        }
    }
    for (; c < c1; ++c) {
        h = fmaf(exp2_hw(a2 * sd[(int64_t)(c - 1) * D]), h, st[(int64_t)c * DN]);
        if (WRITE) st[(int64_t)c * DN] = h;
    }
    return h;
}

__global__ void __launch_bounds__(kWave * kCarrySegs)
scan_carry(const float *__restrict__ A, const float *h0, float *ws_state,
           const float *__restrict__ ws_sumdt, int64_t batch, int64_t D, int N, int n_chunks)
{
    __shared__ float decay[kCarrySegs][kWave], offset[kCarrySegs][kWave];
    const int lane = threadIdx.x, seg = threadIdx.y;
    const int64_t DN = D * N;
    const int64_t idx_raw = (int64_t)blockIdx.x * kWave + lane;
    const bool live = idx_raw < batch * DN;
    const int64_t idx = live ? idx_raw : batch * DN - 1;
    const int64_t b = idx / DN;
    const int64_t dn = idx - b * DN;
    const int64_t d = dn / N;
    const float a2 = A[dn] * kLog2e;
    float *st = ws_state + b * n_chunks * DN + dn;
    const float *sd = ws_sumdt + b * n_chunks * D + d;
    // chunks 1 .. n_chunks-1 split evenly over the segments
    const int per = (n_chunks - 1 + kCarrySegs - 1) / kCarrySegs;
    int c0 = 1 + seg * per, c1 = c0 + per;
    if (c0 > n_chunks) c0 = n_chunks;
    if (c1 > n_chunks) c1 = n_chunks;

    float sum = 0.0f;
    for (int c = c0; c < c1; ++c) sum += sd[(int64_t)(c - 1) * D];
    decay[seg][lane] = exp2_hw(a2 * sum);
    offset[seg][lane] = carry_walk<false>(0.0f, a2, st, sd, c0, c1, DN, D);
    __syncthreads();
    float h = h0 ? h0[idx] : 0.0f;
    for (int s = 0; s < seg; ++s) h = fmaf(decay[s][lane], h, offset[s][lane]);
    if (!live) return;
    if (seg == 0) st[0] = h;
    carry_walk<true>(h, a2, st, sd, c0, c1, DN, D);
}

// The same carry for up to kFastSegs * PER links with a single trip to memory: 16 segments of at most PER
// chunks; a lane owns VEC adjacent states of one channel (N % 4 == 0), fetches all local states and delta sums
// of its segment at once (8- or 16-byte loads, 512 B or 1 KiB per wavefront and chunk), folds them in registers,
// and after the exchange walks the registers again, so the second walk loads nothing.  <4, 8> serves up to 128
// links, <2, 16> up to 256 (both hold 32 state registers per lane).
// block: (64 lanes over (b, d, n / VEC), 16 segments)
constexpr int kFastSegs = 16;

template <int VEC, int PER>
__global__ void __launch_bounds__(kWave * kFastSegs)
scan_carry_fast(const float *__restrict__ A, const float *h0, float *ws_state,
                const float *__restrict__ ws_sumdt, int64_t batch, int64_t D, int N, int n_chunks)
{
    typedef float vec_t __attribute__((ext_vector_type(VEC)));
    __shared__ vec_t decay[kFastSegs][kWave], offset[kFastSegs][kWave];
    const int lane = threadIdx.x, seg = threadIdx.y;
    const int64_t DNV = D * N / VEC;
    const int64_t idx_raw = (int64_t)blockIdx.x * kWave + lane;
    const bool live = idx_raw < batch * DNV;
    const int64_t idx = live ? idx_raw : batch * DNV - 1;
    const int64_t b = idx / DNV;
    const int64_t dnv = idx - b * DNV;
    const int64_t d = dnv / (N / VEC);
    const vec_t a2 = reinterpret_cast<const vec_t *>(A)[dnv] * kLog2e;
    vec_t *st = reinterpret_cast<vec_t *>(ws_state) + b * n_chunks * DNV + dnv;
    const float *sd = ws_sumdt + b * n_chunks * D + d;
    const int per = (n_chunks - 1 + kFastSegs - 1) / kFastSegs;   // <= PER, checked by the launcher
    int c0 = 1 + seg * per, c1 = c0 + per;
    if (c0 > n_chunks) c0 = n_chunks;
    if (c1 > n_chunks) c1 = n_chunks;

    vec_t loc[PER];
    float e[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const bool in = c0 + i < c1;
        loc[i] = in ? st[(int64_t)(c0 + i) * DNV] : vec_t(0.0f);
        e[i] = in ? sd[(int64_t)(c0 + i - 1) * D] : 0.0f;         // delta sum of the chunk before; 0 for the unused tail
    }
    auto step = [&](vec_t h, int i) __attribute__((always_inline)) {
        // decay 1 for the unused tail (delta sum 0), with loc 0: no effect
#pragma unroll
        for (int v = 0; v < VEC; ++v) h[v] = fmaf(exp2_hw(a2[v] * e[i]), h[v], loc[i][v]);
        return h;
    };
    float sum = 0.0f;
    vec_t h = vec_t(0.0f);
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        sum += e[i];
        h = step(h, i);
    }
    vec_t dc;
#pragma unroll
    for (int v = 0; v < VEC; ++v) dc[v] = exp2_hw(a2[v] * sum);
    decay[seg][lane] = dc;
    offset[seg][lane] = h;
    __syncthreads();
    h = h0 ? reinterpret_cast<const vec_t *>(h0)[idx] : vec_t(0.0f);
    for (int s = 0; s < seg; ++s) {
        const vec_t ds = decay[s][lane], of = offset[s][lane];
#pragma unroll
        for (int v = 0; v < VEC; ++v) h[v] = fmaf(ds[v], h[v], of[v]);
    }
    if (!live) return;
    if (seg == 0) st[0] = h;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        h = step(h, i);
        if (c0 + i < c1) st[(int64_t)(c0 + i) * DNV] = h;
    }
}

// Few slots (the segment states of the scalar-decay scan, or a short selective scan): one lane per (b, d, n)
// walks them all; every load is issued before the first is used.  grid: ceil(batch * D * N / 256)
constexpr int kSerialSlots = 32;

__global__ void __launch_bounds__(256)
scan_carry_serial(const float *__restrict__ A, const float *h0, float *ws_state, const float *__restrict__ ws_sumdt,
                  int64_t batch, int64_t D, int N, int n_chunks)
{
    const int64_t DN = D * N;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= batch * DN) return;
    const int64_t b = idx / DN, dn = idx - b * DN, d = dn / N;
    const float a2 = A[dn] * kLog2e;
    float *st = ws_state + b * n_chunks * DN + dn;
    const float *sd = ws_sumdt + b * n_chunks * D + d;
    float loc[kSerialSlots], sm[kSerialSlots];
#pragma unroll
    for (int c = 1; c < kSerialSlots; ++c) {
        const bool in = c < n_chunks;
        loc[c] = in ? st[(int64_t)c * DN] : 0.0f;
        sm[c] = in ? sd[(int64_t)(c - 1) * D] : 0.0f;
    }
    float h = h0 ? h0[idx] : 0.0f;
    st[0] = h;
#pragma unroll
    for (int c = 1; c < kSerialSlots; ++c) {
        h = fmaf(exp2_hw(a2 * sm[c]), h, loc[c]);
        if (c < n_chunks) st[(int64_t)c * DN] = h;
    }
}

// launches the carry over the chunk states
inline void launch_carry(const ScanArgs &a, int N, int nc, float *ws_state, const float *ws_sumdt, hipStream_t stream)
{
    (void)launch_chunk_carry(a.A, a.h0, ws_state, ws_sumdt, a.batch, a.D, N, nc, stream);
}

// copies h0 (or zeros) to h_final when L == 0
__global__ void copy_state(const float *h0, float *h_final, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) h_final[i] = h0 ? h0[i] : 0.0f;
}

template <typename T, int N, int CPL>
hipError_t launch_scan_t(const ScanArgs &a, hipStream_t stream)
{
    const T *x = static_cast<const T *>(a.x), *dt = static_cast<const T *>(a.dt);
    const T *Bm = static_cast<const T *>(a.Bm), *Cm = static_cast<const T *>(a.Cm);
    const T *z = static_cast<const T *>(a.z);
    T *out = static_cast<T *>(a.out);
    const unsigned groups = (unsigned)((a.D + kWave * CPL - 1) / (kWave * CPL));
    const int nc = (int)a.n_chunks;
    const float *h_start = a.h0;
    int chunked = 0;
    if (nc > 1) {
        float *ws_state = a.ws;
        float *ws_sumdt = a.ws + (size_t)a.batch * nc * a.D * N;
        dim3 g1(groups, nc - 1, (unsigned)a.batch);
        if (a.dt_softplus)
            scan_chunk_state<T, N, CPL, true><<<g1, kWave, 0, stream>>>(
                x, dt, a.A, Bm, a.dt_bias, ws_state, ws_sumdt, a.L, a.D, a.chunk_len, nc);
        else
            scan_chunk_state<T, N, CPL, false><<<g1, kWave, 0, stream>>>(
                x, dt, a.A, Bm, a.dt_bias, ws_state, ws_sumdt, a.L, a.D, a.chunk_len, nc);
        launch_carry(a, N, nc, ws_state, ws_sumdt, stream);
        h_start = ws_state;
        chunked = 1;
    }
    dim3 g2(groups, nc, (unsigned)a.batch);
#define MAMBA_LAUNCH_OUT(HZ, SP)                                                                  \
    scan_chunk_out<T, N, CPL, HZ, SP><<<g2, kWave, 0, stream>>>(                                  \
        x, dt, a.A, Bm, Cm, a.Dskip, z, a.dt_bias, h_start, chunked, out, a.h_final, a.L, a.D,    \
        a.chunk_len, nc)
    if (z) {
        if (a.dt_softplus) MAMBA_LAUNCH_OUT(true, true);
        else MAMBA_LAUNCH_OUT(true, false);
    } else {
        if (a.dt_softplus) MAMBA_LAUNCH_OUT(false, true);
        else MAMBA_LAUNCH_OUT(false, false);
    }
#undef MAMBA_LAUNCH_OUT
    return hipGetLastError();
}

// Channels per lane.  Two halve the instruction overhead per state update, but also the number of
// wavefronts and double every wavefront's serial walk, so they pay only when there is work for
// several wavefronts per SIMD even so (measured: from about 2^25 channel-tokens on).  Two channels
// per lane need even D so that every row keeps the pair's alignment.
int scan_channels_per_lane(int64_t batch, int64_t L, int64_t D)
{
    if (D % 2 != 0) return 1;
    const double work = (double)batch * (double)L * (double)D;
    return work >= 33554432.0 ? 2 : 1;
}

template <typename T, int N>
hipError_t launch_scan_n(const ScanArgs &a, hipStream_t stream)
{
    if (scan_channels_per_lane(a.batch, a.L, a.D) == 2) return launch_scan_t<T, N, 2>(a, stream);
    return launch_scan_t<T, N, 1>(a, stream);
}

template <typename T> hipError_t launch_scan_io(const ScanArgs &a, hipStream_t stream)
{
    switch (a.N) {
    case 4: return launch_scan_n<T, 4>(a, stream);
    case 8: return launch_scan_n<T, 8>(a, stream);
    case 16: return launch_scan_n<T, 16>(a, stream);
    case 32: return launch_scan_n<T, 32>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_chunk_carry(const float *A, const float *h0, float *ws_state, const float *ws_sumdt, int64_t batch,
                              int64_t D, int N, int n_slots, hipStream_t stream)
{
    const int64_t total = batch * D * N;
    const unsigned blocks = (unsigned)((total + kWave - 1) / kWave);
    if (n_slots <= kSerialSlots)
        scan_carry_serial<<<(unsigned)((total + 255) / 256), 256, 0, stream>>>(A, h0, ws_state, ws_sumdt, batch, D, N, n_slots);
    else if (n_slots - 1 <= kFastSegs * 8)
        scan_carry_fast<4, 8><<<(unsigned)((total / 4 + kWave - 1) / kWave), dim3(kWave, kFastSegs), 0, stream>>>(A, h0, ws_state, ws_sumdt, batch, D, N, n_slots);
    else if (n_slots - 1 <= kFastSegs * 16)
        scan_carry_fast<2, 16><<<(unsigned)((total / 2 + kWave - 1) / kWave), dim3(kWave, kFastSegs), 0, stream>>>(A, h0, ws_state, ws_sumdt, batch, D, N, n_slots);
    else
        scan_carry<<<blocks, dim3(kWave, kCarrySegs), 0, stream>>>(A, h0, ws_state, ws_sumdt, batch, D, N, n_slots);
    return hipGetLastError();
}

hipError_t launch_copy_state(const float *src, float *dst, int64_t n, hipStream_t stream)
{
    copy_state<<<(unsigned)((n + 255) / 256), 256, 0, stream>>>(src, dst, n);
    return hipGetLastError();
}

// Chunking policy.  A wavefront column covers 64 * CPL channels of one batch row; the chip has
// 256 CUs x 4 SIMDs.  Sequences are cut only as far as needed to put about two wavefronts on
// every SIMD, because every extra chunk costs a second walk over its tokens (pass 1).
void scan_plan(int64_t batch, int64_t L, int64_t D, int64_t N, int64_t chunk_len_req,
               int64_t *chunk_len, int64_t *n_chunks)
{
    if (L <= 0 || batch <= 0 || D <= 0) {
        *chunk_len = L > 0 ? L : 1;
        *n_chunks = 1;
        return;
    }
    int64_t cl;
    if (chunk_len_req > 0) {
        cl = chunk_len_req;
    } else if (scan_kernel_choice(batch, L, D, N) != kScanChunked) {
        cl = L;  // one of the single-pass kernels: no chunks
    } else {
        const int64_t cpl = scan_channels_per_lane(batch, L, D);
        const int64_t columns = batch * ((D + kWave * cpl - 1) / (kWave * cpl));
        const int64_t target_waves = 3072;  // 3 resident wavefronts on each of 1024 SIMDs
        if (columns >= target_waves) {
            cl = L;
        } else {
            const int64_t want = (target_waves + columns - 1) / columns;
            cl = (L + want - 1) / want;
            if (cl > 256) cl = 256;  // short chunks balance better across the chip
            const int64_t shortest = cpl == 2 ? 32 : 16;
            if (cl < shortest) cl = shortest;  // long enough to amortize the chunk prologue and carry
            cl = (cl + kTile - 1) / kTile * kTile;
        }
    }
    if (cl > L) cl = L;
    // the chunk index is a grid dimension: the library's own choice never asks for more chunks than that allows
    if (chunk_len_req <= 0 && (L + cl - 1) / cl > 65535) cl = ((L + 65534) / 65535 + kTile - 1) / kTile * kTile;
    *chunk_len = cl;
    *n_chunks = (L + cl - 1) / cl;
}

int scan_kernel_choice(int64_t batch, int64_t L, int64_t D, int64_t N)
{
    if (scan_direct_applies(batch, L, D, N)) return kScanDirect;
    if (scan_lanes_applies(batch, L, D, N)) return kScanLanes;
    return kScanChunked;
}

size_t scan_workspace_bytes(int64_t batch, int64_t D, int64_t N, int64_t n_chunks)
{
    if (n_chunks <= 1) return 0;
    return (size_t)batch * (size_t)n_chunks * (size_t)D * (size_t)(N + 1) * sizeof(float);
}

// ---------------------------------------------------------------------------------------
// Address of the allocation-free entry point's chunk-state buffer (file scope, top of this file) on the current
// device.  In host code the array's name only stands for the symbol: the address comes from hipGetSymbolAddress,
// once per device with that device current, and only that pointer is ever handed to kernels.
hipError_t scan_static_scratch(float **ptr)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void *per_device[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!per_device[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(::scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        per_device[dev] = p;
    }
    *ptr = static_cast<float *>(per_device[dev]);
    return hipSuccess;
}

hipError_t launch_scan(const ScanArgs &a, hipStream_t stream)
{
    if (a.L == 0) {
        if (a.h_final && a.h_final != a.h0) {
            const int64_t n = a.batch * a.D * a.N;
            copy_state<<<(unsigned)((n + 255) / 256), 256, 0, stream>>>(a.h0, a.h_final, n);
            return hipGetLastError();
        }
        return hipSuccess;
    }
    if (a.single_pass == kScanDirect) return launch_scan_direct(a, stream);
    if (a.single_pass == kScanLanes) return launch_scan_lanes(a, stream);
    if (a.io == kIoBf16) return launch_scan_io<bf16_t>(a, stream);
    return launch_scan_io<float>(a, stream);
}

}  // namespace mamba
