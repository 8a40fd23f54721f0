// Scalar-decay (Mamba-2 style, "state-space dual") layer core for gfx950.  The paper names Mamba-2 as a
// drafter its method carries over to (Sec. 1); the layer is the SSD layer of Dao & Gu (2024):
//
//   delta[t,h] = softplus(dt[t,h] + dt_bias[h])
//   H_t[h] = exp(delta[t,h] A[h]) H_{t-1}[h] + delta[t,h] x_t[h,:] (outer) B_t        (P x N per head)
//   y_t[h,:] = H_t[h] C_t + D[h] x_t[h,:];  out = y silu(z)
//
// One decay per head and step makes the layer a sum of dense contractions over chunks of 64 steps,
// so unlike the selective scan this one runs on the matrix cores (v_mfma_f32_32x32x16_bf16).  With
// s_t the running sum of delta A inside a chunk (s_t <= 0) and H the state at the start of the chunk:
//   outputs G[t,s]  = C_t . B_s;  M[t,s] = G[t,s] exp(s_t - s_s) delta_s for s <= t, else 0
//           y_t[p]  = sum_s M[t,s] x_s[p] + exp(s_t) (C_t . H[p,:]) + D x_t[p]
//   state   H      <- exp(s_end) H + S,   S[p,n] = sum_s exp(s_end - s_s) delta_s x_s[p] B_s[n]
// A workgroup of four wavefronts walks the chunks of one segment of a (batch row, head) in order and
// keeps H (P x N float32) in MFMA accumulators, so chunk states never travel through memory; the
// sequence is cut into segments only to fill the chip, and as in the selective scan a first pass
// gives every segment's end state from zero, the carry kernel stitches them, and a second pass
// walks the segments again from their true incoming state and writes the outputs.  Tiles enter
// LDS once per chunk (those whose contraction index is the slow one in memory, x and B over s,
// transposed) and are read as MFMA fragments (lane l: row l % 32, eight consecutive k from
// 8 (l / 32)).  Products run in bf16 with float32 accumulation; of
// every product one factor is an input as it stands (x, B, C) and the other (M, the weighted x of pass 1,
// the incoming state) is carried as two bf16 terms, the rounded value and the remainder, i.e. with about
// 16 significant bits: single rounding showed wherever large terms cancel (errors of 2^-9 of the terms,
// not of the result), which the bf16 I/O tolerance does not allow for.
#include "device_math.h"
#include "launch.h"

namespace mamba {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kLc = 64;       // chunk length
constexpr int kP = 64;        // head dimension
constexpr int kThreads = 256;

constexpr int kRowS = kLc + 8;    // LDS row of 64 bf16 (steps or channels) + 16 bytes of padding

__device__ __forceinline__ bf16x8 frag(const uint16_t *base, int row_stride, int row, int k0)
{
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(base + row * row_stride + k0));
}

// Tiles that are written transposed (a lane holds 8 consecutive rows of one column, lanes 8 rows apart)
// get 16 more bytes of padding after every 8 rows: with a plain row stride of 144 bytes rows 8 apart fall
// into the same LDS bank and the 2-byte writes of a wavefront serialize 16 ways.
__device__ __forceinline__ int trow(int row) { return row * kRowS + (row >> 3) * 8; }
constexpr int tsize(int rows) { return rows * kRowS + (rows / 8) * 8; }
__device__ __forceinline__ bf16x8 tfrag(const uint16_t *base, int row, int k0)
{
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(base + trow(row) + k0));
}

// value -> rounded bf16 and the bf16 of what the rounding dropped
__device__ __forceinline__ void split2(float v, uint16_t *top, uint16_t *rem)
{
    const uint32_t t = f32_to_bf16(v);
    *top = (uint16_t)t;
    *rem = (uint16_t)f32_to_bf16(v - bf16_to_f32(t));
}

// ---------------------------------------------------------------------------------------------------
// A workgroup walks the chunks of one segment of one (batch row, head) in order, the head's state
// (P x N float32) living in MFMA accumulators: per chunk acc <- exp(s_end) acc + S.
//   PASS2 = false: from a zero state; leaves the segment's end state in slot seg + 1 of ws_state
//       ((batch, n_seg + 1, H * P, N)) and the segment's sum of deltas in ws_sumdt; the carry kernel
//       of the selective scan then turns the slots into the states at the segment starts;
//   PASS2 = true: from the true incoming state (slot seg), with outputs.
// The raw tiles of the next chunk (x, B, C, z, dt) are fetched into registers while the current one
// is multiplied.  grid: (n_seg, H, batch), 4 wavefronts.
template <int N, bool PASS2, bool HAS_Z>
__global__ void __launch_bounds__(kThreads)
ssd_segment(const bf16_t *__restrict__ x, const bf16_t *__restrict__ dt, const float *__restrict__ A,
            const bf16_t *__restrict__ Bm, const bf16_t *__restrict__ Cm, const float *__restrict__ Dskip,
            const bf16_t *__restrict__ z, const float *__restrict__ dt_bias, float *__restrict__ ws_state,
            float *__restrict__ ws_sumdt, float *__restrict__ a_rows, bf16_t *__restrict__ out, float *h_final,
            int64_t L, int64_t H, int chunks_per_seg, int n_seg, int n_chunks, int softplus)
{
    constexpr int kRowN = N + 8;                              // LDS row of N bf16 + padding
    constexpr int NB = N / 32;                                // 16-byte chunks of a B / C tile per thread
    constexpr int PPW = (2 * (N / 32)) / 4;                   // state tiles (32 x 32) per wavefront: 2 p tiles x N / 32 n tiles
    __shared__ float delta[kLc], cum[kLc];
    __shared__ __attribute__((aligned(16))) uint16_t bt[tsize(N)];                       // B as [n][s]
    __shared__ __attribute__((aligned(16))) uint16_t xw_hi[tsize(kP)], xw_lo[tsize(kP)]; // weight_s x_s[p] as [p][s]
    __shared__ __attribute__((aligned(16))) uint16_t xt[PASS2 ? tsize(kP) : 8];          // x as [p][s]
    __shared__ __attribute__((aligned(16))) uint16_t zt[PASS2 ? kLc * kRowS : 8];         // z as [t][p]
    __shared__ __attribute__((aligned(16))) uint16_t c_rows[PASS2 ? kLc * kRowN : 8];     // C as [t][n]
    __shared__ __attribute__((aligned(16))) uint16_t b_rows[PASS2 ? kLc * kRowN : 8];     // B as [s][n]
    __shared__ __attribute__((aligned(16))) uint16_t mm_hi[PASS2 ? kLc * kRowS : 8], mm_lo[PASS2 ? kLc * kRowS : 8];
    __shared__ __attribute__((aligned(16))) uint16_t h_hi[PASS2 ? kP * kRowN : 8], h_lo[PASS2 ? kP * kRowN : 8];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int seg = blockIdx.x;
    const int64_t h = blockIdx.y, b = blockIdx.z;
    const int64_t row0 = b * L, D = H * kP;
    const float A_h = A[h], bias_h = dt_bias ? dt_bias[h] : 0.0f;
    const int r = lane & 31, hk = (lane >> 5) * 8;
    const int tt = wave >> 1, half = wave & 1;                // output block of this wavefront in pass 2
    const int c_first = seg * chunks_per_seg;
    const int c_last = min(c_first + chunks_per_seg, n_chunks);

    // raw tiles of one chunk, as this thread's 16-byte pieces
    struct Raw {
        uint4 x[2], z[2], bq[NB], cq[NB];
        float dt;
    };
    auto fetch = [&](int chunk) {
        Raw q;
        const int64_t tok0 = (int64_t)chunk * kLc;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int ch = tid + i * kThreads, s = ch >> 3, p0 = (ch & 7) * 8;
            const bool ok = tok0 + s < L;
            const int64_t o = ((row0 + tok0 + s) * H + h) * kP + p0;
            q.x[i] = ok ? *reinterpret_cast<const uint4 *>(x + o) : make_uint4(0, 0, 0, 0);
            q.z[i] = (PASS2 && HAS_Z && ok) ? *reinterpret_cast<const uint4 *>(z + o) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int ch = tid + i * kThreads, s = ch / (N / 8), n0 = (ch % (N / 8)) * 8;
            const bool ok = tok0 + s < L;
            const int64_t o = (row0 + tok0 + s) * N + n0;
            q.bq[i] = ok ? *reinterpret_cast<const uint4 *>(Bm + o) : make_uint4(0, 0, 0, 0);
            q.cq[i] = (PASS2 && ok) ? *reinterpret_cast<const uint4 *>(Cm + o) : make_uint4(0, 0, 0, 0);
        }
        q.dt = 0.0f;
        if (tid < kLc && tok0 + tid < L) q.dt = bf16_to_f32(dt[(row0 + tok0 + tid) * H + h]);
        return q;
    };

    // the head's state: tile j of this wavefront is (p tile pt, n tile nt); acc[j][i] is
    // H[p = 32 pt + 8 (i / 4) + 4 (lane / 32) + i % 4][n = 32 nt + lane % 32]
    f32x16 acc[PPW];
    float *slot_in = ws_state + (((int64_t)b * (n_seg + 1) + seg) * D + h * kP) * N;
#pragma unroll
    for (int j = 0; j < PPW; ++j) {
        const int pair = wave * PPW + j, pt = pair & 1, nt = pair >> 1;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int p = pt * 32 + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
            acc[j][i] = PASS2 ? slot_in[(int64_t)p * N + nt * 32 + r] : 0.0f;
        }
    }
    float seg_sum = 0.0f;
    if (!PASS2 && seg == 0 && b == 0)
        for (int i = tid; i < kP * N; i += kThreads) a_rows[h * kP * N + i] = A_h;   // decay matrix for the carry kernel

    Raw raw = fetch(c_first);
    for (int chunk = c_first; chunk < c_last; ++chunk) {
        const int64_t tok0 = (int64_t)chunk * kLc;
        // delta and the inclusive running sum of delta * A over the chunk (wavefront 0, one lane per step)
        if (wave == 0) {
            const float dl = (tok0 + lane < L) ? (softplus ? softplus_f32(raw.dt + bias_h) : raw.dt + bias_h) : 0.0f;
            float sc = dl * A_h;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const float o = __shfl_up(sc, off, 64);
                if (lane >= off) sc += o;
            }
            delta[lane] = dl;
            cum[lane] = sc;
            seg_sum += dl;
        }
        // raw B (and C, x, z in pass 2) into LDS
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int ch = tid + i * kThreads, s = ch / (N / 8), n0 = (ch % (N / 8)) * 8;
            const uint32_t w[4] = {raw.bq[i].x, raw.bq[i].y, raw.bq[i].z, raw.bq[i].w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                bt[trow(n0 + 2 * k) + s] = (uint16_t)(w[k] & 0xffffu);
                bt[trow(n0 + 2 * k + 1) + s] = (uint16_t)(w[k] >> 16);
            }
            if constexpr (PASS2) {
                *reinterpret_cast<uint4 *>(&b_rows[s * kRowN + n0]) = raw.bq[i];
                *reinterpret_cast<uint4 *>(&c_rows[s * kRowN + n0]) = raw.cq[i];
            }
        }
        if constexpr (PASS2) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int ch = tid + i * kThreads, s = ch >> 3, p0 = (ch & 7) * 8;
                const uint32_t w[4] = {raw.x[i].x, raw.x[i].y, raw.x[i].z, raw.x[i].w};
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    xt[trow(p0 + 2 * k) + s] = (uint16_t)(w[k] & 0xffffu);
                    xt[trow(p0 + 2 * k + 1) + s] = (uint16_t)(w[k] >> 16);
                }
                *reinterpret_cast<uint4 *>(&zt[s * kRowS + p0]) = raw.z[i];
            }
            // the state at the start of the chunk, as two bf16 terms, for the incoming-state product
#pragma unroll
            for (int j = 0; j < PPW; ++j) {
                const int pair = wave * PPW + j, pt = pair & 1, nt = pair >> 1;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int p = pt * 32 + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
                    split2(acc[j][i], &h_hi[p * kRowN + nt * 32 + r], &h_lo[p * kRowN + nt * 32 + r]);
                }
            }
        }
        __syncthreads();                                          // delta, cum and the raw tiles are in LDS
        // weighted x for the state update, two bf16 terms: weight_s = exp(s_end - s_s) delta_s
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int ch = tid + i * kThreads, s = ch >> 3, p0 = (ch & 7) * 8;
            const float w = exp2_hw((cum[kLc - 1] - cum[s]) * kLog2e) * delta[s];
            const uint4 q = raw.x[i];
            const float v[8] = {bf16_lo(q.x) * w, bf16_hi(q.x) * w, bf16_lo(q.y) * w, bf16_hi(q.y) * w,
                                bf16_lo(q.z) * w, bf16_hi(q.z) * w, bf16_lo(q.w) * w, bf16_hi(q.w) * w};
#pragma unroll
            for (int k = 0; k < 8; ++k) split2(v[k], &xw_hi[trow(p0 + k) + s], &xw_lo[trow(p0 + k) + s]);
        }
        if (chunk + 1 < c_last) raw = fetch(chunk + 1);           // in flight during the products below

        f32x16 gacc;
        if constexpr (PASS2) {
            // G block (t tile tt, s tile half); above the diagonal it is masked out entirely
#pragma unroll
            for (int i = 0; i < 16; ++i) gacc[i] = 0.0f;
            if (half <= tt) {
#pragma unroll
                for (int ks = 0; ks < N / 16; ++ks)
                    gacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(c_rows, kRowN, tt * 32 + r, ks * 16 + hk),
                                                                   frag(b_rows, kRowN, half * 32 + r, ks * 16 + hk), gacc, 0, 0, 0);
            }
            // M = G * exp(s_t - s_s) * delta_s for s <= t (steps past L have delta = 0)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int t = tt * 32 + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3), s = half * 32 + r;
                const float v = (s <= t) ? gacc[i] * exp2_hw((cum[t] - cum[s]) * kLog2e) * delta[s] : 0.0f;
                split2(v, &mm_hi[t * kRowS + s], &mm_lo[t * kRowS + s]);
            }
        }
        __syncthreads();                                          // M and the weighted x are in LDS

        if constexpr (PASS2) {
            f32x16 inter, intra;
#pragma unroll
            for (int i = 0; i < 16; ++i) inter[i] = intra[i] = 0.0f;
#pragma unroll
            for (int ks = 0; ks < N / 16; ++ks) {
                const bf16x8 cf = frag(c_rows, kRowN, tt * 32 + r, ks * 16 + hk);
                inter = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cf, frag(h_hi, kRowN, half * 32 + r, ks * 16 + hk), inter, 0, 0, 0);
                inter = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cf, frag(h_lo, kRowN, half * 32 + r, ks * 16 + hk), inter, 0, 0, 0);
            }
#pragma unroll
            for (int ks = 0; ks < kLc / 16; ++ks)
                if (ks < 2 * (tt + 1)) {                          // M is zero right of the diagonal block
                    const bf16x8 xf = tfrag(xt, half * 32 + r, ks * 16 + hk);
                    intra = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(mm_hi, kRowS, tt * 32 + r, ks * 16 + hk), xf, intra, 0, 0, 0);
                    intra = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(mm_lo, kRowS, tt * 32 + r, ks * 16 + hk), xf, intra, 0, 0, 0);
                }
            const float dsk = Dskip ? Dskip[h] : 0.0f;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int t = tt * 32 + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3), p = half * 32 + r;
                if (tok0 + t >= L) continue;
                float y = intra[i] + exp2_hw(cum[t] * kLog2e) * inter[i] + dsk * bf16_to_f32(xt[trow(p) + t]);
                if constexpr (HAS_Z) y *= silu_f32(bf16_to_f32(zt[t * kRowS + p]));
                out[((row0 + tok0 + t) * H + h) * kP + p] = (bf16_t)f32_to_bf16(y);
            }
        }
        // state: acc <- exp(s_end) acc + sum_s xw[p][s] bt[n][s]
        const float dec = exp2_hw(cum[kLc - 1] * kLog2e);
#pragma unroll
        for (int j = 0; j < PPW; ++j) {
            const int pair = wave * PPW + j, pt = pair & 1, nt = pair >> 1;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[j][i] *= dec;
#pragma unroll
            for (int ks = 0; ks < kLc / 16; ++ks) {
                const bf16x8 bf = tfrag(bt, nt * 32 + r, ks * 16 + hk);
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tfrag(xw_hi, pt * 32 + r, ks * 16 + hk), bf, acc[j], 0, 0, 0);
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tfrag(xw_lo, pt * 32 + r, ks * 16 + hk), bf, acc[j], 0, 0, 0);
            }
        }
        __syncthreads();                                          // the chunk's LDS tiles are free again
    }

    // end of the segment: pass 1 leaves the local end state and the sum of deltas, pass 2 the final state
    float *dst = nullptr;
    if (!PASS2) dst = ws_state + (((int64_t)b * (n_seg + 1) + seg + 1) * D + h * kP) * N;
    else if (h_final && seg == n_seg - 1) dst = h_final + (b * D + h * kP) * N;
    if (dst) {
#pragma unroll
        for (int j = 0; j < PPW; ++j) {
            const int pair = wave * PPW + j, pt = pair & 1, nt = pair >> 1;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int p = pt * 32 + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
                dst[(int64_t)p * N + nt * 32 + r] = acc[j][i];
            }
        }
    }
    if (!PASS2 && wave == 0) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) seg_sum += __shfl_xor(seg_sum, off, 64);
        ws_sumdt[((int64_t)b * (n_seg + 1) + seg) * D + h * kP + lane] = seg_sum;   // kP == 64 lanes
    }
}

// ---------------------------------------------------------------------------------------------------
// one step for every live draft branch (the counterpart of the selective state update): a lane owns a
// float4 of the branch's (H, P, N) state, the N / 4 lanes of a channel add their partial C.h.
// grid: (ceil(H * P * N / 4 / 256), n_out)
template <typename T, int N>
__global__ void __launch_bounds__(kThreads)
ssd_step_kernel(float *h_out, const float *h_in, const int32_t *__restrict__ parent, const T *__restrict__ x,
                const T *__restrict__ dt, const float *__restrict__ A, const T *__restrict__ Bm, const T *__restrict__ Cm,
                const float *__restrict__ Dskip, const T *__restrict__ z, const float *__restrict__ dt_bias,
                T *__restrict__ out, int64_t n_in, int64_t H, int P, int softplus)
{
    constexpr int Q = N / 4;                                     // lanes per channel: 16 or 32
    const int64_t j = blockIdx.y;
    const int64_t row4 = H * P * Q;
    const int64_t f_raw = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const bool live = f_raw < row4;
    const int64_t f = live ? f_raw : row4 - 1;
    const int64_t d = f / Q, hh = d / P;
    const int q = (int)(f - d * Q);
    float bq[4], cq[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        bq[i] = ld_io(Bm, j * N + 4 * q + i);
        cq[i] = ld_io(Cm, j * N + 4 * q + i);
    }
    const float xv = ld_io(x, j * H * P + d);
    const float v = ld_io(dt, j * H + hh) + (dt_bias ? dt_bias[hh] : 0.0f);
    const float delta = softplus ? softplus_f32(v) : v;
    const float a = exp2_hw(delta * A[hh] * kLog2e), u = delta * xv;
    const int64_t p = parent ? (int64_t)parent[j] : j;
    const bool p_ok = p >= 0 && p < n_in;
    float4 hv = reinterpret_cast<const float4 *>(h_in)[(p_ok ? p : 0) * row4 + f];
    hv.x = fmaf(a, hv.x, u * bq[0]);
    hv.y = fmaf(a, hv.y, u * bq[1]);
    hv.z = fmaf(a, hv.z, u * bq[2]);
    hv.w = fmaf(a, hv.w, u * bq[3]);
    float y = hv.x * cq[0];
    y = fmaf(hv.y, cq[1], y);
    y = fmaf(hv.z, cq[2], y);
    y = fmaf(hv.w, cq[3], y);
#pragma unroll
    for (int off = 1; off < Q; off <<= 1) y += __shfl_xor(y, off, 64);
    if (!p_ok) {
        const float nan = __int_as_float(0x7fc00000);
        hv = make_float4(nan, nan, nan, nan);
        y = nan;
    }
    if (!live) return;
    reinterpret_cast<float4 *>(h_out)[j * row4 + f] = hv;
    if (q == 0) {
        y = fmaf(Dskip ? Dskip[hh] : 0.0f, xv, y);
        if (z) y *= silu_f32(ld_io(z, j * H * P + d));
        st_io(out, j * H * P + d, y);
    }
}

int64_t chunks_of(int64_t L) { return (L + kLc - 1) / kLc; }

// Segments: about one workgroup per CU (a workgroup holds most of a CU's LDS), never more than chunks.
void ssd_plan(int64_t batch, int64_t L, int64_t H, int *chunks_per_seg, int *n_seg)
{
    const int64_t nc = chunks_of(L);
    int64_t want = 256 / (batch * H > 0 ? batch * H : 1);
    if (want < 1) want = 1;
    if (want > nc) want = nc;
    const int64_t cps = (nc + want - 1) / want;
    *chunks_per_seg = (int)cps;
    *n_seg = (int)((nc + cps - 1) / cps);
}

}  // namespace

size_t ssd_workspace_bytes(int64_t batch, int64_t L, int64_t H, int64_t P, int64_t N)
{
    int cps, n_seg;
    ssd_plan(batch, L, H, &cps, &n_seg);
    const int64_t slots = n_seg + 1, D = H * P;
    return (size_t)(batch * slots * D * (N + 1) + D * N) * sizeof(float);
}

hipError_t launch_ssd(const SsdArgs &a, hipStream_t stream)
{
    int cps, n_seg;
    ssd_plan(a.batch, a.L, a.H, &cps, &n_seg);
    const int nc = (int)chunks_of(a.L);
    const int64_t D = a.H * a.P;
    float *ws_state = a.ws;
    float *ws_sumdt = ws_state + (size_t)a.batch * (n_seg + 1) * D * a.N;
    float *a_rows = ws_sumdt + (size_t)a.batch * (n_seg + 1) * D;
    const bf16_t *x = static_cast<const bf16_t *>(a.x), *dt = static_cast<const bf16_t *>(a.dt);
    const bf16_t *Bm = static_cast<const bf16_t *>(a.Bm), *Cm = static_cast<const bf16_t *>(a.Cm);
    const bf16_t *z = static_cast<const bf16_t *>(a.z);
    bf16_t *out = static_cast<bf16_t *>(a.out);
    dim3 grid((unsigned)n_seg, (unsigned)a.H, (unsigned)a.batch);
#define MAMBA_SSD(NN, P2, HZ)                                                                                     \
    ssd_segment<NN, P2, HZ><<<grid, kThreads, 0, stream>>>(x, dt, a.A, Bm, Cm, a.Dskip, z, a.dt_bias, ws_state,    \
                                                          ws_sumdt, a_rows, out, a.h_final, a.L, a.H, cps, n_seg, \
                                                          nc, a.dt_softplus)
    if (n_seg > 1) {
        if (a.N == 64) MAMBA_SSD(64, false, false);
        else MAMBA_SSD(128, false, false);
        if (hipError_t e = launch_chunk_carry(a_rows, a.h0, ws_state, ws_sumdt, a.batch, D, a.N, n_seg + 1, stream)) return e;
    } else {
        // a single segment starts from h0 itself: slot 0 <- h0 (or zeros)
        for (int64_t b = 0; b < a.batch; ++b)
            if (hipError_t e = launch_copy_state(a.h0 ? a.h0 + b * D * a.N : nullptr, ws_state + (size_t)b * 2 * D * a.N, D * a.N, stream))
                return e;
    }
    if (a.N == 64) {
        if (z) MAMBA_SSD(64, true, true);
        else MAMBA_SSD(64, true, false);
    } else {
        if (z) MAMBA_SSD(128, true, true);
        else MAMBA_SSD(128, true, false);
    }
#undef MAMBA_SSD
    return hipGetLastError();
}

hipError_t launch_ssd_step(const SsdStepArgs &a, hipStream_t stream)
{
    const int64_t row4 = a.H * a.P * (a.N / 4);
    dim3 grid((unsigned)((row4 + kThreads - 1) / kThreads), (unsigned)a.n_out);
#define MAMBA_SSD_STEP(T, NN)                                                                                     \
    ssd_step_kernel<T, NN><<<grid, kThreads, 0, stream>>>(a.h_out, a.h_in, a.parent, static_cast<const T *>(a.x),  \
        static_cast<const T *>(a.dt), a.A, static_cast<const T *>(a.Bm), static_cast<const T *>(a.Cm), a.Dskip,   \
        static_cast<const T *>(a.z), a.dt_bias, static_cast<T *>(a.out), a.n_in, a.H, a.P, a.dt_softplus)
    if (a.io == kIoBf16) {
        if (a.N == 64) MAMBA_SSD_STEP(bf16_t, 64);
        else MAMBA_SSD_STEP(bf16_t, 128);
    } else {
        if (a.N == 64) MAMBA_SSD_STEP(float, 64);
        else MAMBA_SSD_STEP(float, 128);
    }
#undef MAMBA_SSD_STEP
    return hipGetLastError();
}

}  // namespace mamba
