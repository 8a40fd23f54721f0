// Scalar-decay (Mamba-2 style, "state-space dual") layer core for gfx950.  The paper names Mamba-2 as a
// drafter its method carries over to (Sec. 1); the layer is the SSD layer of Dao & Gu (2024):
//
//   delta[t,h] = softplus(dt[t,h] + dt_bias[h])
//   H_t[h] = exp(delta[t,h] A[h]) H_{t-1}[h] + delta[t,h] x_t[h,:] (outer) B_t        (P x N per head)
//   y_t[h,:] = H_t[h] C_t + D[h] x_t[h,:];  out = y silu(z)
//
// One decay per head and step makes the layer a sum of dense contractions over chunks of 64 steps,
// so unlike the selective scan this one runs on the matrix cores (v_mfma_f32_32x32x16_bf16).  With
// s_t the running sum of delta A inside a chunk (s_t <= 0):
//   pass 1  S[p,n]  = sum_s exp(s_end - s_s) delta_s x_s[p] B_s[n]            local end state of the chunk
//   carry   H_in[c+1] = exp(s_end) H_in[c] + S_c                              same kernel as the selective scan
//   pass 2  G[t,s]  = C_t . B_s;  M[t,s] = G[t,s] exp(s_t - s_s) delta_s for s <= t, else 0
//           y_t[p]  = sum_s M[t,s] x_s[p] + exp(s_t) (C_t . H_in[p,:]) + D x_t[p]
// A workgroup of four wavefronts owns one (batch row, head, chunk).  Operands whose contraction index
// is the slow one in memory (x and B over s) are transposed through LDS on the way in; C, B and the
// incoming state are read from global memory directly in MFMA fragment order (lane l: row l % 32,
// eight consecutive k starting at 8 (l / 32)).  Products run in bf16 with float32 accumulation; of
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
constexpr int kRowU16 = kLc + 8;   // LDS row of 64 bf16 + 16 bytes of padding

// delta, inclusive running sum of delta * A over the chunk (wavefront 0, one lane per step)
__device__ __forceinline__ void chunk_decay(const bf16_t *dt, const float *dt_bias, float A_h, int64_t tok0, int64_t L,
                                            int64_t H, int64_t h, int64_t row0, int softplus, float *delta_out,
                                            float *cum_out)
{
    const int t = threadIdx.x;                                   // < 64
    const int64_t tok = tok0 + t;
    float delta = 0.0f;
    if (tok < L) {
        const float v = bf16_to_f32(dt[(row0 + tok) * H + h]) + (dt_bias ? dt_bias[h] : 0.0f);
        delta = softplus ? softplus_f32(v) : v;
    }
    float s = delta * A_h;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const float o = __shfl_up(s, off, 64);
        if (t >= off) s += o;
    }
    delta_out[t] = delta;
    cum_out[t] = s;
}

// x tile (64 steps x 64 channels of one head), scaled per step when scale is given, to LDS as [channel][step] bf16;
// with xt_rem the scaled value is kept as two bf16 terms (rounded value and remainder)
__device__ __forceinline__ void stage_x_transposed(const bf16_t *x, int64_t row0, int64_t tok0, int64_t L, int64_t H,
                                                   int64_t h, const float *scale, uint16_t (*xt)[kRowU16],
                                                   uint16_t (*xt_rem)[kRowU16] = nullptr)
{
    for (int ch = threadIdx.x; ch < kLc * (kP / 8); ch += kThreads) {
        const int s = ch / (kP / 8), p0 = (ch % (kP / 8)) * 8;
        const int64_t tok = tok0 + s;
        uint4 r = make_uint4(0, 0, 0, 0);
        if (tok < L) r = *reinterpret_cast<const uint4 *>(x + ((row0 + tok) * H + h) * kP + p0);
        const float w = scale ? scale[s] : 1.0f;                 // times 1: the bits of x unchanged
        const float v[8] = {bf16_lo(r.x) * w, bf16_hi(r.x) * w, bf16_lo(r.y) * w, bf16_hi(r.y) * w,
                            bf16_lo(r.z) * w, bf16_hi(r.z) * w, bf16_lo(r.w) * w, bf16_hi(r.w) * w};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t top = f32_to_bf16(v[i]);
            xt[p0 + i][s] = (uint16_t)top;
            if (xt_rem) xt_rem[p0 + i][s] = (uint16_t)f32_to_bf16(v[i] - bf16_to_f32(top));   // what the rounding dropped
        }
    }
}

__device__ __forceinline__ bf16x8 lds_frag(const uint16_t (*m)[kRowU16], int row, int k0)
{
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(&m[row][k0]));
}

// ---------------------------------------------------------------------------------------------------
// pass 1.  grid: (n_chunks, H, batch).  Writes slot chunk + 1 of ws_state ((batch, n_chunks + 1, H * P, N)),
// entry chunk of ws_sumdt ((batch, n_chunks + 1, H * P), the sum of deltas repeated over the head's channels)
// and, from the first workgroups, the decay matrix the carry kernel expects (A[h] repeated, (H * P, N)).
template <int N>
__global__ void __launch_bounds__(kThreads)
ssd_chunk_state(const bf16_t *__restrict__ x, const bf16_t *__restrict__ dt, const float *__restrict__ A,
                const bf16_t *__restrict__ Bm, const float *__restrict__ dt_bias, float *__restrict__ ws_state,
                float *__restrict__ ws_sumdt, float *__restrict__ a_rows, int64_t L, int64_t H, int n_chunks, int softplus)
{
    __shared__ float delta[kLc], cum[kLc], weight[kLc];
    __shared__ __attribute__((aligned(16))) uint16_t xt[kP][kRowU16], xt_rem[kP][kRowU16];
    __shared__ __attribute__((aligned(16))) uint16_t bt[N][kRowU16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int chunk = blockIdx.x;
    const int64_t h = blockIdx.y, b = blockIdx.z;
    const int64_t row0 = b * L, tok0 = (int64_t)chunk * kLc, D = H * kP;
    const float A_h = A[h];

    if (wave == 0) chunk_decay(dt, dt_bias, A_h, tok0, L, H, h, row0, softplus, delta, cum);
    __syncthreads();
    if (tid < kLc) weight[tid] = exp2_hw((cum[kLc - 1] - cum[tid]) * kLog2e) * delta[tid];
    if (tid < kP) {
        // the sum of deltas: the carry kernel forms the chunk's decay as exp(A * sum)
        float sum = 0.0f;
        for (int t = 0; t < kLc; ++t) sum += delta[t];
        ws_sumdt[((int64_t)b * (n_chunks + 1) + chunk) * D + h * kP + tid] = sum;
    }
    if (chunk == 0 && b == 0)
        for (int i = tid; i < kP * N; i += kThreads) a_rows[h * kP * N + i] = A_h;
    __syncthreads();
    stage_x_transposed(x, row0, tok0, L, H, h, weight, xt, xt_rem);
    for (int ch = tid; ch < kLc * (N / 8); ch += kThreads) {     // B tile to LDS as [state][step]
        const int s = ch / (N / 8), n0 = (ch % (N / 8)) * 8;
        const int64_t tok = tok0 + s;
        uint4 r = make_uint4(0, 0, 0, 0);
        if (tok < L) r = *reinterpret_cast<const uint4 *>(Bm + (row0 + tok) * N + n0);
        const uint32_t q[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            bt[n0 + 2 * i][s] = (uint16_t)(q[i] & 0xffffu);
            bt[n0 + 2 * i + 1][s] = (uint16_t)(q[i] >> 16);
        }
    }
    __syncthreads();

    // S[p][n] = sum_s xt[p][s] bt[n][s]: 2 tiles along p, N / 32 along n, dealt to the four wavefronts
    const int r = lane & 31, hk = (lane >> 5) * 8;
    float *dst = ws_state + (((int64_t)b * (n_chunks + 1) + chunk + 1) * D + h * kP) * N;
    for (int pair = wave; pair < 2 * (N / 32); pair += 4) {
        const int pt = pair & 1, ntile = pair >> 1;
        f32x16 acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.0f;
#pragma unroll
        for (int ks = 0; ks < kLc / 16; ++ks) {
            const bf16x8 bf = lds_frag(bt, ntile * 32 + r, ks * 16 + hk);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag(xt, pt * 32 + r, ks * 16 + hk), bf, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag(xt_rem, pt * 32 + r, ks * 16 + hk), bf, acc, 0, 0, 0);
        }
        // acc[i] is S[p = 32 pt + 8 (i / 4) + 4 (lane / 32) + i % 4][n = 32 ntile + lane % 32]
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int p = pt * 32 + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
            dst[(int64_t)p * N + ntile * 32 + r] = acc[i];
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// pass 2.  grid: (n_chunks, H, batch).  Wavefront w owns the 32 x 32 block (t tile w / 2, p tile w % 2) of
// the chunk's outputs and the block (t tile w / 2, s tile w % 2) of G.
template <int N, bool HAS_Z>
__global__ void __launch_bounds__(kThreads)
ssd_chunk_out(const bf16_t *__restrict__ x, const bf16_t *__restrict__ dt, const float *__restrict__ A,
              const bf16_t *__restrict__ Bm, const bf16_t *__restrict__ Cm, const float *__restrict__ Dskip,
              const bf16_t *__restrict__ z, const float *__restrict__ dt_bias, const float *__restrict__ ws_state,
              bf16_t *__restrict__ out, int64_t L, int64_t H, int n_chunks, int softplus)
{
    __shared__ float delta[kLc], cum[kLc];
    __shared__ __attribute__((aligned(16))) uint16_t xt[kP][kRowU16];     // x_s[p] as [p][s]
    __shared__ __attribute__((aligned(16))) uint16_t mm[kLc][kRowU16], mm_rem[kLc][kRowU16];   // M[t][s], two bf16 terms
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int chunk = blockIdx.x;
    const int64_t h = blockIdx.y, b = blockIdx.z;
    const int64_t row0 = b * L, tok0 = (int64_t)chunk * kLc, D = H * kP;
    const int tt = wave >> 1, half = wave & 1;
    const int r = lane & 31, hk = (lane >> 5) * 8;

    if (wave == 0) chunk_decay(dt, dt_bias, A[h], tok0, L, H, h, row0, softplus, delta, cum);
    __syncthreads();
    stage_x_transposed(x, row0, tok0, L, H, h, nullptr, xt);

    // C fragments of this wavefront's t tile (kept for G and for the incoming-state term); rows past L
    // repeat the last token and are never stored
    int64_t tok_c = tok0 + tt * 32 + r;
    tok_c = tok_c < L ? tok_c : L - 1;
    const uint4 *crow = reinterpret_cast<const uint4 *>(Cm + (row0 + tok_c) * N);
    bf16x8 cf[N / 16];
#pragma unroll
    for (int ks = 0; ks < N / 16; ++ks) cf[ks] = __builtin_bit_cast(bf16x8, crow[ks * 2 + (lane >> 5)]);

    // G block (t tile tt, s tile half); above the diagonal it is masked out entirely
    f32x16 g;
#pragma unroll
    for (int i = 0; i < 16; ++i) g[i] = 0.0f;
    if (half <= tt) {
        int64_t tok_b = tok0 + half * 32 + r;
        tok_b = tok_b < L ? tok_b : L - 1;
        const uint4 *brow = reinterpret_cast<const uint4 *>(Bm + (row0 + tok_b) * N);
#pragma unroll
        for (int ks = 0; ks < N / 16; ++ks)
            g = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cf[ks], __builtin_bit_cast(bf16x8, brow[ks * 2 + (lane >> 5)]), g, 0, 0, 0);
    }
    // M = G * exp(s_t - s_s) * delta_s for s <= t (steps past L have delta = 0 and x = 0, so they add nothing)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int t = tt * 32 + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3), s = half * 32 + r;
        const float v = (s <= t) ? g[i] * exp2_hw((cum[t] - cum[s]) * kLog2e) * delta[s] : 0.0f;
        const uint32_t top = f32_to_bf16(v);
        mm[t][s] = (uint16_t)top;
        mm_rem[t][s] = (uint16_t)f32_to_bf16(v - bf16_to_f32(top));
    }
    __syncthreads();

    // output block (t tile tt, p tile half)
    f32x16 inter, intra;
#pragma unroll
    for (int i = 0; i < 16; ++i) inter[i] = intra[i] = 0.0f;
    {
        // incoming state of the chunk, rows p of this p tile, as two bf16 terms (value and rounding
        // remainder): this is the one sum where single rounding shows, a long contraction with a state
        // that can be large and cancel
        const float *hrow = ws_state + (((int64_t)b * (n_chunks + 1) + chunk) * D + h * kP + half * 32 + r) * N;
#pragma unroll
        for (int ks = 0; ks < N / 16; ++ks) {
            const float4 lo4 = *reinterpret_cast<const float4 *>(hrow + ks * 16 + hk);
            const float4 hi4 = *reinterpret_cast<const float4 *>(hrow + ks * 16 + hk + 4);
            const float v[8] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};
            uint32_t top[4], rem[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                top[i] = f32x2_to_bf16x2(v[2 * i], v[2 * i + 1]);
                rem[i] = f32x2_to_bf16x2(v[2 * i] - bf16_lo(top[i]), v[2 * i + 1] - bf16_hi(top[i]));
            }
            inter = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cf[ks], __builtin_bit_cast(bf16x8, make_uint4(top[0], top[1], top[2], top[3])), inter, 0, 0, 0);
            inter = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cf[ks], __builtin_bit_cast(bf16x8, make_uint4(rem[0], rem[1], rem[2], rem[3])), inter, 0, 0, 0);
        }
    }
#pragma unroll
    for (int ks = 0; ks < kLc / 16; ++ks)
        if (ks < 2 * (tt + 1)) {                                 // M is zero right of the diagonal block
            const bf16x8 xf = lds_frag(xt, half * 32 + r, ks * 16 + hk);
            intra = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag(mm, tt * 32 + r, ks * 16 + hk), xf, intra, 0, 0, 0);
            intra = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag(mm_rem, tt * 32 + r, ks * 16 + hk), xf, intra, 0, 0, 0);
        }
    const float dsk = Dskip ? Dskip[h] : 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int t = tt * 32 + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
        const int64_t tok = tok0 + t;
        if (tok >= L) continue;
        const int64_t o = ((row0 + tok) * H + h) * kP + half * 32 + r;
        float y = intra[i] + exp2_hw(cum[t] * kLog2e) * inter[i] + dsk * bf16_to_f32(x[o]);
        if constexpr (HAS_Z) y *= silu_f32(bf16_to_f32(z[o]));
        out[o] = (bf16_t)f32_to_bf16(y);
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

}  // namespace

size_t ssd_workspace_bytes(int64_t batch, int64_t L, int64_t H, int64_t P, int64_t N)
{
    const int64_t slots = chunks_of(L) + 1, D = H * P;
    return (size_t)(batch * slots * D * (N + 1) + D * N) * sizeof(float);
}

hipError_t launch_ssd(const SsdArgs &a, hipStream_t stream)
{
    const int nc = (int)chunks_of(a.L);
    const int64_t D = a.H * a.P;
    float *ws_state = a.ws;
    float *ws_sumdt = ws_state + (size_t)a.batch * (nc + 1) * D * a.N;
    float *a_rows = ws_sumdt + (size_t)a.batch * (nc + 1) * D;
    const bf16_t *x = static_cast<const bf16_t *>(a.x), *dt = static_cast<const bf16_t *>(a.dt);
    const bf16_t *Bm = static_cast<const bf16_t *>(a.Bm), *Cm = static_cast<const bf16_t *>(a.Cm);
    const bf16_t *z = static_cast<const bf16_t *>(a.z);
    bf16_t *out = static_cast<bf16_t *>(a.out);
    dim3 grid((unsigned)nc, (unsigned)a.H, (unsigned)a.batch);
    if (a.N == 64)
        ssd_chunk_state<64><<<grid, kThreads, 0, stream>>>(x, dt, a.A, Bm, a.dt_bias, ws_state, ws_sumdt, a_rows, a.L, a.H, nc, a.dt_softplus);
    else
        ssd_chunk_state<128><<<grid, kThreads, 0, stream>>>(x, dt, a.A, Bm, a.dt_bias, ws_state, ws_sumdt, a_rows, a.L, a.H, nc, a.dt_softplus);
    if (hipError_t e = launch_chunk_carry(a_rows, a.h0, ws_state, ws_sumdt, a.batch, D, a.N, nc + 1, stream)) return e;
#define MAMBA_SSD_OUT(NN, HZ)                                                                                    \
    ssd_chunk_out<NN, HZ><<<grid, kThreads, 0, stream>>>(x, dt, a.A, Bm, Cm, a.Dskip, z, a.dt_bias, ws_state, out, \
                                                        a.L, a.H, nc, a.dt_softplus)
    if (a.N == 64) {
        if (z) MAMBA_SSD_OUT(64, true);
        else MAMBA_SSD_OUT(64, false);
    } else {
        if (z) MAMBA_SSD_OUT(128, true);
        else MAMBA_SSD_OUT(128, false);
    }
#undef MAMBA_SSD_OUT
    if (a.h_final) {
        // the carry left the state after the last chunk in the last slot of every batch row
        for (int64_t b = 0; b < a.batch; ++b)
            if (hipError_t e = launch_copy_state(ws_state + ((size_t)b * (nc + 1) + nc) * D * a.N, a.h_final + b * D * a.N, D * a.N, stream))
                return e;
    }
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
