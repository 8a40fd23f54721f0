// Selective scan in a single pass for shapes with few independent channels (one sequence, or a few, of a
// Mamba-130M-sized layer: the contexts of a few thousand tokens the paper's drafter encodes, Sec. 3.1 and the
// long-context experiments), gfx950, N = 16.  Same arithmetic as scan.hip:
//
//   delta = softplus(dt + dt_bias);  h_t = exp(delta_t A) h_{t-1} + delta_t B_t x_t
//   y_t = C_t . h_t + D x_t;  out_t = y_t silu(z_t)
//
// With 1536 channels there is not enough channel parallelism for 1024 SIMDs, so time has to run in
// parallel somewhere.  Here it runs across the lanes of a wavefront instead of across workgroups: no chunk
// states in memory, no carry kernel, every token read once, exp evaluated once per state update.
//
// (Every workgroup then reads its own 12 bytes of every token row, a 64-byte request each: at a few thousand
// tokens this beats the two-pass kernels' launches and hand-overs, on long sequences their full-line accesses
// win; scan_lanes_applies draws the line.)
//
// A workgroup owns 6 adjacent channels (256 workgroups for 1536 channels) and walks the sequence in
// super-steps of 512 tokens.  Its 12 wavefronts are (channel pair, group of 4 states); the 64 lanes of a
// wavefront are 64 consecutive blocks of 8 tokens.  Per super-step a lane
//   1. integrates its 8 tokens from a zero state (lane 0 from the true state that enters the super-step),
//      keeping the 8 x 8 decay factors a = exp(delta A) in registers: mul, exp2, mul, fma per update;
//   2. forms the decay over its whole block, P = exp(A * sum of its deltas);
//   3. takes part in an inclusive scan over the 64 lanes of the pairs (P, H) under
//      (P1, H1) o (P2, H2) = (P1 P2, P2 H1 + H2): four row_shr steps inside each row of 16 lanes, then
//      row_bcast:15 and row_bcast:31 across the rows (DPP, no LDS): afterwards H is the true state at the
//      end of the lane's block, and a one-lane rotation hands every lane the state its block starts from
//      (lane 0 thereby receives the state that enters the next super-step);
//   4. walks its 8 tokens again from that state with the stored decays (mul, fma) and accumulates
//      C . h (fma); the four state groups of a channel leave their parts in LDS.
// Loads, per-token arithmetic (softplus, delta * x, skip term, gate) and stores happen in a token layout:
// thread (j, i) of the first 8 wavefronts owns token 8 i + j of the super-step, all 6 channels (B_t and C_t are
// fetched by all threads in consecutive 16-byte pieces);
// operands go to LDS as float32 in layouts in which consecutive lanes touch consecutive 16-byte slots.
// The next super-step's rows are requested before the second walk of the current one and used after it.
#include "device_math.h"
#include "launch.h"

namespace mamba {
namespace {

constexpr int kG = 6;                    // channels per workgroup
constexpr int kN = 16;                   // states per channel
constexpr int kParts = 4;                // groups of 4 states
constexpr int kWaves = (kG / 2) * kParts;
constexpr int kThreadsL = 64 * kWaves;   // 768
constexpr int kTau = 8;                  // tokens per lane and super-step
constexpr int kT = 64 * kTau;            // tokens per super-step
constexpr int kTokenThreads = kT;        // one token row per thread of the first 8 wavefronts
constexpr int kBcPart = 66, kBcTau = kParts * kBcPart + 1;   // slots per state group and per token j of lds_B / lds_C

__device__ __forceinline__ void lds_barrier_l()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// One level of the scan for the 8 (P, H) pairs of a lane.  Lanes whose DPP source is valid combine with it,
//   H <- P * H_src + H,  P <- P * P_src,
// the others are left alone (a DPP instruction does not write lanes without a source, and row_mask picks the
// receiving rows of a broadcast).  Written as DPP forms of v_fmac / v_mul, one instruction per update; the
// compiler, given the builtin, moves the source lane into a register first and doubles the count.  Within a
// block every instruction reads registers written at least eight instructions earlier; the s_nop covers the two
// wait states a DPP read needs after a VALU write by whatever precedes the block.
#define MAMBA_SCAN_H(CTRL)                                                   \
    "v_fmac_f32_dpp %0, %0, %8 " CTRL " bank_mask:0xf\n"                     \
    "v_fmac_f32_dpp %1, %1, %9 " CTRL " bank_mask:0xf\n"                     \
    "v_fmac_f32_dpp %2, %2, %10 " CTRL " bank_mask:0xf\n"                    \
    "v_fmac_f32_dpp %3, %3, %11 " CTRL " bank_mask:0xf\n"                    \
    "v_fmac_f32_dpp %4, %4, %12 " CTRL " bank_mask:0xf\n"                    \
    "v_fmac_f32_dpp %5, %5, %13 " CTRL " bank_mask:0xf\n"                    \
    "v_fmac_f32_dpp %6, %6, %14 " CTRL " bank_mask:0xf\n"                    \
    "v_fmac_f32_dpp %7, %7, %15 " CTRL " bank_mask:0xf\n"
#define MAMBA_SCAN_P(CTRL)                                                   \
    "v_mul_f32_dpp %8, %8, %8 " CTRL " bank_mask:0xf\n"                      \
    "v_mul_f32_dpp %9, %9, %9 " CTRL " bank_mask:0xf\n"                      \
    "v_mul_f32_dpp %10, %10, %10 " CTRL " bank_mask:0xf\n"                   \
    "v_mul_f32_dpp %11, %11, %11 " CTRL " bank_mask:0xf\n"                   \
    "v_mul_f32_dpp %12, %12, %12 " CTRL " bank_mask:0xf\n"                   \
    "v_mul_f32_dpp %13, %13, %13 " CTRL " bank_mask:0xf\n"                   \
    "v_mul_f32_dpp %14, %14, %14 " CTRL " bank_mask:0xf\n"                   \
    "v_mul_f32_dpp %15, %15, %15 " CTRL " bank_mask:0xf\n"
#define MAMBA_SCAN_OPERANDS(H, P)                                                                              \
    "+v"(H[0]), "+v"(H[1]), "+v"(H[2]), "+v"(H[3]), "+v"(H[4]), "+v"(H[5]), "+v"(H[6]), "+v"(H[7]),            \
    "+v"(P[0]), "+v"(P[1]), "+v"(P[2]), "+v"(P[3]), "+v"(P[4]), "+v"(P[5]), "+v"(P[6]), "+v"(P[7])

// inclusive scan over the 64 lanes; afterwards H is the state at the end of the lane's block (P is used up)
__device__ __forceinline__ void lane_scan(float (&H)[8], float (&P)[8])
{
    asm volatile("s_nop 1\n" MAMBA_SCAN_H("row_shr:1 row_mask:0xf") MAMBA_SCAN_P("row_shr:1 row_mask:0xf") : MAMBA_SCAN_OPERANDS(H, P));
    asm volatile("s_nop 1\n" MAMBA_SCAN_H("row_shr:2 row_mask:0xf") MAMBA_SCAN_P("row_shr:2 row_mask:0xf") : MAMBA_SCAN_OPERANDS(H, P));
    asm volatile("s_nop 1\n" MAMBA_SCAN_H("row_shr:4 row_mask:0xf") MAMBA_SCAN_P("row_shr:4 row_mask:0xf") : MAMBA_SCAN_OPERANDS(H, P));
    asm volatile("s_nop 1\n" MAMBA_SCAN_H("row_shr:8 row_mask:0xf") MAMBA_SCAN_P("row_shr:8 row_mask:0xf") : MAMBA_SCAN_OPERANDS(H, P));
    // lane 15 of rows 0 and 2 into rows 1 and 3, then lane 31 into rows 2 and 3
    asm volatile("s_nop 1\n" MAMBA_SCAN_H("row_bcast:15 row_mask:0xa") MAMBA_SCAN_P("row_bcast:15 row_mask:0xa") : MAMBA_SCAN_OPERANDS(H, P));
    asm volatile("s_nop 1\n" MAMBA_SCAN_H("row_bcast:31 row_mask:0xc") : MAMBA_SCAN_OPERANDS(H, P));
}

// lane i <- lane i - 1, lane 0 <- lane 63
__device__ __forceinline__ float wave_rotate1(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x13C, 0xf, 0xf, false));
}

// six adjacent channels of one token row, as they lie in memory
template <typename T> struct Row6;
template <> struct Row6<bf16_t> {
    uint32_t v[3];
    __device__ __forceinline__ void load(const bf16_t *p)
    {
        const uint32_t *q = reinterpret_cast<const uint32_t *>(p);
        v[0] = q[0]; v[1] = q[1]; v[2] = q[2];
    }
    __device__ __forceinline__ void unpack(float *f) const
    {
        f[0] = bf16_lo(v[0]); f[1] = bf16_hi(v[0]); f[2] = bf16_lo(v[1]); f[3] = bf16_hi(v[1]);
        f[4] = bf16_lo(v[2]); f[5] = bf16_hi(v[2]);
    }
};
template <> struct Row6<float> {
    float2 v[3];
    __device__ __forceinline__ void load(const float *p)
    {
        const float2 *q = reinterpret_cast<const float2 *>(p);
        v[0] = q[0]; v[1] = q[1]; v[2] = q[2];
    }
    __device__ __forceinline__ void unpack(float *f) const
    {
        f[0] = v[0].x; f[1] = v[0].y; f[2] = v[1].x; f[3] = v[1].y; f[4] = v[2].x; f[5] = v[2].y;
    }
};
__device__ __forceinline__ void store_row6(bf16_t *p, const float *f)
{
    uint32_t *q = reinterpret_cast<uint32_t *>(p);
    q[0] = f32x2_to_bf16x2(f[0], f[1]);
    q[1] = f32x2_to_bf16x2(f[2], f[3]);
    q[2] = f32x2_to_bf16x2(f[4], f[5]);
}
__device__ __forceinline__ void store_row6(float *p, const float *f)
{
    float2 *q = reinterpret_cast<float2 *>(p);
    q[0] = make_float2(f[0], f[1]);
    q[1] = make_float2(f[2], f[3]);
    q[2] = make_float2(f[4], f[5]);
}

// the channel pairs from `first` on only (first even)
__device__ __forceinline__ void store_pairs(bf16_t *p, const float *f, int first)
{
    uint32_t *q = reinterpret_cast<uint32_t *>(p);
#pragma unroll
    for (int c = 0; c < kG; c += 2)
        if (c >= first) q[c / 2] = f32x2_to_bf16x2(f[c], f[c + 1]);
}
__device__ __forceinline__ void store_pairs(float *p, const float *f, int first)
{
    float2 *q = reinterpret_cast<float2 *>(p);
#pragma unroll
    for (int c = 0; c < kG; c += 2)
        if (c >= first) q[c / 2] = make_float2(f[c], f[c + 1]);
}

// B_t and C_t of a super-step are fetched by all threads in 16-byte chunks, consecutive threads on consecutive
// chunks (fully coalesced), and land in LDS as float32 groups of 4 states.
template <typename T> struct BcChunk;
template <> struct BcChunk<bf16_t> {     // 8 values: two groups of 4 states
    static constexpr int kGroups = 2;
    uint4 v;
    __device__ __forceinline__ void load(const bf16_t *p) { v = *reinterpret_cast<const uint4 *>(p); }
    __device__ __forceinline__ float4 group(int g) const
    {
        const uint32_t a = g ? v.z : v.x, b = g ? v.w : v.y;
        return make_float4(bf16_lo(a), bf16_hi(a), bf16_lo(b), bf16_hi(b));
    }
};
template <> struct BcChunk<float> {      // 4 values: one group
    static constexpr int kGroups = 1;
    float4 v;
    __device__ __forceinline__ void load(const float *p) { v = *reinterpret_cast<const float4 *>(p); }
    __device__ __forceinline__ float4 group(int) const { return v; }
};

// grid: (ceil(D / 6) rounded up to a multiple of 8, batch); block: 768.  N = 16, D even and >= 6.
template <typename T, bool HAS_Z, bool SOFTPLUS>
__global__ void __launch_bounds__(kThreadsL)
scan_lanes_kernel(const T *x, const T *dt, const float *__restrict__ A, const T *Bm, const T *Cm,
                  const float *__restrict__ Dskip, const T *z, const float *__restrict__ dt_bias,
                  const float *h0 /* may alias h_final */, T *out, float *h_final, int64_t L, int64_t D)
{
    // [token j of the lane's block][state group][lane][4 states]: the lanes of a wavefront read consecutive slots.
    // The threads that fill them write, eight lanes at a time, four consecutive tokens (j) x two state groups two
    // apart: with rows of 66 slots and 265 slots per j those eight 16-byte slots fall on eight different quarters
    // of the banks (j * 265 + 2 * 66 * pos = j + 4 * pos mod 8).
    __shared__ __attribute__((aligned(16))) float4 lds_B[kTau * kBcTau];
    __shared__ __attribute__((aligned(16))) float4 lds_C[kTau * kBcTau];
    // [channel][half of the block][lane][4 tokens]
    __shared__ __attribute__((aligned(16))) float4 lds_d[kG][kTau / 4][64];   // delta
    __shared__ __attribute__((aligned(16))) float4 lds_u[kG][kTau / 4][64];   // delta * x
    __shared__ __attribute__((aligned(16))) float4 lds_y[kParts][kG][kTau / 4][64];   // C . h per token, same layout: one part per state group
    __shared__ float lds_par[2][kG];                                           // dt_bias, D of the workgroup's channels

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int64_t b = blockIdx.y;
    // the last workgroup of a row may have fewer than 6 channels of its own (2 or 4, D being even): it then loads
    // the last 6 of the row, works on all of them, and keeps results only for its own (the leading `dead` ones
    // belong to its neighbour and are neither stored nor taken as a state)
    // Workgroups are dealt to the 8 XCDs in turn (workgroup i runs on XCD i % 8, each with an L2 of its own) and
    // neighbouring channel groups share every 128-byte line of a token row, so the groups are numbered to put
    // neighbours on the same XCD: XCD x takes groups x * per_xcd .. (x + 1) * per_xcd - 1.  The grid is padded to a
    // multiple of 8; a workgroup without a group leaves at once.
    const int64_t n_groups = (D + kG - 1) / kG;
    const int64_t per_xcd = (n_groups + 7) / 8;
    const int64_t group = (int64_t)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((int64_t)(blockIdx.x >> 3) >= per_xcd || group >= n_groups) return;
    int64_t c0 = group * kG;
    int dead = 0;
    if (c0 + kG > D) {
        dead = (int)(c0 + kG - D);
        c0 = D - kG;
    }
    const int64_t row0 = b * L;

    // ---- token layout (threads of the first 8 wavefronts): thread t has token t of the super-step, which is token
    // tj of the block of lane ti.  (A wavefront's 4-byte accesses to the [..][lane][4 tokens] arrays then cover all
    // banks: 8 lanes x 4 positions.)
    const bool token_thread = tid < kTokenThreads;
    const int tj = tid & (kTau - 1), ti = (tid >> 3) & 63;
    // dt_bias and D of the workgroup's channels: one load per thread, requested here and put into LDS only after the
    // first rows have been requested as well (written where it is fetched, wavefront 0 would sit through two
    // memory round trips before it asks for anything else, and the whole workgroup waits for it at the barrier)
    float par = 0.0f;
    if (tid < 2 * kG) {
        const float *src = tid < kG ? dt_bias : Dskip;
        if (src) par = src[c0 + (tid < kG ? tid : tid - kG)];
    }

    // ---- state layout: channels ca, ca + 1 of the workgroup, states 4 * part .. 4 * part + 3, tokens 8 * lane ..
    const int pair = wave / kParts, part = wave % kParts;
    const int ca = 2 * pair;
    float a2[2][4];              // A * log2(e)
    float hp[2][4];              // the state that enters the next super-step: one value per wavefront (scalar registers)
#pragma unroll
    for (int ch = 0; ch < 2; ++ch)
#pragma unroll
        for (int n = 0; n < 4; ++n) {
            const int64_t idx = (c0 + ca + ch) * kN + 4 * part + n;
            a2[ch][n] = A[idx] * kLog2e;
            hp[ch][n] = (h0 && ca >= dead) ? h0[b * D * kN + idx] : 0.0f;   // wave-uniform address
        }

    // With 2-byte elements everything a super-step needs is requested during the one before; with float32 (twice
    // the registers) only x and dt are, and z, B_t, C_t are fetched where they are used.
    constexpr bool kAhead = sizeof(T) == 2;
    Row6<T> x_nxt, dt_nxt, z_nxt, x_cur, z_cur;
    constexpr int kChunkGroups = BcChunk<T>::kGroups;
    constexpr int kChunksPerRow = kParts / kChunkGroups;             // 2 (bf16) or 4 (float32)
    constexpr int kChunks = 2 * kT * kChunksPerRow;                  // B and C of a super-step
    constexpr int kBcIters = (kChunks + kThreadsL - 1) / kThreadsL;  // 3 or 6
    constexpr int kBcHeld = 3;                                       // chunks a thread holds at a time
    BcChunk<T> bc_nxt[kBcHeld];

    // chunk q of a super-step: (array, token, position in the row); `first`: 0, or 3 for the second half of float32
    auto fetch_bc = [&](int64_t t_base, int first) {
#pragma unroll
        for (int it = 0; it < kBcHeld; ++it) {
            const int q = tid + (first + it) * kThreadsL;
            if (kChunks % kThreadsL == 0 || q < kChunks) {
                const int arr = q / (kT * kChunksPerRow), r = q % (kT * kChunksPerRow);
                int64_t t = t_base + r / kChunksPerRow;
                t = t < L ? t : L - 1;
                bc_nxt[it].load((arr ? Cm : Bm) + (row0 + t) * kN + (r % kChunksPerRow) * (kN / kChunksPerRow));
            }
        }
    };
    auto publish_bc = [&](int first) {
#pragma unroll
        for (int it = 0; it < kBcHeld; ++it) {
            const int q = tid + (first + it) * kThreadsL;
            if (kChunks % kThreadsL == 0 || q < kChunks) {
                const int arr = q / (kT * kChunksPerRow), r = q % (kT * kChunksPerRow);
                const int tok = r / kChunksPerRow, pos = r % kChunksPerRow;
                // (a token past the end re-reads the last row: its delta is zero, which alone keeps the state as it is)
                float4 *dst = arr ? lds_C : lds_B;
#pragma unroll
                for (int g = 0; g < kChunkGroups; ++g)
                    dst[(tok & (kTau - 1)) * kBcTau + (pos * kChunkGroups + g) * kBcPart + tok / kTau] = bc_nxt[it].group(g);
            }
        }
    };
    auto fetch = [&](int64_t t_base) {
        int64_t t = t_base + kTau * ti + tj;
        t = t < L ? t : L - 1;                       // tokens past the end re-read the last one and are zeroed at use
        const int64_t o = (row0 + t) * D + c0;
        x_nxt.load(x + o);
        dt_nxt.load(dt + o);
        if constexpr (kAhead && HAS_Z) z_nxt.load(z + o);
    };
    auto publish = [&](int64_t t_base) {
        const bool valid = t_base + kTau * ti + tj < L;
        float xv[kG], dv[kG];
        x_nxt.unpack(xv);
        dt_nxt.unpack(dv);
#pragma unroll
        for (int c = 0; c < kG; ++c) {
            const float v = dv[c] + lds_par[0][c];
            float d = SOFTPLUS ? softplus_f32(v) : v;
            d = valid ? d : 0.0f;                    // a token past the end leaves the state as it is
            reinterpret_cast<float *>(&lds_d[c][tj >> 2][ti])[tj & 3] = d;
            reinterpret_cast<float *>(&lds_u[c][tj >> 2][ti])[tj & 3] = d * xv[c];
        }
        x_cur = x_nxt;
        if constexpr (HAS_Z && kAhead) z_cur = z_nxt;
    };
    auto epilogue = [&](int64_t t_base) {
        const int64_t t = t_base + kTau * ti + tj;
        float xv[kG], zv[kG], ov[kG];
        x_cur.unpack(xv);
        if constexpr (HAS_Z && !kAhead) z_cur.load(z + (row0 + (t < L ? t : L - 1)) * D + c0);
        if constexpr (HAS_Z) z_cur.unpack(zv);
#pragma unroll
        for (int c = 0; c < kG; ++c) {
            // the four state groups in a fixed order: the result does not depend on which wavefront was first
            auto part_y = [&](int p) { return reinterpret_cast<const float *>(&lds_y[p][c][tj >> 2][ti])[tj & 3]; };
            const float ch = (part_y(0) + part_y(1)) + (part_y(2) + part_y(3));
            const float y = fmaf(lds_par[1][c], xv[c], ch);
            ov[c] = HAS_Z ? y * silu_f32(zv[c]) : y;
        }
        if (t < L) {
            if (dead == 0) store_row6(out + (row0 + t) * D + c0, ov);
            else store_pairs(out + (row0 + t) * D + c0, ov, dead);
        }
    };

    const int64_t n_super = (L + kT - 1) / kT;
    if (token_thread) fetch(0);
    fetch_bc(0, 0);
    if (tid < 2 * kG) (&lds_par[0][0])[tid] = par;
    lds_barrier_l();   // the channel parameters are in LDS
    if (token_thread) publish(0);
    publish_bc(0);
    if constexpr (kBcIters > kBcHeld) {
        fetch_bc(0, kBcHeld);
        publish_bc(kBcHeld);
    }
    lds_barrier_l();

    for (int64_t k = 0; k < n_super; ++k) {
        const int64_t t_base = k * kT;
        const bool more = k + 1 < n_super;
        if (token_thread && more) fetch(t_base + kT);

        // ---- 1. the lane's 8 tokens from zero (lane 0: from the state entering the super-step), decays kept
        // (delta and delta * x are taken from LDS four tokens at a time: fewer registers held at once)
        float a[kTau][2][4], h[2][4], P[2][4], dsum[2] = {0.0f, 0.0f};
#pragma unroll
        for (int ch = 0; ch < 2; ++ch)
#pragma unroll
            for (int n = 0; n < 4; ++n) h[ch][n] = lane == 0 ? hp[ch][n] : 0.0f;
#pragma unroll
        for (int jh = 0; jh < kTau / 4; ++jh) {
            float4 d4[2], u4[2];
#pragma unroll
            for (int ch = 0; ch < 2; ++ch) {
                d4[ch] = lds_d[ca + ch][jh][lane];
                u4[ch] = lds_u[ca + ch][jh][lane];
            }
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const int j = 4 * jh + jj;
                const float4 b4 = lds_B[j * kBcTau + part * kBcPart + lane];
                const float bv[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
                for (int ch = 0; ch < 2; ++ch) {
                    const float d = jj == 0 ? d4[ch].x : jj == 1 ? d4[ch].y : jj == 2 ? d4[ch].z : d4[ch].w;
                    const float u = jj == 0 ? u4[ch].x : jj == 1 ? u4[ch].y : jj == 2 ? u4[ch].z : u4[ch].w;
                    dsum[ch] += d;
#pragma unroll
                    for (int n = 0; n < 4; ++n) {
                        a[j][ch][n] = exp2_hw(d * a2[ch][n]);
                        h[ch][n] = fmaf(a[j][ch][n], h[ch][n], u * bv[n]);
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // ---- 2. decay over the whole block
#pragma unroll
        for (int ch = 0; ch < 2; ++ch)
#pragma unroll
            for (int n = 0; n < 4; ++n) P[ch][n] = exp2_hw(dsum[ch] * a2[ch][n]);
        // ---- 3. inclusive scan over the 64 lanes, then every lane takes the state at the end of the block before it
        float hin[2][4];
        {
            float Hs[8], Ps[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                Hs[r] = h[r >> 2][r & 3];
                Ps[r] = P[r >> 2][r & 3];
            }
            lane_scan(Hs, Ps);
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const float rot = wave_rotate1(Hs[r]);
                hin[r >> 2][r & 3] = lane == 0 ? hp[r >> 2][r & 3] : rot;
                // lane 63's end state enters the next super-step
                hp[r >> 2][r & 3] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(Hs[r]), 63));
            }
        }
        // The next super-step's rows are requested here rather than at the top: their registers would otherwise be
        // held through the first walk, where the decays pile up; the second walk, the barrier and the gating of
        // this super-step's outputs are what their latency hides behind.
        if (more) {
            if constexpr (kAhead) fetch_bc(t_base + kT, 0);
        }
        // ---- 4. the 8 tokens again from the true state, with outputs (delta * x is read again rather than kept)
#pragma unroll
        for (int jh = 0; jh < kTau / 4; ++jh) {
            __builtin_amdgcn_sched_barrier(0);
            float4 u4[2];
            float yq[2][4];
#pragma unroll
            for (int ch = 0; ch < 2; ++ch) u4[ch] = lds_u[ca + ch][jh][lane];
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const int j = 4 * jh + jj;
                const float4 b4 = lds_B[j * kBcTau + part * kBcPart + lane], c4 = lds_C[j * kBcTau + part * kBcPart + lane];
                const float bv[4] = {b4.x, b4.y, b4.z, b4.w}, cv[4] = {c4.x, c4.y, c4.z, c4.w};
#pragma unroll
                for (int ch = 0; ch < 2; ++ch) {
                    const float u = jj == 0 ? u4[ch].x : jj == 1 ? u4[ch].y : jj == 2 ? u4[ch].z : u4[ch].w;
                    float yp = 0.0f;
#pragma unroll
                    for (int n = 0; n < 4; ++n) {
                        hin[ch][n] = fmaf(a[j][ch][n], hin[ch][n], u * bv[n]);
                        yp = fmaf(hin[ch][n], cv[n], yp);
                    }
                    yq[ch][jj] = yp;
                }
            }
#pragma unroll
            for (int ch = 0; ch < 2; ++ch) lds_y[part][ca + ch][jh][lane] = make_float4(yq[ch][0], yq[ch][1], yq[ch][2], yq[ch][3]);
        }
        lds_barrier_l();   // y of the super-step is complete; its operands are used up

        if constexpr (!kAhead) {
            if (more) fetch_bc(t_base + kT, 0);
        }
        if (token_thread) {
            epilogue(t_base);
            if (more) publish(t_base + kT);
        }
        if (more) {
            publish_bc(0);
            if constexpr (kBcIters > kBcHeld) {
                fetch_bc(t_base + kT, kBcHeld);
                publish_bc(kBcHeld);
            }
        }
        lds_barrier_l();   // the next super-step is in LDS
    }

    if (h_final && lane == 0 && ca >= dead) {
#pragma unroll
        for (int ch = 0; ch < 2; ++ch)
#pragma unroll
            for (int n = 0; n < 4; ++n)
                h_final[b * D * kN + (c0 + ca + ch) * kN + 4 * part + n] = hp[ch][n];
    }
}

}  // namespace

// Shapes the lane-scan kernel serves: 16 states, token rows that can be read in 4-byte pieces from any even
// channel, at least one full workgroup; and among those the ones it is expected to finish before the two-pass
// kernels of scan.hip.  Its time is rounds x (about 6 us + 11.6 ns per token), a round being 256 workgroups of 6
// channels (every workgroup walks the whole sequence); the two-pass kernels take about 24 us + 9.8 ns per token
// and 1536 channels.  Measured in one run, lanes against two-pass, 1536 channels: 2048 tokens 31 against 43 us,
// 5120 tokens 71 against 78, 8192 tokens 101 against 104, 10240 tokens 121 against 122, 32768 tokens 461 against
// 353; two sequences of 2048 tokens 56 against 60, of 4096 tokens 102 against 101; 768 channels x 4096 tokens 48
// against 44; 2048 channels (342 workgroups, two rounds) x 4096 tokens 105 against 76.
bool scan_lanes_applies(int64_t batch, int64_t L, int64_t D, int64_t N)
{
    if (N != kN || D % 2 != 0 || D < kG || L < 64 || batch > 65535) return false;
    const double groups = (double)batch * (double)((D + kG - 1) / kG);
    const double rounds = (double)(int64_t)((groups + 255.0) / 256.0);
    const double lanes_ns = rounds * (6000.0 + 11.6 * (double)L);
    const double two_pass_ns = 24000.0 + 9.8 * (double)L * ((double)batch * (double)D / 1536.0);
    return lanes_ns < two_pass_ns;
}

hipError_t launch_scan_lanes(const ScanArgs &a, hipStream_t stream)
{
    const int64_t n_groups = (a.D + kG - 1) / kG;
    const dim3 grid((unsigned)(8 * ((n_groups + 7) / 8)), (unsigned)a.batch);   // padded for the XCD-aware numbering
#define MAMBA_LAUNCH_LANES(T, HZ, SP)                                                                       \
    scan_lanes_kernel<T, HZ, SP><<<grid, kThreadsL, 0, stream>>>(                                           \
        static_cast<const T *>(a.x), static_cast<const T *>(a.dt), a.A, static_cast<const T *>(a.Bm),       \
        static_cast<const T *>(a.Cm), a.Dskip, static_cast<const T *>(a.z), a.dt_bias, a.h0,                \
        static_cast<T *>(a.out), a.h_final, a.L, a.D)
#define MAMBA_LAUNCH_LANES_T(T)                                  \
    do {                                                         \
        if (a.z) {                                               \
            if (a.dt_softplus) MAMBA_LAUNCH_LANES(T, true, true);  \
            else MAMBA_LAUNCH_LANES(T, true, false);             \
        } else {                                                 \
            if (a.dt_softplus) MAMBA_LAUNCH_LANES(T, false, true); \
            else MAMBA_LAUNCH_LANES(T, false, false);            \
        }                                                        \
    } while (0)
    if (a.io == kIoBf16) MAMBA_LAUNCH_LANES_T(bf16_t);
    else MAMBA_LAUNCH_LANES_T(float);
#undef MAMBA_LAUNCH_LANES_T
#undef MAMBA_LAUNCH_LANES
    return hipGetLastError();
}

}  // namespace mamba
