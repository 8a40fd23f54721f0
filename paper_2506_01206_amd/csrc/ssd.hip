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

// Workgroup barrier that orders LDS traffic only: the tiles exchanged between wavefronts live in LDS, and a
// barrier that also ordered global memory would wait for every output store and every prefetch in flight.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}


// four values -> their bf16 roundings and the bf16 of what the roundings dropped, packed in order
__device__ __forceinline__ void split4(const float *v, uint2 *top, uint2 *rem)
{
    const uint32_t t01 = f32x2_to_bf16x2(v[0], v[1]), t23 = f32x2_to_bf16x2(v[2], v[3]);
    *top = make_uint2(t01, t23);
    *rem = make_uint2(f32x2_to_bf16x2(v[0] - bf16_lo(t01), v[1] - bf16_hi(t01)),
                      f32x2_to_bf16x2(v[2] - bf16_lo(t23), v[3] - bf16_hi(t23)));
}

// element k (0 .. 7) of a 16-byte piece of bf16, as float / the 16-bit halves of two pieces side by side
__device__ __forceinline__ uint32_t piece_word(const uint4 &q, int k2) { return k2 == 0 ? q.x : k2 == 1 ? q.y : k2 == 2 ? q.z : q.w; }
__device__ __forceinline__ float piece_el(const uint4 &q, int k)
{
    const uint32_t w = piece_word(q, k >> 1);
    return (k & 1) ? bf16_hi(w) : bf16_lo(w);
}
__device__ __forceinline__ uint32_t pair_el(const uint4 &a, const uint4 &b, int k)   // element k of a (low half), of b (high half)
{
    const uint32_t wa = piece_word(a, k >> 1), wb = piece_word(b, k >> 1);
    return (k & 1) ? ((wa >> 16) | (wb & 0xffff0000u)) : ((wa & 0xffffu) | (wb << 16));
}

// ---------------------------------------------------------------------------------------------------
// A workgroup walks the chunks of one segment of one (batch row, head) in order, the head's state
// living transposed (N x P float32) in MFMA accumulators: per chunk acc <- exp(s_end) acc + S.
//   PASS2 = false: from a zero state; leaves the segment's end state in slot seg + 1 of ws_state
//       ((batch, n_slots, H * P, N)) and the segment's sum of deltas in ws_sumdt; the carry kernel
//       of the selective scan then turns the slots into the states at the segment starts;
//   PASS2 = true: from the true incoming state (slot seg * slot_step: pass 1 may cut the sequence
//       slot_step times finer than pass 2, its workgroups being small enough to share a CU), with outputs.
// Two roles.  The four "state" wavefronts hold the accumulators: per chunk they multiply the transposed B and
// the weighted x (two bf16 terms), which they parked in LDS one phase earlier, into the state; in pass 2 they
// also lay out B row-major, x transposed and the state at the chunk start (two bf16 terms) for the output
// products.  Pass 2 adds four "output" wavefronts, one 32 x 32 block of the chunk's 64 x 64 outputs each,
// computed transposed so that a lane owns one step and four adjacent channels at a time: they lay out C and
// z, form G^T and M (D goes onto M's diagonal, which adds D x_t to the outputs), after the barrier multiply M
// with x and C with the incoming state, and gate and store during the next chunk's first phase, when the
// state role is busy filling LDS.  With one wavefront of each role on every SIMD the conversions of one
// overlap the products of the other.  Everything a thread moves into LDS transposed is a run of 2 or 4 steps
// of one row (its pieces are adjacent steps), so the writes are 4 or 8 bytes wide.  Raw tiles are fetched
// unconditionally (steps past L re-read step L - 1 and are zeroed at use), B and x two chunks ahead into
// register sets used in turn, C and z one chunk ahead; delta and its running sum are formed one chunk ahead
// into the other half of a double buffer.
// grid: (n_seg, H, batch); 256 threads in pass 1, 512 in pass 2.
template <int N, bool PASS2, bool HAS_Z>
__global__ void __launch_bounds__(PASS2 ? 2 * kThreads : kThreads) __attribute__((amdgpu_waves_per_eu(2)))
ssd_segment(const bf16_t *x, const bf16_t *dt, const float *__restrict__ A, const bf16_t *Bm, const bf16_t *Cm,
            const float *__restrict__ Dskip, const bf16_t *z, const float *__restrict__ dt_bias, float *ws_state,
            float *ws_sumdt, float *a_rows, bf16_t *out, float *h_final, int64_t L, int64_t H, int chunks_per_seg,
            int n_seg, int n_slots, int slot_step, int n_chunks, int softplus)
{
    // (x, dt, B, C, z are deliberately not declared restrict: as possibly aliased by the stores to out they
    // stay where they are written, a chunk ahead of their use, instead of being sunk to it by the compiler)
    constexpr int kRowN = N + 8;                              // LDS row of N bf16 + padding
    constexpr int NB = N / 32;                                // 16-byte pieces of a B / C tile per state thread
    constexpr int PPR = N / 8;                                // pieces per B / C row
    constexpr int PPW = N / 64;                               // state tiles (32 x 32) per state wavefront: N / 32 n tiles x 2 p tiles
    __shared__ float4 delta4[2][kLc / 4], cum4[2][kLc / 4];      // delta and its running sum times A, per step; two chunks
    float (*delta)[kLc] = reinterpret_cast<float (*)[kLc]>(delta4), (*cum)[kLc] = reinterpret_cast<float (*)[kLc]>(cum4);
    __shared__ __attribute__((aligned(16))) uint16_t bt[tsize(N)];                       // B as [n][s]
    __shared__ __attribute__((aligned(16))) uint16_t xw_hi[tsize(kP)], xw_lo[tsize(kP)]; // weight_s x_s[p] as [p][s]
    __shared__ __attribute__((aligned(16))) uint16_t xt[PASS2 ? tsize(kP) : 8];          // x as [p][s]
    __shared__ __attribute__((aligned(16))) uint16_t zt[(PASS2 && HAS_Z) ? kLc * kRowS : 8];   // z as [t][p]
    __shared__ __attribute__((aligned(16))) uint16_t c_rows[PASS2 ? kLc * kRowN : 8];     // C as [t][n]
    __shared__ __attribute__((aligned(16))) uint16_t b_rows[PASS2 ? kLc * kRowN : 8];     // B as [s][n]
    __shared__ __attribute__((aligned(16))) uint16_t mm_hi[PASS2 ? kLc * kRowS : 8], mm_lo[PASS2 ? kLc * kRowS : 8];   // M as [t][s]
    __shared__ __attribute__((aligned(16))) uint16_t h_hi[PASS2 ? kP * kRowN : 8], h_lo[PASS2 ? kP * kRowN : 8];       // state as [p][n]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool role_y = PASS2 && wave < 4;                    // output role: wavefronts 0 .. 3 of pass 2
    const int yt = tid & (kThreads - 1);                      // thread index inside a role
    const int sw = wave & 3;                                  // wavefront index inside a role
    const bool scan_wave = !role_y && sw == 0;                // keeps delta and its running sum
    const int seg = blockIdx.x;
    const int64_t h = blockIdx.y, b = blockIdx.z;
    const int64_t row0 = b * L, D = H * kP;
    const float A_h = A[h], bias_h = dt_bias ? dt_bias[h] : 0.0f;
    const float dsk = Dskip ? Dskip[h] : 0.0f;
    const int r = lane & 31, up = lane >> 5, hk = up * 8;
    const int tt = sw >> 1, half = sw & 1;                    // output role: block (channel tile half, step tile tt)
    const int c_first = seg * chunks_per_seg;
    const int c_last = min(c_first + chunks_per_seg, n_chunks);

    // State role: this thread's 16-byte pieces of a chunk's raw tiles: NB adjacent steps sb0 .. of B and of
    // C (states nb0 .. + 7), two adjacent steps sx0, sx0 + 1 of x and of z (channels px0 .. + 7).
    const int sb0 = NB * (yt / PPR), nb0 = (yt % PPR) * 8;
    const int sx0 = 2 * (yt >> 3), px0 = (yt & 7) * 8;
    // B and x are needed twice, a phase before their chunk starts (transposed B and weighted x for the state
    // update) and in its first phase (row-major B, transposed x): two register sets used in turn, each
    // refilled for the chunk after the next as soon as its chunk has gone to LDS.  C and z (output role, which
    // uses the same piece-to-thread map): one set, fetched a chunk ahead.
    struct Early {
        uint4 b[NB], x[2];
    };
    Early E2[2];
    uint4 Pc[NB], Pz0 = make_uint4(0, 0, 0, 0), Pz1 = Pz0;
    // Every fetch is unconditional: chunks past the segment re-read its last chunk, steps past L the row of
    // step L - 1 (zeroed where used).  Addresses: a per-thread base plus (step inside the batch row) x (row size).
    const uint32_t last_tok = (uint32_t)(L - 1);
    auto tok_of = [&](int chunk, int s) { return min((uint32_t)min(chunk, c_last - 1) * kLc + s, last_tok); };
    const bf16_t *b_base = Bm + row0 * N + nb0, *c_base = Cm + row0 * N + nb0;
    const bf16_t *x_base = x + (row0 * H + h) * kP + px0;
    const bf16_t *z_base = (PASS2 && HAS_Z) ? z + (row0 * H + h) * kP + px0 : x_base;
    const uint32_t xz_row = (uint32_t)(H * kP);
    auto fetch_early = [&](int chunk, Early &e) {                 // state role: B and x
#pragma unroll
        for (int i = 0; i < NB; ++i) e.b[i] = *reinterpret_cast<const uint4 *>(b_base + (uint64_t)tok_of(chunk, sb0 + i) * (uint32_t)N);
#pragma unroll
        for (int i = 0; i < 2; ++i) e.x[i] = *reinterpret_cast<const uint4 *>(x_base + (uint64_t)tok_of(chunk, sx0 + i) * xz_row);
    };
    auto fetch_late = [&](int chunk) {                            // output role: C and z
#pragma unroll
        for (int i = 0; i < NB; ++i) Pc[i] = *reinterpret_cast<const uint4 *>(c_base + (uint64_t)tok_of(chunk, sb0 + i) * (uint32_t)N);
        if constexpr (HAS_Z) {
            Pz0 = *reinterpret_cast<const uint4 *>(z_base + (uint64_t)tok_of(chunk, sx0) * xz_row);
            Pz1 = *reinterpret_cast<const uint4 *>(z_base + (uint64_t)tok_of(chunk, sx0 + 1) * xz_row);
        }
    };
    // steps past L (only in the last chunk of a row) count as zeros
    auto mask_early = [&](int chunk, Early &e) {
        const int64_t tok0 = (int64_t)chunk * kLc;
        if (tok0 + kLc > L) {
#pragma unroll
            for (int i = 0; i < NB; ++i)
                if (tok0 + sb0 + i >= L) e.b[i] = make_uint4(0, 0, 0, 0);
#pragma unroll
            for (int i = 0; i < 2; ++i)
                if (tok0 + sx0 + i >= L) e.x[i] = make_uint4(0, 0, 0, 0);
        }
    };
    // B transposed and the weighted x (two bf16 terms: weight_s = exp(s_end - s_s) delta_s) of a chunk into
    // LDS, for its state update; buf: where the chunk's delta and running sums are
    auto park_state_operands = [&](const Early &e, int buf) {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            if constexpr (NB == 4)
                *reinterpret_cast<uint2 *>(&bt[trow(nb0 + k) + sb0]) = make_uint2(pair_el(e.b[0], e.b[1], k), pair_el(e.b[2], e.b[3], k));
            else
                *reinterpret_cast<uint32_t *>(&bt[trow(nb0 + k) + sb0]) = pair_el(e.b[0], e.b[1], k);
        }
        const float cend = cum[buf][kLc - 1];
        const float w0 = exp2_hw((cend - cum[buf][sx0]) * kLog2e) * delta[buf][sx0];
        const float w1 = exp2_hw((cend - cum[buf][sx0 + 1]) * kLog2e) * delta[buf][sx0 + 1];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const float v0 = piece_el(e.x[0], k) * w0, v1 = piece_el(e.x[1], k) * w1;
            const uint32_t top = f32x2_to_bf16x2(v0, v1);
            *reinterpret_cast<uint32_t *>(&xw_hi[trow(px0 + k) + sx0]) = top;
            *reinterpret_cast<uint32_t *>(&xw_lo[trow(px0 + k) + sx0]) = f32x2_to_bf16x2(v0 - bf16_lo(top), v1 - bf16_hi(top));
        }
    };
    auto fetch_dt = [&](int chunk) {                              // one lane per step, raw bits (converted where used)
        return dt[(row0 + tok_of(chunk, lane)) * H + h];
    };
    // delta and the inclusive running sum of delta * A over a chunk (steps past L: delta = 0), one lane per
    // step: sums inside rows of 16 lanes by shifted adds, then the totals of the rows before
    float seg_sum = 0.0f;
    auto prefix = [&](int chunk, bf16_t dt_raw, int buf) {
        const float dtv = bf16_to_f32(dt_raw);
        const float dl = ((int64_t)chunk * kLc + lane < L) ? (softplus ? softplus_f32(dtv + bias_h) : dtv + bias_h) : 0.0f;
        float sc = dl * A_h;
        sc += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, sc), 0x111, 0xf, 0xf, false));
        sc += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, sc), 0x112, 0xf, 0xf, false));
        sc += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, sc), 0x114, 0xf, 0xf, false));
        sc += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, sc), 0x118, 0xf, 0xf, false));
        const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, sc), 15));
        const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, sc), 31));
        const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, sc), 47));
        const int row = lane >> 4;
        sc += row == 0 ? 0.0f : row == 1 ? r0 : row == 2 ? r0 + r1 : (r0 + r1) + r2;
        delta[buf][lane] = dl;
        cum[buf][lane] = sc;
        seg_sum += dl;
    };

    // State role: the head's state, transposed: tile j of a state wavefront is (n tile nt, p tile pt);
    // acc[j][4 g + q] is H[p = 32 pt + lane % 32][n = 32 nt + 8 g + 4 (lane / 32) + q].
    f32x16 acc[PPW];
    float *slot_in = ws_state + (((int64_t)b * n_slots + (int64_t)seg * slot_step) * D + h * kP) * N;
#pragma unroll
    for (int j = 0; j < PPW; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.0f;
    if (PASS2 && !role_y) {
#pragma unroll
        for (int j = 0; j < PPW; ++j) {
            const int id = sw * PPW + j, pt = id & 1, nt = id >> 1;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float4 v = *reinterpret_cast<const float4 *>(slot_in + (int64_t)(pt * 32 + r) * N + nt * 32 + 8 * g + 4 * up);
                acc[j][4 * g] = v.x, acc[j][4 * g + 1] = v.y, acc[j][4 * g + 2] = v.z, acc[j][4 * g + 3] = v.w;
            }
        }
    }
    if (!PASS2 && seg == 0 && b == 0)
        for (int i = tid; i < kP * N; i += kThreads) a_rows[h * kP * N + i] = A_h;   // decay matrix for the carry kernel

    bf16_t dt_next = 0, dt_after = 0;                             // dt of the next chunk and of the one after
    if (role_y) {
        if constexpr (PASS2) fetch_late(c_first);
    } else {
        fetch_early(c_first, E2[0]);
        fetch_early(c_first + 1, E2[1]);
        dt_next = fetch_dt(c_first + 1);
        dt_after = fetch_dt(c_first + 2);
        if (scan_wave) prefix(c_first, fetch_dt(c_first), 0);
    }
    lds_barrier();                                                // delta, cum of the first chunk
    if (!role_y) {
        mask_early(c_first, E2[0]);
        park_state_operands(E2[0], 0);
    }
    if constexpr (!PASS2) lds_barrier();                          // (pass 2 has a barrier ahead of the first state update anyway)

    // Each role runs its own loop over the chunks, with the same three barriers per chunk (two in pass 1):
    //   A  state role: row-major B, transposed x and the state at the chunk start into LDS; fetches.
    //      output role: gate and store the outputs of the chunk before; C and z into LDS; fetches. | barrier (pass 2)
    //   B  state role: state update; delta sums of the next chunk.  output role: G^T and M.   | barrier
    //   C  state role: transposed B and weighted x of the next chunk into LDS.
    //      output role: the two output products.                                              | barrier
    // (a wavefront never changes role, so both sides meet at every barrier; with the loops apart the
    // compiler counts each role's loads in flight exactly)
    if (role_y) {
        if constexpr (PASS2) {
            const int t = tt * 32 + r;
            f32x16 inter, intra;                                      // outputs of the chunk before, not yet gated
            uint2 zq[4];
            float e_t = 0.0f;
            int64_t tok_prev = -1;                                    // its token (none yet)
#pragma unroll
            for (int i = 0; i < 16; ++i) inter[i] = intra[i] = 0.0f;
#pragma unroll
            for (int g = 0; g < 4; ++g) zq[g] = make_uint2(0, 0);
            auto epilogue = [&]() {
                if (tok_prev < 0 || tok_prev >= L) return;
                bf16_t *orow = out + ((row0 + tok_prev) * H + h) * kP + half * 32 + 4 * up;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    float y[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) y[q] = intra[4 * g + q] + e_t * inter[4 * g + q];
                    if constexpr (HAS_Z) {
                        y[0] *= silu_f32(bf16_lo(zq[g].x)), y[1] *= silu_f32(bf16_hi(zq[g].x));
                        y[2] *= silu_f32(bf16_lo(zq[g].y)), y[3] *= silu_f32(bf16_hi(zq[g].y));
                    }
                    *reinterpret_cast<uint2 *>(orow + 8 * g) = make_uint2(f32x2_to_bf16x2(y[0], y[1]), f32x2_to_bf16x2(y[2], y[3]));
                }
            };
            for (int chunk = c_first; chunk < c_last; ++chunk) {
                const int buf = (chunk - c_first) & 1;
                epilogue();
                if ((int64_t)chunk * kLc + kLc > L) {                 // only the last chunk of a row: zero C past L
#pragma unroll
                    for (int i = 0; i < NB; ++i)
                        if ((int64_t)chunk * kLc + sb0 + i >= L) Pc[i] = make_uint4(0, 0, 0, 0);
                }
#pragma unroll
                for (int i = 0; i < NB; ++i) *reinterpret_cast<uint4 *>(&c_rows[(sb0 + i) * kRowN + nb0]) = Pc[i];
                if constexpr (HAS_Z) {
                    *reinterpret_cast<uint4 *>(&zt[sx0 * kRowS + px0]) = Pz0;
                    *reinterpret_cast<uint4 *>(&zt[(sx0 + 1) * kRowS + px0]) = Pz1;
                }
                fetch_late(chunk + 1);
                lds_barrier();                                        // the raw tiles are in LDS
                if (half <= tt) {                                     // the block above the diagonal is masked out entirely
                    float4 cs[4], ds[4];                              // running sums and deltas of the lane's 16 steps s
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        cs[g] = cum4[buf][half * 8 + 2 * g + up];
                        ds[g] = delta4[buf][half * 8 + 2 * g + up];
                    }
                    const float ct = cum[buf][t];
                    f32x16 gacc;
#pragma unroll
                    for (int i = 0; i < 16; ++i) gacc[i] = 0.0f;
                    {
                        // all fragments are requested before the first product, so that the products do not
                        // each wait out an LDS round trip
                        bf16x8 bf[N / 16], cf[N / 16];
#pragma unroll
                        for (int ks = 0; ks < N / 16; ++ks) {
                            bf[ks] = frag(b_rows, kRowN, half * 32 + r, ks * 16 + hk);
                            cf[ks] = frag(c_rows, kRowN, tt * 32 + r, ks * 16 + hk);
                        }
#pragma unroll
                        for (int ks = 0; ks < N / 16; ++ks) gacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[ks], cf[ks], gacc, 0, 0, 0);
                    }
                    // gacc[4 g + q] = C_t . B_s, t = 32 tt + lane % 32, s = 32 half + 8 g + 4 (lane / 32) + q
                    // M = G * exp(s_t - s_s) * delta_s for s <= t (steps past L have delta = 0), + D on the diagonal
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int s0 = half * 32 + 8 * g + 4 * up;
                        const float c4[4] = {cs[g].x, cs[g].y, cs[g].z, cs[g].w}, d4[4] = {ds[g].x, ds[g].y, ds[g].z, ds[g].w};
                        float v[4];
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            v[q] = (s0 + q <= t) ? gacc[4 * g + q] * exp2_hw((ct - c4[q]) * kLog2e) * d4[q] : 0.0f;
                            if (s0 + q == t) v[q] += dsk;
                        }
                        split4(v, reinterpret_cast<uint2 *>(&mm_hi[t * kRowS + s0]), reinterpret_cast<uint2 *>(&mm_lo[t * kRowS + s0]));
                    }
                }
                lds_barrier();                                        // M is in LDS
#pragma unroll
                for (int i = 0; i < 16; ++i) inter[i] = intra[i] = 0.0f;
                {
                    // C with the incoming state, then M (with D) with x (M is zero right of the diagonal block);
                    // again the fragments of a product are requested before it starts
                    bf16x8 cf[N / 16], hh[N / 16], hl[N / 16], xf[kLc / 16], mh[kLc / 16], ml[kLc / 16];
#pragma unroll
                    for (int ks = 0; ks < N / 16; ++ks) {
                        cf[ks] = frag(c_rows, kRowN, tt * 32 + r, ks * 16 + hk);
                        hh[ks] = frag(h_hi, kRowN, half * 32 + r, ks * 16 + hk);
                    }
#pragma unroll
                    for (int ks = 0; ks < N / 16; ++ks) hl[ks] = frag(h_lo, kRowN, half * 32 + r, ks * 16 + hk);
#pragma unroll
                    for (int ks = 0; ks < N / 16; ++ks) inter = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hh[ks], cf[ks], inter, 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int ks = 0; ks < kLc / 16; ++ks)
                        if (ks < 2 * (tt + 1)) {
                            xf[ks] = tfrag(xt, half * 32 + r, ks * 16 + hk);
                            mh[ks] = frag(mm_hi, kRowS, tt * 32 + r, ks * 16 + hk);
                            ml[ks] = frag(mm_lo, kRowS, tt * 32 + r, ks * 16 + hk);
                        }
#pragma unroll
                    for (int ks = 0; ks < N / 16; ++ks) inter = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hl[ks], cf[ks], inter, 0, 0, 0);
#pragma unroll
                    for (int ks = 0; ks < kLc / 16; ++ks)
                        if (ks < 2 * (tt + 1)) {
                            intra = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf[ks], mh[ks], intra, 0, 0, 0);
                            intra = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf[ks], ml[ks], intra, 0, 0, 0);
                        }
                }
                // inter / intra [4 g + q]: step t = 32 tt + lane % 32, channel p = 32 half + 8 g + 4 (lane / 32) + q;
                // what the gate needs leaves LDS now, the arithmetic waits for the next chunk's first phase
                e_t = exp2_hw(cum[buf][t] * kLog2e);
                if constexpr (HAS_Z) {
#pragma unroll
                    for (int g = 0; g < 4; ++g) zq[g] = *reinterpret_cast<const uint2 *>(&zt[t * kRowS + half * 32 + 8 * g + 4 * up]);
                }
                tok_prev = (int64_t)chunk * kLc + t;
                lds_barrier();                                        // the chunk's LDS tiles are free again
            }
            epilogue();
        }
    } else {
        // one chunk; cur holds its B and x pieces (and takes those of the chunk after the next), nxt the next chunk's
        auto walk = [&](int chunk, Early &cur, Early &nxt) {
            const int buf = (chunk - c_first) & 1;
            if constexpr (PASS2) {
#pragma unroll
                for (int i = 0; i < NB; ++i) *reinterpret_cast<uint4 *>(&b_rows[(sb0 + i) * kRowN + nb0]) = cur.b[i];
#pragma unroll
                for (int k = 0; k < 8; ++k) *reinterpret_cast<uint32_t *>(&xt[trow(px0 + k) + sx0]) = pair_el(cur.x[0], cur.x[1], k);
                // the state at the start of the chunk, as two bf16 terms, for the incoming-state product
#pragma unroll
                for (int j = 0; j < PPW; ++j) {
                    const int id = sw * PPW + j, pt = id & 1, nt = id >> 1;
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const float v[4] = {acc[j][4 * g], acc[j][4 * g + 1], acc[j][4 * g + 2], acc[j][4 * g + 3]};
                        const int o = (pt * 32 + r) * kRowN + nt * 32 + 8 * g + 4 * up;
                        split4(v, reinterpret_cast<uint2 *>(&h_hi[o]), reinterpret_cast<uint2 *>(&h_lo[o]));
                    }
                }
            }
            fetch_early(chunk + 2, cur);
            if constexpr (PASS2) lds_barrier();                   // the raw tiles are in LDS
            if (scan_wave && chunk + 1 < c_last) prefix(chunk + 1, dt_next, buf ^ 1);
            dt_next = dt_after;
            dt_after = fetch_dt(chunk + 3);
            // state: acc <- exp(s_end) acc + sum_s bt[n][s] xw[p][s]
            const float dec = exp2_hw(cum[buf][kLc - 1] * kLog2e);
#pragma unroll
            for (int j = 0; j < PPW; ++j) {
                const int id = sw * PPW + j, pt = id & 1, nt = id >> 1;
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[j][i] *= dec;
#pragma unroll
                for (int ks = 0; ks < kLc / 16; ++ks) {
                    const bf16x8 bf = tfrag(bt, nt * 32 + r, ks * 16 + hk);
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf, tfrag(xw_hi, pt * 32 + r, ks * 16 + hk), acc[j], 0, 0, 0);
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf, tfrag(xw_lo, pt * 32 + r, ks * 16 + hk), acc[j], 0, 0, 0);
                }
            }
            lds_barrier();                                        // the state operands are used up; the next delta sums are in LDS
            if (chunk + 1 < c_last) {
                mask_early(chunk + 1, nxt);
                park_state_operands(nxt, buf ^ 1);
            }
            lds_barrier();                                        // the chunk's LDS tiles are free again
        };
        for (int chunk = c_first; chunk < c_last; chunk += 2) {
            walk(chunk, E2[0], E2[1]);
            if (chunk + 1 < c_last) walk(chunk + 1, E2[1], E2[0]);
        }
    }

    // end of the segment: pass 1 leaves the local end state and the sum of deltas, pass 2 the final state
    float *dst = nullptr;
    if (!PASS2) dst = ws_state + (((int64_t)b * n_slots + seg + 1) * D + h * kP) * N;
    else if (h_final && seg == n_seg - 1) dst = h_final + (b * D + h * kP) * N;
    if (dst && !role_y) {
#pragma unroll
        for (int j = 0; j < PPW; ++j) {
            const int id = sw * PPW + j, pt = id & 1, nt = id >> 1;
#pragma unroll
            for (int g = 0; g < 4; ++g)
                *reinterpret_cast<float4 *>(dst + (int64_t)(pt * 32 + r) * N + nt * 32 + 8 * g + 4 * up) =
                    make_float4(acc[j][4 * g], acc[j][4 * g + 1], acc[j][4 * g + 2], acc[j][4 * g + 3]);
        }
    }
    if (!PASS2 && scan_wave) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) seg_sum += __shfl_xor(seg_sum, off, 64);
        ws_sumdt[((int64_t)b * n_slots + seg) * D + h * kP + lane] = seg_sum;   // kP == 64 lanes
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
    // the state is touched once per step: streaming accesses, as in the selective step
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const f32x4 hraw = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(h_in) + (p_ok ? p : 0) * row4 + f);
    float4 hv = make_float4(hraw.x, hraw.y, hraw.z, hraw.w);
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
    f32x4 hst;
    hst.x = hv.x; hst.y = hv.y; hst.z = hv.z; hst.w = hv.w;
    __builtin_nontemporal_store(hst, reinterpret_cast<f32x4 *>(h_out) + j * row4 + f);
    if (q == 0) {
        y = fmaf(Dskip ? Dskip[hh] : 0.0f, xv, y);
        if (z) y *= silu_f32(ld_io(z, j * H * P + d));
        st_io(out, j * H * P + d, y);
    }
}

int64_t chunks_of(int64_t L) { return (L + kLc - 1) / kLc; }

// Segments.  Pass 2: about one workgroup per CU (a workgroup holds most of a CU's LDS), never more than
// chunks.  Pass 1 cuts every such segment in two when its length is even: its workgroups are small, and two
// on a CU hide each other's waits.  chunks1 / n_seg1 describe pass 1 (and the state slots: n_seg1 + 1),
// chunks2 / n_seg2 pass 2.
struct SsdPlan {
    int chunks1, n_seg1, chunks2, n_seg2;
};
SsdPlan ssd_plan(int64_t batch, int64_t L, int64_t H)
{
    const int64_t nc = chunks_of(L);
    int64_t want = 256 / (batch * H > 0 ? batch * H : 1);
    if (want < 1) want = 1;
    if (want > nc) want = nc;
    int64_t cps = (nc + want - 1) / want;
    if (cps > 1 && cps % 2) ++cps;
    SsdPlan p;
    p.chunks2 = (int)cps;
    p.n_seg2 = (int)((nc + cps - 1) / cps);
    p.chunks1 = (cps % 2 || p.n_seg2 == 1) ? (int)cps : (int)(cps / 2);   // one segment: it starts from h0, no first pass
    p.n_seg1 = (int)((nc + p.chunks1 - 1) / p.chunks1);
    return p;
}

}  // namespace

size_t ssd_workspace_bytes(int64_t batch, int64_t L, int64_t H, int64_t P, int64_t N)
{
    const SsdPlan p = ssd_plan(batch, L, H);
    const int64_t slots = p.n_seg1 + 1, D = H * P;
    return (size_t)(batch * slots * D * (N + 1) + D * N) * sizeof(float);
}

hipError_t launch_ssd(const SsdArgs &a, hipStream_t stream)
{
    const SsdPlan p = ssd_plan(a.batch, a.L, a.H);
    const int nc = (int)chunks_of(a.L);
    const int n_slots = p.n_seg1 + 1, slot_step = p.chunks2 / p.chunks1;
    const int64_t D = a.H * a.P;
    float *ws_state = a.ws;
    float *ws_sumdt = ws_state + (size_t)a.batch * n_slots * D * a.N;
    float *a_rows = ws_sumdt + (size_t)a.batch * n_slots * D;
    const bf16_t *x = static_cast<const bf16_t *>(a.x), *dt = static_cast<const bf16_t *>(a.dt);
    const bf16_t *Bm = static_cast<const bf16_t *>(a.Bm), *Cm = static_cast<const bf16_t *>(a.Cm);
    const bf16_t *z = static_cast<const bf16_t *>(a.z);
    bf16_t *out = static_cast<bf16_t *>(a.out);
#define MAMBA_SSD(NN, P2, HZ)                                                                                       \
    ssd_segment<NN, P2, HZ><<<dim3((unsigned)((P2) ? p.n_seg2 : p.n_seg1), (unsigned)a.H, (unsigned)a.batch),        \
                              (P2) ? 2 * kThreads : kThreads, 0, stream>>>(                                         \
        x, dt, a.A, Bm, Cm, a.Dskip, z, a.dt_bias, ws_state, ws_sumdt, a_rows, out, a.h_final, a.L, a.H,             \
        (P2) ? p.chunks2 : p.chunks1, (P2) ? p.n_seg2 : p.n_seg1, n_slots, slot_step, nc, a.dt_softplus)
    if (p.n_seg1 > 1) {
        if (a.N == 64) MAMBA_SSD(64, false, false);
        else MAMBA_SSD(128, false, false);
        if (hipError_t e = launch_chunk_carry(a_rows, a.h0, ws_state, ws_sumdt, a.batch, D, a.N, n_slots, stream)) return e;
    } else {
        // a single segment starts from h0 itself: slot 0 <- h0 (or zeros)
        for (int64_t b = 0; b < a.batch; ++b)
            if (hipError_t e = launch_copy_state(a.h0 ? a.h0 + b * D * a.N : nullptr, ws_state + (size_t)b * n_slots * D * a.N, D * a.N, stream))
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
