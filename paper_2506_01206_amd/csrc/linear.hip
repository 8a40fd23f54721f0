// Dense projections of the Mamba block (in_proj, x_proj, dt_proj, out_proj of the Mamba-130M
// drafter the paper uses, Sec. 3.1) on the gfx950 matrix cores.
//
//   out[m, n] = sum_k x[m, k] * w[n, k]  (+ bias[n]) (+ residual[m, n])
//
// x: (M, K) bf16, w: (N, K) bf16 (one row per output feature, K contiguous in both operands, which
// is the order MFMA operands want), fp32 accumulation, bf16 output.  The N output columns may be
// split over up to three contiguous output tensors (in_proj -> x | z; x_proj -> dt_low | B | C), so
// that the consumers get the dense (tokens, features) tensors they expect without a copy.
//
// Tiling: a workgroup of 4 wavefronts (2 x 2) owns a BM x BN output tile (128 x 128, or 64 x 128 or
// 64 x 64 when that is needed to give every CU a few workgroups); each wavefront a (BM/2) x (BN/2) part as
// MFMA tiles of v_mfma_f32_32x32x16_bf16.  K is walked in slabs of BK = 64: the x and w slabs are
// fetched with 16-byte loads one slab ahead into registers, parked in LDS (rows padded by 16 B)
// and read back as MFMA fragments with 16-byte LDS reads: lane l holds row l % 32,
// k = 8 * (l / 32) .. + 7 of each k16 step.  Three resident workgroups per CU hide the latencies.  (Larger
// tiles on this scheme, with its register staging and full barriers, measured slower; long contexts
// take the 256-row tiles of linear_wide_kernel below, which is built differently.)
// Rows past M or N re-read the last valid row and are never stored; a K tail is zero-filled.
// Epilogue: the accumulators (+ bias) are rounded to bf16 into LDS, then leave as 16-byte row
// chunks (+ residual), so that stores are coalesced; output splits that are not multiples of 8
// columns take an element-wise path.
#include <type_traits>

#include "device_math.h"
#include "launch.h"

namespace mamba {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;

// barrier that orders LDS traffic only: global loads in flight stay in flight
__device__ __forceinline__ void lds_barrier_linear()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// tile counts from which each kernel shape takes over (measured crossovers, see launch_linear)
constexpr int64_t kTilesBig = 512, kTilesMid = 512, kTilesWide = 96, kTilesWideSmall = 192, kTilesWideSmallMax = 512,
                  kTilesDeep = 513;

struct OutSplit {
    bf16_t *ptr[3];
    int64_t width[3];
};

// one step of the depthwise causal conv + SiLU applied to the first output tensor on its way out
struct ConvTail {
    const float *w, *bias;      // (channels, k), (channels) or nullptr; w == nullptr: no conv
    const bf16_t *src;          // (rows_in, channels, k - 1) carried windows
    bf16_t *dst;                // (M, channels, k - 1)
    const int32_t *parent;      // row m continues from src[parent[m]]; nullptr: src[m]
    int64_t n_in;
    int k;
};

// the next projection applied to the first output tensor on its way out, as partial sums per column block
struct XprojTail {
    const bf16_t *w;            // (n, ldw) bf16; nullptr: off
    float *part;                // (M, n, column blocks of the first output tensor)
    int n;
    int64_t ldw;                // row length of w = width of the first output tensor
};

// column n of the virtual (M, N) output -> tensor and column inside it
__device__ __forceinline__ int locate(const OutSplit &o, int64_t n, int64_t *col)
{
    int64_t c = n;
    int s = 0;
    if (c >= o.width[0]) { c -= o.width[0]; s = 1; if (c >= o.width[1]) { c -= o.width[1]; s = 2; } }
    *col = c;
    return s;
}

// grid: (ceil(N / BN), ceil(M / BM)).  WSTREAM: w is read once and is large (the LM head on a draft position): its
// loads are streaming, so that they do not push the blocks' weights, which the next position reads again, out of
// the last-level cache.
template <int BM, int BN, int BK, bool WSTREAM = false>
__global__ void __launch_bounds__(kThreads)
linear_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ w, const float *__restrict__ bias,
              const bf16_t *residual, OutSplit out, int64_t M, int64_t N, int64_t K, int vector_out)
{
    constexpr int MT = BM / 64, NT = BN / 64;                 // 32 x 32 MFMA tiles per wavefront along m, n
    constexpr int kBN = BN, kBK = BK;
    constexpr int kStageCols = BN < 128 ? BN : 128;           // the output tile is staged at most 128 columns at a time
    constexpr int kOutRowBytes = kStageCols * 2 + 16;
    constexpr int kRowBytes = BK * 2 + 16;                    // data + 16 B pad against bank conflicts
    constexpr int kOperandBytes = (BM + kBN) * kRowBytes;
    constexpr int kStageBytes = BM * kOutRowBytes;
    constexpr int kLdsBytes = kOperandBytes > kStageBytes ? kOperandBytes : kStageBytes;
    __shared__ __attribute__((aligned(16))) unsigned char lds[kLdsBytes];
    unsigned char *lds_x = lds, *lds_w = lds + BM * kRowBytes;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t m0 = (int64_t)blockIdx.y * BM, n0 = (int64_t)blockIdx.x * kBN;

    // global -> LDS staging: (BM + BN) rows x BK/8 chunks of 16 B, NCH chunks per thread
    constexpr int kCpr = BK / 8;                              // chunks per row
    constexpr int NCH = (BM + kBN) * kCpr / kThreads;
    const uint4 *src[NCH];
    int dst_off[NCH], chunk[NCH];
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int c = tid + i * kThreads;
        const int row = c / kCpr;                             // 0 .. BM + BN - 1: x rows first, then w rows
        chunk[i] = c % kCpr;
        if (row < BM) {
            int64_t r = m0 + row;
            r = r < M ? r : M - 1;
            src[i] = reinterpret_cast<const uint4 *>(x + r * K);
        } else {
            int64_t r = n0 + (row - BM);
            r = r < N ? r : N - 1;
            src[i] = reinterpret_cast<const uint4 *>(w + r * K);
        }
        dst_off[i] = row * kRowBytes + chunk[i] * 16;
    }
    const int64_t kchunks = K / 8;                            // K is a multiple of 8 (checked on the host)
    uint4 regs[NCH];
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int64_t ch = k0 / 8 + chunk[i];
            if (WSTREAM && i * kThreads >= BM * kCpr) {         // chunks of w rows (whole multiples of the block: BM * kCpr % kThreads == 0)
                const u32x4 t = ch < kchunks ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src[i] + ch)) : u32x4(0u);
                regs[i] = make_uint4(t.x, t.y, t.z, t.w);
            } else {
                regs[i] = ch < kchunks ? src[i][ch] : make_uint4(0, 0, 0, 0);
            }
        }
    };
    auto park = [&]() {
#pragma unroll
        for (int i = 0; i < NCH; ++i) *reinterpret_cast<uint4 *>(lds + dst_off[i]) = regs[i];
    };

    f32x16 acc[MT][NT];
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int b = 0; b < NT; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;

    const int frag_row = lane & 31, frag_k = (lane >> 5) * 16;    // byte offset of the lane's 8 k values
    fetch(0);
    for (int64_t k0 = 0; k0 < K; k0 += kBK) {
        __syncthreads();                                          // everyone is done reading the last slab
        park();
        __syncthreads();
        if (k0 + kBK < K) fetch(k0 + kBK);                        // in flight while this slab is multiplied
#pragma unroll
        for (int ks = 0; ks < kBK / 16; ++ks) {
            bf16x8 af[MT], bfr[NT];
#pragma unroll
            for (int t = 0; t < MT; ++t)
                af[t] = *reinterpret_cast<const bf16x8 *>(lds_x + (wm * (BM / 2) + t * 32 + frag_row) * kRowBytes + ks * 32 + frag_k);
#pragma unroll
            for (int t = 0; t < NT; ++t)
                bfr[t] = *reinterpret_cast<const bf16x8 *>(lds_w + (wn * (BN / 2) + t * 32 + frag_row) * kRowBytes + ks * 32 + frag_k);
#pragma unroll
            for (int a = 0; a < MT; ++a)
#pragma unroll
                for (int b = 0; b < NT; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bfr[b], acc[a][b], 0, 0, 0);
        }
    }

    // epilogue.  acc[a][b][i] is C[8 * (i / 4) + 4 * (lane / 32) + i % 4][lane % 32] of its 32 x 32 tile.
    // The tile leaves through LDS 128 columns at a time.
#pragma unroll
    for (int half = 0; half < BN / kStageCols; ++half) {
        __syncthreads();                                          // LDS (operands or the last half) is free
#pragma unroll
        for (int a = 0; a < MT; ++a)
#pragma unroll
            for (int b = 0; b < NT; ++b) {
                const int tile_col = wn * (BN / 2) + b * 32;      // column of this MFMA tile in the BN-wide tile
                if (tile_col / kStageCols != half) continue;      // compile-time per (wn is uniform per wavefront)
                const int col = tile_col - half * kStageCols + (lane & 31);
                const int64_t n = n0 + half * kStageCols + col;
                const float bv = (bias && n < N) ? bias[n] : 0.0f;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int row = wm * (BM / 2) + a * 32 + 8 * (i / 4) + 4 * (lane >> 5) + (i & 3);
                    *reinterpret_cast<uint16_t *>(lds + row * kOutRowBytes + col * 2) = (uint16_t)f32_to_bf16(acc[a][b][i] + bv);
                }
            }
        __syncthreads();
        const int64_t nh = n0 + half * kStageCols;
        if (vector_out) {
            // every output width is a multiple of 8 columns: 16-byte chunks never straddle two tensors
            constexpr int kChunks = BM * (kStageCols / 8);
#pragma unroll
            for (int c = tid; c < kChunks; c += kThreads) {
                const int row = c / (kStageCols / 8), cc = c % (kStageCols / 8);
                const int64_t m = m0 + row, n = nh + cc * 8;
                if (m >= M || n >= N) continue;
                uint4 v = *reinterpret_cast<const uint4 *>(lds + row * kOutRowBytes + cc * 16);
                int64_t col;
                const int s = locate(out, n, &col);
                const int64_t off = m * out.width[s] + col;
                if (residual) {
                    const uint4 r = *reinterpret_cast<const uint4 *>(residual + off);   // single output: same offset
                    v.x = f32x2_to_bf16x2(bf16_lo(v.x) + bf16_lo(r.x), bf16_hi(v.x) + bf16_hi(r.x));
                    v.y = f32x2_to_bf16x2(bf16_lo(v.y) + bf16_lo(r.y), bf16_hi(v.y) + bf16_hi(r.y));
                    v.z = f32x2_to_bf16x2(bf16_lo(v.z) + bf16_lo(r.z), bf16_hi(v.z) + bf16_hi(r.z));
                    v.w = f32x2_to_bf16x2(bf16_lo(v.w) + bf16_lo(r.w), bf16_hi(v.w) + bf16_hi(r.w));
                }
                *reinterpret_cast<uint4 *>(out.ptr[s] + off) = v;
            }
        } else {
            for (int e = tid; e < BM * kStageCols; e += kThreads) {
                const int row = e / kStageCols, cl = e % kStageCols;
                const int64_t m = m0 + row, n = nh + cl;
                if (m >= M || n >= N) continue;
                float v = bf16_to_f32(*reinterpret_cast<const uint16_t *>(lds + row * kOutRowBytes + cl * 2));
                int64_t col;
                const int s = locate(out, n, &col);
                const int64_t off = m * out.width[s] + col;
                if (residual) v += bf16_to_f32(residual[off]);
                out.ptr[s][off] = (bf16_t)f32_to_bf16(v);
            }
        }
    }
}


// ---------------------------------------------------------------------------------------------------
// Many rows (the projections of a long context).  A 128 x 128 tile asks the L1 for 512 bytes per k and
// multiplies 8 cycles per k on every SIMD, so the cache, which delivers 64 bytes a cycle, can feed the
// matrix cores half the time at best.  This kernel takes 256 x 256 (or 256 x 128) tiles, one workgroup
// per CU and one wavefront per SIMD, each wavefront a 128 x 128 (128 x 64) part held in 256 (128)
// accumulator registers: per k the same 8 (6) cycles of cache traffic now feed 32 (16) cycles of MFMA.
// (With BM = 128 it also runs 128 x 128 tiles, two workgroups to a CU, for products too small to give every CU
// a 256-row tile: the feeding scheme below, not the tile size, is what those gain from.)
//
// Operands go from memory straight into LDS (global_load_lds_dwordx4: lane l of a wavefront lands at
// M0 + 16 l, so one instruction fills eight 128-byte rows): no staging registers, and none of the LDS
// write instructions whose data path the counters showed full when the slabs were parked from registers.
// Rows lie 128 bytes apart without padding; the 16-byte slot c of row r sits at slot c ^ ((r >> 1) & 7), chosen
// on the memory side of the load, which makes the fragment reads (32 rows, one slot each) conflict-free.
// The instruction is issued from inline assembly so that the compiler's wait-count pass does not see an LDS
// write it cannot place (it would wait for every load in flight before each LDS read); the waits are explicit:
// vmcnt(0) before the one barrier per slab.  Slabs of 64 k alternate between two stages.  The barrier of
// slab s comes when its last fragments have been read, a quarter before its end; slab s + 2 is requested
// right after it into the stage just freed and has a whole slab of multiplications to arrive.
// The product is formed transposed (w fragments as the row operand), so that a lane's four accumulators
// of a group are four adjacent output columns of one row and leave as one 8-byte write.
// Requires M % 256 == 0, N % BN == 0, K % 128 == 0 and output widths that are multiples of 8.
// grid: 8 * ceil(tiles / 8) workgroups; consecutive workgroups go to different XCDs, so tile numbers are
// dealt such that each XCD (each L2) works on a contiguous range of tiles, column tiles of one row block
// adjacent.
constexpr int kWideBM = 256, kWideBK = 64, kWideRow = kWideBK * 2;

// 16 bytes per lane from base + lane_off into LDS at lds_addr + 16 * lane (lds_addr wave-uniform)
__device__ __forceinline__ void load_to_lds16(const char *base, uint32_t lane_off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(lane_off), "s"(base) : "memory");
}

template <int BM, int BN>
__global__ void __launch_bounds__(256)
linear_wide_kernel(const bf16_t *x, const bf16_t *w, const float *__restrict__ bias, const bf16_t *residual,
                   OutSplit out, int64_t M, int64_t N, int64_t K, int tiles_n, int n_tiles)
{
    constexpr int MT = BM / 64, NT = BN / 64;                     // 32 x 32 MFMA tiles per wavefront along m and n
    constexpr int kRows = BM + BN;
    constexpr int kStage = kRows * kWideRow;
    constexpr int kOutRow = BN * 2 + 16;
    constexpr int kLds = 2 * kStage > BM * kOutRow ? 2 * kStage : BM * kOutRow;
    __shared__ __attribute__((aligned(1024))) unsigned char lds[kLds];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;

    const int per_xcd = (n_tiles + 7) / 8;
    const int tile = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if (tile >= n_tiles) return;
    const int64_t m0 = (int64_t)(tile / tiles_n) * BM, n0 = (int64_t)(tile % tiles_n) * BN;

    // Loads: wavefront v takes the row groups g = 4 j + v (rows 8 g .. 8 g + 7 of the stage; x rows first, then w);
    // lane l lands in row 8 g + l / 8, slot l % 8, and therefore fetches slot (l % 8) ^ ((4 (g & 1) + l / 16) & 7)
    // of that row (g & 1 == v & 1).
    constexpr int NLX = BM / 32, NLW = BN / 32;              // loads per wavefront and slab
    const uint32_t lane_off = (uint32_t)((lane >> 3) * K * 2 + (((lane & 7) ^ ((4 * (wave & 1) + (lane >> 4)) & 7)) << 4));
    const char *xrow = reinterpret_cast<const char *>(x + (m0 + 8 * wave) * K);
    const char *wrow = reinterpret_cast<const char *>(w + (n0 + 8 * wave) * K);
    const int64_t rows32 = 64 * K;                                 // bytes between rows 32 apart
    const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) unsigned char *)lds;
    // loads [first, last) of the slab at k0 into the stage at byte `stage`
    auto request = [&](int64_t k0, int stage, auto first, auto last) __attribute__((always_inline)) {
#pragma unroll
        for (int i = decltype(first)::value; i < decltype(last)::value; ++i) {
            const char *base = i < NLX ? xrow + (i * rows32 + 2 * k0) : wrow + ((i - NLX) * rows32 + 2 * k0);
            load_to_lds16(base, lane_off, lds0 + stage + (i < NLX ? 0 : BM * kWideRow) + wave * 1024 + (i < NLX ? i : i - NLX) * 4096);
        }
    };
    typedef std::integral_constant<int, 0> L0;
    typedef std::integral_constant<int, (NLX + NLW) / 4> L1;
    typedef std::integral_constant<int, (NLX + NLW) / 2> L2;
    typedef std::integral_constant<int, 3 * (NLX + NLW) / 4> L3;
    typedef std::integral_constant<int, NLX + NLW> L4;

    f32x16 acc[MT][NT];
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int b = 0; b < NT; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;

    // fragment of k16 step ks: row lane % 32 of a 32-row block, slot (2 ks + lane / 32) ^ ((lane >> 1) & 7)
    int frag_x[4], frag_w[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        const int slot = ((2 * ks + (lane >> 5)) ^ ((lane >> 1) & 7)) << 4;
        frag_x[ks] = (wm * (BM / 2) + (lane & 31)) * kWideRow + slot;
        frag_w[ks] = (BM + wn * (BN / 2) + (lane & 31)) * kWideRow + slot;
    }
    struct Frags { bf16x8 xf[MT], wf[NT]; };
    auto load_x = [&](const unsigned char *stage, int ks, Frags &f, int t) __attribute__((always_inline)) {
        f.xf[t] = *reinterpret_cast<const bf16x8 *>(stage + frag_x[ks] + t * 32 * kWideRow);
    };
    auto load_w = [&](const unsigned char *stage, int ks, Frags &f, int t) __attribute__((always_inline)) {
        f.wf[t] = *reinterpret_cast<const bf16x8 *>(stage + frag_w[ks] + t * 32 * kWideRow);
    };
    auto load_frags = [&](const unsigned char *stage, int ks, Frags &f) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < MT; ++t) load_x(stage, ks, f, t);
#pragma unroll
        for (int t = 0; t < NT; ++t) load_w(stage, ks, f, t);
    };
    auto multiply_row = [&](const Frags &f, int a) __attribute__((always_inline)) {
#pragma unroll
        for (int b = 0; b < NT; ++b)
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.wf[b], f.xf[a], acc[a][b], 0, 0, 0);
    };
    auto multiply = [&](const Frags &f) __attribute__((always_inline)) {
#pragma unroll
        for (int a = 0; a < MT; ++a) multiply_row(f, a);
    };
    // Slab s, read from stage s % 2, whose first fragments are already in f0.  Four quarters of MT NT MFMAs; the
    // fragments of a quarter are read during the one before it (the instruction groups keep the scheduler from
    // moving the reads next to their use).  After the third quarter every read of this stage has been issued: the
    // slab s + 1 must have landed by then (requested a slab ago), the barrier publishes it, the stage of slab s is
    // free, and the last quarter requests slab s + 2 into it (REQUEST) and reads the first fragments of slab s + 1
    // (NEXT) between its multiplications.
    Frags f0, f1;
    auto slab = [&](auto parity, int64_t k_next, auto do_request, auto do_next) __attribute__((always_inline)) {
        constexpr int P = decltype(parity)::value;
        constexpr bool REQUEST = decltype(do_request)::value, NEXT = decltype(do_next)::value;
        const unsigned char *cur = lds + P * kStage;
        const unsigned char *nxt = lds + (1 - P) * kStage;
/* one fragment read per two MFMAs */
#define MAMBA_WIDE_SPREAD __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); __builtin_amdgcn_sched_group_barrier(0x008, NT / 2, 0);
#define MAMBA_WIDE_QUARTER(KS, FA, FB)                                                                                \
        load_frags(cur, KS, FB);                                                                                      \
        multiply(FA);                                                                                                 \
        MAMBA_WIDE_SPREAD MAMBA_WIDE_SPREAD                                                                           \
        if constexpr (MT == 4) { MAMBA_WIDE_SPREAD MAMBA_WIDE_SPREAD }                                                \
        __builtin_amdgcn_sched_group_barrier(0x100, NT, 0);                                                           \
        __builtin_amdgcn_sched_group_barrier(0x008, MT * NT / 2, 0);                                                  \
        __builtin_amdgcn_sched_barrier(0);
        MAMBA_WIDE_QUARTER(1, f0, f1)
        MAMBA_WIDE_QUARTER(2, f1, f0)
        MAMBA_WIDE_QUARTER(3, f0, f1)
#undef MAMBA_WIDE_QUARTER
#undef MAMBA_WIDE_SPREAD
        __builtin_amdgcn_s_waitcnt(0x0F70);                       // vmcnt(0): this wavefront's part of slab s + 1 is in LDS
        lds_barrier_linear();
#define MAMBA_WIDE_LAST(A, FROM, TO)                                                                                  \
        if constexpr (REQUEST) request(k_next, P * kStage, FROM(), TO());                                             \
        if constexpr (NEXT) {                                                                                         \
            if constexpr (A < MT) load_x(nxt, 0, f0, A);                                                              \
            if constexpr (A < NT) load_w(nxt, 0, f0, A);                                                              \
        }                                                                                                             \
        if constexpr (A < MT) multiply_row(f1, A);                                                                    \
        __builtin_amdgcn_sched_barrier(0);
        MAMBA_WIDE_LAST(0, L0, L1)
        MAMBA_WIDE_LAST(1, L1, L2)
        MAMBA_WIDE_LAST(2, L2, L3)
        MAMBA_WIDE_LAST(3, L3, L4)
#undef MAMBA_WIDE_LAST
    };
    typedef std::integral_constant<int, 0> Even;
    typedef std::integral_constant<int, 1> Odd;
    const int S = (int)(K / kWideBK);
    request(0, 0, L0(), L4());
    request(kWideBK, kStage, L0(), L4());
    // vmcnt(loads of one slab): slab 0 is in, slab 1 may be under way (vmcnt is split over bits 3:0 and 15:14)
    __builtin_amdgcn_s_waitcnt(0x0F70 | ((NLX + NLW) & 15) | (((NLX + NLW) >> 4) << 14));
    lds_barrier_linear();
    load_frags(lds, 0, f0);
    int s = 0;
    for (; s + 2 < S; s += 2) {
        slab(Even(), (int64_t)(s + 2) * kWideBK, std::true_type(), std::true_type());
        slab(Odd(), (int64_t)(s + 3) * kWideBK, std::true_type(), std::true_type());
    }
    slab(Even(), 0, std::false_type(), std::true_type());         // S is even: two slabs left, nothing more to request
    slab(Odd(), 0, std::false_type(), std::false_type());
    // Epilogue.  The residual chunks this thread will add are requested first, all at once: with one workgroup per
    // CU nothing else would hide their latency, and fetched four at a time inside the store loop they cost a third
    // of the tile's time.
    constexpr int kCpr = BN / 8, kChunks = BM * kCpr / 256;
    u32x4 res[kChunks];
    if (residual) {
#pragma unroll
        for (int i = 0; i < kChunks; ++i) {
            const int c = tid + i * 256, row = c / kCpr, cc = c % kCpr;
            int64_t col;
            const int sp = locate(out, n0 + cc * 8, &col);
            res[i] = *reinterpret_cast<const u32x4 *>(residual + (m0 + row) * out.width[sp] + col);
        }
    }
    lds_barrier_linear();                                         // the stages are free for the output tile (the requests stay in flight)

    // acc[a][b][4 g + j] is C[m = 32 a + lane % 32][n = 32 b + 8 g + 4 (lane / 32) + j] of the wavefront's part
#pragma unroll
    for (int b = 0; b < NT; ++b)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int nl = wn * (BN / 2) + b * 32 + 8 * g + 4 * (lane >> 5);
            float4 bv = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (bias) bv = *reinterpret_cast<const float4 *>(bias + n0 + nl);
#pragma unroll
            for (int a = 0; a < MT; ++a) {
                const int ml = wm * (BM / 2) + a * 32 + (lane & 31);
                uint2 v;
                v.x = f32x2_to_bf16x2(acc[a][b][4 * g + 0] + bv.x, acc[a][b][4 * g + 1] + bv.y);
                v.y = f32x2_to_bf16x2(acc[a][b][4 * g + 2] + bv.z, acc[a][b][4 * g + 3] + bv.w);
                *reinterpret_cast<uint2 *>(lds + ml * kOutRow + nl * 2) = v;
            }
            __builtin_amdgcn_sched_barrier(0);                    // one group at a time: the accumulators stay where they are until used
        }
    lds_barrier_linear();
#pragma unroll
    for (int i = 0; i < kChunks; ++i) {
        const int c = tid + i * 256, row = c / kCpr, cc = c % kCpr;
        uint4 v = *reinterpret_cast<const uint4 *>(lds + row * kOutRow + cc * 16);
        int64_t col;
        const int sp = locate(out, n0 + cc * 8, &col);
        const int64_t off = (m0 + row) * out.width[sp] + col;
        if (residual) {
            const u32x4 r = res[i];
            v.x = f32x2_to_bf16x2(bf16_lo(v.x) + bf16_lo(r.x), bf16_hi(v.x) + bf16_hi(r.x));
            v.y = f32x2_to_bf16x2(bf16_lo(v.y) + bf16_lo(r.y), bf16_hi(v.y) + bf16_hi(r.y));
            v.z = f32x2_to_bf16x2(bf16_lo(v.z) + bf16_lo(r.z), bf16_hi(v.z) + bf16_hi(r.z));
            v.w = f32x2_to_bf16x2(bf16_lo(v.w) + bf16_lo(r.w), bf16_hi(v.w) + bf16_hi(r.w));
        }
        *reinterpret_cast<uint4 *>(out.ptr[sp] + off) = v;
    }
}

// ---------------------------------------------------------------------------------------------------
// Few rows (M <= 64: the branches of one draft position, Sec. 4.1).  The product is then bound by
// reading w once and by latency, so the work is cut finely: one workgroup per 32 output columns,
// its NW wavefronts take the 64-wide k blocks of the row round robin and their partial 32 x 32 tiles
// are added through LDS.  A wavefront fetches a k block of 32 rows x 128 bytes with four 16-byte
// loads per lane, eight lanes on one row, so that every load instruction covers whole 128-byte
// lines; the block then goes through a 4 KiB LDS patch private to the wavefront (16-byte slots
// xor-swizzled by the row, conflict-free both ways) and comes back as MFMA fragments: lane (r, h)
// takes the slots 4 h .. 4 h + 3 of row r, one per k16 step.  Both operands use the same slot
// order, so the sum over k is complete.  (Run over a grid of row blocks for more rows with a long k loop and
// few output tiles it measured slower than the tiled kernel with 256-deep slabs: x_proj 10.4 vs 10.5 us,
// out_proj 30 vs 17 us on 2048 tokens.)
// grid: (ceil(N / 32), ceil(M / (32 MB)))
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int NW, int MB>
__global__ void __launch_bounds__(NW * 64)
linear_skinny_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ w, const float *__restrict__ bias,
                     const bf16_t *residual, OutSplit out, int64_t M, int64_t N, int64_t K,
                     const float *__restrict__ norm_w, float eps, ConvTail conv, XprojTail xp)
{
    // LDS: in the main loop two 4 KiB patches per wavefront (w block, x block); afterwards the same
    // memory holds the partial tiles, the sums of x^2 (with norm_w) and the row factors
    __shared__ __attribute__((aligned(16))) unsigned char lds[NW * 8192];
    float (*part)[16][64] = reinterpret_cast<float (*)[16][64]>(lds);
    float (*ssq)[MB][4][64] = reinterpret_cast<float (*)[MB][4][64]>(lds + NW * 4096);
    float *row_scale = reinterpret_cast<float *>(lds + NW * 4096 + NW * MB * 1024);
    static_assert(NW * 4096 + NW * MB * 1024 + 128 <= NW * 8192, "LDS reuse");
    // with eight wavefronts there is room for the finished columns of the first output (float32), which the
    // projection tail multiplies on
    constexpr bool kTailRoom = NW * 4096 + NW * MB * 1024 + 128 + MB * 4096 <= NW * 8192;
    float (*xc)[32][32] = reinterpret_cast<float (*)[32][32]>(lds + NW * 4096 + NW * MB * 1024 + 128);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 31, h = lane >> 5;                       // fragment view: row, k half
    const int lrow = lane >> 3, lch = lane & 7;                   // load view: row (+ 8 i), 16-byte slot
    const int64_t n0 = (int64_t)blockIdx.x * 32, m0 = (int64_t)blockIdx.y * (32 * MB);
    const int64_t kchunks = K / 8, kblocks = (K + 63) / 64;
    uint4 *patch_w = reinterpret_cast<uint4 *>(lds + wave * 8192), *patch_x = patch_w + 256;
    const int put = lrow * 8 + (lch ^ lrow);                      // + 64 i: slot of row lrow + 8 i ((lrow + 8 i) & 7 == lrow)
    int get[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) get[s] = r * 8 + ((4 * h + s) ^ (r & 7));

    const uint4 *wptr[4];
    const uint4 *xptr[MB][4];
    bool xlive[MB][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int64_t wr = n0 + lrow + 8 * i;
        wr = wr < N ? wr : N - 1;                                 // columns past N repeat the last one, never stored
        wptr[i] = reinterpret_cast<const uint4 *>(w + wr * K);
#pragma unroll
        for (int b = 0; b < MB; ++b) {
            const int64_t m = m0 + b * 32 + lrow + 8 * i;
            xlive[b][i] = m < M;                                  // rows past M stay zero
            xptr[b][i] = reinterpret_cast<const uint4 *>(x + (xlive[b][i] ? m : 0) * K);
        }
    }
    f32x16 acc[MB];
#pragma unroll
    for (int b = 0; b < MB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[b][i] = 0.0f;
    float ss[MB][4];
#pragma unroll
    for (int b = 0; b < MB; ++b)
#pragma unroll
        for (int i = 0; i < 4; ++i) ss[b][i] = 0.0f;

    // What an output element needs besides the sums: bias, residual, and for the conv tail the carried
    // window (through the parent index), the taps and the conv bias.  With one row block these loads
    // are issued ahead of and inside the main loop, so that the epilogue does not wait for them: first what needs no
    // parent index, and the index itself; then, once the first group of the main loop's loads is on its way, the
    // window behind the index.  No fetch is used where it is issued (a value converted, selected or compared there
    // is waited for there, one memory latency each): raw bits are kept, taps and window entries a short conv does not
    // have re-read the last one and are dropped at use, and the width and pointer of an output tensor are picked
    // from values held in registers (indexing the argument struct by a per-lane number goes through memory).
    struct Tail {
        float bias, cb, wk[4];
        uint16_t res, carried[3];
        int32_t parent;
    };
    int64_t ow0 = out.width[0], ow1 = out.width[1], ow2 = out.width[2];
    bf16_t *op0 = out.ptr[0], *op1 = out.ptr[1], *op2 = out.ptr[2];
    asm volatile("" : "+s"(ow0), "+s"(ow1), "+s"(ow2), "+s"(op0), "+s"(op1), "+s"(op2));
    auto locate_tail = [&](int64_t n, int64_t *col, int64_t *width, bf16_t **ptr) {
        int64_t c = n, wd = ow0;
        bf16_t *pt = op0;
        int sp = 0;
        if (c >= ow0) {
            c -= ow0; sp = 1; wd = ow1; pt = op1;
            if (c >= ow1) { c -= ow1; sp = 2; wd = ow2; pt = op2; }
        }
        *col = c; *width = wd; *ptr = pt;
        return sp;
    };
    constexpr int OPT = 16 * 64 / (NW * 64);                      // outputs per thread and row block
    auto tail_first = [&](int b, int j, Tail &t) {
        t.bias = t.cb = 0.0f;
        t.res = 0;
        t.parent = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) t.wk[k] = 0.0f;
#pragma unroll
        for (int k = 0; k < 3; ++k) t.carried[k] = 0;
        const int o = tid + j * NW * 64, i = o >> 6, l = o & 63;
        const int64_t m = m0 + b * 32 + 8 * (i >> 2) + 4 * (l >> 5) + (i & 3), n = n0 + (l & 31);
        if (m >= M || n >= N) return;
        if (bias) t.bias = bias[n];
        int64_t col, width;
        bf16_t *ptr;
        const int sp = locate_tail(n, &col, &width, &ptr);
        if (residual) t.res = residual[m * width + col];
        if (conv.w && sp == 0 && conv.parent) t.parent = conv.parent[m];
    };
    // (all parent indices are turned into addresses before the first window fetch: the wait for an index also
    // waits for every fetch issued before it)
    struct WinAddr {
        int64_t win, col;                                         // window's first element in conv.src; channel
        bool on;
    };
    auto tail_address = [&](int b, int j, const Tail &t) {
        WinAddr a;
        const int o = tid + j * NW * 64, i = o >> 6, l = o & 63;
        const int64_t m = m0 + b * 32 + 8 * (i >> 2) + 4 * (l >> 5) + (i & 3), n = n0 + (l & 31);
        a.on = !(m >= M || n >= N || !conv.w || n >= ow0);
        a.col = a.on ? n : 0;
        const int64_t p = conv.parent ? (int64_t)t.parent : m;
        const bool p_ok = !conv.parent || (p >= 0 && p < conv.n_in);
        a.win = (((a.on && p_ok) ? p : 0) * ow0 + a.col) * (conv.k - 1);
        return a;
    };
    auto tail_window = [&](const WinAddr &a, Tail &t) {
        if (!a.on) return;
        const int H = conv.k - 1;
        if (conv.bias) t.cb = conv.bias[a.col];
#pragma unroll
        for (int k = 0; k < 4; ++k) t.wk[k] = conv.w[a.col * conv.k + (k <= H ? k : H)];
#pragma unroll
        for (int k = 0; k < 3; ++k) t.carried[k] = conv.src[a.win + (k < H ? k : H - 1)];
    };
    auto tail_windows = [&](int b, Tail *ts) {
        if (!conv.w) return;
        WinAddr wa[OPT];
#pragma unroll
        for (int j = 0; j < OPT; ++j) wa[j] = tail_address(b, j, ts[j]);
#pragma unroll
        for (int j = 0; j < OPT; ++j) asm volatile("" : "+v"(wa[j].win));  // formed here, not where it is first used
#pragma unroll
        for (int j = 0; j < OPT; ++j) tail_window(wa[j], ts[j]);
    };
    // projection tail: thread (group g, output j) of NW * 64 / n groups takes rows g, g + groups, ... of the
    // block; its 32 weights are fetched here, ahead of the main loop
    uint4 xw4[4] = {make_uint4(0, 0, 0, 0), make_uint4(0, 0, 0, 0), make_uint4(0, 0, 0, 0), make_uint4(0, 0, 0, 0)};
    const bool tail_on = kTailRoom && xp.w && n0 < out.width[0];  // uniform: a column block lies in one output tensor
    const int tail_groups = tail_on ? (NW * 64) / xp.n : 0, tail_g = tail_on ? tid / xp.n : 0, tail_j = tail_on ? tid - tail_g * xp.n : 0;
    if (tail_on && tail_g < tail_groups) {
        const uint4 *wr = reinterpret_cast<const uint4 *>(xp.w + (int64_t)tail_j * xp.ldw + n0);
#pragma unroll
        for (int c = 0; c < 4; ++c) xw4[c] = wr[c];
    }
    Tail early[OPT];
    bool window_pending = MB == 1;
    if constexpr (MB == 1) {
#pragma unroll
        for (int j = 0; j < OPT; ++j) tail_first(0, j, early[j]);
    }

    // A wavefront's k blocks are taken G at a time: all loads of a group are issued before its first
    // MFMA, so that a row of up to 64 * NW * G values costs one trip to memory, not one per block.
    constexpr int G = MB == 1 ? 3 : 2;
    for (int64_t blk0 = wave; blk0 < kblocks; blk0 += (int64_t)NW * G) {
        uint4 wf[G][4], xf[G][MB][4];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int64_t c = (blk0 + (int64_t)g * NW) * 8 + lch;
            const bool ok = c < kchunks;                          // also false for blocks past the last
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                wf[g][i] = ok ? wptr[i][c] : make_uint4(0, 0, 0, 0);
#pragma unroll
                for (int b = 0; b < MB; ++b) xf[g][b][i] = (ok && xlive[b][i]) ? xptr[b][i][c] : make_uint4(0, 0, 0, 0);
            }
        }
        // the norm weights of all groups go out with the group's own loads (fetched group by group where they are
        // used, each costs a trip of its own); chunks past the end re-read the last one and are not used
        float4 nw[G][2];
        if (norm_w) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const int64_t c = (blk0 + (int64_t)g * NW) * 8 + lch;
                const int64_t cc = c < kchunks ? c : kchunks - 1;
                nw[g][0] = reinterpret_cast<const float4 *>(norm_w)[2 * cc];
                nw[g][1] = reinterpret_cast<const float4 *>(norm_w)[2 * cc + 1];
            }
        }
        if (MB == 1 && window_pending) {
            tail_windows(0, early);
            window_pending = false;
        }
        if (norm_w) {
            // RMSNorm on the way in: the element-wise weight now, the row factor after the sums
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const int64_t c = (blk0 + (int64_t)g * NW) * 8 + lch;
                if (c >= kchunks) continue;
                const float4 g0 = nw[g][0], g1 = nw[g][1];
#pragma unroll
                for (int b = 0; b < MB; ++b)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        uint4 &q = xf[g][b][i];
                        const float v0 = bf16_lo(q.x), v1 = bf16_hi(q.x), v2 = bf16_lo(q.y), v3 = bf16_hi(q.y);
                        const float v4 = bf16_lo(q.z), v5 = bf16_hi(q.z), v6 = bf16_lo(q.w), v7 = bf16_hi(q.w);
                        ss[b][i] += v0 * v0 + v1 * v1 + v2 * v2 + v3 * v3 + v4 * v4 + v5 * v5 + v6 * v6 + v7 * v7;
                        q = make_uint4(f32x2_to_bf16x2(v0 * g0.x, v1 * g0.y), f32x2_to_bf16x2(v2 * g0.z, v3 * g0.w),
                                       f32x2_to_bf16x2(v4 * g1.x, v5 * g1.y), f32x2_to_bf16x2(v6 * g1.z, v7 * g1.w));
                    }
            }
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            bf16x8 wv[4], xv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                patch_w[put + 64 * i] = wf[g][i];
                patch_x[put + 64 * i] = xf[g][0][i];
            }
            wave_sync();
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                wv[s] = __builtin_bit_cast(bf16x8, patch_w[get[s]]);
                xv[s] = __builtin_bit_cast(bf16x8, patch_x[get[s]]);
            }
#pragma unroll
            for (int s = 0; s < 4; ++s) acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xv[s], wv[s], acc[0], 0, 0, 0);
#pragma unroll
            for (int b = 1; b < MB; ++b) {
                wave_sync();                                      // the x patch has been read
#pragma unroll
                for (int i = 0; i < 4; ++i) patch_x[put + 64 * i] = xf[g][b][i];
                wave_sync();
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, patch_x[get[s]]), wv[s], acc[b], 0, 0, 0);
            }
            wave_sync();
        }
    }
    if (MB == 1 && window_pending) tail_windows(0, early);        // a wavefront without a k block of its own
    __syncthreads();                                              // patches are done with: their memory is reused below

    // acc[b][i] is C[m = 32 b + 8 (i / 4) + 4 (lane / 32) + i % 4][n = n0 + lane % 32]
#pragma unroll
    for (int b = 0; b < MB; ++b) {
        if (b > 0) __syncthreads();
#pragma unroll
        for (int i = 0; i < 16; ++i) part[wave][i][lane] = acc[b][i];
        if (norm_w) {
#pragma unroll
            for (int i = 0; i < 4; ++i) ssq[wave][b][i][lane] = ss[b][i];
        }
        __syncthreads();
        if (norm_w) {
            if (tid < 32) {                                       // row tid = (tid & 7) + 8 (tid >> 3): lanes 8 (tid & 7) .. + 7, i = tid >> 3
                float t = 0.0f;
#pragma unroll
                for (int q = 0; q < NW; ++q)
#pragma unroll
                    for (int j = 0; j < 8; ++j) t += ssq[q][b][tid >> 3][8 * (tid & 7) + j];
                row_scale[tid] = __builtin_amdgcn_rsqf(t / (float)K + eps);
            }
            __syncthreads();
        }
        Tail late[OPT];
        if constexpr (MB != 1) {
#pragma unroll
            for (int j = 0; j < OPT; ++j) tail_first(b, j, late[j]);
            tail_windows(b, late);
        }
#pragma unroll
        for (int j = 0; j < OPT; ++j) {
            const int o = tid + j * NW * 64, i = o >> 6, l = o & 63;
            const Tail t = MB == 1 ? early[j] : late[j];
            float v = 0.0f;
#pragma unroll
            for (int q = 0; q < NW; ++q) v += part[q][i][l];
            if (norm_w) v *= row_scale[8 * (i >> 2) + 4 * (l >> 5) + (i & 3)];
            const int64_t m = m0 + b * 32 + 8 * (i >> 2) + 4 * (l >> 5) + (i & 3), n = n0 + (l & 31);
            if (m >= M || n >= N) continue;
            v = bf16_to_f32(f32_to_bf16(v + t.bias));             // same two roundings as the tiled kernel
            int64_t col, width;
            bf16_t *optr;
            const int sp = locate_tail(n, &col, &width, &optr);
            const int64_t off = m * width + col;
            if (residual) v += bf16_to_f32(t.res);
            if (conv.w && sp == 0) {
                // the window of this (row, channel): K - 1 carried values, then v; same order of operations
                // as the stand-alone conv kernel.  A bad parent index leaves NaN in the carried places.
                const int H = conv.k - 1;
                const bool p_ok = !conv.parent || (t.parent >= 0 && (int64_t)t.parent < conv.n_in);
                uint16_t carried[3];
#pragma unroll
                for (int k = 0; k < 3; ++k) carried[k] = p_ok ? t.carried[k] : (uint16_t)0x7fc0;
                bf16_t *nwin = conv.dst + off * H;
                float a = t.cb;
#pragma unroll
                for (int k = 0; k < 3; ++k)
                    if (k < H) a = fmaf(t.wk[k], bf16_to_f32(carried[k]), a);
                float wlast = t.wk[0];
#pragma unroll
                for (int k = 1; k < 4; ++k)
                    if (k == H) wlast = t.wk[k];
                a = fmaf(wlast, v, a);
#pragma unroll
                for (int k = 0; k < 2; ++k)
                    if (k + 1 < H) nwin[k] = carried[k + 1];
                if (H > 0) nwin[H - 1] = (bf16_t)f32_to_bf16(v);
                v = silu_f32(a);
            }
            const uint32_t stored = f32_to_bf16(v);
            optr[off] = (bf16_t)stored;
            if constexpr (kTailRoom) {
                if (xp.w && sp == 0) xc[b][8 * (i >> 2) + 4 * (l >> 5) + (i & 3)][l & 31] = bf16_to_f32(stored);
            }
        }
    }
    if constexpr (kTailRoom) {
        if (tail_on) {
            __syncthreads();
            const int rows = (int)((M - m0 < 32 * MB) ? M - m0 : 32 * MB);
            for (int ml = tail_g; ml < rows && tail_g < tail_groups; ml += tail_groups) {
                const int j = tail_j;
                const float *xr = xc[ml >> 5][ml & 31];
                float acc = 0.0f;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const uint4 q = xw4[c];
                    acc = fmaf(xr[8 * c + 0], bf16_lo(q.x), acc);
                    acc = fmaf(xr[8 * c + 1], bf16_hi(q.x), acc);
                    acc = fmaf(xr[8 * c + 2], bf16_lo(q.y), acc);
                    acc = fmaf(xr[8 * c + 3], bf16_hi(q.y), acc);
                    acc = fmaf(xr[8 * c + 4], bf16_lo(q.z), acc);
                    acc = fmaf(xr[8 * c + 5], bf16_hi(q.z), acc);
                    acc = fmaf(xr[8 * c + 6], bf16_lo(q.w), acc);
                    acc = fmaf(xr[8 * c + 7], bf16_hi(q.w), acc);
                }
                xp.part[((m0 + ml) * xp.n + j) * (xp.ldw / 32) + blockIdx.x] = acc;
            }
        }
    }
}

}  // namespace

hipError_t launch_linear(const LinearArgs &a, hipStream_t stream)
{
    OutSplit o;
    for (int s = 0; s < 3; ++s) {
        o.ptr[s] = static_cast<bf16_t *>(a.out[s]);
        o.width[s] = a.width[s];
    }
    const int64_t N = a.width[0] + a.width[1] + a.width[2];
    const int vec = (a.width[0] % 8 == 0 && a.width[1] % 8 == 0 && a.width[2] % 8 == 0) ? 1 : 0;
    const bf16_t *x = static_cast<const bf16_t *>(a.x), *w = static_cast<const bf16_t *>(a.w);
    const bf16_t *res = static_cast<const bf16_t *>(a.residual);
    // few rows: the split-k kernel, except for very wide outputs (the LM head), where the tiled kernel's
    // shared x tile reads less
    const int64_t col_blocks = (N + 31) / 32;
    const bool few_rows = a.M <= 64 && (N < 8192 || a.norm_w || a.conv_w);
    if (few_rows) {
        const ConvTail ct{a.conv_w, a.conv_b, static_cast<const bf16_t *>(a.conv_src), static_cast<bf16_t *>(a.conv_dst),
                          a.conv_parent, a.conv_n_in, a.conv_k};
        const bool deep = a.K > 512;                              // more wavefronts share a long k loop
        const XprojTail xt{deep ? static_cast<const bf16_t *>(a.xproj_w) : nullptr, a.xproj_part, a.xproj_n, a.width[0]};
        if (a.M <= 32) {
            const dim3 grid((unsigned)col_blocks, 1);
            if (deep) linear_skinny_kernel<8, 1><<<grid, 512, 0, stream>>>(x, w, a.bias, res, o, a.M, N, a.K, a.norm_w, a.eps, ct, xt);
            else      linear_skinny_kernel<4, 1><<<grid, 256, 0, stream>>>(x, w, a.bias, res, o, a.M, N, a.K, a.norm_w, a.eps, ct, xt);
        } else {
            const dim3 grid((unsigned)col_blocks, (unsigned)((a.M + 63) / 64));
            if (deep) linear_skinny_kernel<8, 2><<<grid, 512, 0, stream>>>(x, w, a.bias, res, o, a.M, N, a.K, a.norm_w, a.eps, ct, xt);
            else      linear_skinny_kernel<4, 2><<<grid, 256, 0, stream>>>(x, w, a.bias, res, o, a.M, N, a.K, a.norm_w, a.eps, ct, xt);
        }
        return hipGetLastError();
    }
    // Few output columns and a long k loop (x_proj on a context of a few thousand tokens): the tiled kernel would walk
    // k slab by slab on a few dozen CUs; the split-k kernel over a grid of 32-row blocks fetches a block's whole k range
    // in one trip, as long as all of its workgroups are resident at once (2048 tokens: 10.4 -> 6.5 us; with a second
    // round of workgroups, at 4096 tokens, it is slower than the tiles: 13.6 against 10.7 us).
    if (N <= 128 && a.K > 512 && col_blocks * ((a.M + 31) / 32) <= 256) {
        const ConvTail ct{nullptr, nullptr, nullptr, nullptr, nullptr, 0, 0};
        const XprojTail xt{nullptr, nullptr, 0, 0};
        const dim3 grid((unsigned)col_blocks, (unsigned)((a.M + 31) / 32));
        linear_skinny_kernel<8, 1><<<grid, 512, 0, stream>>>(x, w, a.bias, res, o, a.M, N, a.K, nullptr, a.eps, ct, xt);
        return hipGetLastError();
    }
    auto tiles = [&](int64_t bm, int64_t bn) { return ((N + bn - 1) / bn) * ((a.M + bm - 1) / bm); };
    if (vec && a.M % 128 == 0 && a.K % (2 * kWideBK) == 0 && a.K >= 2 * kWideBK) {
        // The memory-to-LDS kernel with 128 x 128 tiles (two workgroups to a CU) from 192 tiles on, while 256 x 128
        // ones would come to fewer than two per CU: in_proj on 2048 tokens 17.6 -> 16.3 us, on 4096 tokens 32 -> 29 us,
        // out_proj on 4096 tokens 22 -> 16 us.  (With fewer tiles it wins only on operands that are already in cache
        // -- out_proj on 2048 tokens, 96 tiles: 17.2 -> 12.7 us alone in a loop, but 17.6 -> 19.5 us inside the block,
        // where two 32 KiB stages per CU are too little in flight for operands that come from memory.)  Beyond that
        // 256-row tiles (in_proj on 32768 tokens 222 -> 172 us), 256 columns wide unless that leaves a ragged last round.
        const bool m256 = a.M % kWideBM == 0;
        const int64_t t256 = m256 && N % 256 == 0 ? (a.M / kWideBM) * (N / 256) : 0;
        const int64_t t128 = m256 && N % 128 == 0 ? (a.M / kWideBM) * (N / 128) : 0;
        const int64_t t128s = N % 128 == 0 ? (a.M / 128) * (N / 128) : 0;
        if (t128s >= kTilesWideSmall && t128 < kTilesWideSmallMax) {
            linear_wide_kernel<128, 128><<<(unsigned)(8 * ((t128s + 7) / 8)), 256, 0, stream>>>(x, w, a.bias, res, o, a.M, N, a.K, (int)(N / 128), (int)t128s);
            return hipGetLastError();
        }
        if (t256 >= kTilesWide && (t256 % 256 == 0 || t256 >= 4 * 256 || t128 == 0)) {
            linear_wide_kernel<256, 256><<<(unsigned)(8 * ((t256 + 7) / 8)), 256, 0, stream>>>(x, w, a.bias, res, o, a.M, N, a.K, (int)(N / 256), (int)t256);
            return hipGetLastError();
        }
        if (t128 >= kTilesWide) {
            linear_wide_kernel<256, 128><<<(unsigned)(8 * ((t128 + 7) / 8)), 256, 0, stream>>>(x, w, a.bias, res, o, a.M, N, a.K, (int)(N / 128), (int)t128);
            return hipGetLastError();
        }
    }
    if (tiles(128, 128) >= kTilesBig) {
        dim3 grid((unsigned)((N + 127) / 128), (unsigned)((a.M + 127) / 128));
        linear_kernel<128, 128, 64><<<grid, kThreads, 0, stream>>>(x, w, a.bias, res, o, a.M, N, a.K, vec);
    } else if (tiles(64, 128) >= kTilesMid) {
        dim3 grid((unsigned)((N + 127) / 128), (unsigned)((a.M + 63) / 64));
        linear_kernel<64, 128, 64><<<grid, kThreads, 0, stream>>>(x, w, a.bias, res, o, a.M, N, a.K, vec);
    } else if (a.K >= 512 && tiles(64, 64) < kTilesDeep) {
        // few tiles and a long k loop (x_proj, out_proj on a context of a few thousand tokens): with one or two
        // workgroups per CU nothing hides the fetch of the next slab, so the slabs are made four times deeper
        // and the loop four times shorter
        dim3 grid((unsigned)((N + 63) / 64), (unsigned)((a.M + 63) / 64));
        linear_kernel<64, 64, 256><<<grid, kThreads, 0, stream>>>(x, w, a.bias, res, o, a.M, N, a.K, vec);
    } else {
        dim3 grid((unsigned)((N + 63) / 64), (unsigned)((a.M + 63) / 64));
        if (a.M <= 64 && N >= 8192)
            linear_kernel<64, 64, 64, true><<<grid, kThreads, 0, stream>>>(x, w, a.bias, res, o, a.M, N, a.K, vec);
        else
            linear_kernel<64, 64, 64><<<grid, kThreads, 0, stream>>>(x, w, a.bias, res, o, a.M, N, a.K, vec);
    }
    return hipGetLastError();
}

}  // namespace mamba
