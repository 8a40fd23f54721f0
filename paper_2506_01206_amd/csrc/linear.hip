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
// Tiling: a workgroup of 4 wavefronts owns a 128 x 128 output tile, each wavefront a 64 x 64
// quadrant as 2 x 2 MFMA tiles of v_mfma_f32_32x32x16_bf16 (64 fp32 accumulators per lane).  K is
// walked in slabs of 32: the x and w slabs (128 rows x 64 B each) are fetched with 16-byte loads
// one slab ahead into registers, parked in one of two LDS buffers (rows padded to 80 B), and read
// back as MFMA fragments with 16-byte LDS reads: lane l holds row l % 32, k = 8 * (l / 32) .. + 7.
// Rows past M or N re-read the last valid row and are never stored; a K tail is zero-filled.
#include "device_math.h"
#include "launch.h"

namespace mamba {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBM = 128, kBN = 128, kBK = 32;
constexpr int kThreads = 256;
constexpr int kRowBytes = 80;                 // 64 B of data + 16 B pad against bank conflicts
constexpr int kTileBytes = 128 * kRowBytes;   // one operand slab in LDS

struct OutSplit {
    bf16_t *ptr[3];
    int64_t width[3];
};

__device__ __forceinline__ void store_out(const OutSplit &o, int64_t m, int64_t n, float v)
{
    int64_t c = n;
#pragma unroll
    for (int s = 0; s < 3; ++s) {
        if (c < o.width[s]) {
            o.ptr[s][m * o.width[s] + c] = (bf16_t)f32_to_bf16(v);
            return;
        }
        c -= o.width[s];
    }
}

__device__ __forceinline__ float load_res(const OutSplit &o, const bf16_t *const *res, int64_t m, int64_t n)
{
    int64_t c = n;
#pragma unroll
    for (int s = 0; s < 3; ++s) {
        if (c < o.width[s]) return res[s] ? bf16_to_f32(res[s][m * o.width[s] + c]) : 0.0f;
        c -= o.width[s];
    }
    return 0.0f;
}

// grid: (ceil(N / 128), ceil(M / 128))
__global__ void __launch_bounds__(kThreads)
linear_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ w, const float *__restrict__ bias,
              const bf16_t *res0, OutSplit out, int64_t M, int64_t N, int64_t K)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[2][2][kTileBytes];  // [buffer][x | w]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;                  // quadrant of the wavefront
    const int64_t m0 = (int64_t)blockIdx.y * kBM, n0 = (int64_t)blockIdx.x * kBN;

    // global -> LDS staging: 128 rows x 4 chunks of 16 B per operand, 2 chunks per thread each
    int ld_row[2], ld_chunk[2];
    const uint4 *xg[2], *wg[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int c = tid + i * kThreads;      // 0 .. 511
        ld_row[i] = c >> 2;
        ld_chunk[i] = c & 3;
        int64_t xm = m0 + ld_row[i], wn_ = n0 + ld_row[i];
        xm = xm < M ? xm : M - 1;
        wn_ = wn_ < N ? wn_ : N - 1;
        xg[i] = reinterpret_cast<const uint4 *>(x + xm * K);
        wg[i] = reinterpret_cast<const uint4 *>(w + wn_ * K);
    }
    const int64_t kchunks = K / 8;             // K is a multiple of 8 (checked on the host)
    auto fetch = [&](int64_t k0, uint4 *xr, uint4 *wr) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int64_t ch = k0 / 8 + ld_chunk[i];
            const bool in = ch < kchunks;
            xr[i] = in ? xg[i][ch] : make_uint4(0, 0, 0, 0);
            wr[i] = in ? wg[i][ch] : make_uint4(0, 0, 0, 0);
        }
    };
    auto park = [&](int buf, const uint4 *xr, const uint4 *wr) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int off = ld_row[i] * kRowBytes + ld_chunk[i] * 16;
            *reinterpret_cast<uint4 *>(&lds[buf][0][off]) = xr[i];
            *reinterpret_cast<uint4 *>(&lds[buf][1][off]) = wr[i];
        }
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;

    uint4 xr[2], wr[2];
    fetch(0, xr, wr);
    park(0, xr, wr);
    __syncthreads();
    const int frag_row = lane & 31, frag_k = (lane >> 5) * 16;   // byte offset of the lane's 8 k values
    int buf = 0;
    for (int64_t k0 = 0; k0 < K; k0 += kBK) {
        const bool more = k0 + kBK < K;
        if (more) fetch(k0 + kBK, xr, wr);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {                          // two k16 sub-steps per slab
            bf16x8 af[2], bfr[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int ar = wm * 64 + t * 32 + frag_row, br = wn * 64 + t * 32 + frag_row;
                af[t] = *reinterpret_cast<const bf16x8 *>(&lds[buf][0][ar * kRowBytes + ks * 32 + frag_k]);
                bfr[t] = *reinterpret_cast<const bf16x8 *>(&lds[buf][1][br * kRowBytes + ks * 32 + frag_k]);
            }
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bfr[b], acc[a][b], 0, 0, 0);
        }
        if (more) park(buf ^ 1, xr, wr);
        __syncthreads();
        buf ^= 1;
    }

    // epilogue: acc[a][b][i] is C[8 * (i / 4) + 4 * (lane / 32) + i % 4][lane % 32] of its 32 x 32 tile
    const bf16_t *res[3] = {res0, nullptr, nullptr};
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int64_t n = n0 + wn * 64 + b * 32 + (lane & 31);
            if (n >= N) continue;
            const float bv = bias ? bias[n] : 0.0f;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int64_t m = m0 + wm * 64 + a * 32 + 8 * (i / 4) + 4 * (lane >> 5) + (i & 3);
                if (m >= M) continue;
                float v = acc[a][b][i] + bv;
                if (res0) v += load_res(out, res, m, n);
                store_out(out, m, n, v);
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
    dim3 grid((unsigned)((N + kBN - 1) / kBN), (unsigned)((a.M + kBM - 1) / kBM));
    linear_kernel<<<grid, kThreads, 0, stream>>>(static_cast<const bf16_t *>(a.x), static_cast<const bf16_t *>(a.w),
                                                 a.bias, static_cast<const bf16_t *>(a.residual), o, a.M, N, a.K);
    return hipGetLastError();
}

}  // namespace mamba
