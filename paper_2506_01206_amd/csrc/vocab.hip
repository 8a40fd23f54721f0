// Token-side ends of the drafter around the blocks (the paper's drafter is a Mamba-130M language
// model, Sec. 3.1; in tree drafting every node proposes N_i children, Sec. 4.1): the embedding
// lookup that turns draft tokens into hidden rows, and the selection of the k most probable next
// tokens of every branch from the LM head's logits.
#include "device_math.h"
#include "launch.h"

namespace mamba {
namespace {

constexpr int kBlock = 256;

// out[m, :] = table[tokens[m], :]; rows of dm bf16 moved as 16-byte vectors (dm % 8 == 0).
// A token outside [0, V) yields a row of NaN instead of an out-of-bounds read.
__global__ void __launch_bounds__(kBlock)
embedding_kernel(const int32_t *__restrict__ tokens, const uint4 *__restrict__ table, uint4 *__restrict__ out,
                 int64_t V, int64_t vecs)
{
    const int64_t m = blockIdx.x;
    const int64_t t = tokens[m];
    const bool ok = t >= 0 && t < V;
    for (int64_t v = threadIdx.x; v < vecs; v += kBlock)
        out[m * vecs + v] = ok ? table[t * vecs + v] : make_uint4(~0u, ~0u, ~0u, ~0u);
}

// larger value first; equal values: lower index first (a total order, so the result is unique)
__device__ __forceinline__ bool better(float va, int32_t ia, float vb, int32_t ib)
{
    return va > vb || (va == vb && ia < ib);
}

// One workgroup per row: every lane keeps the KMAX best of its strided share in registers, then the
// 256 candidate lists are merged k rounds in a row through LDS (arg-max of the heads, pop the winner).
template <int KMAX>
__global__ void __launch_bounds__(kBlock)
topk_kernel(const bf16_t *__restrict__ logits, int32_t *__restrict__ idx, float *__restrict__ val, int64_t V, int k)
{
    const int64_t m = blockIdx.x;
    const bf16_t *row = logits + m * V;
    float bv[KMAX];
    int32_t bi[KMAX];
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
        bv[j] = -INFINITY;
        bi[j] = 0x7fffffff;
    }
    for (int64_t v = threadIdx.x; v < V; v += kBlock) {
        float x = bf16_to_f32(row[v]);
        if (x != x) x = -INFINITY;                     // NaN logits never win
        int32_t xi = (int32_t)v;
#pragma unroll
        for (int j = 0; j < KMAX; ++j) {               // insertion into the sorted list
            if (better(x, xi, bv[j], bi[j])) {
                const float tv = bv[j];
                const int32_t ti = bi[j];
                bv[j] = x;
                bi[j] = xi;
                x = tv;
                xi = ti;
            }
        }
    }
    __shared__ float sv[kBlock];
    __shared__ int32_t si[kBlock];
    __shared__ int winner;
    for (int r = 0; r < k; ++r) {
        sv[threadIdx.x] = bv[0];
        si[threadIdx.x] = bi[0];
        __syncthreads();
        for (int s = kBlock / 2; s > 0; s >>= 1) {
            if ((int)threadIdx.x < s && better(sv[threadIdx.x + s], si[threadIdx.x + s], sv[threadIdx.x], si[threadIdx.x])) {
                sv[threadIdx.x] = sv[threadIdx.x + s];
                si[threadIdx.x] = si[threadIdx.x + s];
            }
            __syncthreads();
        }
        if (threadIdx.x == 0) {
            idx[m * k + r] = si[0] == 0x7fffffff ? -1 : si[0];
            val[m * k + r] = sv[0];
            winner = si[0];
        }
        __syncthreads();
        if (bi[0] == winner && winner != 0x7fffffff) { // the owner pops its head
#pragma unroll
            for (int j = 0; j + 1 < KMAX; ++j) {
                bv[j] = bv[j + 1];
                bi[j] = bi[j + 1];
            }
            bv[KMAX - 1] = -INFINITY;
            bi[KMAX - 1] = 0x7fffffff;
        }
        __syncthreads();
    }
}

}  // namespace

hipError_t launch_embedding(const int32_t *tokens, const void *table, void *out, int64_t M, int64_t V, int64_t dm,
                            hipStream_t stream)
{
    embedding_kernel<<<(unsigned)M, kBlock, 0, stream>>>(tokens, static_cast<const uint4 *>(table),
                                                       static_cast<uint4 *>(out), V, dm / 8);
    return hipGetLastError();
}

hipError_t launch_topk(const void *logits, int32_t *idx, float *val, int64_t M, int64_t V, int k, hipStream_t stream)
{
    topk_kernel<8><<<(unsigned)M, kBlock, 0, stream>>>(static_cast<const bf16_t *>(logits), idx, val, V, k);
    return hipGetLastError();
}

}  // namespace mamba
