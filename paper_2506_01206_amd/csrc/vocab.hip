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

// Ranking works on integer keys that order like (value, then lower index first), a total order, so
// the result is unique.  The bf16 logit is mapped to 16 bits that order like the float (NaN ranks
// as -inf and so never wins against a number).  While a lane scans its share of a row a candidate
// is a 32-bit key: these 16 bits, then the complement of the candidate's sequence number in the
// lane (the lane meets its elements in index order).  For the merge over the workgroup the key is
// widened to 64 bits: the same 16 bits, then the complement of the index in the row.  0 = none.
__device__ __forceinline__ uint32_t ordered16(uint32_t b)
{
    if ((b & 0x7fffu) > 0x7f80u) b = 0xff80u;
    return b ^ ((b & 0x8000u) ? 0xffffu : 0x8000u);
}
__device__ __forceinline__ float ordered16_value(uint32_t o)
{
    const uint32_t b = o ^ ((o & 0x8000u) ? 0x8000u : 0xffffu);
    return __uint_as_float(b << 16);
}

constexpr int kTopkBlock = 1024;
constexpr uint32_t kSeqHead = 0, kSeqTail = 0xfffe;                  // sequence numbers of the scalar ends

// One workgroup per row.  Every lane keeps the KMAX best keys of its share in a sorted register
// list; the row is read as 16-byte vectors where it is aligned, the few elements before and after
// as scalars.  Then k rounds pick the best head over the workgroup (butterfly inside a wavefront,
// LDS across the wavefronts) and its owner pops it.
template <int KMAX>
__global__ void __launch_bounds__(kTopkBlock)
topk_kernel(const bf16_t *__restrict__ logits, int32_t *__restrict__ idx, float *__restrict__ val, int64_t V, int k)
{
    const int64_t m = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bf16_t *row = logits + m * V;
    uint32_t best[KMAX];
#pragma unroll
    for (int j = 0; j < KMAX; ++j) best[j] = 0;
    auto offer = [&](uint32_t bits, uint32_t seq) {
        uint32_t key = (ordered16(bits) << 16) | (0xffffu - seq);
#pragma unroll
        for (int j = 0; j < KMAX; ++j) {
            const uint32_t hi = max(key, best[j]);
            key = min(key, best[j]);
            best[j] = hi;
        }
    };
    const int64_t head = min<int64_t>((8 - (m * V) % 8) % 8, V);     // elements before the first aligned vector
    const int64_t nvec = (V - head) / 8, tail0 = head + nvec * 8;
    const uint4 *vrow = reinterpret_cast<const uint4 *>(row + head);
    if (tid < head) offer(row[tid], kSeqHead);
    uint32_t seq = 1;
    for (int64_t v = tid; v < nvec; v += kTopkBlock, seq += 8) {
        const uint4 q = vrow[v];
        offer(q.x & 0xffffu, seq);
        offer(q.x >> 16, seq + 1);
        offer(q.y & 0xffffu, seq + 2);
        offer(q.y >> 16, seq + 3);
        offer(q.z & 0xffffu, seq + 4);
        offer(q.z >> 16, seq + 5);
        offer(q.w & 0xffffu, seq + 6);
        offer(q.w >> 16, seq + 7);
    }
    if (tail0 + tid < V) offer(row[tail0 + tid], kSeqTail);

    uint64_t wide[KMAX];                                              // (ordered value, ~index in the row)
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
        const uint32_t sq = 0xffffu - (best[j] & 0xffffu);
        const int64_t e = sq == kSeqHead ? tid : sq == kSeqTail ? tail0 + tid
                        : head + ((int64_t)tid + (int64_t)((sq - 1) >> 3) * kTopkBlock) * 8 + ((sq - 1) & 7);
        wide[j] = best[j] ? ((uint64_t)(best[j] >> 16) << 32) | (uint32_t)~(uint32_t)e : 0;
    }

    __shared__ uint64_t heads[kTopkBlock / 64];
    for (int r = 0; r < k; ++r) {
        uint64_t w = wide[0];
#pragma unroll
        for (int s = 32; s > 0; s >>= 1) {
            const uint64_t o = __shfl_xor(w, s, 64);
            w = o > w ? o : w;
        }
        if (lane == 0) heads[wave] = w;
        __syncthreads();
        uint64_t win = heads[lane & (kTopkBlock / 64 - 1)];
#pragma unroll
        for (int s = kTopkBlock / 128; s > 0; s >>= 1) {
            const uint64_t o = __shfl_xor(win, s, 64);
            win = o > win ? o : win;
        }
        if (tid == 0) {
            idx[m * k + r] = win ? (int32_t)~(uint32_t)win : -1;
            val[m * k + r] = win ? ordered16_value((uint32_t)(win >> 32)) : -INFINITY;
        }
        if (win != 0 && wide[0] == win) {                             // keys are distinct: one owner pops its head
#pragma unroll
            for (int j = 0; j + 1 < KMAX; ++j) wide[j] = wide[j + 1];
            wide[KMAX - 1] = 0;
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
    const bf16_t *lg = static_cast<const bf16_t *>(logits);
    if (k <= 2)      topk_kernel<2><<<(unsigned)M, kTopkBlock, 0, stream>>>(lg, idx, val, V, k);
    else if (k <= 4) topk_kernel<4><<<(unsigned)M, kTopkBlock, 0, stream>>>(lg, idx, val, V, k);
    else             topk_kernel<8><<<(unsigned)M, kTopkBlock, 0, stream>>>(lg, idx, val, V, k);
    return hipGetLastError();
}

}  // namespace mamba
