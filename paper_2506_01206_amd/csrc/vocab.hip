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

// A candidate is one 64-bit key: the logit mapped to an unsigned integer that orders like the float
// (high word), then the complemented index (low word), so that a larger key means a larger value or,
// for equal values, the lower index: a total order, hence a unique result.  Key 0 is "no candidate".
__device__ __forceinline__ uint64_t make_key(uint32_t bf16_bits, int32_t index)
{
    uint32_t u = bf16_bits << 16;
    if ((u & 0x7fffffffu) > 0x7f800000u) u = 0xff800000u;          // NaN logits never win: they rank as -inf
    u ^= (u >> 31) ? 0xffffffffu : 0x80000000u;
    return ((uint64_t)u << 32) | (uint32_t)~index;
}
__device__ __forceinline__ float key_value(uint64_t key)
{
    uint32_t u = (uint32_t)(key >> 32);
    u ^= (u >> 31) ? 0x80000000u : 0xffffffffu;
    return __uint_as_float(u);
}

constexpr int kTopkBlock = 1024;

// One workgroup per row.  Every lane keeps the KMAX best keys of its share in a sorted register
// list (a key that does not beat the list's tail is dropped after one comparison); the row is read
// as 16-byte vectors where it is aligned, the few elements before and after as scalars.  Then k
// rounds pick the best head over the workgroup (butterfly inside a wavefront, LDS across the
// wavefronts) and its owner pops it.
template <int KMAX>
__global__ void __launch_bounds__(kTopkBlock)
topk_kernel(const bf16_t *__restrict__ logits, int32_t *__restrict__ idx, float *__restrict__ val, int64_t V, int k)
{
    const int64_t m = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bf16_t *row = logits + m * V;
    uint64_t best[KMAX];
#pragma unroll
    for (int j = 0; j < KMAX; ++j) best[j] = 0;
    auto offer = [&](uint64_t key) {
        if (key <= best[KMAX - 1]) return;
#pragma unroll
        for (int j = 0; j < KMAX; ++j) {
            const uint64_t hi = key > best[j] ? key : best[j], lo = key > best[j] ? best[j] : key;
            best[j] = hi;
            key = lo;
        }
    };
    const int64_t head = min<int64_t>((8 - (m * V) % 8) % 8, V);     // elements before the first aligned vector
    const int64_t nvec = (V - head) / 8, tail0 = head + nvec * 8;
    const uint4 *vrow = reinterpret_cast<const uint4 *>(row + head);
    for (int64_t v = tid; v < nvec; v += kTopkBlock) {
        const uint4 q = vrow[v];
        const int32_t e = (int32_t)(head + v * 8);
        offer(make_key(q.x & 0xffffu, e));
        offer(make_key(q.x >> 16, e + 1));
        offer(make_key(q.y & 0xffffu, e + 2));
        offer(make_key(q.y >> 16, e + 3));
        offer(make_key(q.z & 0xffffu, e + 4));
        offer(make_key(q.z >> 16, e + 5));
        offer(make_key(q.w & 0xffffu, e + 6));
        offer(make_key(q.w >> 16, e + 7));
    }
    if (tid < head) offer(make_key(row[tid], tid));
    if (tail0 + tid < V) offer(make_key(row[tail0 + tid], (int32_t)(tail0 + tid)));

    __shared__ uint64_t heads[kTopkBlock / 64];
    for (int r = 0; r < k; ++r) {
        uint64_t w = best[0];
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
            val[m * k + r] = win ? key_value(win) : -INFINITY;
        }
        if (win != 0 && best[0] == win) {                             // keys are distinct: one owner pops its head
#pragma unroll
            for (int j = 0; j + 1 < KMAX; ++j) best[j] = best[j + 1];
            best[KMAX - 1] = 0;
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
    topk_kernel<8><<<(unsigned)M, kTopkBlock, 0, stream>>>(static_cast<const bf16_t *>(logits), idx, val, V, k);
    return hipGetLastError();
}

}  // namespace mamba
