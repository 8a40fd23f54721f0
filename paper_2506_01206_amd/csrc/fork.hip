// State copy by parent index (Sec. 4.1 of the paper: the children of a node start from a copy
// of its state; the copy goes into the pre-allocated cache of the next batch size), gfx950.
//
//   dst[l, j, :] = src[l, parent[j], :]      rows of row_bytes bytes, all layers in one launch
//
// A pure byte gather: rows are moved as the widest vectors (16, 8, 4 or 2 bytes) that divide the
// row size, a few per lane so that several loads are in flight, consecutive lanes on consecutive
// vectors.  The conv-state rows and the SSM-state rows of all layers go in a single launch.
#include "device_math.h"
#include "launch.h"

namespace mamba {
namespace {

constexpr int kBlock = 256;
constexpr int kUnroll = 4;

template <typename V> __device__ __forceinline__ V fill_ff();
template <> __device__ __forceinline__ uint4 fill_ff<uint4>() { return make_uint4(~0u, ~0u, ~0u, ~0u); }
template <> __device__ __forceinline__ uint2 fill_ff<uint2>() { return make_uint2(~0u, ~0u); }
template <> __device__ __forceinline__ uint32_t fill_ff<uint32_t>() { return ~0u; }
template <> __device__ __forceinline__ uint16_t fill_ff<uint16_t>() { return (uint16_t)0xffffu; }

template <typename V>
__device__ __forceinline__ void gather_row(V *__restrict__ dst, const V *__restrict__ src,
                                           int64_t row_vecs, int64_t first, bool p_ok)
{
    V v[kUnroll];
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) {
        const int64_t k = first + (int64_t)i * kBlock;
        v[i] = (p_ok && k < row_vecs) ? src[k] : fill_ff<V>();
    }
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) {
        const int64_t k = first + (int64_t)i * kBlock;
        if (k < row_vecs) dst[k] = v[i];
    }
}

// grid: (conv_blocks + ssm_blocks, n_out, n_layers).  The first conv_blocks workgroups of a
// (branch, layer) move its conv row, the rest its SSM row.
template <typename VC, typename VS>
__global__ void __launch_bounds__(kBlock)
state_fork_kernel(VC *__restrict__ conv_dst, const VC *__restrict__ conv_src,
                  VS *__restrict__ ssm_dst, const VS *__restrict__ ssm_src,
                  const int32_t *__restrict__ parent, int64_t n_out, int64_t n_in,
                  int64_t conv_vecs, int64_t ssm_vecs, int conv_blocks)
{
    const int64_t j = blockIdx.y, l = blockIdx.z;
    const int64_t p = parent[j];
    const bool p_ok = p >= 0 && p < n_in;
    const int64_t ps = p_ok ? p : 0;
    if ((int)blockIdx.x < conv_blocks) {
        const int64_t first = (int64_t)blockIdx.x * (kBlock * kUnroll) + threadIdx.x;
        gather_row<VC>(conv_dst + (l * n_out + j) * conv_vecs, conv_src + (l * n_in + ps) * conv_vecs,
                       conv_vecs, first, p_ok);
    } else {
        const int64_t first = (int64_t)(blockIdx.x - conv_blocks) * (kBlock * kUnroll) + threadIdx.x;
        gather_row<VS>(ssm_dst + (l * n_out + j) * ssm_vecs, ssm_src + (l * n_in + ps) * ssm_vecs,
                       ssm_vecs, first, p_ok);
    }
}

__global__ void __launch_bounds__(kBlock)
tree_parents_kernel(int32_t *__restrict__ parent, int64_t n, int32_t fanout)
{
    const int64_t j = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (j < n) parent[j] = (int32_t)(j / fanout);
}

int vec_bytes(int64_t row_bytes)
{
    if (row_bytes % 16 == 0) return 16;
    if (row_bytes % 8 == 0) return 8;
    if (row_bytes % 4 == 0) return 4;
    return 2;
}

template <typename VC, typename VS> hipError_t launch_fork_t(const ForkArgs &a, hipStream_t stream)
{
    const int64_t conv_vecs = a.conv_dst ? a.conv_row_bytes / (int64_t)sizeof(VC) : 0;
    const int64_t ssm_vecs = a.ssm_dst ? a.ssm_row_bytes / (int64_t)sizeof(VS) : 0;
    const int per_block = kBlock * kUnroll;
    const int conv_blocks = (int)((conv_vecs + per_block - 1) / per_block);
    const int ssm_blocks = (int)((ssm_vecs + per_block - 1) / per_block);
    if (conv_blocks + ssm_blocks == 0) return hipSuccess;
    dim3 grid((unsigned)(conv_blocks + ssm_blocks), (unsigned)a.n_out, (unsigned)a.n_layers);
    state_fork_kernel<VC, VS><<<grid, kBlock, 0, stream>>>(
        static_cast<VC *>(a.conv_dst), static_cast<const VC *>(a.conv_src),
        static_cast<VS *>(a.ssm_dst), static_cast<const VS *>(a.ssm_src), a.parent, a.n_out, a.n_in,
        conv_vecs, ssm_vecs, conv_blocks);
    return hipGetLastError();
}

template <typename VC> hipError_t launch_fork_c(const ForkArgs &a, hipStream_t stream)
{
    // SSM rows are D * N floats: at least 4-byte granular
    switch (a.ssm_dst ? vec_bytes(a.ssm_row_bytes) : 16) {
    case 16: return launch_fork_t<VC, uint4>(a, stream);
    case 8: return launch_fork_t<VC, uint2>(a, stream);
    default: return launch_fork_t<VC, uint32_t>(a, stream);
    }
}

}  // namespace

hipError_t launch_tree_parents(int32_t *parent, int64_t n, int32_t fanout, hipStream_t stream)
{
    if (n <= 0) return hipSuccess;
    tree_parents_kernel<<<(unsigned)((n + kBlock - 1) / kBlock), kBlock, 0, stream>>>(parent, n, fanout);
    return hipGetLastError();
}

hipError_t launch_fork(const ForkArgs &a, hipStream_t stream)
{
    switch (a.conv_dst ? vec_bytes(a.conv_row_bytes) : 16) {
    case 16: return launch_fork_c<uint4>(a, stream);
    case 8: return launch_fork_c<uint2>(a, stream);
    case 4: return launch_fork_c<uint32_t>(a, stream);
    default: return launch_fork_c<uint16_t>(a, stream);
    }
}

}  // namespace mamba
