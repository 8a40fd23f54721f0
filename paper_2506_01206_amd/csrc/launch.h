// Internal launch interface between the host-side C ABI (api.cpp) and the kernel files.
// Arguments are already validated; every function enqueues on `stream` and returns the
// hipError_t of its last launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mamba {

constexpr int kIoF32 = 0;
constexpr int kIoBf16 = 1;

struct ConvArgs {
    const void *x;
    const float *w, *bias;
    const void *state_in;
    void *y;
    void *state_out;
    int64_t batch, L, D;
    int K, apply_silu, io;
    // tree drafting: sequence b takes the carried rows of state_in[parent[b]] (n_in rows there; an index
    // outside [0, n_in) gives NaN); nullptr: state_in[b].  Needs state_in != state_out.
    const int32_t *parent = nullptr;
    int64_t n_in = 0;
};
hipError_t launch_conv1d(const ConvArgs &a, hipStream_t stream);

struct ScanArgs {
    const void *x, *dt, *Bm, *Cm, *z;
    const float *A, *Dskip, *dt_bias, *h0;
    void *out;
    float *h_final;
    float *ws;  // chunk-boundary workspace or nullptr when n_chunks == 1
    int64_t batch, L, D;
    int N, io, dt_softplus;
    int64_t chunk_len, n_chunks;
    int single_pass = 0;  // kScanDirect / kScanLanes: one of the single-pass kernels (n_chunks == 1, no workspace)
};
constexpr int kScanChunked = 0, kScanDirect = 1, kScanLanes = 2;
// The library's own choice (chunk_len = 0) of kernel for a shape: channels across lanes (scan_direct.hip) when
// there are many independent channels, time across lanes (scan_lanes.hip) for one or a few sequences of a
// narrow layer, else time chunks across workgroups (scan.hip).
int scan_kernel_choice(int64_t batch, int64_t L, int64_t D, int64_t N);
bool scan_direct_applies(int64_t batch, int64_t L, int64_t D, int64_t N);
bool scan_lanes_applies(int64_t batch, int64_t L, int64_t D, int64_t N);
hipError_t launch_scan_direct(const ScanArgs &a, hipStream_t stream);
hipError_t launch_scan_lanes(const ScanArgs &a, hipStream_t stream);
// Token tensors with element strides {batch, token, channel} (strided.hip): plain kernels, one lane per channel.
struct ConvStridedArgs {
    const void *x;
    const float *w, *bias;
    const void *state_in;
    void *y;
    void *state_out;
    int64_t batch, L, D;
    int K, apply_silu, io;
    int64_t xs[3], ys[3];
};
struct ScanStridedArgs {
    const void *x, *dt, *Bm, *Cm, *z;
    const float *A, *Dskip, *dt_bias, *h0;
    void *out;
    float *h_final;
    int64_t batch, L, D;
    int N, io, dt_softplus;
    int64_t xs[3], ds[3], zs[3], os[3];
};
hipError_t launch_conv1d_strided(const ConvStridedArgs &a, hipStream_t stream);
hipError_t launch_scan_strided(const ScanStridedArgs &a, hipStream_t stream);
// Chunking chosen for a shape when the caller passes chunk_len = 0 (pure function of the shape).
void scan_plan(int64_t batch, int64_t L, int64_t D, int64_t N, int64_t chunk_len_req,
               int64_t *chunk_len, int64_t *n_chunks);
size_t scan_workspace_bytes(int64_t batch, int64_t D, int64_t N, int64_t n_chunks);
hipError_t launch_scan(const ScanArgs &a, hipStream_t stream);
// Device address, on the current device, of the chunk-state buffer that is part of the code object (the
// allocation-free scan entry point); looked up once per device.
hipError_t scan_static_scratch(float **ptr);
// Carry over chunk states, in place: slot 0 <- h0 (or 0); slot c <- exp(A * sumdt[c-1]) * slot[c-1] + slot[c].
// ws_state: (batch, n_slots, D, N) fp32, slot c holding the local end state of chunk c - 1 on entry;
// ws_sumdt: (batch, n_slots, D) fp32, entry c the sum of deltas of chunk c; A: (D, N).
hipError_t launch_chunk_carry(const float *A, const float *h0, float *ws_state, const float *ws_sumdt, int64_t batch,
                              int64_t D, int N, int n_slots, hipStream_t stream);
hipError_t launch_copy_state(const float *src /* nullptr: zeros */, float *dst, int64_t n, hipStream_t stream);

// Scalar-decay (Mamba-2 style) layer core.  x, z, out: (batch, L, H, P); dt: (batch, L, H); Bm, Cm: (batch, L, N);
// A, Dskip, dt_bias: (H); h0, h_final: (batch, H, P, N) fp32.  P = 64, N in {64, 128}; bf16 I/O for the scan.
struct SsdArgs {
    const void *x, *dt, *Bm, *Cm, *z;
    const float *A, *Dskip, *dt_bias, *h0;
    void *out;
    float *h_final;
    float *ws;
    int64_t batch, L, H;
    int P, N, dt_softplus;
};
size_t ssd_workspace_bytes(int64_t batch, int64_t L, int64_t H, int64_t P, int64_t N);
hipError_t launch_ssd(const SsdArgs &a, hipStream_t stream);

struct SsdStepArgs {
    float *h_out;
    const float *h_in;
    const int32_t *parent;
    const void *x, *dt, *Bm, *Cm, *z;
    const float *A, *Dskip, *dt_bias;
    void *out;
    int64_t n_out, n_in, H;
    int P, N, io, dt_softplus;
};
hipError_t launch_ssd_step(const SsdStepArgs &a, hipStream_t stream);

struct StepArgs {
    float *h_out;
    const float *h_in;
    const int32_t *parent;
    const void *x, *dt, *Bm, *Cm, *z;
    const float *A, *Dskip, *dt_bias;
    void *out;
    int64_t n_out, n_in, D;
    int N, io, dt_softplus;
    // with dt_w (D, dt_rank) bf16 the kernel also does the dt projection: ``dt`` is then the low-rank
    // (n_out, dt_rank) tensor and delta_raw[j,d] = sum_r dt[j,r] dt_w[d,r]  (bf16 I/O only, dt_rank % 4 == 0)
    const void *dt_w = nullptr;
    int64_t dt_rank = 0;
    // with xpart ((n_out, dt_rank + 2 N, n_parts) float32 partial sums of the x projection, n_parts % 4 == 0) the
    // kernel adds the parts up itself and takes dt (low rank), Bm and Cm from the sums, rounded to bf16 as the stored tensors
    // would be; dt, Bm, Cm are then not read (needs dt_w, dt_rank + 2 N <= 256)
    const float *xpart = nullptr;
    int n_parts = 0;
    // with conv_w ((D, conv_k) float32) the kernel also does the conv step: ``x`` is then the input before the conv,
    // conv_src (n_in, D, conv_k - 1) the carried windows (read through the parent index), conv_dst (n_out, D, conv_k - 1)
    // the new ones, xc_out (n_out, D) the conv output if wanted; conv_k in 2..4
    const float *conv_w = nullptr, *conv_bias = nullptr;
    const void *conv_src = nullptr;
    void *conv_dst = nullptr, *xc_out = nullptr;
    int conv_k = 0, conv_silu = 1;
};
hipError_t launch_step(const StepArgs &a, hipStream_t stream);

struct ForkArgs {
    void *conv_dst;
    const void *conv_src;
    void *ssm_dst;
    const void *ssm_src;
    const int32_t *parent;
    int64_t n_layers, n_out, n_in;
    int64_t conv_row_bytes, ssm_row_bytes;
};
hipError_t launch_fork(const ForkArgs &a, hipStream_t stream);

// parent[j] = j / fanout for j < n (children of a node sit next to each other)
hipError_t launch_tree_parents(int32_t *parent, int64_t n, int32_t fanout, hipStream_t stream);

struct LinearArgs {
    const void *x, *w;       // (M, K), (N, K) bf16
    const float *bias;       // (N) or nullptr
    const void *residual;    // (M, N) bf16 or nullptr (single output only)
    void *out[3];            // up to three output tensors (M, width[i]) bf16
    int64_t width[3];
    int64_t M, K;
    // with norm_w (K) the rows of x are RMS-normalised on the way in: x[m,k] * norm_w[k] enters the
    // product and the row factor rsqrt(mean_k x[m,k]^2 + eps) is applied to the sums (M <= 64 only)
    const float *norm_w = nullptr;
    float eps = 0.0f;
    // with conv_w the columns of the first output tensor (the x half of in_proj, width[0] channels) go
    // through one step of the causal depthwise conv + SiLU before they are stored (M <= 64 only): row m
    // takes the window conv_src[parent[m]] (or conv_src[m]), and the shifted window goes to conv_dst[m].
    // conv_src / conv_dst: (rows, width[0], conv_k - 1) bf16; may be the same buffer when parent is null.
    const float *conv_w = nullptr, *conv_b = nullptr;
    const void *conv_src = nullptr;
    void *conv_dst = nullptr;
    const int32_t *conv_parent = nullptr;
    int64_t conv_n_in = 0;
    int conv_k = 0;
    // with xproj_w (xproj_n, width[0]) bf16 every workgroup also multiplies its 32 finished columns of the first
    // output tensor (as stored, i.e. after the conv step) into the next projection and leaves the partial sums in
    // xproj_part[(row, j, column block)] (float32, (M, xproj_n, width[0] / 32)); whoever consumes them adds the
    // column blocks up in order.  (M <= 64, K > 512 and width[0] % 32 == 0 only.)
    const void *xproj_w = nullptr;
    float *xproj_part = nullptr;
    int xproj_n = 0;
};
hipError_t launch_linear(const LinearArgs &a, hipStream_t stream);

struct NormArgs {
    const void *x;           // (M, C) bf16
    const float *w;          // (C)
    void *y;                 // (M, C) bf16
    int64_t M, C;
    float eps;
};
hipError_t launch_rmsnorm(const NormArgs &a, hipStream_t stream);

hipError_t launch_embedding(const int32_t *tokens, const void *table, void *out, int64_t M, int64_t V, int64_t dm,
                            hipStream_t stream);
hipError_t launch_topk(const void *logits, int32_t *idx, float *val, int64_t M, int64_t V, int k, hipStream_t stream);

}  // namespace mamba
