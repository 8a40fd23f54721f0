/*
 * mamba_hip.h - C ABI of the selective-SSM layer core of a Mamba drafter on
 * AMD MI355X (gfx950).
 *
 * The paper drafts with a Mamba model: the context is encoded once (prefill),
 * then tokens are generated one step at a time from a fixed-size recurrent
 * state (Sec. 1, Sec. 3.1), and a draft tree is generated as a batch in which
 * every child starts from a copy of its parent's state (Sec. 4.1).  The four
 * operations below are the per-layer core of that path: causal depthwise
 * conv1d and selective scan for the prefill, a one-step state update for all
 * branches of the tree at once, and the state copy by parent index; a fifth
 * entry point does copy, conv step and state update of a layer in one launch.
 *
 * Conventions common to all entry points
 *  - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *    allocates nothing, keeps no global state and never synchronizes: each call
 *    validates its arguments on the host, enqueues kernels on `hip_stream`
 *    (a hipStream_t passed as void*; NULL = the default stream) and returns.
 *  - Layout is row-major and contiguous, time-major for token tensors:
 *      x, dt, z, out, y : (batch, L, D)        I/O dtype `io`
 *      Bm, Cm           : (batch, L, N)        I/O dtype `io`
 *      A                : (D, N)               float32, the (negative) real
 *                                              diagonal itself, not its log
 *      Dskip, dt_bias   : (D)                  float32
 *      w                : (D, K), bias : (D)   float32
 *      h (SSM state)    : (rows, D, N)         float32
 *      conv state       : (rows, D, K-1)       I/O dtype, oldest sample first
 *    One B_t, C_t vector per (batch row, token) is shared by all D channels.
 *  - All arithmetic is float32; bf16 inputs are widened exactly and outputs
 *    rounded to nearest-even once, at the store.
 *  - Supported ranges: N (d_state) in {4, 8, 16, 32}; K (d_conv) in {2, 3, 4};
 *    batch, n_out and n_layers up to 65535; anything else returns
 *    MAMBA_ERR_UNSUPPORTED.  D is arbitrary (the widest vector path is taken
 *    when D allows it).  Data pointers must be 16-byte aligned
 *    (MAMBA_ERR_MISALIGNED).
 *  - Return value: MAMBA_OK (0); a negative mamba_status_t for an argument
 *    error, detected before any HIP call (so nothing was enqueued); a positive
 *    value is the hipError_t of a failed launch.  A call with zero work
 *    (L == 0, batch == 0, n_out == 0, ...) succeeds and launches nothing,
 *    except where stated (scan with L == 0 still copies h0 to h_final).
 */
#ifndef MAMBA_HIP_H
#define MAMBA_HIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* I/O element type of a call.  A plain int in the signatures, so that a value outside the list is an
 * ordinary argument the library can refuse (MAMBA_ERR_UNSUPPORTED), not an invalid enumeration value. */
typedef int mamba_dtype_t;
enum { MAMBA_F32 = 0, MAMBA_BF16 = 1 };

typedef enum {
    MAMBA_OK = 0,
    MAMBA_ERR_NULL_POINTER = -1, /* a required pointer is NULL */
    MAMBA_ERR_BAD_SHAPE = -2,    /* negative size, size overflow, n_in == 0 with work to do */
    MAMBA_ERR_UNSUPPORTED = -3,  /* dtype, N or K outside the compiled range */
    MAMBA_ERR_MISALIGNED = -4,   /* a data pointer is not 16-byte aligned */
    MAMBA_ERR_WORKSPACE = -5,    /* workspace NULL or smaller than the query says */
    MAMBA_ERR_ALIAS = -6         /* output overlaps an input where that is not allowed */
} mamba_status_t;

#define MAMBA_MAX_N 32
#define MAMBA_MAX_K 4

/* Human-readable text for a status returned by any function here (static storage). */
const char *mamba_status_string(int status);

/*
 * Causal depthwise conv1d over time (first stage of the layer, applied to the
 * context during encoding and to one token per branch during drafting):
 *   y[b,t,d] = act( bias[d] + sum_{k=0..K-1} w[d,k] * xpad[b,t+k,d] ),
 *   xpad = [ conv_state_in[b,d,0..K-2] ; x[b,0..L-1,d] ]   (zeros when NULL),
 *   act  = SiLU if apply_silu else identity,
 *   conv_state_out[b,d,k] = xpad[b,L+k,d], k = 0..K-2  (the last K-1 samples).
 * With L = 1 this is the decode-time window shift.
 *   x, y: (batch,L,D) io.  w: (D,K) f32.  bias: (D) f32 or NULL (zero).
 *   conv_state_in: (batch,D,K-1) io or NULL.  conv_state_out: same shape or NULL.
 * conv_state_out may be the same buffer as conv_state_in (in-place window
 * update); then time is not split across workgroups, which is meant for short L.
 * y must not overlap x.  Partial overlap of the two states is an error.
 */
int mamba_conv1d_fwd(const void *x, const float *w, const float *bias,
                     const void *conv_state_in, void *y, void *conv_state_out,
                     int64_t batch, int64_t L, int64_t D, int K, int apply_silu,
                     mamba_dtype_t io, void *hip_stream);

/*
 * Selective scan over L tokens (context encoding; Sec. 3.1 "encoding"):
 *   delta = softplus(dt + dt_bias) if dt_softplus else dt + dt_bias
 *   h_t[d,n] = exp(delta_t[d] * A[d,n]) * h_{t-1}[d,n] + delta_t[d] * Bm_t[n] * x_t[d]
 *   y_t[d]   = sum_n Cm_t[n] * h_t[d,n] + Dskip[d] * x_t[d]
 *   out_t[d] = y_t[d] * silu(z_t[d])            (no gate when z is NULL)
 *   h_{-1} = h0 (zeros when NULL);  h_final = h_{L-1}.
 * Nullable: Dskip (no skip term), z, dt_bias (zero), h0, h_final (not written).
 * Time has to run in parallel somewhere when batch x D channels do not fill the
 * chip.  With chunk_len > 0 the sequence is cut into time chunks of that many
 * tokens that run in parallel across workgroups, the chunk-boundary states
 * carried through `workspace`; chunk_len >= L means one chunk.  chunk_len = 0
 * lets the library choose by shape: such chunks, or one of two single-pass
 * kernels that need no workspace (channels across lanes when batch x D is large,
 * time across the lanes of a wavefront for one or a few short sequences); see
 * mamba_scan_kernel.  The result does not depend on the choice beyond float32
 * rounding order, and is bitwise reproducible from run to run.
 * mamba_scan_workspace_bytes gives the bytes needed for the same
 * (batch, L, D, N, chunk_len); workspace may be NULL when that is 0.
 * h_final may alias h0.  out must not overlap any input.
 */
size_t mamba_scan_workspace_bytes(int64_t batch, int64_t L, int64_t D, int64_t N,
                                  int64_t chunk_len);
/*
 * Which kernels mamba_scan_fwd runs for a shape (a pure function of the shape, static storage):
 *   "chunked": time chunks across workgroups, two passes and a carry (needs the workspace);
 *   "direct":  one pass, channels across lanes: shapes with many independent channels (batch x D);
 *   "lanes":   one pass, time across the lanes of a wavefront: one or a few short sequences, N = 16;
 *   "single":  one chunk (a chunk_len >= L was asked for, or the sequence is short).
 * The library chooses among them only when chunk_len = 0; an explicit chunk_len always means "chunked"
 * or "single".  "" for a shape mamba_scan_fwd would refuse.
 */
const char *mamba_scan_kernel(int64_t batch, int64_t L, int64_t D, int64_t N, int64_t chunk_len);
int mamba_scan_fwd(const void *x, const void *dt, const float *A, const void *Bm,
                   const void *Cm, const float *Dskip, const void *z,
                   const float *dt_bias, const float *h0, void *out, float *h_final,
                   void *workspace, size_t workspace_bytes, int64_t batch, int64_t L,
                   int64_t D, int64_t N, int64_t chunk_len, int dt_softplus,
                   mamba_dtype_t io, void *hip_stream);

/*
 * mamba_scan_fwd for callers that cannot allocate device memory or hand over a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels, with the
 * chunk-boundary states in a buffer that is part of the library's code object (MAMBA_SCAN_STATIC_BYTES
 * of device memory per GPU the library runs on, held until the process ends).  Same arguments without
 * the workspace pair.  Calls no allocating routine.  A shape whose mamba_scan_workspace_bytes exceeds
 * MAMBA_SCAN_STATIC_BYTES is refused with MAMBA_ERR_WORKSPACE and nothing is launched.
 * Every call on a GPU uses that GPU's one buffer: calls that overlap in time on the same GPU (two
 * streams, two threads) race on it; calls on one stream, or ordered by events, are safe, and nothing in
 * the buffer has to be cleared between calls (every slot is written before it is read).
 * The buffer's address is looked up once per device on the first call there, with that device current.
 */
#define MAMBA_SCAN_STATIC_BYTES (32u << 20)
int mamba_scan_fwd_static(const void *x, const void *dt, const float *A, const void *Bm,
                          const void *Cm, const float *Dskip, const void *z, const float *dt_bias,
                          const float *h0, void *out, float *h_final, int64_t batch, int64_t L,
                          int64_t D, int64_t N, int64_t chunk_len, int dt_softplus,
                          mamba_dtype_t io, void *hip_stream);

/*
 * The conv1d and the scan above for token tensors in another layout (the layer's equations, Sec. 3.1, do not
 * fix one; a channel-major (batch, D, L) caller, or tensors that are column ranges of a wider row such as
 * x | z side by side, are expressible this way).  A stride triple is a HOST array of three element counts
 * {batch, token, channel}: element (b, t, d) lies at b * s[0] + t * s[1] + d * s[2] elements from the base;
 * NULL means contiguous time-major, {L * D, D, 1}.  Strided tensors: x, y of the conv; x, dt, z, out of the
 * scan.  Everything else (w, bias, the conv states, A, Bm, Cm, Dskip, dt_bias, h0, h_final) is laid out as in
 * mamba_conv1d_fwd / mamba_scan_fwd.
 * When every triple describes the contiguous layout and the strided tensors' bases are 16-byte aligned the call
 * IS mamba_conv1d_fwd / mamba_scan_fwd (chunk_len 0; their aliasing and workspace rules, same kernels, same
 * bits).  Otherwise a plain kernel runs:
 * one lane per channel walking time, no workspace, not tuned (the tuned kernels need contiguous rows), results
 * within the same tolerance.  Rules of that path: strides >= 0, and for an output (y, out) a layout in which
 * different (b, t, d) never share an element (checked: sorted by stride, each stride covers the extent below
 * it), else MAMBA_ERR_BAD_SHAPE; base pointers aligned to the element size, the rest to 16 bytes; the byte
 * range an output spans must not overlap the range any input spans (MAMBA_ERR_ALIAS; ranges, not elements:
 * interleaved views of one buffer are refused); conv_state_out must not be conv_state_in; L <= 65535 * 128
 * for the conv.  workspace / workspace_bytes are only looked at on the contiguous path.
 */
int mamba_conv1d_fwd_strided(const void *x, const int64_t *x_strides, const float *w, const float *bias,
                             const void *conv_state_in, void *y, const int64_t *y_strides,
                             void *conv_state_out, int64_t batch, int64_t L, int64_t D, int K,
                             int apply_silu, mamba_dtype_t io, void *hip_stream);
int mamba_scan_fwd_strided(const void *x, const int64_t *x_strides, const void *dt, const int64_t *dt_strides,
                           const float *A, const void *Bm, const void *Cm, const float *Dskip,
                           const void *z, const int64_t *z_strides, const float *dt_bias, const float *h0,
                           void *out, const int64_t *out_strides, float *h_final, void *workspace,
                           size_t workspace_bytes, int64_t batch, int64_t L, int64_t D, int64_t N,
                           int dt_softplus, mamba_dtype_t io, void *hip_stream);

/*
 * One recurrence step for all n_out live branches of a draft tree at once
 * (Sec. 4.1: batch generation with batch size B_i at draft position i; a child
 * continues from its parent's state).  Same equations as the scan with L = 1:
 *   p = parent_idx[j] (j itself when parent_idx is NULL, which needs n_in == n_out)
 *   h_out[j,d,n] = exp(delta_j[d]*A[d,n]) * h_in[p,d,n] + delta_j[d]*Bm_j[n]*x_j[d]
 *   out[j,d] = (sum_n Cm_j[n]*h_out[j,d,n] + Dskip[d]*x_j[d]) * silu(z_j[d])
 *   h_in: (n_in,D,N) f32.  h_out: (n_out,D,N) f32.  parent_idx: device int32[n_out],
 *   values in [0,n_in).  x, dt, z, out: (n_out,D) io.  Bm, Cm: (n_out,N) io.
 * With parent_idx the state copy is fused into the step: the result is bit-identical
 * to mamba_state_fork followed by a step without parent_idx.  A parent index outside
 * [0,n_in) never reads out of bounds: that branch's state and output become NaN.
 * h_out == h_in is allowed only when parent_idx is NULL (in-place sequential decode).
 */
int mamba_state_step(float *h_out, const float *h_in, const int32_t *parent_idx,
                     const void *x, const void *dt, const float *A, const void *Bm,
                     const void *Cm, const float *Dskip, const void *z,
                     const float *dt_bias, void *out, int64_t n_out, int64_t n_in,
                     int64_t D, int64_t N, int dt_softplus, mamba_dtype_t io,
                     void *hip_stream);

/*
 * Fork, conv step and state update of one layer for all branches in ONE launch (Sec. 4.1: tree
 * drafting advances every branch of a depth at once, each child from a copy of its parent's conv
 * and SSM state; this is the body of that loop for one layer).  x is the input BEFORE the conv:
 *   p = parent_idx[j] (or j);  win = conv_state_in[p,d,:]
 *   x_c[j,d] = act(conv_bias[d] + sum_{k<K-1} conv_w[d,k] win[k] + conv_w[d,K-1] x[j,d])
 *   conv_state_out[j,d,:] = (win[1:], x[j,d])
 *   then mamba_state_step on x_c rounded to the I/O type (h_out, out as there).
 * The result is bit for bit what mamba_conv1d_fwd (L = 1, carried window gathered by parent) followed
 * by mamba_state_step (same parent_idx) gives.
 *   conv_state_in (n_in,D,K-1), conv_state_out (n_out,D,K-1), x, dt, z, out, xc_out (n_out,D),
 *   Bm, Cm (n_out,N) in the I/O type; conv_w (D,K), conv_bias (D) or NULL, A, Dskip, dt_bias f32.
 *   xc_out may be NULL (x_c is then not stored).  K in 2..4, N as for mamba_state_step.
 * conv_state_out == conv_state_in and h_out == h_in are allowed only when parent_idx is NULL.
 * A parent index outside [0,n_in) reads nothing out of bounds: that branch's states and outputs
 * become NaN (its new window still ends with x[j,d]).
 */
int mamba_conv_state_step(float *h_out, const float *h_in, void *conv_state_out,
                          const void *conv_state_in, const int32_t *parent_idx, const void *x,
                          const float *conv_w, const float *conv_bias, const void *dt,
                          const float *A, const void *Bm, const void *Cm, const float *Dskip,
                          const void *z, const float *dt_bias, void *out, void *xc_out,
                          int64_t n_out, int64_t n_in, int64_t D, int64_t N, int K, int apply_silu,
                          int dt_softplus, mamba_dtype_t io, void *hip_stream);

/*
 * State copy by parent index for all layers at once (Sec. 4.1: creating the children
 * of a node "only requires copying the current state"; destination buffers are the
 * pre-allocated caches of the next batch size, hence out of place):
 *   conv_dst[l,j,:,:] = conv_src[l,parent_idx[j],:,:]   (n_layers,n_out,D,K-1) <- (n_layers,n_in,D,K-1)
 *   ssm_dst [l,j,:,:] = ssm_src [l,parent_idx[j],:,:]   (n_layers,n_out,D,N)   <- (n_layers,n_in,D,N)
 * A byte copy: bit-exact, NaN payloads included.  Either the conv pair or the ssm pair
 * may be NULL (both pointers) to copy only the other.  Source and destination must not
 * overlap (MAMBA_ERR_ALIAS).  A parent index outside [0,n_in) copies nothing for that
 * branch and fills its destination rows with 0xFF bytes (NaN).
 */
int mamba_state_fork(void *conv_dst, const void *conv_src, float *ssm_dst,
                     const float *ssm_src, const int32_t *parent_idx, int64_t n_layers,
                     int64_t n_out, int64_t n_in, int64_t D, int64_t N, int K,
                     mamba_dtype_t conv_dtype, void *hip_stream);

/*
 * The dense parts of a Mamba block around the four operations above (the paper's drafter is a
 * Mamba-130M, Sec. 3.1: per layer RMSNorm, in_proj, conv1d, x_proj, dt_proj, selective SSM,
 * out_proj, residual).  bfloat16 tensors only (MAMBA_ERR_UNSUPPORTED otherwise), fp32 accumulation.
 *
 * mamba_linear_fwd:  out[m,n] = sum_k x[m,k] * w[n,k] (+ bias[n]) (+ residual[m,n])
 *   x: (M,K) bf16; w: (N,K) bf16, N = n0 + n1 + n2; bias: (N) f32 or NULL.
 *   The N output columns go to up to three dense tensors out0 (M,n0), out1 (M,n1), out2 (M,n2)
 *   (n1, n2 may be 0 with NULL pointers): in_proj writes x | z, x_proj writes dt_low | B | C.
 *   residual: (M,N) bf16 or NULL, only with a single output (n1 = n2 = 0); may be out0 itself.
 *   K must be a multiple of 8; M up to 65535 * 128 rows.  Outputs must not overlap x or w.
 *
 * mamba_rmsnorm_fwd:  y[m,:] = x[m,:] * rsqrt(mean(x[m,:]^2) + eps) * w,  x, y: (M,C) bf16, w: (C) f32,
 *   C a multiple of 8, C <= 4096.  y may be x itself.
 */
int mamba_linear_fwd(const void *x, const void *w, const float *bias, const void *residual,
                     void *out0, int64_t n0, void *out1, int64_t n1, void *out2, int64_t n2,
                     int64_t M, int64_t K, mamba_dtype_t io, void *hip_stream);
int mamba_rmsnorm_fwd(const void *x, const float *w, void *y, int64_t M, int64_t C, float eps,
                      mamba_dtype_t io, void *hip_stream);

/*
 * One whole Mamba block of the drafter (Mamba-130M shape in the paper, Sec. 3.1), built from the
 * entry points above; bf16 activations, fp32 parameters of the SSM core, bf16 projection weights:
 *   u = rmsnorm(hidden) ; [x | z] = u W_in^T ; x_c = silu(conv1d(x)) ;
 *   [dt_low | B | C] = x_c W_x^T ; dt = dt_low W_dt^T ; y = selective_scan(x_c, dt, A, B, C, D, z, dt_bias) ;
 *   hidden_out = hidden + y W_out^T
 * Tensors between the stages live in the workspace in bf16 (rounded once when stored).
 *
 * mamba_block_fwd encodes L tokens of `batch` sequences (prefill): hidden, hidden_out (batch,L,d_model);
 * conv_state_in / h0 (nullable) carry a previous piece of the sequence, conv_state_out / h_final
 * (nullable) receive the states after the last token.  hidden_out may be hidden itself.
 * mamba_block_step advances n_out draft branches by one token (decode): branch j continues from
 * the states of branch parent_idx[j] of the source caches (n_in rows); with parent_idx NULL the
 * step is in place (sources == destinations, n_in == n_out).  hidden, hidden_out: (n_out, d_model).
 * workspace: device memory of at least mamba_block_workspace_bytes(p, rows) bytes for
 * rows = batch * L (or n_out), 16-byte aligned.  d_model, d_inner, dt_rank multiples of 8.
 */
typedef struct {
    int64_t d_model, d_inner, d_state, dt_rank;
    int32_t d_conv;
    float eps;                 /* RMSNorm epsilon */
    const float *norm_w;       /* (d_model)                                              */
    const void *in_proj_w;     /* (2 d_inner, d_model) bf16: rows of x, then rows of z   */
    const float *conv_w;       /* (d_inner, d_conv)                                      */
    const float *conv_b;       /* (d_inner) or NULL                                      */
    const void *x_proj_w;      /* (dt_rank + 2 d_state, d_inner) bf16: dt_low | B | C    */
    const void *dt_proj_w;     /* (d_inner, dt_rank) bf16                                */
    const float *dt_bias;      /* (d_inner)                                              */
    const float *A;            /* (d_inner, d_state)                                     */
    const float *Dskip;        /* (d_inner)                                              */
    const void *out_proj_w;    /* (d_model, d_inner) bf16                                */
} mamba_block_params_t;

size_t mamba_block_workspace_bytes(const mamba_block_params_t *p, int64_t batch, int64_t L);
/*
 * Where mamba_block_fwd leaves the stage tensors of its last call in the workspace (byte offsets from
 * its start; host arithmetic only), so that a caller can inspect every stage on its own inputs:
 *   offsets[0] dt (rows, d_inner)      offsets[1] z (rows, d_inner)     offsets[2] x_c (rows, d_inner)
 *   offsets[3] y (rows, d_inner): the gated scan output               offsets[4] dt_low (rows, dt_rank)
 *   offsets[5] B (rows, d_state)       offsets[6] C (rows, d_state)     all bf16, rows = batch * L.
 * (x, the conv's input, shares dt's place and is overwritten by it.)  Returns MAMBA_OK or the error
 * mamba_block_fwd would give for these parameters.
 */
int mamba_block_workspace_layout(const mamba_block_params_t *p, int64_t batch, int64_t L, int64_t offsets[7]);
int mamba_block_fwd(const mamba_block_params_t *p, const void *hidden, void *hidden_out,
                    const void *conv_state_in, void *conv_state_out, const float *h0,
                    float *h_final, void *workspace, size_t workspace_bytes, int64_t batch,
                    int64_t L, void *hip_stream);
int mamba_block_step(const mamba_block_params_t *p, const void *hidden, void *hidden_out,
                     const void *conv_src, void *conv_dst, const float *ssm_src, float *ssm_dst,
                     const int32_t *parent_idx, void *workspace, size_t workspace_bytes,
                     int64_t n_out, int64_t n_in, void *hip_stream);

/*
 * Token-side ends of the drafter (a language model: embedding in front of the blocks, LM head =
 * mamba_linear_fwd with the (V, d_model) vocabulary matrix behind them).
 * mamba_embedding_fwd: out[m,:] = table[tokens[m],:]; tokens: device int32[M]; table: (V,dm) bf16,
 *   dm a multiple of 8; M up to 2^31 - 1.  A token outside [0,V) gives a row of NaN (0xFF bytes).
 * mamba_topk_fwd: for every row of logits (M,V) bf16 the k largest entries, largest first, ties to
 *   the lower index; idx: device int32 (M,k), val: device float (M,k); 1 <= k <= 8; V <= 2^25.
 *   A NaN logit ranks as -inf (so it never wins against a number); when V < k the tail is
 *   idx -1, val -inf.  These are the
 *   children every node of a draft tree proposes (Sec. 4.1) when the N_i candidates are taken
 *   greedily instead of sampled.
 */
int mamba_embedding_fwd(const int32_t *tokens, const void *table, void *out, int64_t M, int64_t V,
                        int64_t dm, mamba_dtype_t io, void *hip_stream);
int mamba_topk_fwd(const void *logits, int32_t *idx, float *val, int64_t M, int64_t V, int k,
                   mamba_dtype_t io, void *hip_stream);

/*
 * Batch-wise state caches of a draft tree (Sec. 4.1, "efficient cache utilization for batch
 * generation": for a tree configuration T = (N_1..N_gamma) the batch size at draft position i is
 * B_i = N_1 * ... * N_i; one state cache per possible batch size is allocated in advance so that
 * duplicating states never re-allocates).
 *
 * mamba_tree_plan is pure host arithmetic: from the tree (HOST int32[gamma]) and the layer
 * shapes it lays out, inside one caller-allocated device slab, a cache per DISTINCT batch size
 * (conv rows (n_layers,B,D,K-1) in conv_dtype and SSM rows (n_layers,B,D,N) float32; cache 0
 * is the root's, B = 1, filled by the prefill) and an int32 parent-index array for every draft
 * position that branches (N_i > 1).  A position with N_i = 1 keeps its batch size: it steps in
 * place in the same cache and has no parent array (parent_offset = -1).  All offsets are
 * multiples of 256 bytes; the slab must hold total_bytes.  Children of node p at position i
 * occupy rows p*N_i .. p*N_i+N_i-1, so parent[j] = j / N_i.
 * Errors: gamma outside [1, MAMBA_MAX_DEPTH] or N_i < 1 -> BAD_SHAPE; a batch size above 65535,
 * unsupported N / K / dtype -> UNSUPPORTED; size overflow -> BAD_SHAPE.
 *
 * mamba_tree_parents writes those parent arrays into the slab (device), one small kernel per
 * branching position, on hip_stream.  plan and tree are HOST pointers.
 */
#define MAMBA_MAX_DEPTH 16

typedef struct {
    int32_t gamma;                                /* draft length; positions are 1..gamma          */
    int32_t n_caches;                             /* distinct batch sizes, the root's (1) included */
    int64_t batch[MAMBA_MAX_DEPTH + 1];           /* batch[0] = 1, batch[i] = N_1 * ... * N_i       */
    int32_t cache_of_depth[MAMBA_MAX_DEPTH + 1];  /* cache holding the states after position i     */
    int64_t parent_offset[MAMBA_MAX_DEPTH + 1];   /* byte offset of int32[batch[i]], -1 if N_i = 1 */
    int64_t cache_batch[MAMBA_MAX_DEPTH + 1];     /* per cache: its batch size                     */
    int64_t conv_offset[MAMBA_MAX_DEPTH + 1];     /* per cache: byte offset of its conv rows       */
    int64_t ssm_offset[MAMBA_MAX_DEPTH + 1];      /* per cache: byte offset of its SSM rows        */
    int64_t total_bytes;
} mamba_tree_plan_t;

int mamba_tree_plan(const int32_t *tree, int gamma, int64_t n_layers, int64_t D, int64_t N,
                    int K, mamba_dtype_t conv_dtype, mamba_tree_plan_t *plan);
int mamba_tree_parents(void *slab, const mamba_tree_plan_t *plan, const int32_t *tree,
                       void *hip_stream);

/*
 * Scalar-decay (Mamba-2 style) layer core.  The paper names Mamba-2 as a drafter its method carries over
 * to (Sec. 1); the layer is the state-space-dual layer of Dao & Gu (2024).  Per head h with P channels and
 * N states, one decay per head and step:
 *   delta[t,h] = softplus(dt[t,h] + dt_bias[h])      (dt_softplus = 0: delta = dt + dt_bias)
 *   H_t[h] = exp(delta[t,h] A[h]) H_{t-1}[h] + delta[t,h] x_t[h,:] (outer) B_t
 *   y_t[h,:] = H_t[h] C_t + Dskip[h] x_t[h,:];  out = y silu(z) when z is given
 * Layout (device pointers, 16-byte aligned): x, z, out (batch, L, H, P) and dt (batch, L, H) in the I/O
 * dtype; Bm, Cm (batch, L, N), one group shared by all heads; A, Dskip, dt_bias float[H] (Dskip, dt_bias,
 * z, h0, h_final nullable); states h0, h_final (batch, H, P, N) float.  P = 64, N in {64, 128}.
 *
 * mamba2_ssd_fwd encodes a sequence in chunks of 64 steps on the matrix cores (bf16 I/O only);
 * workspace: device scratch of mamba2_ssd_workspace_bytes(batch, L, H, P, N) bytes (0 for an unsupported
 * shape), caller-owned.  mamba2_state_step advances n_out draft branches by one token (x, z, out
 * (n_out, H, P), dt (n_out, H), Bm, Cm (n_out, N); h_in (n_in, H, P, N), h_out (n_out, H, P, N)); branch j
 * continues from h_in[parent_idx[j]] (device int32[n_out]; NULL: h_in[j], and then h_out may be h_in);
 * an index outside [0, n_in) gives NaN for that branch.  mamba_state_fork copies such states too
 * (pass D = H * P).  Errors as for the selective scan; batch, H, n_out <= 65535.
 */
size_t mamba2_ssd_workspace_bytes(int64_t batch, int64_t L, int64_t H, int64_t P, int64_t N);
int mamba2_ssd_fwd(const void *x, const void *dt, const float *A, const void *Bm, const void *Cm,
                   const float *Dskip, const void *z, const float *dt_bias, const float *h0, void *out,
                   float *h_final, void *workspace, size_t workspace_bytes, int64_t batch, int64_t L,
                   int64_t H, int64_t P, int64_t N, int dt_softplus, mamba_dtype_t io, void *hip_stream);
int mamba2_state_step(float *h_out, const float *h_in, const int32_t *parent_idx, const void *x,
                      const void *dt, const float *A, const void *Bm, const void *Cm, const float *Dskip,
                      const void *z, const float *dt_bias, void *out, int64_t n_out, int64_t n_in,
                      int64_t H, int64_t P, int64_t N, int dt_softplus, mamba_dtype_t io, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MAMBA_HIP_H */
