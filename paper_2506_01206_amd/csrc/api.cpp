// Host side of the C ABI declared in include/mamba_hip.h: argument validation (all of it before
// any HIP call, so it can be exercised without a GPU), then dispatch to the kernel launchers.
#include "../../include/mamba_hip.h"
#include "launch.h"

#include <stdint.h>

namespace {

using namespace mamba;

constexpr int64_t kMaxGridYZ = 65535;

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool mul_ok(int64_t a, int64_t b, int64_t *r) { return !__builtin_mul_overflow(a, b, r) && *r >= 0; }

// total = a * b * c * elem without overflow, below 2^62
bool size3(int64_t a, int64_t b, int64_t c, int64_t elem, int64_t *bytes)
{
    int64_t t;
    if (a < 0 || b < 0 || c < 0) return false;
    if (!mul_ok(a, b, &t) || !mul_ok(t, c, &t) || !mul_ok(t, elem, &t)) return false;
    if (t > (int64_t)1 << 62) return false;
    *bytes = t;
    return true;
}

bool overlap(const void *p, int64_t pn, const void *q, int64_t qn)
{
    if (!p || !q || pn <= 0 || qn <= 0) return false;
    const uintptr_t a = reinterpret_cast<uintptr_t>(p), b = reinterpret_cast<uintptr_t>(q);
    return a < b + (uintptr_t)qn && b < a + (uintptr_t)pn;
}

int io_size(int io) { return io == MAMBA_F32 ? 4 : io == MAMBA_BF16 ? 2 : 0; }
bool n_supported(int64_t N) { return N == 4 || N == 8 || N == 16 || N == 32; }
bool k_supported(int K) { return K >= 2 && K <= MAMBA_MAX_K; }

}  // namespace

extern "C" {

const char *mamba_status_string(int status)
{
    switch (status) {
    case MAMBA_OK: return "success";
    case MAMBA_ERR_NULL_POINTER: return "a required pointer is NULL";
    case MAMBA_ERR_BAD_SHAPE: return "negative, overflowing or inconsistent sizes";
    case MAMBA_ERR_UNSUPPORTED: return "dtype, d_state, d_conv or a size outside the supported range";
    case MAMBA_ERR_MISALIGNED: return "a data pointer is not 16-byte aligned";
    case MAMBA_ERR_WORKSPACE: return "workspace is NULL or too small";
    case MAMBA_ERR_ALIAS: return "an output buffer overlaps an input where that is not allowed";
    default: break;
    }
    if (status > 0) return hipGetErrorString(static_cast<hipError_t>(status));
    return "unknown status";
}

int mamba_conv1d_fwd(const void *x, const float *w, const float *bias, const void *conv_state_in,
                     void *y, void *conv_state_out, int64_t batch, int64_t L, int64_t D, int K,
                     int apply_silu, mamba_dtype_t io, void *hip_stream)
{
    const int e = io_size(io);
    if (e == 0 || !k_supported(K)) return MAMBA_ERR_UNSUPPORTED;
    int64_t tok_bytes, st_bytes;
    if (!size3(batch, L, D, e, &tok_bytes) || !size3(batch, D, K - 1, e, &st_bytes)) return MAMBA_ERR_BAD_SHAPE;
    if (batch > kMaxGridYZ) return MAMBA_ERR_UNSUPPORTED;
    if (batch == 0 || D == 0) return MAMBA_OK;
    if (!w || (L > 0 && (!x || !y))) return MAMBA_ERR_NULL_POINTER;
    if (!aligned16(x) || !aligned16(w) || !aligned16(bias) || !aligned16(conv_state_in) ||
        !aligned16(y) || !aligned16(conv_state_out))
        return MAMBA_ERR_MISALIGNED;
    if (overlap(x, tok_bytes, y, tok_bytes)) return MAMBA_ERR_ALIAS;
    if (conv_state_in != conv_state_out && overlap(conv_state_in, st_bytes, conv_state_out, st_bytes))
        return MAMBA_ERR_ALIAS;
    if (overlap(y, tok_bytes, conv_state_in, st_bytes) || overlap(y, tok_bytes, conv_state_out, st_bytes) ||
        overlap(x, tok_bytes, conv_state_out, st_bytes))
        return MAMBA_ERR_ALIAS;
    if (L == 0 && (!conv_state_out || conv_state_out == conv_state_in)) return MAMBA_OK;
    ConvArgs a{x, w, bias, conv_state_in, y, conv_state_out, batch, L, D, K, apply_silu, (int)io};
    return (int)launch_conv1d(a, static_cast<hipStream_t>(hip_stream));
}

size_t mamba_scan_workspace_bytes(int64_t batch, int64_t L, int64_t D, int64_t N, int64_t chunk_len)
{
    int64_t t;
    if (batch <= 0 || L <= 0 || D <= 0 || N <= 0 || chunk_len < 0) return 0;
    if (!size3(batch, L, D, 4, &t) || !size3(batch, D, N + 1, 4, &t)) return 0;
    int64_t cl, nc;
    scan_plan(batch, L, D, N, chunk_len, &cl, &nc);
    return scan_workspace_bytes(batch, D, N, nc);
}

const char *mamba_scan_kernel(int64_t batch, int64_t L, int64_t D, int64_t N, int64_t chunk_len)
{
    int64_t t;
    if (batch <= 0 || L <= 0 || D <= 0 || chunk_len < 0 || !n_supported(N) || batch > kMaxGridYZ) return "";
    if (!size3(batch, L, D, 4, &t) || !size3(batch, D, N + 1, 4, &t)) return "";
    if (chunk_len == 0) {
        const int k = scan_kernel_choice(batch, L, D, N);
        if (k == kScanDirect) return "direct";
        if (k == kScanLanes) return "lanes";
    }
    int64_t cl, nc;
    scan_plan(batch, L, D, N, chunk_len, &cl, &nc);
    if (nc > kMaxGridYZ) return "";
    return nc > 1 ? "chunked" : "single";
}

namespace {

// validation and launch shared by the two scan entry points; static_ws: take the library's own buffer
int scan_checked(const void *x, const void *dt, const float *A, const void *Bm, const void *Cm,
                 const float *Dskip, const void *z, const float *dt_bias, const float *h0,
                 void *out, float *h_final, void *workspace, size_t workspace_bytes, bool static_ws,
                 int64_t batch, int64_t L, int64_t D, int64_t N, int64_t chunk_len,
                 int dt_softplus, mamba_dtype_t io, void *hip_stream)
{
    const int e = io_size(io);
    if (e == 0) return MAMBA_ERR_UNSUPPORTED;
    if (N < 0 || chunk_len < 0) return MAMBA_ERR_BAD_SHAPE;
    int64_t tok_bytes, bc_bytes, st_bytes;
    if (!size3(batch, L, D, e, &tok_bytes) || !size3(batch, L, N, e, &bc_bytes) ||
        !size3(batch, D, N, 4, &st_bytes))
        return MAMBA_ERR_BAD_SHAPE;
    if (!n_supported(N) || batch > kMaxGridYZ) return MAMBA_ERR_UNSUPPORTED;
    if (batch == 0 || D == 0) return MAMBA_OK;
    if (!A || (L > 0 && (!x || !dt || !Bm || !Cm || !out))) return MAMBA_ERR_NULL_POINTER;
    if (!aligned16(x) || !aligned16(dt) || !aligned16(A) || !aligned16(Bm) || !aligned16(Cm) ||
        !aligned16(Dskip) || !aligned16(z) || !aligned16(dt_bias) || !aligned16(h0) ||
        !aligned16(out) || !aligned16(h_final) || !aligned16(workspace))
        return MAMBA_ERR_MISALIGNED;
    if (overlap(out, tok_bytes, x, tok_bytes) || overlap(out, tok_bytes, dt, tok_bytes) ||
        overlap(out, tok_bytes, z, tok_bytes) || overlap(out, tok_bytes, Bm, bc_bytes) ||
        overlap(out, tok_bytes, Cm, bc_bytes) || overlap(out, tok_bytes, h0, st_bytes) ||
        overlap(out, tok_bytes, h_final, st_bytes))
        return MAMBA_ERR_ALIAS;
    if (h_final != h0 && overlap(h_final, st_bytes, h0, st_bytes)) return MAMBA_ERR_ALIAS;
    int64_t cl, nc;
    scan_plan(batch, L, D, N, chunk_len, &cl, &nc);
    if (nc > kMaxGridYZ) return MAMBA_ERR_UNSUPPORTED;
    const size_t need = scan_workspace_bytes(batch, D, N, nc);
    float *ws = nullptr;
    if (static_ws) {
        if (need > (size_t)MAMBA_SCAN_STATIC_BYTES) return MAMBA_ERR_WORKSPACE;
        if (need > 0) {
            const hipError_t he = scan_static_scratch(&ws);
            if (he != hipSuccess) return (int)he;
        }
    } else if (need > 0) {
        if (!workspace || workspace_bytes < need) return MAMBA_ERR_WORKSPACE;
        if (overlap(workspace, (int64_t)need, out, tok_bytes) || overlap(workspace, (int64_t)need, x, tok_bytes) ||
            overlap(workspace, (int64_t)need, dt, tok_bytes) || overlap(workspace, (int64_t)need, h_final, st_bytes))
            return MAMBA_ERR_ALIAS;
        ws = static_cast<float *>(workspace);
    }
    ScanArgs a{x, dt, Bm, Cm, z, A, Dskip, dt_bias, h0, out, h_final, ws,
               batch, L, D, (int)N, (int)io, dt_softplus, cl, nc};
    a.single_pass = (chunk_len == 0 && L > 0) ? scan_kernel_choice(batch, L, D, N) : kScanChunked;
    return (int)launch_scan(a, static_cast<hipStream_t>(hip_stream));
}

}  // namespace

int mamba_scan_fwd(const void *x, const void *dt, const float *A, const void *Bm, const void *Cm,
                   const float *Dskip, const void *z, const float *dt_bias, const float *h0,
                   void *out, float *h_final, void *workspace, size_t workspace_bytes,
                   int64_t batch, int64_t L, int64_t D, int64_t N, int64_t chunk_len,
                   int dt_softplus, mamba_dtype_t io, void *hip_stream)
{
    return scan_checked(x, dt, A, Bm, Cm, Dskip, z, dt_bias, h0, out, h_final, workspace, workspace_bytes, false,
                        batch, L, D, N, chunk_len, dt_softplus, io, hip_stream);
}

int mamba_scan_fwd_static(const void *x, const void *dt, const float *A, const void *Bm, const void *Cm,
                          const float *Dskip, const void *z, const float *dt_bias, const float *h0,
                          void *out, float *h_final, int64_t batch, int64_t L, int64_t D, int64_t N,
                          int64_t chunk_len, int dt_softplus, mamba_dtype_t io, void *hip_stream)
{
    return scan_checked(x, dt, A, Bm, Cm, Dskip, z, dt_bias, h0, out, h_final, nullptr, 0, true,
                        batch, L, D, N, chunk_len, dt_softplus, io, hip_stream);
}

namespace {

// A stride triple {batch, token, channel} resolved for a (batch, L, D) tensor of e-byte elements (all sizes >= 1).
struct Layout {
    int64_t s[3];
    int64_t bytes;      // bytes from the base to the end of the last element
    bool contiguous;    // time-major without gaps (strides of axes of length 1 do not matter)
};

bool resolve_layout(const int64_t *strides, int64_t batch, int64_t L, int64_t D, int e, Layout *o)
{
    const int64_t dims[3] = {batch, L, D};
    int64_t ld;
    if (!mul_ok(L, D, &ld)) return false;
    const int64_t dense[3] = {ld, D, 1};
    int64_t last = 0;
    o->contiguous = true;
    for (int i = 0; i < 3; ++i) {
        o->s[i] = strides ? strides[i] : dense[i];
        if (o->s[i] < 0) return false;
        int64_t t;
        if (!mul_ok(dims[i] - 1, o->s[i], &t) || __builtin_add_overflow(last, t, &last)) return false;
        if (dims[i] > 1 && o->s[i] != dense[i]) o->contiguous = false;
    }
    if (__builtin_add_overflow(last, (int64_t)1, &last) || !mul_ok(last, e, &o->bytes)) return false;
    return o->bytes <= (int64_t)1 << 62;
}

// no two (b, t, d) of an output may share an element.  Sufficient and easy to state: taken in order of
// increasing stride, every axis steps past everything the axes before it can reach.
bool injective(const Layout &l, int64_t batch, int64_t L, int64_t D)
{
    const int64_t dims[3] = {batch, L, D};
    int order[3] = {0, 1, 2};
    for (int i = 0; i < 3; ++i)
        for (int j = i + 1; j < 3; ++j)
            if (l.s[order[j]] < l.s[order[i]]) { const int t = order[i]; order[i] = order[j]; order[j] = t; }
    int64_t reach = 0;   // largest offset the axes handled so far can produce (resolve_layout showed no overflow)
    for (int i = 0; i < 3; ++i) {
        const int a = order[i];
        if (dims[a] == 1) continue;
        if (l.s[a] <= reach) return false;
        reach += (dims[a] - 1) * l.s[a];
    }
    return true;
}

bool aligned_to(const void *p, int e) { return (reinterpret_cast<uintptr_t>(p) & (uintptr_t)(e - 1)) == 0; }

}  // namespace

int mamba_conv1d_fwd_strided(const void *x, const int64_t *x_strides, const float *w, const float *bias,
                             const void *conv_state_in, void *y, const int64_t *y_strides,
                             void *conv_state_out, int64_t batch, int64_t L, int64_t D, int K,
                             int apply_silu, mamba_dtype_t io, void *hip_stream)
{
    const int e = io_size(io);
    if (e == 0 || !k_supported(K)) return MAMBA_ERR_UNSUPPORTED;
    int64_t tok_bytes, st_bytes;
    if (!size3(batch, L, D, e, &tok_bytes) || !size3(batch, D, K - 1, e, &st_bytes)) return MAMBA_ERR_BAD_SHAPE;
    if (batch == 0 || D == 0 || L == 0)   // nothing strided to touch: the contiguous call's own rules
        return mamba_conv1d_fwd(x, w, bias, conv_state_in, y, conv_state_out, batch, L, D, K, apply_silu, io, hip_stream);
    Layout lx, ly;
    if (!resolve_layout(x_strides, batch, L, D, e, &lx) || !resolve_layout(y_strides, batch, L, D, e, &ly))
        return MAMBA_ERR_BAD_SHAPE;
    if (lx.contiguous && ly.contiguous && aligned16(x) && aligned16(y))
        return mamba_conv1d_fwd(x, w, bias, conv_state_in, y, conv_state_out, batch, L, D, K, apply_silu, io, hip_stream);
    if (!injective(ly, batch, L, D)) return MAMBA_ERR_BAD_SHAPE;
    if (batch > kMaxGridYZ || (L + 127) / 128 > kMaxGridYZ) return MAMBA_ERR_UNSUPPORTED;
    if (!w || !x || !y) return MAMBA_ERR_NULL_POINTER;
    if (!aligned_to(x, e) || !aligned_to(y, e) || !aligned16(w) || !aligned16(bias) || !aligned16(conv_state_in) ||
        !aligned16(conv_state_out))
        return MAMBA_ERR_MISALIGNED;
    if (overlap(y, ly.bytes, x, lx.bytes) || overlap(y, ly.bytes, conv_state_in, st_bytes) ||
        overlap(y, ly.bytes, conv_state_out, st_bytes) || overlap(x, lx.bytes, conv_state_out, st_bytes) ||
        overlap(conv_state_in, st_bytes, conv_state_out, st_bytes))
        return MAMBA_ERR_ALIAS;
    ConvStridedArgs a{x, w, bias, conv_state_in, y, conv_state_out, batch, L, D, K, apply_silu, (int)io,
                      {lx.s[0], lx.s[1], lx.s[2]}, {ly.s[0], ly.s[1], ly.s[2]}};
    return (int)launch_conv1d_strided(a, static_cast<hipStream_t>(hip_stream));
}

int mamba_scan_fwd_strided(const void *x, const int64_t *x_strides, const void *dt, const int64_t *dt_strides,
                           const float *A, const void *Bm, const void *Cm, const float *Dskip,
                           const void *z, const int64_t *z_strides, const float *dt_bias, const float *h0,
                           void *out, const int64_t *out_strides, float *h_final, void *workspace,
                           size_t workspace_bytes, int64_t batch, int64_t L, int64_t D, int64_t N,
                           int dt_softplus, mamba_dtype_t io, void *hip_stream)
{
    const int e = io_size(io);
    if (e == 0) return MAMBA_ERR_UNSUPPORTED;
    if (N < 0) return MAMBA_ERR_BAD_SHAPE;
    int64_t tok_bytes, bc_bytes, st_bytes;
    if (!size3(batch, L, D, e, &tok_bytes) || !size3(batch, L, N, e, &bc_bytes) || !size3(batch, D, N, 4, &st_bytes))
        return MAMBA_ERR_BAD_SHAPE;
    if (batch == 0 || D == 0 || L == 0)
        return mamba_scan_fwd(x, dt, A, Bm, Cm, Dskip, z, dt_bias, h0, out, h_final, workspace, workspace_bytes,
                              batch, L, D, N, 0, dt_softplus, io, hip_stream);
    Layout lx, ld, lz, lo;
    if (!resolve_layout(x_strides, batch, L, D, e, &lx) || !resolve_layout(dt_strides, batch, L, D, e, &ld) ||
        !resolve_layout(z_strides, batch, L, D, e, &lz) || !resolve_layout(out_strides, batch, L, D, e, &lo))
        return MAMBA_ERR_BAD_SHAPE;
    if (lx.contiguous && ld.contiguous && (lz.contiguous || !z) && lo.contiguous && aligned16(x) && aligned16(dt) &&
        aligned16(z) && aligned16(out))
        return mamba_scan_fwd(x, dt, A, Bm, Cm, Dskip, z, dt_bias, h0, out, h_final, workspace, workspace_bytes,
                              batch, L, D, N, 0, dt_softplus, io, hip_stream);
    if (!injective(lo, batch, L, D)) return MAMBA_ERR_BAD_SHAPE;
    if (!n_supported(N) || batch > kMaxGridYZ) return MAMBA_ERR_UNSUPPORTED;
    if (!A || !x || !dt || !Bm || !Cm || !out) return MAMBA_ERR_NULL_POINTER;
    if (!aligned_to(x, e) || !aligned_to(dt, e) || !aligned_to(z, e) || !aligned_to(out, e) || !aligned16(A) ||
        !aligned16(Bm) || !aligned16(Cm) || !aligned16(Dskip) || !aligned16(dt_bias) || !aligned16(h0) ||
        !aligned16(h_final))
        return MAMBA_ERR_MISALIGNED;
    if (overlap(out, lo.bytes, x, lx.bytes) || overlap(out, lo.bytes, dt, ld.bytes) ||
        overlap(out, lo.bytes, z, lz.bytes) || overlap(out, lo.bytes, Bm, bc_bytes) ||
        overlap(out, lo.bytes, Cm, bc_bytes) || overlap(out, lo.bytes, h0, st_bytes) ||
        overlap(out, lo.bytes, h_final, st_bytes))
        return MAMBA_ERR_ALIAS;
    if (h_final != h0 && overlap(h_final, st_bytes, h0, st_bytes)) return MAMBA_ERR_ALIAS;
    ScanStridedArgs a{x, dt, Bm, Cm, z, A, Dskip, dt_bias, h0, out, h_final, batch, L, D, (int)N, (int)io, dt_softplus,
                      {lx.s[0], lx.s[1], lx.s[2]}, {ld.s[0], ld.s[1], ld.s[2]}, {lz.s[0], lz.s[1], lz.s[2]},
                      {lo.s[0], lo.s[1], lo.s[2]}};
    return (int)launch_scan_strided(a, static_cast<hipStream_t>(hip_stream));
}

int mamba_state_step(float *h_out, const float *h_in, const int32_t *parent_idx, const void *x,
                     const void *dt, const float *A, const void *Bm, const void *Cm,
                     const float *Dskip, const void *z, const float *dt_bias, void *out,
                     int64_t n_out, int64_t n_in, int64_t D, int64_t N, int dt_softplus,
                     mamba_dtype_t io, void *hip_stream)
{
    const int e = io_size(io);
    if (e == 0) return MAMBA_ERR_UNSUPPORTED;
    if (N < 0) return MAMBA_ERR_BAD_SHAPE;
    int64_t out_bytes, hin_bytes, hout_bytes;
    if (!size3(n_out, D, 1, e, &out_bytes) || !size3(n_in, D, N, 4, &hin_bytes) ||
        !size3(n_out, D, N, 4, &hout_bytes))
        return MAMBA_ERR_BAD_SHAPE;
    if (!parent_idx && n_in != n_out) return MAMBA_ERR_BAD_SHAPE;
    if (n_out > 0 && n_in == 0) return MAMBA_ERR_BAD_SHAPE;
    if (!n_supported(N) || n_out > kMaxGridYZ) return MAMBA_ERR_UNSUPPORTED;
    if (n_out == 0 || D == 0) return MAMBA_OK;
    if (!h_out || !h_in || !x || !dt || !A || !Bm || !Cm || !out) return MAMBA_ERR_NULL_POINTER;
    if (!aligned16(h_out) || !aligned16(h_in) || !aligned16(parent_idx) || !aligned16(x) ||
        !aligned16(dt) || !aligned16(A) || !aligned16(Bm) || !aligned16(Cm) || !aligned16(Dskip) ||
        !aligned16(z) || !aligned16(dt_bias) || !aligned16(out))
        return MAMBA_ERR_MISALIGNED;
    if (!(h_out == h_in && !parent_idx) && overlap(h_out, hout_bytes, h_in, hin_bytes))
        return MAMBA_ERR_ALIAS;
    if (overlap(out, out_bytes, x, out_bytes) || overlap(out, out_bytes, dt, out_bytes) ||
        overlap(out, out_bytes, z, out_bytes) || overlap(out, out_bytes, h_in, hin_bytes) ||
        overlap(out, out_bytes, h_out, hout_bytes) || overlap(h_out, hout_bytes, x, out_bytes) ||
        overlap(h_out, hout_bytes, dt, out_bytes) || overlap(h_out, hout_bytes, z, out_bytes))
        return MAMBA_ERR_ALIAS;
    StepArgs a{h_out, h_in, parent_idx, x, dt, Bm, Cm, z, A, Dskip, dt_bias, out,
               n_out, n_in, D, (int)N, (int)io, dt_softplus};
    return (int)launch_step(a, static_cast<hipStream_t>(hip_stream));
}

int mamba_conv_state_step(float *h_out, const float *h_in, void *conv_state_out, const void *conv_state_in,
                          const int32_t *parent_idx, const void *x, const float *conv_w, const float *conv_bias,
                          const void *dt, const float *A, const void *Bm, const void *Cm, const float *Dskip,
                          const void *z, const float *dt_bias, void *out, void *xc_out, int64_t n_out, int64_t n_in,
                          int64_t D, int64_t N, int K, int apply_silu, int dt_softplus, mamba_dtype_t io,
                          void *hip_stream)
{
    const int e = io_size(io);
    if (e == 0) return MAMBA_ERR_UNSUPPORTED;
    if (N < 0) return MAMBA_ERR_BAD_SHAPE;
    if (K < 2 || K > 4) return MAMBA_ERR_UNSUPPORTED;
    int64_t out_bytes, hin_bytes, hout_bytes, cin_bytes, cout_bytes;
    if (!size3(n_out, D, 1, e, &out_bytes) || !size3(n_in, D, N, 4, &hin_bytes) ||
        !size3(n_out, D, N, 4, &hout_bytes) || !size3(n_in, D, K - 1, e, &cin_bytes) ||
        !size3(n_out, D, K - 1, e, &cout_bytes))
        return MAMBA_ERR_BAD_SHAPE;
    if (!parent_idx && n_in != n_out) return MAMBA_ERR_BAD_SHAPE;
    if (n_out > 0 && n_in == 0) return MAMBA_ERR_BAD_SHAPE;
    if (!n_supported(N) || n_out > kMaxGridYZ) return MAMBA_ERR_UNSUPPORTED;
    if (n_out == 0 || D == 0) return MAMBA_OK;
    if (!h_out || !h_in || !conv_state_out || !conv_state_in || !x || !conv_w || !dt || !A || !Bm || !Cm || !out)
        return MAMBA_ERR_NULL_POINTER;
    if (!aligned16(h_out) || !aligned16(h_in) || !aligned16(conv_state_out) || !aligned16(conv_state_in) ||
        !aligned16(parent_idx) || !aligned16(x) || !aligned16(conv_w) || !aligned16(conv_bias) || !aligned16(dt) ||
        !aligned16(A) || !aligned16(Bm) || !aligned16(Cm) || !aligned16(Dskip) || !aligned16(z) ||
        !aligned16(dt_bias) || !aligned16(out) || !aligned16(xc_out))
        return MAMBA_ERR_MISALIGNED;
    if (!(h_out == h_in && !parent_idx) && overlap(h_out, hout_bytes, h_in, hin_bytes)) return MAMBA_ERR_ALIAS;
    if (!(conv_state_out == conv_state_in && !parent_idx) && overlap(conv_state_out, cout_bytes, conv_state_in, cin_bytes))
        return MAMBA_ERR_ALIAS;
    // no output may overlap an input or another output
    const void *outs[4] = {h_out, conv_state_out, out, xc_out};
    const int64_t out_sz[4] = {hout_bytes, cout_bytes, out_bytes, out_bytes};
    const void *ins[5] = {x, dt, z, h_in, conv_state_in};
    const int64_t in_sz[5] = {out_bytes, out_bytes, out_bytes, hin_bytes, cin_bytes};
    for (int i = 0; i < 4; ++i) {
        if (!outs[i]) continue;
        for (int k = i + 1; k < 4; ++k)
            if (outs[k] && overlap(outs[i], out_sz[i], outs[k], out_sz[k])) return MAMBA_ERR_ALIAS;
        for (int k = 0; k < 5; ++k) {
            if (!ins[k]) continue;
            if ((i == 0 && k == 3) || (i == 1 && k == 4)) continue;      // the in-place pairs were judged above
            if (overlap(outs[i], out_sz[i], ins[k], in_sz[k])) return MAMBA_ERR_ALIAS;
        }
    }
    StepArgs a{h_out, h_in, parent_idx, x, dt, Bm, Cm, z, A, Dskip, dt_bias, out,
               n_out, n_in, D, (int)N, (int)io, dt_softplus};
    a.conv_w = conv_w;
    a.conv_bias = conv_bias;
    a.conv_src = conv_state_in;
    a.conv_dst = conv_state_out;
    a.xc_out = xc_out;
    a.conv_k = K;
    a.conv_silu = apply_silu ? 1 : 0;
    return (int)launch_step(a, static_cast<hipStream_t>(hip_stream));
}

int mamba_state_fork(void *conv_dst, const void *conv_src, float *ssm_dst, const float *ssm_src,
                     const int32_t *parent_idx, int64_t n_layers, int64_t n_out, int64_t n_in,
                     int64_t D, int64_t N, int K, mamba_dtype_t conv_dtype, void *hip_stream)
{
    const bool has_conv = conv_dst || conv_src, has_ssm = ssm_dst || ssm_src;
    const int e = io_size(conv_dtype);
    if (has_conv && (e == 0 || K < 1)) return MAMBA_ERR_UNSUPPORTED;
    if (N < 0 || n_layers < 0) return MAMBA_ERR_BAD_SHAPE;
    int64_t conv_row = 0, ssm_row = 0, t, cs = 0, cd = 0, ss = 0, sd = 0;
    if (has_conv && (!size3(D, K - 1, 1, e, &conv_row) || !size3(n_layers, n_in, conv_row, 1, &cs) ||
                     !size3(n_layers, n_out, conv_row, 1, &cd)))
        return MAMBA_ERR_BAD_SHAPE;
    if (has_ssm && (!size3(D, N, 1, 4, &ssm_row) || !size3(n_layers, n_in, ssm_row, 1, &ss) ||
                    !size3(n_layers, n_out, ssm_row, 1, &sd)))
        return MAMBA_ERR_BAD_SHAPE;
    if (!size3(n_layers, n_out, 1, 1, &t) || !size3(n_layers, n_in, 1, 1, &t) || D < 0) return MAMBA_ERR_BAD_SHAPE;
    if (n_out > 0 && n_in == 0) return MAMBA_ERR_BAD_SHAPE;
    if (n_out > kMaxGridYZ || n_layers > kMaxGridYZ) return MAMBA_ERR_UNSUPPORTED;
    if (n_layers == 0 || n_out == 0 || (!has_conv && !has_ssm)) return MAMBA_OK;
    if ((has_conv && (!conv_dst || !conv_src)) || (has_ssm && (!ssm_dst || !ssm_src)) || !parent_idx)
        return MAMBA_ERR_NULL_POINTER;
    if (!aligned16(conv_dst) || !aligned16(conv_src) || !aligned16(ssm_dst) || !aligned16(ssm_src) ||
        !aligned16(parent_idx))
        return MAMBA_ERR_MISALIGNED;
    if (overlap(conv_dst, cd, conv_src, cs) || overlap(ssm_dst, sd, ssm_src, ss) ||
        overlap(conv_dst, cd, ssm_src, ss) || overlap(ssm_dst, sd, conv_src, cs) ||
        overlap(conv_dst, cd, ssm_dst, sd))
        return MAMBA_ERR_ALIAS;
    ForkArgs a{conv_row ? conv_dst : nullptr, conv_src, ssm_row ? ssm_dst : nullptr, ssm_src,
               parent_idx, n_layers, n_out, n_in, conv_row, ssm_row};
    return (int)launch_fork(a, static_cast<hipStream_t>(hip_stream));
}

int mamba_linear_fwd(const void *x, const void *w, const float *bias, const void *residual, void *out0,
                     int64_t n0, void *out1, int64_t n1, void *out2, int64_t n2, int64_t M, int64_t K,
                     mamba_dtype_t io, void *hip_stream)
{
    if (io != MAMBA_BF16) return MAMBA_ERR_UNSUPPORTED;
    if (n0 < 0 || n1 < 0 || n2 < 0 || M < 0 || K < 0) return MAMBA_ERR_BAD_SHAPE;
    int64_t N;
    if (__builtin_add_overflow(n0, n1, &N) || __builtin_add_overflow(N, n2, &N)) return MAMBA_ERR_BAD_SHAPE;
    int64_t xb, wb, ob[3];
    const int64_t widths[3] = {n0, n1, n2};
    void *outs[3] = {out0, out1, out2};
    if (!size3(M, K, 1, 2, &xb) || !size3(N, K, 1, 2, &wb)) return MAMBA_ERR_BAD_SHAPE;
    for (int i = 0; i < 3; ++i)
        if (!size3(M, widths[i], 1, 2, &ob[i])) return MAMBA_ERR_BAD_SHAPE;
    if (K % 8 != 0 || M > kMaxGridYZ * 128) return MAMBA_ERR_UNSUPPORTED;
    if (residual && (n1 != 0 || n2 != 0)) return MAMBA_ERR_UNSUPPORTED;
    if (M == 0 || N == 0) return MAMBA_OK;
    if (K == 0) return MAMBA_ERR_BAD_SHAPE;
    if (!x || !w) return MAMBA_ERR_NULL_POINTER;
    for (int i = 0; i < 3; ++i)
        if (widths[i] > 0 && !outs[i]) return MAMBA_ERR_NULL_POINTER;
    if (!aligned16(x) || !aligned16(w) || !aligned16(bias) || !aligned16(residual) || !aligned16(out0) ||
        !aligned16(out1) || !aligned16(out2))
        return MAMBA_ERR_MISALIGNED;
    for (int i = 0; i < 3; ++i) {
        if (widths[i] == 0) continue;
        if (overlap(outs[i], ob[i], x, xb) || overlap(outs[i], ob[i], w, wb)) return MAMBA_ERR_ALIAS;
        for (int j = i + 1; j < 3; ++j)
            if (widths[j] > 0 && overlap(outs[i], ob[i], outs[j], ob[j])) return MAMBA_ERR_ALIAS;
    }
    if (residual && residual != out0 && overlap(residual, ob[0], out0, ob[0])) return MAMBA_ERR_ALIAS;
    LinearArgs a{x, w, bias, residual, {out0, out1, out2}, {n0, n1, n2}, M, K};
    return (int)launch_linear(a, static_cast<hipStream_t>(hip_stream));
}

int mamba_rmsnorm_fwd(const void *x, const float *w, void *y, int64_t M, int64_t C, float eps,
                      mamba_dtype_t io, void *hip_stream)
{
    if (io != MAMBA_BF16) return MAMBA_ERR_UNSUPPORTED;
    int64_t bytes;
    if (!size3(M, C, 1, 2, &bytes) || !(eps >= 0.0f)) return MAMBA_ERR_BAD_SHAPE;
    if (C % 8 != 0 || C > 4096 || M > (int64_t)1 << 31) return MAMBA_ERR_UNSUPPORTED;
    if (M == 0 || C == 0) return MAMBA_OK;
    if (!x || !w || !y) return MAMBA_ERR_NULL_POINTER;
    if (!aligned16(x) || !aligned16(w) || !aligned16(y)) return MAMBA_ERR_MISALIGNED;
    if (x != y && overlap(x, bytes, y, bytes)) return MAMBA_ERR_ALIAS;
    NormArgs a{x, w, y, M, C, eps};
    return (int)launch_rmsnorm(a, static_cast<hipStream_t>(hip_stream));
}

namespace {

struct BlockBuffers {
    char *a, *b, *c, *d;        // four (rows, d_inner) bf16 buffers: x then dt | z | x_c | normed then y
    char *dtl, *bm, *cm;        // (rows, dt_rank), (rows, d_state), (rows, d_state) bf16
    char *xpart;                // one token on up to 64 rows: (rows, dt_rank + 2 d_state, d_inner / 32) float32 partial sums
    char *scan_ws;
    size_t scan_ws_bytes, total;
};

int64_t align256(int64_t v) { return (v + 255) / 256 * 256; }

// lays the intermediate tensors of a block out in the workspace; false on a size overflow
bool block_layout(const mamba_block_params_t *p, int64_t batch, int64_t L, void *base, BlockBuffers *bb)
{
    int64_t rows, big, dtl, bc;
    if (!mul_ok(batch, L, &rows)) return false;
    const int64_t wide = p->d_inner > p->d_model ? p->d_inner : p->d_model;
    if (!size3(rows, wide, 1, 2, &big) || !size3(rows, p->dt_rank, 1, 2, &dtl) || !size3(rows, p->d_state, 1, 2, &bc))
        return false;
    int64_t cl, nc;
    scan_plan(batch, L, p->d_inner, p->d_state, 0, &cl, &nc);
    const size_t sws = scan_workspace_bytes(batch, p->d_inner, p->d_state, nc);
    // integer arithmetic on the address: the size queries lay out from a null base
    const uintptr_t q = reinterpret_cast<uintptr_t>(base);
    int64_t off = 0;
    auto take = [&](int64_t n) { char *r = reinterpret_cast<char *>(q + (uintptr_t)off); off += align256(n); return r; };
    bb->a = take(big); bb->b = take(big); bb->c = take(big); bb->d = take(big);
    bb->dtl = take(dtl); bb->bm = take(bc); bb->cm = take(bc);
    int64_t xp = 0;
    if (L == 1 && rows <= 64 && !size3(p->d_inner / 32 + 1, rows, p->dt_rank + 2 * p->d_state, 4, &xp)) return false;
    bb->xpart = take(xp);
    bb->scan_ws = take((int64_t)sws);
    bb->scan_ws_bytes = sws;
    bb->total = (size_t)off;
    return true;
}

int block_params_ok(const mamba_block_params_t *p)
{
    if (!p) return MAMBA_ERR_NULL_POINTER;
    if (p->d_model < 1 || p->d_inner < 1 || p->d_state < 1 || p->dt_rank < 1 || !(p->eps >= 0.0f)) return MAMBA_ERR_BAD_SHAPE;
    if (!n_supported(p->d_state) || !k_supported(p->d_conv) || p->d_model % 8 || p->d_inner % 8 || p->dt_rank % 8 ||
        p->d_model > 4096)
        return MAMBA_ERR_UNSUPPORTED;
    if (!p->norm_w || !p->in_proj_w || !p->conv_w || !p->x_proj_w || !p->dt_proj_w || !p->A || !p->out_proj_w)
        return MAMBA_ERR_NULL_POINTER;
    if (!aligned16(p->norm_w) || !aligned16(p->in_proj_w) || !aligned16(p->conv_w) || !aligned16(p->conv_b) ||
        !aligned16(p->x_proj_w) || !aligned16(p->dt_proj_w) || !aligned16(p->dt_bias) || !aligned16(p->A) ||
        !aligned16(p->Dskip) || !aligned16(p->out_proj_w))
        return MAMBA_ERR_MISALIGNED;
    return MAMBA_OK;
}

}  // namespace

size_t mamba_block_workspace_bytes(const mamba_block_params_t *p, int64_t batch, int64_t L)
{
    if (block_params_ok(p) != MAMBA_OK || batch <= 0 || L <= 0) return 0;
    BlockBuffers bb;
    if (!block_layout(p, batch, L, nullptr, &bb)) return 0;
    return bb.total;
}

int mamba_block_workspace_layout(const mamba_block_params_t *p, int64_t batch, int64_t L, int64_t offsets[7])
{
    const int st = block_params_ok(p);
    if (st != MAMBA_OK) return st;
    if (!offsets) return MAMBA_ERR_NULL_POINTER;
    if (batch <= 0 || L <= 0) return MAMBA_ERR_BAD_SHAPE;
    BlockBuffers bb;
    if (!block_layout(p, batch, L, nullptr, &bb)) return MAMBA_ERR_BAD_SHAPE;
    const void *at[7] = {bb.a, bb.b, bb.c, bb.d, bb.dtl, bb.bm, bb.cm};
    for (int i = 0; i < 7; ++i) offsets[i] = (int64_t)reinterpret_cast<uintptr_t>(at[i]);   // laid out from a null base
    return MAMBA_OK;
}

int mamba_block_fwd(const mamba_block_params_t *p, const void *hidden, void *hidden_out,
                    const void *conv_state_in, void *conv_state_out, const float *h0, float *h_final,
                    void *workspace, size_t workspace_bytes, int64_t batch, int64_t L, void *hip_stream)
{
    const int st = block_params_ok(p);
    if (st != MAMBA_OK) return st;
    if (batch < 0 || L < 0) return MAMBA_ERR_BAD_SHAPE;
    if (batch == 0 || L == 0) return MAMBA_OK;
    if (!hidden || !hidden_out) return MAMBA_ERR_NULL_POINTER;
    if (!aligned16(hidden) || !aligned16(hidden_out) || !aligned16(workspace)) return MAMBA_ERR_MISALIGNED;
    BlockBuffers bb;
    if (!block_layout(p, batch, L, workspace, &bb)) return MAMBA_ERR_BAD_SHAPE;
    if (!workspace || workspace_bytes < bb.total) return MAMBA_ERR_WORKSPACE;
    const int64_t rows = batch * L, Di = p->d_inner, N = p->d_state, R = p->dt_rank;
    const mamba_dtype_t io = MAMBA_BF16;
    int rc;
    // u = rmsnorm(hidden)                                   -> d
    if ((rc = mamba_rmsnorm_fwd(hidden, p->norm_w, bb.d, rows, p->d_model, p->eps, io, hip_stream))) return rc;
    // [x | z] = u W_in^T                                    -> a, b
    if ((rc = mamba_linear_fwd(bb.d, p->in_proj_w, nullptr, nullptr, bb.a, Di, bb.b, Di, nullptr, 0, rows, p->d_model, io, hip_stream))) return rc;
    // x_c = silu(conv1d(x))                                 -> c
    if ((rc = mamba_conv1d_fwd(bb.a, p->conv_w, p->conv_b, conv_state_in, bb.c, conv_state_out, batch, L, Di, p->d_conv, 1, io, hip_stream))) return rc;
    // [dt_low | B | C] = x_c W_x^T
    if ((rc = mamba_linear_fwd(bb.c, p->x_proj_w, nullptr, nullptr, bb.dtl, R, bb.bm, N, bb.cm, N, rows, Di, io, hip_stream))) return rc;
    // dt = dt_low W_dt^T                                    -> a (x is dead)
    if ((rc = mamba_linear_fwd(bb.dtl, p->dt_proj_w, nullptr, nullptr, bb.a, Di, nullptr, 0, nullptr, 0, rows, R, io, hip_stream))) return rc;
    // y = scan(...) gated by silu(z)                        -> d (u is dead)
    if ((rc = mamba_scan_fwd(bb.c, bb.a, p->A, bb.bm, bb.cm, p->Dskip, bb.b, p->dt_bias, h0, bb.d, h_final,
                             bb.scan_ws_bytes ? bb.scan_ws : nullptr, bb.scan_ws_bytes, batch, L, Di, N, 0, 1, io, hip_stream)))
        return rc;
    // hidden_out = hidden + y W_out^T
    return mamba_linear_fwd(bb.d, p->out_proj_w, nullptr, hidden, hidden_out, p->d_model, nullptr, 0, nullptr, 0, rows, Di, io, hip_stream);
}

int mamba_block_step(const mamba_block_params_t *p, const void *hidden, void *hidden_out, const void *conv_src,
                     void *conv_dst, const float *ssm_src, float *ssm_dst, const int32_t *parent_idx,
                     void *workspace, size_t workspace_bytes, int64_t n_out, int64_t n_in, void *hip_stream)
{
    const int st = block_params_ok(p);
    if (st != MAMBA_OK) return st;
    if (n_out < 0 || n_in < 0 || (n_out > 0 && n_in == 0)) return MAMBA_ERR_BAD_SHAPE;
    if (!parent_idx && (n_in != n_out || conv_src != conv_dst || ssm_src != ssm_dst)) return MAMBA_ERR_BAD_SHAPE;
    if (parent_idx && (conv_src == conv_dst || ssm_src == ssm_dst)) return MAMBA_ERR_ALIAS;
    if (n_out == 0) return MAMBA_OK;
    if (!hidden || !hidden_out || !conv_src || !conv_dst || !ssm_src || !ssm_dst) return MAMBA_ERR_NULL_POINTER;
    if (!aligned16(hidden) || !aligned16(hidden_out) || !aligned16(workspace)) return MAMBA_ERR_MISALIGNED;
    BlockBuffers bb;
    if (!block_layout(p, n_out, 1, workspace, &bb)) return MAMBA_ERR_BAD_SHAPE;
    if (!workspace || workspace_bytes < bb.total) return MAMBA_ERR_WORKSPACE;
    const int64_t Di = p->d_inner, N = p->d_state, R = p->dt_rank;
    const mamba_dtype_t io = MAMBA_BF16;
    int rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (n_out > kMaxGridYZ) return MAMBA_ERR_UNSUPPORTED;
    {
        int64_t conv_in_bytes, conv_out_bytes, ssm_in_bytes, ssm_out_bytes, hid_bytes;
        if (!size3(n_in, Di, p->d_conv - 1, 2, &conv_in_bytes) || !size3(n_out, Di, p->d_conv - 1, 2, &conv_out_bytes) ||
            !size3(n_in, Di, N, 4, &ssm_in_bytes) || !size3(n_out, Di, N, 4, &ssm_out_bytes) ||
            !size3(n_out, p->d_model, 1, 2, &hid_bytes))
            return MAMBA_ERR_BAD_SHAPE;
        if (!aligned16(conv_src) || !aligned16(conv_dst) || !aligned16(ssm_src) || !aligned16(ssm_dst) || !aligned16(parent_idx))
            return MAMBA_ERR_MISALIGNED;
        if (parent_idx && (overlap(conv_dst, conv_out_bytes, conv_src, conv_in_bytes) ||
                           overlap(ssm_dst, ssm_out_bytes, ssm_src, ssm_in_bytes)))
            return MAMBA_ERR_ALIAS;
        if (hidden != hidden_out && overlap(hidden, hid_bytes, hidden_out, hid_bytes)) return MAMBA_ERR_ALIAS;
        const void *state_bufs[4] = {conv_src, conv_dst, ssm_src, ssm_dst};
        const int64_t state_bytes[4] = {conv_in_bytes, conv_out_bytes, ssm_in_bytes, ssm_out_bytes};
        for (int i = 0; i < 4; ++i)
            if (overlap(state_bufs[i], state_bytes[i], workspace, (int64_t)bb.total) ||
                overlap(state_bufs[i], state_bytes[i], hidden, hid_bytes) ||
                overlap(state_bufs[i], state_bytes[i], hidden_out, hid_bytes))
                return MAMBA_ERR_ALIAS;
        if (overlap(hidden, hid_bytes, workspace, (int64_t)bb.total) || overlap(hidden_out, hid_bytes, workspace, (int64_t)bb.total))
            return MAMBA_ERR_ALIAS;
    }
    if (n_out <= 64) {
        // A draft position has a few rows and lives on launch latency, so the chain is shortened to four
        // launches: RMSNorm rides into in_proj and the conv step (with the copy of the parent's window)
        // out of it, the dt projection rides in the state step.  (Buffers: z -> b, x_c -> c, y -> d.)
        // [x_c | z] = [silu(conv step(.)) | .] of rmsnorm(hidden) W_in^T; the conv windows move to conv_dst
        LinearArgs in{hidden, p->in_proj_w, nullptr, nullptr, {bb.c, bb.b, nullptr}, {Di, Di, 0}, n_out, p->d_model};
        in.norm_w = p->norm_w;
        in.eps = p->eps;
        in.conv_w = p->conv_w;
        in.conv_b = p->conv_b;
        in.conv_src = conv_src;
        in.conv_dst = conv_dst;
        in.conv_parent = parent_idx;
        in.conv_n_in = n_in;
        in.conv_k = p->d_conv;
        // With a wide enough model the x projection rides along as well: every in_proj workgroup multiplies its 32
        // finished x_c columns into it and the state step adds the partial sums up, which takes the launch of a
        // product with three output tiles out of the chain.
        const bool fuse_xproj = p->d_model > 512 && Di % 128 == 0 && R + 2 * N <= 256;
        if (fuse_xproj) {
            in.xproj_w = p->x_proj_w;
            in.xproj_part = reinterpret_cast<float *>(bb.xpart);
            in.xproj_n = (int)(R + 2 * N);
        }
        if (hipError_t e = launch_linear(in, stream)) return (int)e;
        if (!fuse_xproj &&
            (rc = mamba_linear_fwd(bb.c, p->x_proj_w, nullptr, nullptr, bb.dtl, R, bb.bm, N, bb.cm, N, n_out, Di, io, hip_stream)))
            return rc;
        StepArgs sa{ssm_dst, ssm_src, parent_idx, bb.c, bb.dtl, bb.bm, bb.cm, bb.b, p->A, p->Dskip, p->dt_bias, bb.d,
                    n_out, n_in, Di, (int)N, kIoBf16, 1};
        sa.dt_w = p->dt_proj_w;
        sa.dt_rank = R;
        if (fuse_xproj) {
            sa.xpart = reinterpret_cast<const float *>(bb.xpart);
            sa.n_parts = (int)(Di / 32);
        }
        if (hipError_t e = launch_step(sa, stream)) return (int)e;
        return mamba_linear_fwd(bb.d, p->out_proj_w, nullptr, hidden, hidden_out, p->d_model, nullptr, 0, nullptr, 0, n_out, Di, io, hip_stream);
    }
    if ((rc = mamba_rmsnorm_fwd(hidden, p->norm_w, bb.d, n_out, p->d_model, p->eps, io, hip_stream))) return rc;
    if ((rc = mamba_linear_fwd(bb.d, p->in_proj_w, nullptr, nullptr, bb.a, Di, bb.b, Di, nullptr, 0, n_out, p->d_model, io, hip_stream))) return rc;
    // children read their parent's conv window and leave the shifted window in the destination cache
    {
        ConvArgs cv{bb.a, p->conv_w, p->conv_b, conv_src, bb.c, conv_dst, n_out, 1, Di, p->d_conv, 1, kIoBf16};
        cv.parent = parent_idx;
        cv.n_in = n_in;
        if (hipError_t e = launch_conv1d(cv, stream)) return (int)e;
    }
    if ((rc = mamba_linear_fwd(bb.c, p->x_proj_w, nullptr, nullptr, bb.dtl, R, bb.bm, N, bb.cm, N, n_out, Di, io, hip_stream))) return rc;
    if ((rc = mamba_linear_fwd(bb.dtl, p->dt_proj_w, nullptr, nullptr, bb.a, Di, nullptr, 0, nullptr, 0, n_out, R, io, hip_stream))) return rc;
    if ((rc = mamba_state_step(ssm_dst, ssm_src, parent_idx, bb.c, bb.a, p->A, bb.bm, bb.cm, p->Dskip, bb.b, p->dt_bias, bb.d,
                               n_out, n_in, Di, N, 1, io, hip_stream)))
        return rc;
    return mamba_linear_fwd(bb.d, p->out_proj_w, nullptr, hidden, hidden_out, p->d_model, nullptr, 0, nullptr, 0, n_out, Di, io, hip_stream);
}

int mamba_embedding_fwd(const int32_t *tokens, const void *table, void *out, int64_t M, int64_t V, int64_t dm,
                        mamba_dtype_t io, void *hip_stream)
{
    if (io != MAMBA_BF16) return MAMBA_ERR_UNSUPPORTED;
    int64_t tb, ob;
    if (!size3(V, dm, 1, 2, &tb) || !size3(M, dm, 1, 2, &ob)) return MAMBA_ERR_BAD_SHAPE;
    if (dm % 8 != 0 || M > 0x7fffffff) return MAMBA_ERR_UNSUPPORTED;
    if (M == 0 || dm == 0) return MAMBA_OK;
    if (V == 0) return MAMBA_ERR_BAD_SHAPE;
    if (!tokens || !table || !out) return MAMBA_ERR_NULL_POINTER;
    if (!aligned16(tokens) || !aligned16(table) || !aligned16(out)) return MAMBA_ERR_MISALIGNED;
    if (overlap(out, ob, table, tb) || overlap(out, ob, tokens, M * 4)) return MAMBA_ERR_ALIAS;
    return (int)launch_embedding(tokens, table, out, M, V, dm, static_cast<hipStream_t>(hip_stream));
}

int mamba_topk_fwd(const void *logits, int32_t *idx, float *val, int64_t M, int64_t V, int k, mamba_dtype_t io,
                   void *hip_stream)
{
    if (io != MAMBA_BF16) return MAMBA_ERR_UNSUPPORTED;
    int64_t lb;
    if (!size3(M, V, 1, 2, &lb)) return MAMBA_ERR_BAD_SHAPE;
    if (k < 1 || k > 8 || M > 0x7fffffff || V > ((int64_t)1 << 25)) return MAMBA_ERR_UNSUPPORTED;
    if (M == 0) return MAMBA_OK;
    if (V == 0) return MAMBA_ERR_BAD_SHAPE;
    if (!logits || !idx || !val) return MAMBA_ERR_NULL_POINTER;
    if (!aligned16(logits) || !aligned16(idx) || !aligned16(val)) return MAMBA_ERR_MISALIGNED;
    if (overlap(idx, M * k * 4, logits, lb) || overlap(val, M * k * 4, logits, lb) || overlap(idx, M * k * 4, val, M * k * 4))
        return MAMBA_ERR_ALIAS;
    return (int)launch_topk(logits, idx, val, M, V, k, static_cast<hipStream_t>(hip_stream));
}

namespace {
bool ssd_shape_ok(int64_t P, int64_t N) { return P == 64 && (N == 64 || N == 128); }
}  // namespace

size_t mamba2_ssd_workspace_bytes(int64_t batch, int64_t L, int64_t H, int64_t P, int64_t N)
{
    int64_t t;
    if (batch <= 0 || L <= 0 || H <= 0 || !ssd_shape_ok(P, N)) return 0;
    if (!size3(batch, L / 64 + 2, H, 1, &t) || !size3(t, P, N + 1, 4, &t)) return 0;
    return ssd_workspace_bytes(batch, L, H, P, N);
}

int mamba2_ssd_fwd(const void *x, const void *dt, const float *A, const void *Bm, const void *Cm, const float *Dskip,
                   const void *z, const float *dt_bias, const float *h0, void *out, float *h_final, void *workspace,
                   size_t workspace_bytes, int64_t batch, int64_t L, int64_t H, int64_t P, int64_t N, int dt_softplus,
                   mamba_dtype_t io, void *hip_stream)
{
    if (io != MAMBA_BF16) return MAMBA_ERR_UNSUPPORTED;
    if (batch < 0 || L < 0 || H < 0 || P < 0 || N < 0) return MAMBA_ERR_BAD_SHAPE;
    int64_t hp, tok_bytes, dt_bytes, bc_bytes, st_bytes, t;
    if (!mul_ok(H, P, &hp) || !size3(batch, L, hp, 2, &tok_bytes) || !size3(batch, L, H, 2, &dt_bytes) ||
        !size3(batch, L, N, 2, &bc_bytes) || !size3(batch, hp, N, 4, &st_bytes) ||
        !size3(batch, L / 64 + 2, H, 1, &t) || !size3(t, P, N + 1, 4, &t))
        return MAMBA_ERR_BAD_SHAPE;
    if (!ssd_shape_ok(P, N) || batch > kMaxGridYZ || H > kMaxGridYZ || L > ((int64_t)1 << 31)) return MAMBA_ERR_UNSUPPORTED;
    if (batch == 0 || H == 0) return MAMBA_OK;
    if (L == 0) {
        if (h_final && h_final != h0) {
            if (!aligned16(h_final) || !aligned16(h0)) return MAMBA_ERR_MISALIGNED;
            return (int)launch_copy_state(h0, h_final, batch * hp * N, static_cast<hipStream_t>(hip_stream));
        }
        return MAMBA_OK;
    }
    if (!x || !dt || !A || !Bm || !Cm || !out) return MAMBA_ERR_NULL_POINTER;
    if (!aligned16(x) || !aligned16(dt) || !aligned16(A) || !aligned16(Bm) || !aligned16(Cm) || !aligned16(Dskip) ||
        !aligned16(z) || !aligned16(dt_bias) || !aligned16(h0) || !aligned16(out) || !aligned16(h_final) || !aligned16(workspace))
        return MAMBA_ERR_MISALIGNED;
    const size_t need = ssd_workspace_bytes(batch, L, H, P, N);
    if (!workspace || workspace_bytes < need) return MAMBA_ERR_WORKSPACE;
    if (overlap(out, tok_bytes, x, tok_bytes) || overlap(out, tok_bytes, z, tok_bytes) || overlap(out, tok_bytes, dt, dt_bytes) ||
        overlap(out, tok_bytes, Bm, bc_bytes) || overlap(out, tok_bytes, Cm, bc_bytes) || overlap(out, tok_bytes, h0, st_bytes) ||
        overlap(out, tok_bytes, h_final, st_bytes) || overlap(out, tok_bytes, workspace, (int64_t)need) ||
        overlap(workspace, (int64_t)need, x, tok_bytes) || overlap(workspace, (int64_t)need, z, tok_bytes) ||
        overlap(workspace, (int64_t)need, dt, dt_bytes) || overlap(workspace, (int64_t)need, Bm, bc_bytes) ||
        overlap(workspace, (int64_t)need, Cm, bc_bytes) || overlap(workspace, (int64_t)need, h0, st_bytes) ||
        overlap(workspace, (int64_t)need, h_final, st_bytes) ||
        overlap(h_final, st_bytes, x, tok_bytes) || overlap(h_final, st_bytes, z, tok_bytes))
        return MAMBA_ERR_ALIAS;
    SsdArgs a{x, dt, Bm, Cm, z, A, Dskip, dt_bias, h0, out, h_final, static_cast<float *>(workspace), batch, L, H, (int)P, (int)N,
              dt_softplus};
    return (int)launch_ssd(a, static_cast<hipStream_t>(hip_stream));
}

int mamba2_state_step(float *h_out, const float *h_in, const int32_t *parent_idx, const void *x, const void *dt,
                      const float *A, const void *Bm, const void *Cm, const float *Dskip, const void *z,
                      const float *dt_bias, void *out, int64_t n_out, int64_t n_in, int64_t H, int64_t P, int64_t N,
                      int dt_softplus, mamba_dtype_t io, void *hip_stream)
{
    const int e = io_size(io);
    if (e == 0) return MAMBA_ERR_UNSUPPORTED;
    if (n_out < 0 || n_in < 0 || H < 0 || P < 0 || N < 0) return MAMBA_ERR_BAD_SHAPE;
    int64_t hp, out_bytes, hin_bytes, hout_bytes;
    if (!mul_ok(H, P, &hp) || !size3(n_out, hp, 1, e, &out_bytes) || !size3(n_in, hp, N, 4, &hin_bytes) ||
        !size3(n_out, hp, N, 4, &hout_bytes))
        return MAMBA_ERR_BAD_SHAPE;
    if (!parent_idx && n_in != n_out) return MAMBA_ERR_BAD_SHAPE;
    if (n_out > 0 && n_in == 0) return MAMBA_ERR_BAD_SHAPE;
    if (!ssd_shape_ok(P, N) || n_out > kMaxGridYZ) return MAMBA_ERR_UNSUPPORTED;
    if (n_out == 0 || H == 0) return MAMBA_OK;
    if (!h_out || !h_in || !x || !dt || !A || !Bm || !Cm || !out) return MAMBA_ERR_NULL_POINTER;
    if (!aligned16(h_out) || !aligned16(h_in) || !aligned16(parent_idx) || !aligned16(x) || !aligned16(dt) || !aligned16(A) ||
        !aligned16(Bm) || !aligned16(Cm) || !aligned16(Dskip) || !aligned16(z) || !aligned16(dt_bias) || !aligned16(out))
        return MAMBA_ERR_MISALIGNED;
    if (!(h_out == h_in && !parent_idx) && overlap(h_out, hout_bytes, h_in, hin_bytes)) return MAMBA_ERR_ALIAS;
    if (overlap(out, out_bytes, x, out_bytes) || overlap(out, out_bytes, z, out_bytes) || overlap(out, out_bytes, h_in, hin_bytes) ||
        overlap(out, out_bytes, h_out, hout_bytes) || overlap(h_out, hout_bytes, x, out_bytes) ||
        overlap(h_out, hout_bytes, z, out_bytes))
        return MAMBA_ERR_ALIAS;
    SsdStepArgs a{h_out, h_in, parent_idx, x, dt, Bm, Cm, z, A, Dskip, dt_bias, out, n_out, n_in, H, (int)P, (int)N, (int)io,
                  dt_softplus};
    return (int)launch_ssd_step(a, static_cast<hipStream_t>(hip_stream));
}

int mamba_tree_plan(const int32_t *tree, int gamma, int64_t n_layers, int64_t D, int64_t N, int K,
                    mamba_dtype_t conv_dtype, mamba_tree_plan_t *plan)
{
    if (!tree || !plan) return MAMBA_ERR_NULL_POINTER;
    const int e = io_size(conv_dtype);
    if (e == 0 || !n_supported(N) || !k_supported(K)) return MAMBA_ERR_UNSUPPORTED;
    if (gamma < 1 || gamma > MAMBA_MAX_DEPTH || n_layers < 0 || D < 0) return MAMBA_ERR_BAD_SHAPE;
    int64_t conv_row, ssm_row;
    if (!size3(n_layers, D, K - 1, e, &conv_row) || !size3(n_layers, D, N, 4, &ssm_row)) return MAMBA_ERR_BAD_SHAPE;
    mamba_tree_plan_t p = {};
    p.gamma = gamma;
    p.batch[0] = 1;
    p.cache_of_depth[0] = 0;
    p.parent_offset[0] = -1;
    p.n_caches = 1;
    p.cache_batch[0] = 1;
    for (int i = 1; i <= gamma; ++i) {
        const int64_t fan = tree[i - 1];
        if (fan < 1) return MAMBA_ERR_BAD_SHAPE;
        int64_t b;
        if (!mul_ok(p.batch[i - 1], fan, &b)) return MAMBA_ERR_BAD_SHAPE;
        if (b > kMaxGridYZ) return MAMBA_ERR_UNSUPPORTED;
        p.batch[i] = b;
        if (fan == 1) {
            p.cache_of_depth[i] = p.cache_of_depth[i - 1];
        } else {
            p.cache_of_depth[i] = p.n_caches;
            p.cache_batch[p.n_caches++] = b;
        }
    }
    auto align = [](int64_t v) { return (v + 255) / 256 * 256; };
    int64_t off = 0;
    for (int c = 0; c < p.n_caches; ++c) {
        int64_t cb, sb;
        if (!mul_ok(conv_row, p.cache_batch[c], &cb) || !mul_ok(ssm_row, p.cache_batch[c], &sb) ||
            cb > ((int64_t)1 << 60) || sb > ((int64_t)1 << 60))
            return MAMBA_ERR_BAD_SHAPE;
        p.conv_offset[c] = off;
        off = align(off + cb);
        p.ssm_offset[c] = off;
        off = align(off + sb);
    }
    for (int i = 1; i <= gamma; ++i) {
        if (tree[i - 1] == 1) {
            p.parent_offset[i] = -1;
        } else {
            p.parent_offset[i] = off;
            off = align(off + p.batch[i] * 4);
        }
    }
    p.total_bytes = off;
    *plan = p;
    return MAMBA_OK;
}

int mamba_tree_parents(void *slab, const mamba_tree_plan_t *plan, const int32_t *tree, void *hip_stream)
{
    if (!slab || !plan || !tree) return MAMBA_ERR_NULL_POINTER;
    if (!aligned16(slab)) return MAMBA_ERR_MISALIGNED;
    if (plan->gamma < 1 || plan->gamma > MAMBA_MAX_DEPTH) return MAMBA_ERR_BAD_SHAPE;
    for (int i = 1; i <= plan->gamma; ++i) {
        const bool forks = tree[i - 1] > 1;
        if (tree[i - 1] < 1 || forks != (plan->parent_offset[i] >= 0) ||
            (forks && (plan->parent_offset[i] % 16 != 0 || plan->parent_offset[i] + plan->batch[i] * 4 > plan->total_bytes)))
            return MAMBA_ERR_BAD_SHAPE;  // the plan was not made for this tree
    }
    for (int i = 1; i <= plan->gamma; ++i) {
        if (plan->parent_offset[i] < 0) continue;
        int32_t *dst = reinterpret_cast<int32_t *>(static_cast<char *>(slab) + plan->parent_offset[i]);
        const hipError_t err = launch_tree_parents(dst, plan->batch[i], tree[i - 1], static_cast<hipStream_t>(hip_stream));
        if (err != hipSuccess) return (int)err;
    }
    return MAMBA_OK;
}

}  // extern "C"
