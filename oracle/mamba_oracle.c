/*
 * fp64 CPU oracle for the selective-SSM layer core of a Mamba drafter.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file:
 * it exists so that the GPU kernels can be compared, element by element, with
 * the plain definition of what they compute.  It shares no code, header, table
 * or helper with the GPU library.
 *
 * What is computed (the paper uses Mamba as its drafter and relies on two
 * properties of it: a linear recurrence with a fixed-size state, Sec. 1 and
 * Sec. 3.1, and "the next token needs only the current state", Sec. 4.1; the
 * layer equations themselves are those of the selective SSM it cites):
 *
 *   conv   x_c[b,t,d] = act( bias[d] + sum_{k<K} w[d,k] * xpad[b,t+k,d] )
 *          xpad = [ K-1 carried rows (or zeros) ; x ],  act = SiLU or identity
 *   scan   delta = softplus(dt + dt_bias)            (or dt + dt_bias as is)
 *          h_t[n] = exp(delta_t*A[d,n]) * h_{t-1}[n] + delta_t * B_t[n] * x_t
 *          y_t    = sum_n C_t[n]*h_t[n] + D[d]*x_t
 *          out_t  = y_t * silu(z_t)                  (no gate when z absent)
 *   step   the scan with L = 1 for every draft branch j, the previous state
 *          taken from branch parent[j] (Sec. 4.1: a child copies the state of
 *          its parent node and continues from there)
 *   fork   dst[l,j] = src[l,parent[j]]: a byte copy (Sec. 4.1, state copy;
 *          separate pre-allocated buffers per batch size => out of place)
 *
 * Everything is plain loops in double precision, in the order of the
 * definition: no blocking, no fusion, no reordering.  OpenMP only distributes
 * independent (batch, channel) recurrences over threads; each recurrence is
 * evaluated sequentially in time.
 *
 * Layout (row-major, contiguous): x, dt, z, out: (B, L, D); Bm, Cm: (B, L, N);
 * A: (D, N); Dskip, dt_bias, bias: (D); w: (D, K); h: (B, D, N);
 * conv_state: (B, D, K-1), oldest sample first.
 *
 * Pins (tests/test_oracle_pins.py): geometric-series closed form, A = 0 ->
 * cumulative sum, independent unrolled form on tiny inputs, scan == repeated
 * step, chunk carry, delta -> 0, linearity, special cases, conv == Toeplitz /
 * numpy.convolve, fork == fancy indexing.  No function is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double softplus_exact(double v)
{
    /* log(1 + e^v) without overflow or cancellation, no threshold */
    return fmax(v, 0.0) + log1p(exp(-fabs(v)));
}

static double silu(double v)
{
    return v / (1.0 + exp(-v));
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* Depthwise causal conv1d over time, one filter of K taps per channel. */
void oracle_conv1d_fwd(const double *x, const double *w, const double *bias,
                       const double *conv_state_in, double *y,
                       double *conv_state_out, long B, long L, long D, int K,
                       int apply_silu)
{
    const long H = K - 1; /* rows of left context */
#pragma omp parallel for collapse(2) schedule(static)
    for (long b = 0; b < B; ++b) {
        for (long d = 0; d < D; ++d) {
            /* xpad(r): row r of [state ; x] for this (b, d) */
#define XPAD(r)                                                               \
    ((r) < H ? (conv_state_in ? conv_state_in[(b * D + d) * H + (r)] : 0.0)   \
             : x[(b * L + ((r) - H)) * D + d])
            for (long t = 0; t < L; ++t) {
                double acc = bias ? bias[d] : 0.0;
                for (int k = 0; k < K; ++k)
                    acc += w[d * K + k] * XPAD(t + k);
                y[(b * L + t) * D + d] = apply_silu ? silu(acc) : acc;
            }
            if (conv_state_out) {
                double tmp[64];
                for (long k = 0; k < H; ++k) tmp[k] = XPAD(L + k);
                for (long k = 0; k < H; ++k)
                    conv_state_out[(b * D + d) * H + k] = tmp[k];
            }
#undef XPAD
        }
    }
}

/* Selective scan over L tokens. */
void oracle_scan_fwd(const double *x, const double *dt, const double *A,
                     const double *Bm, const double *Cm, const double *Dskip,
                     const double *z, const double *dt_bias, const double *h0,
                     double *out, double *h_final, long B, long L, long D,
                     long N, int dt_softplus)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (long b = 0; b < B; ++b) {
        for (long d = 0; d < D; ++d) {
            double h[256];
            for (long n = 0; n < N; ++n)
                h[n] = h0 ? h0[(b * D + d) * N + n] : 0.0;
            for (long t = 0; t < L; ++t) {
                const long i = (b * L + t) * D + d;
                const double xv = x[i];
                double v = dt[i] + (dt_bias ? dt_bias[d] : 0.0);
                const double delta = dt_softplus ? softplus_exact(v) : v;
                double yv = 0.0;
                for (long n = 0; n < N; ++n) {
                    const double abar = exp(delta * A[d * N + n]);
                    h[n] = abar * h[n] + delta * Bm[(b * L + t) * N + n] * xv;
                    yv += Cm[(b * L + t) * N + n] * h[n];
                }
                if (Dskip) yv += Dskip[d] * xv;
                out[i] = z ? yv * silu(z[i]) : yv;
            }
            if (h_final)
                for (long n = 0; n < N; ++n)
                    h_final[(b * D + d) * N + n] = h[n];
        }
    }
}

/* One recurrence step for n_out branches; branch j continues from the state of
 * branch parent[j] (identity when parent is NULL).  h_out may not alias h_in
 * unless parent is NULL. */
void oracle_state_step(double *h_out, const double *h_in,
                       const int32_t *parent, const double *x,
                       const double *dt, const double *A, const double *Bm,
                       const double *Cm, const double *Dskip, const double *z,
                       const double *dt_bias, double *out, long n_out,
                       long n_in, long D, long N, int dt_softplus)
{
    (void)n_in;
#pragma omp parallel for collapse(2) schedule(static)
    for (long j = 0; j < n_out; ++j) {
        for (long d = 0; d < D; ++d) {
            const long p = parent ? (long)parent[j] : j;
            const double xv = x[j * D + d];
            double v = dt[j * D + d] + (dt_bias ? dt_bias[d] : 0.0);
            const double delta = dt_softplus ? softplus_exact(v) : v;
            double yv = 0.0;
            for (long n = 0; n < N; ++n) {
                const double abar = exp(delta * A[d * N + n]);
                const double hn = abar * h_in[(p * D + d) * N + n] +
                                  delta * Bm[j * N + n] * xv;
                h_out[(j * D + d) * N + n] = hn;
                yv += Cm[j * N + n] * hn;
            }
            if (Dskip) yv += Dskip[d] * xv;
            out[j * D + d] = z ? yv * silu(z[j * D + d]) : yv;
        }
    }
}

/* State fork: rows of conv_row_bytes / ssm_row_bytes are copied as bytes.
 * Either pair of pointers may be NULL. */
void oracle_state_fork(void *conv_dst, const void *conv_src, void *ssm_dst,
                       const void *ssm_src, const int32_t *parent,
                       long n_layers, long n_out, long n_in,
                       long conv_row_bytes, long ssm_row_bytes)
{
    for (long l = 0; l < n_layers; ++l) {
        for (long j = 0; j < n_out; ++j) {
            const long p = parent[j];
            if (conv_dst && conv_src)
                memcpy((char *)conv_dst + (l * n_out + j) * conv_row_bytes,
                       (const char *)conv_src + (l * n_in + p) * conv_row_bytes,
                       (size_t)conv_row_bytes);
            if (ssm_dst && ssm_src)
                memcpy((char *)ssm_dst + (l * n_out + j) * ssm_row_bytes,
                       (const char *)ssm_src + (l * n_in + p) * ssm_row_bytes,
                       (size_t)ssm_row_bytes);
        }
    }
}
