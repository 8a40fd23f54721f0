"""float64 oracle of the Mamba-2 style layer core (scalar decay per head), test infrastructure only.

The paper names Mamba-2 as a drafter that its method carries over to (Sec. 1); the layer is the
state-space-dual (SSD) layer of Dao & Gu, "Transformers are SSMs" (2024), restated here:

    delta[t,h] = softplus(dt[t,h] + dt_bias[h])
    H_t[h]     = exp(delta[t,h] A[h]) H_{t-1}[h] + delta[t,h] x_t[h,:] (outer) B_t          (P x N per head)
    y_t[h,:]   = H_t[h] C_t + D[h] x_t[h,:]          out = y * silu(z)  (when z is given)

with one B_t, C_t in R^N per token shared by all heads (a single group).  Plain loop over time in
numpy float64: the definition written out, nothing chunked or reordered.
"""
import numpy as np


def _softplus(v):
    return np.maximum(v, 0.0) + np.log1p(np.exp(-np.abs(v)))


def _silu(v):
    return v / (1.0 + np.exp(-v))


def ssd_scan(x, dt, A, Bm, Cm, Dskip=None, z=None, dt_bias=None, h0=None, dt_softplus=True):
    """x, z (B,L,H,P); dt (B,L,H); A, Dskip, dt_bias (H); Bm, Cm (B,L,N); h0 (B,H,P,N).
    Returns out (B,L,H,P) and the final state (B,H,P,N)."""
    x = np.asarray(x, dtype=np.float64)
    B_, L, H, P = x.shape
    N = Bm.shape[-1]
    h = np.zeros((B_, H, P, N)) if h0 is None else np.array(h0, dtype=np.float64)
    out = np.empty_like(x)
    for t in range(L):
        v = dt[:, t].astype(np.float64) + (0.0 if dt_bias is None else dt_bias[None, :])
        delta = _softplus(v) if dt_softplus else v
        a = np.exp(delta * A[None, :])
        u = delta[:, :, None] * x[:, t]
        h = a[:, :, None, None] * h + u[..., None] * Bm[:, t][:, None, None, :]
        y = np.einsum("bhpn,bn->bhp", h, Cm[:, t].astype(np.float64))
        if Dskip is not None:
            y = y + Dskip[None, :, None] * x[:, t]
        out[:, t] = y if z is None else y * _silu(z[:, t].astype(np.float64))
    return out, h


def ssd_step(h_in, x, dt, A, Bm, Cm, Dskip=None, z=None, dt_bias=None, parent=None, dt_softplus=True):
    """One token for n_out draft branches: h_in (n_in,H,P,N); x, z (n_out,H,P); dt (n_out,H); Bm, Cm (n_out,N);
    branch j continues from h_in[parent[j]] (h_in[j] without parent).  Returns h_out (n_out,H,P,N), out (n_out,H,P)."""
    src = np.asarray(h_in, dtype=np.float64)
    if parent is not None:
        src = src[np.asarray(parent)]
    out, h = ssd_scan(np.asarray(x)[:, None], np.asarray(dt)[:, None], A, np.asarray(Bm)[:, None], np.asarray(Cm)[:, None],
                      Dskip, None if z is None else np.asarray(z)[:, None], dt_bias, src, dt_softplus)
    return h, out[:, 0]
