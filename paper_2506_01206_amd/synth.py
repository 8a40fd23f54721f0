"""Seeded synthetic inputs for the selective-SSM layer core.

This module only draws random numbers and shapes them; it holds none of the
layer's arithmetic and imports neither the GPU binding nor the oracle, so both
can be fed from it.  bfloat16 tensors are carried as uint16 bit patterns
(numpy has no bfloat16); the same rounded bits go to both sides.

Shapes follow a Mamba-130M layer (d_inner 1536, d_state 16, d_conv 4) and a
Mamba-1.4B layer (d_inner 4096); the drafter in the paper is a Mamba-130M
(Sec. 3.1), contexts run to 8k tokens (Sec. 5, long-context table) and trees
are a few steps deep with up to 18 leaves (Sec. 4.1, tree-configuration table).
"""
from __future__ import annotations

import numpy as np

F32 = "f32"
BF16 = "bf16"

# name -> shapes.  "io" is the dtype of x, dt, z, B, C, out and the conv state.
CONFIGS = {
    "cfg0": dict(io=F32, batch=1, L=256, D=256, N=16, K=4, dt_rank=16),
    "cfg1": dict(io=BF16, batch=1, L=2048, D=1536, N=16, K=4, dt_rank=48),
    "cfg2": dict(io=BF16, n_layers=24, branches=32, steps=5, D=1536, N=16, K=4),
    "cfg3": dict(io=BF16, batch=1, L=32768, D=1536, N=16, K=4, dt_rank=48),
    "cfg4": dict(io=BF16, batch=8, L=8192, D=4096, N=16, K=4, dt_rank=128,
                 branches=64, steps=8),
}
SEEDS = {"cfg0": 0, "cfg1": 1, "cfg2": 2, "cfg3": 3, "cfg4": 4}


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns.
    Inputs here are finite, so NaN handling is not needed."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    assert b.dtype == np.uint16
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_io(a: np.ndarray, io: str) -> np.ndarray:
    """float32 values -> storage array of the I/O dtype (float32, or uint16 bf16 bits)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return f32_to_bf16_bits(a) if io == BF16 else a


def io_values(a: np.ndarray, io: str) -> np.ndarray:
    """Storage array -> the float32 values it denotes."""
    return bf16_bits_to_f32(a) if io == BF16 else a


def _normal(rng, shape, std=1.0):
    a = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def layer_params(rng: np.random.Generator, D: int, N: int, K: int, random_A: bool = False):
    """fp32 layer parameters.  A[d,n] = -(n+1) on every row (or -U(0.5,16) when
    random_A); D = 1; dt_bias = inverse softplus of dt0, dt0 log-uniform in
    [1e-3, 0.1] per channel; conv weights U(-0.5, 0.5), conv bias 0."""
    dt0 = np.exp(rng.uniform(np.log(1e-3), np.log(0.1), size=D))
    dt_bias = (dt0 + np.log(-np.expm1(-dt0))).astype(np.float32)
    conv_w = rng.uniform(-0.5, 0.5, size=(D, K)).astype(np.float32)
    if random_A:
        A = -rng.uniform(0.5, 16.0, size=(D, N)).astype(np.float32)
    else:
        A = np.ascontiguousarray(
            np.broadcast_to(-np.arange(1, N + 1, dtype=np.float32), (D, N)))
    return dict(A=A, Dskip=np.ones(D, dtype=np.float32), dt_bias=dt_bias,
                conv_w=conv_w, conv_bias=np.zeros(D, dtype=np.float32))


def token_inputs(rng: np.random.Generator, lead: tuple, D: int, N: int, io: str):
    """x, z ~ N(0,1) (lead..., D); Bm, Cm ~ N(0,1) (lead..., N); dt ~ N(0, std 0.1).
    Draw order: x, z, Bm, Cm, dt.  Returned in the storage dtype of ``io``."""
    x = to_io(_normal(rng, lead + (D,)), io)
    z = to_io(_normal(rng, lead + (D,)), io)
    Bm = to_io(_normal(rng, lead + (N,)), io)
    Cm = to_io(_normal(rng, lead + (N,)), io)
    dt = to_io(_normal(rng, lead + (D,), std=0.1), io)
    return dict(x=x, z=z, Bm=Bm, Cm=Cm, dt=dt)


def prefill_case(batch: int, L: int, D: int, N: int, K: int, io: str, seed: int,
                 random_A: bool = False):
    """One prefill workload: token tensors (B,L,.) then layer parameters."""
    rng = np.random.default_rng(seed)
    case = token_inputs(rng, (batch, L), D, N, io)
    case.update(layer_params(rng, D, N, K, random_A=random_A))
    case.update(io=io, batch=batch, L=L, D=D, N=N, K=K, seed=seed)
    return case


def decode_case(n_layers: int, branches: int, steps: int, D: int, N: int, K: int, io: str,
                seed: int):
    """Tree-decode workload: per layer parameters and N(0,1) initial SSM (fp32) and conv
    (io dtype) states for ``branches`` live branches; per step a parent-index array drawn
    uniformly from [0, branches) and per (step, layer) token inputs for every branch."""
    rng = np.random.default_rng(seed)
    params = [layer_params(rng, D, N, K) for _ in range(n_layers)]
    ssm0 = _normal(rng, (n_layers, branches, D, N))
    conv0 = to_io(_normal(rng, (n_layers, branches, D, K - 1)), io)
    parents = [rng.integers(0, branches, size=branches).astype(np.int32) for _ in range(steps)]
    tokens = [[token_inputs(rng, (branches,), D, N, io) for _ in range(n_layers)]
              for _ in range(steps)]
    return dict(params=params, ssm0=ssm0, conv0=conv0, parents=parents, tokens=tokens,
                io=io, n_layers=n_layers, branches=branches, steps=steps, D=D, N=N, K=K, seed=seed)


def config_prefill(name: str):
    c = CONFIGS[name]
    return prefill_case(c["batch"], c["L"], c["D"], c["N"], c["K"], c["io"], SEEDS[name])


def config_decode(name: str, n_layers=None):
    c = CONFIGS[name]
    nl = c.get("n_layers", 1) if n_layers is None else n_layers
    return decode_case(nl, c["branches"], c["steps"], c["D"], c["N"], c["K"], c["io"],
                       SEEDS[name] + 100)


def block_weights(rng: np.random.Generator, d_model: int, D: int, N: int, K: int, dt_rank: int):
    """Random weights of one Mamba block in storage form: the SSM-core parameters of ``layer_params``
    plus RMSNorm weight ~ 1 + 0.1 N(0,1) (fp32) and projection matrices ~ N(0, 1/fan_in) as bf16 bit
    patterns: in_proj (2D, d_model), x_proj (dt_rank + 2N, D), dt_proj (D, dt_rank), out_proj (d_model, D)."""
    w = layer_params(rng, D, N, K, random_A=True)
    w["conv_b"] = (0.1 * rng.standard_normal(D)).astype(np.float32)
    w.pop("conv_bias")
    w["norm_w"] = (1.0 + 0.1 * rng.standard_normal(d_model)).astype(np.float32)
    mat = lambda n, k: f32_to_bf16_bits((rng.standard_normal((n, k)) / np.sqrt(k)).astype(np.float32))
    w["in_proj_w"] = mat(2 * D, d_model)
    w["x_proj_w"] = mat(dt_rank + 2 * N, D)
    w["dt_proj_w"] = mat(D, dt_rank)
    w["out_proj_w"] = mat(d_model, D)
    return w
