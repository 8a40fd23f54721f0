"""ctypes binding of the host-side tree search and verification in libmamba_hip.so
(include/sd_tree_search.h).  Host arrays only; no GPU is touched."""
from __future__ import annotations

import ctypes

import numpy as np

from .binding import lib, MambaError

SD_MAX_ARMS = 32
EXPORTS = ("sd_bandit_init", "sd_bandit_select", "sd_reward", "sd_bandit_update", "sd_verify")


class Bandit(ctypes.Structure):
    """sd_bandit_t."""
    _fields_ = [("n_arms", ctypes.c_int32), ("t", ctypes.c_int64), ("n", ctypes.c_int64 * SD_MAX_ARMS),
                ("reward_sum", ctypes.c_double * SD_MAX_ARMS), ("lambda_ucb", ctypes.c_double),
                ("lambda_gamma", ctypes.c_double)]


_bp = ctypes.POINTER(Bandit)
lib.sd_bandit_init.argtypes = [_bp, ctypes.c_int, ctypes.c_double, ctypes.c_double]
lib.sd_bandit_select.argtypes = [_bp, ctypes.POINTER(ctypes.c_int32)]
lib.sd_reward.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_double, ctypes.POINTER(ctypes.c_double)]
lib.sd_bandit_update.argtypes = [_bp, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32]
lib.sd_verify.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_float, ctypes.c_int32, ctypes.c_int64, ctypes.c_int,
                                                  ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32)]
for _f in EXPORTS:
    getattr(lib, _f).restype = ctypes.c_int


def _check(fn, st):
    if st != 0:
        raise MambaError(fn, st)


def sd_bandit_init(n_arms, lambda_ucb, lambda_gamma) -> Bandit:
    b = Bandit()
    _check("sd_bandit_init", lib.sd_bandit_init(ctypes.byref(b), n_arms, lambda_ucb, lambda_gamma))
    return b


def sd_bandit_select(b: Bandit) -> int:
    arm = ctypes.c_int32(-1)
    _check("sd_bandit_select", lib.sd_bandit_select(ctypes.byref(b), ctypes.byref(arm)))
    return arm.value


def sd_reward(n_accept, gamma, lambda_gamma) -> float:
    r = ctypes.c_double()
    _check("sd_reward", lib.sd_reward(n_accept, gamma, lambda_gamma, ctypes.byref(r)))
    return r.value


def sd_bandit_update(b: Bandit, arm, n_accept, gamma) -> None:
    _check("sd_bandit_update", lib.sd_bandit_update(ctypes.byref(b), arm, n_accept, gamma))


def sd_verify(p, q, draft, u_accept, u_sample, greedy):
    """p (gamma+1, V), q (gamma, V) float32; draft int32[gamma]; returns the emitted tokens."""
    p = np.ascontiguousarray(p, dtype=np.float32)
    q = np.ascontiguousarray(q, dtype=np.float32)
    draft = np.ascontiguousarray(draft, dtype=np.int32)
    u = np.ascontiguousarray(u_accept, dtype=np.float32)
    gamma, V = q.shape
    assert p.shape == (gamma + 1, V) and draft.shape == (gamma,) and u.shape == (gamma,)
    out = np.empty(gamma + 1, dtype=np.int32)
    n = ctypes.c_int32(0)
    st = lib.sd_verify(p.ctypes.data, q.ctypes.data, draft.ctypes.data, u.ctypes.data, float(u_sample), gamma, V,
                       int(bool(greedy)), out.ctypes.data, ctypes.byref(n))
    _check("sd_verify", st)
    return out[:n.value].tolist()
