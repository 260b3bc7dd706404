"""ctypes front end of ``espo_oracle.c`` (numpy arrays in, numpy arrays out).

TEST INFRASTRUCTURE ONLY: argument marshalling for the plain C oracle; all the
arithmetic lives in the C file next to this one.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "espo_oracle.c")
_LIB = os.path.join(_HERE, "libespo_oracle.so")

F32, BF16 = 0, 1


def build_oracle(force: bool = False) -> str:
    """Compile the oracle with gcc (no GPU toolchain involved)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fPIC", "-shared", "-std=c11", "-ffp-contract=off", "-fno-fast-math",
               "-fopenmp", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Params(C.Structure):
    _fields_ = [("mu_g", C.c_float), ("var_g", C.c_float), ("delta", C.c_float),
                ("clip_c", C.c_float), ("alpha_s", C.c_float), ("beta", C.c_float),
                ("eps", C.c_float), ("stop_enabled", C.c_int32), ("eos_id", C.c_int32),
                ("stop_mode", C.c_int32), ("stop_threshold", C.c_float), ("simulate", C.c_int32),
                ("top_p", C.c_float), ("top_k", C.c_int32)]


@dataclass
class OracleParams:
    """Frozen rollout parameters (Algorithm 1 'Require'; Eq. normalized_gap, Eq. stop_rule)."""
    mu_g: float = 0.0
    var_g: float = 1.0
    delta: float = 1e-8
    clip_c: float = 10.0
    alpha_s: float = 0.9
    beta: float = 7.0
    eps: float = 0.2
    stop_enabled: int = 1
    eos_id: int = -1
    stop_mode: int = 0          # 0 Eq. stop_rule; 1 value only; 2 regret only; 3 random (ablations D, E, F)
    stop_threshold: float = 0.0
    simulate: int = 0           # record the first stop step, keep decoding
    top_p: float = 0.0          # nucleus sampling (0 or >= 1: off)
    top_k: int = 0              # keep the k largest logits (<= 0: off)

    def c_struct(self) -> _Params:
        return _Params(self.mu_g, self.var_g, self.delta, self.clip_c, self.alpha_s, self.beta,
                       self.eps, int(self.stop_enabled), int(self.eos_id), int(self.stop_mode),
                       float(self.stop_threshold), int(self.simulate), float(self.top_p), int(self.top_k))


_lib = None


def _load():
    global _lib
    if _lib is None:
        build_oracle()
        lib = C.CDLL(_LIB)
        vp, i64, i32, u64, f32 = C.c_void_p, C.c_int64, C.c_int32, C.c_uint64, C.c_float
        lib.oracle_step.restype = C.c_int
        lib.oracle_step.argtypes = [vp, C.c_int, i64, i64, i64, f32, u64, i32, vp, C.POINTER(_Params),
                                    vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        lib.oracle_state_update.restype = C.c_int
        lib.oracle_state_update.argtypes = [i64, vp, vp, vp, C.POINTER(_Params), u64, i32, vp, vp, vp]
        lib.oracle_advantages.restype = C.c_int
        lib.oracle_advantages.argtypes = [vp, vp, vp, vp, i64, i64, f32, f32, f32, vp, vp, vp]
        lib.oracle_whiten.restype = C.c_int
        lib.oracle_whiten.argtypes = [vp, vp, i64, i64, f32, C.c_int, C.c_int, vp, vp]
        lib.oracle_advantages_packed.restype = C.c_int
        lib.oracle_advantages_packed.argtypes = [vp, vp, vp, vp, vp, i64, i64, f32, f32, f32, vp, vp, vp, vp]
        lib.oracle_advantages_terminal.restype = C.c_int
        lib.oracle_advantages_terminal.argtypes = [vp, vp, vp, vp, i64, i64, f32, f32, f32, vp, vp, vp]
        lib.oracle_gae_bruteforce.restype = C.c_int
        lib.oracle_gae_bruteforce.argtypes = [vp, vp, vp, vp, i64, i64, f32, f32, f32, vp]
        lib.oracle_batch_stats.restype = C.c_int
        lib.oracle_batch_stats.argtypes = [vp, vp, vp, i64, i64, f32, f32, f32, f32, f32, f32, f32, f32, vp]
        lib.oracle_philox4x32_10.restype = None
        lib.oracle_philox4x32_10.argtypes = [vp, vp, vp]
        lib.oracle_stream_word.restype = C.c_uint32
        lib.oracle_stream_word.argtypes = [u64, i64, i32, i64]
        lib.oracle_uniform.restype = C.c_double
        lib.oracle_uniform.argtypes = [C.c_uint32]
        lib.oracle_gumbel.restype = C.c_double
        lib.oracle_gumbel.argtypes = [C.c_uint32]
        lib.oracle_gumbel_at.restype = C.c_double
        lib.oracle_gumbel_at.argtypes = [u64, i64, i32, i64, i64]
        lib.oracle_block_draw.restype = None
        lib.oracle_block_draw.argtypes = [u64, i64, i32, i64, i64, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        lib.oracle_num_threads.restype = C.c_int
        lib.oracle_set_threads.argtypes = [C.c_int]
        _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(a, dtype, shape=None, name="array"):
    if not isinstance(a, np.ndarray) or a.dtype != dtype or not a.flags.c_contiguous:
        raise TypeError(f"{name}: need C-contiguous numpy array of {dtype}")
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"{name}: shape {a.shape} != {shape}")
    return a


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_threads(n: int) -> None:
    _load().oracle_set_threads(int(n))


def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    assert c.shape == (4,) and k.shape == (2,)
    out = np.zeros(4, dtype=np.uint32)
    _load().oracle_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def stream_word(seed: int, row: int, step_: int, v: int) -> int:
    return int(_load().oracle_stream_word(seed, row, step_, v))


def uniform(word: int) -> float:
    return float(_load().oracle_uniform(word))


def gumbel(word: int) -> float:
    return float(_load().oracle_gumbel(word))


def gumbel_at(seed: int, row: int, step_: int, v: int, V: int) -> float:
    """Gumbel variate G_v of vocabulary index v in a row of V entries."""
    return float(_load().oracle_gumbel_at(seed, row, step_, v, V))


def block_draw(seed: int, row: int, step_: int, q: int, n: int):
    """(M_q, pos_q): maximum of block q's variates and the offset that attains it."""
    M = C.c_double()
    pos = C.c_int64()
    _load().oracle_block_draw(seed, row, step_, q, n, C.byref(M), C.byref(pos))
    return float(M.value), int(pos.value)


def step(logits: np.ndarray, temperature: float, seed: int, step_: int, values: np.ndarray,
         params: OracleParams, z: np.ndarray, alive: np.ndarray, stop_step: np.ndarray,
         V: int | None = None, forced_tokens: np.ndarray | None = None, want_logprob: bool = True,
         want_entropy: bool = False):
    """One decode step.  ``logits`` is [B, row_stride] float32, or uint16 holding bf16 bits.

    ``z``, ``alive``, ``stop_step`` are updated in place.  Returns a dict with tokens,
    regret, logprob and the diagnostics of the draw (best/second score, runner-up,
    softmax sum, row maximum); with ``want_entropy`` also the entropy of the distribution
    the token is drawn from.
    """
    lib = _load()
    if logits.dtype == np.float32:
        dt = F32
    elif logits.dtype == np.uint16:
        dt = BF16
    else:
        raise TypeError("logits must be float32 or uint16 (bf16 bit patterns)")
    assert logits.ndim == 2 and logits.flags.c_contiguous
    B, stride = logits.shape
    V = stride if V is None else int(V)
    _chk(values, np.float32, (B,), "values")
    _chk(z, np.float32, (B,), "z")
    _chk(alive, np.uint8, (B,), "alive")
    _chk(stop_step, np.int32, (B,), "stop_step")
    if forced_tokens is not None:
        _chk(forced_tokens, np.int32, (B,), "forced_tokens")
    out = {
        "tokens": np.empty(B, np.int32), "regret": np.empty(B, np.float32),
        "logprob": np.empty(B, np.float32) if want_logprob else None,
        "best_score": np.empty(B, np.float64), "second_score": np.empty(B, np.float64),
        "second_token": np.empty(B, np.int32), "sum_exp": np.empty(B, np.float64),
        "row_max": np.empty(B, np.float32),
        "entropy": np.empty(B, np.float32) if want_entropy else None,
        "kept": np.empty(B, np.int64),
    }
    ps = params.c_struct()
    rc = lib.oracle_step(_ptr(logits), dt, B, V, stride, float(temperature), int(seed), int(step_),
                         _ptr(values), C.byref(ps), _ptr(z), _ptr(alive), _ptr(stop_step),
                         _ptr(out["tokens"]), _ptr(out["regret"]), _ptr(out["logprob"]),
                         _ptr(forced_tokens), _ptr(out["best_score"]), _ptr(out["second_score"]),
                         _ptr(out["second_token"]), _ptr(out["sum_exp"]), _ptr(out["row_max"]),
                         _ptr(out["entropy"]), _ptr(out["kept"]))
    if rc != 0:
        raise ValueError("oracle_step: invalid arguments")
    return out


def state_update(g: np.ndarray, tokens: np.ndarray, values: np.ndarray, params: OracleParams,
                 step_: int, z: np.ndarray, alive: np.ndarray, stop_step: np.ndarray, seed: int = 0) -> None:
    """Advance (z, alive, stop_step) in place from a given regret/token vector (`seed` only
    matters for the random stop mode)."""
    B = g.shape[0]
    _chk(g, np.float32, (B,), "g")
    _chk(tokens, np.int32, (B,), "tokens")
    _chk(values, np.float32, (B,), "values")
    _chk(z, np.float32, (B,), "z")
    _chk(alive, np.uint8, (B,), "alive")
    _chk(stop_step, np.int32, (B,), "stop_step")
    ps = params.c_struct()
    rc = _load().oracle_state_update(B, _ptr(g), _ptr(tokens), _ptr(values), C.byref(ps), int(seed), int(step_),
                                     _ptr(z), _ptr(alive), _ptr(stop_step))
    if rc != 0:
        raise ValueError("oracle_state_update: invalid arguments")


def advantages(rewards: np.ndarray, values: np.ndarray, lengths: np.ndarray, stopped: np.ndarray,
               r_fail: float, gamma: float, lam: float, want_scale: bool = True):
    """TD errors and GAE (double) on truncated trajectories; also the |.|-weighted scale."""
    assert rewards.ndim == 2
    B, T = rewards.shape
    _chk(rewards, np.float32, (B, T), "rewards")
    _chk(values, np.float32, (B, T), "values")
    _chk(lengths, np.int32, (B,), "lengths")
    _chk(stopped, np.uint8, (B,), "stopped")
    td = np.empty((B, T), np.float64)
    adv = np.empty((B, T), np.float64)
    scale = np.empty((B, T), np.float64) if want_scale else None
    rc = _load().oracle_advantages(_ptr(rewards), _ptr(values), _ptr(lengths), _ptr(stopped), B, T,
                                   float(r_fail), float(gamma), float(lam), _ptr(td), _ptr(adv),
                                   _ptr(scale))
    if rc != 0:
        raise ValueError("oracle_advantages: invalid arguments")
    return td, adv, scale


def advantages_terminal(values: np.ndarray, lengths: np.ndarray, stopped: np.ndarray,
                        terminal_reward: np.ndarray, r_fail: float, gamma: float, lam: float):
    """TD errors, GAE and value targets (double) when every reward but the last is zero."""
    B, T = values.shape
    _chk(values, np.float32, (B, T), "values")
    _chk(lengths, np.int32, (B,), "lengths")
    _chk(stopped, np.uint8, (B,), "stopped")
    _chk(terminal_reward, np.float32, (B,), "terminal_reward")
    td, adv, ret = (np.empty((B, T), np.float64) for _ in range(3))
    rc = _load().oracle_advantages_terminal(_ptr(values), _ptr(lengths), _ptr(stopped), _ptr(terminal_reward), B, T,
                                            float(r_fail), float(gamma), float(lam), _ptr(td), _ptr(adv), _ptr(ret))
    if rc != 0:
        raise ValueError("oracle_advantages_terminal: invalid arguments")
    return td, adv, ret


def advantages_packed(rewards, terminal_reward, values: np.ndarray, cu_seqlens: np.ndarray, stopped: np.ndarray,
                      r_fail: float, gamma: float, lam: float):
    """TD errors, GAE, value targets and the scale (double) for trajectories stored back to
    back: trajectory b is values[cu_seqlens[b]:cu_seqlens[b+1]].  `rewards` (same layout) or,
    if it is None, `terminal_reward` [B] with zero reward before the last step.  Positions no
    trajectory owns come back as NaN."""
    N = values.shape[0]
    B = stopped.shape[0]
    _chk(values, np.float32, (N,), "values")
    _chk(cu_seqlens, np.int64, (B + 1,), "cu_seqlens")
    _chk(stopped, np.uint8, (B,), "stopped")
    if rewards is not None:
        _chk(rewards, np.float32, (N,), "rewards")
    if terminal_reward is not None:
        _chk(terminal_reward, np.float32, (B,), "terminal_reward")
    td, adv, ret, scale = (np.full(N, np.nan, np.float64) for _ in range(4))
    rc = _load().oracle_advantages_packed(_ptr(rewards) if rewards is not None else None,
                                          _ptr(terminal_reward) if terminal_reward is not None else None,
                                          _ptr(values), _ptr(cu_seqlens), _ptr(stopped), B, N, float(r_fail),
                                          float(gamma), float(lam), _ptr(td), _ptr(adv), _ptr(ret), _ptr(scale))
    if rc != 0:
        raise ValueError("oracle_advantages_packed: invalid arguments")
    return td, adv, ret, scale


def whiten(adv: np.ndarray, lengths: np.ndarray, eps: float = 1e-8, shift_mean: bool = True, unbiased: bool = False):
    """Whitened advantages (double; NaN where t >= L) and (mean, var, n) over the valid tokens."""
    B, T = adv.shape
    _chk(adv, np.float32, (B, T), "adv")
    _chk(lengths, np.int32, (B,), "lengths")
    out = np.full((B, T), np.nan, np.float64)
    stats = np.zeros(3, np.float64)
    rc = _load().oracle_whiten(_ptr(adv), _ptr(lengths), B, T, float(eps), int(bool(shift_mean)), int(bool(unbiased)),
                               _ptr(out), _ptr(stats))
    if rc != 0:
        raise ValueError("oracle_whiten: invalid arguments")
    return out, stats


def gae_bruteforce(rewards: np.ndarray, values: np.ndarray, lengths: np.ndarray, stopped: np.ndarray,
                   r_fail: float, gamma: float, lam: float) -> np.ndarray:
    """Eq. gae as the explicit O(L^2) double sum."""
    B, T = rewards.shape
    _chk(rewards, np.float32, (B, T), "rewards")
    _chk(values, np.float32, (B, T), "values")
    _chk(lengths, np.int32, (B,), "lengths")
    _chk(stopped, np.uint8, (B,), "stopped")
    adv = np.empty((B, T), np.float64)
    rc = _load().oracle_gae_bruteforce(_ptr(rewards), _ptr(values), _ptr(lengths), _ptr(stopped), B, T,
                                       float(r_fail), float(gamma), float(lam), _ptr(adv))
    if rc != 0:
        raise ValueError("oracle_gae_bruteforce: invalid arguments")
    return adv


def batch_stats(regret: np.ndarray, lengths: np.ndarray, stopped: np.ndarray, mu_g: float, var_g: float,
                beta: float, alpha_ema: float, eta_beta: float, target_rate: float, beta_min: float,
                beta_max: float) -> dict:
    """Batch mean / variance of the regret over valid tokens, stop rate, and the updated
    (mu_g, var_g, beta) of Section 4.2 and Eq. beta_update."""
    assert regret.ndim == 2
    B, T = regret.shape
    _chk(regret, np.float32, (B, T), "regret")
    _chk(lengths, np.int32, (B,), "lengths")
    _chk(stopped, np.uint8, (B,), "stopped")
    out = np.zeros(7, np.float64)
    rc = _load().oracle_batch_stats(_ptr(regret), _ptr(lengths), _ptr(stopped), B, T, float(mu_g), float(var_g),
                                    float(beta), float(alpha_ema), float(eta_beta), float(target_rate),
                                    float(beta_min), float(beta_max), _ptr(out))
    if rc != 0:
        raise ValueError("oracle_batch_stats: invalid arguments")
    return {"mean": out[0], "var": out[1], "stop_rate": out[2], "mu_g": np.float32(out[3]),
            "var_g": np.float32(out[4]), "beta": np.float32(out[5]), "tokens": int(out[6])}
