"""ctypes binding of libespo.so: same names as the C ABI, argument marshalling only.

Tensors are torch tensors on the GPU (used for their device pointers and the current
HIP stream); every step of the path runs in the library's kernels.  There is no CPU
fallback: if the shared library is missing the first call raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libespo.so")
_lib = None

ESPO_F32, ESPO_BF16 = 0, 1


class EspoError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"espo error {code}: {text}")
        self.code = code


class _Params(C.Structure):
    _fields_ = [("mu_g", C.c_float), ("var_g", C.c_float), ("delta", C.c_float),
                ("clip_c", C.c_float), ("alpha_s", C.c_float), ("beta", C.c_float),
                ("eps", C.c_float), ("stop_enabled", C.c_int32), ("eos_id", C.c_int32),
                ("stop_mode", C.c_int32), ("stop_threshold", C.c_float), ("simulate", C.c_int32),
                ("top_p", C.c_float), ("top_k", C.c_int32)]


@dataclass
class EspoParams:
    """Mirror of `espo_params` (include/espo.h)."""
    mu_g: float = 0.0
    var_g: float = 1.0
    delta: float = 1e-8
    clip_c: float = 10.0
    alpha_s: float = 0.9
    beta: float = 7.0
    eps: float = 0.2
    stop_enabled: int = 1
    eos_id: int = -1
    stop_mode: int = 0          # espo_stop_mode: 0 Eq. stop_rule, 1 value only, 2 regret only, 3 random
    stop_threshold: float = 0.0
    simulate: int = 0
    top_p: float = 0.0          # nucleus filter on the draw (0 or >= 1: off)
    top_k: int = 0              # top-k filter on the draw (<= 0: off)

    def _c(self) -> _Params:
        return _Params(self.mu_g, self.var_g, self.delta, self.clip_c, self.alpha_s, self.beta,
                       self.eps, int(self.stop_enabled), int(self.eos_id), int(self.stop_mode),
                       float(self.stop_threshold), int(self.simulate), float(self.top_p), int(self.top_k))


def library_path() -> str:
    return _LIB_PATH


class _BatchCtrl(C.Structure):
    _fields_ = [("alpha_ema", C.c_float), ("eta_beta", C.c_float), ("target_rate", C.c_float),
                ("beta_min", C.c_float), ("beta_max", C.c_float)]


class _BatchResult(C.Structure):
    _fields_ = [("mean_g", C.c_double), ("var_g_batch", C.c_double), ("stop_rate", C.c_double),
                ("tokens", C.c_int64), ("mu_g", C.c_float), ("var_g", C.c_float), ("beta", C.c_float),
                ("stopped", C.c_int32)]


BATCH_RESULT_BYTES = C.sizeof(_BatchResult)


def load_library():
    """Loads libespo.so (built in-tree by `build.py`); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2605_29860_amd.build` "
                "(there is no fallback path)")
        lib = C.CDLL(_LIB_PATH)
        vp, i64, i32, u64, f32, sz = C.c_void_p, C.c_int64, C.c_int32, C.c_uint64, C.c_float, C.c_size_t
        lib.espo_step.restype = C.c_int
        lib.espo_step.argtypes = [vp, C.c_int, i64, i64, i64, f32, u64, i32, vp, C.POINTER(_Params),
                                  vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.espo_step_workspace_bytes.restype = sz
        lib.espo_step_workspace_bytes.argtypes = [i64, i64, C.c_int]
        lib.espo_advantages.restype = C.c_int
        lib.espo_whiten.restype = C.c_int
        lib.espo_whiten.argtypes = [vp, vp, i64, i64, f32, i32, i32, vp, vp, vp, C.c_size_t, vp]
        lib.espo_whiten_workspace_bytes.restype = C.c_size_t
        lib.espo_whiten_workspace_bytes.argtypes = [i64, i64]
        lib.espo_advantages_packed.restype = C.c_int
        lib.espo_advantages_packed.argtypes = [vp, vp, vp, vp, vp, i64, i64, f32, f32, f32, vp, vp, vp, vp]
        lib.espo_advantages_terminal.restype = C.c_int
        lib.espo_advantages_terminal.argtypes = [vp, vp, vp, vp, i64, i64, f32, f32, f32, i32, vp, vp, vp, vp]
        lib.espo_advantages.argtypes = [vp, vp, vp, vp, i64, i64, f32, f32, f32, vp, vp, vp]
        lib.espo_advantages_ws.restype = C.c_int
        lib.espo_advantages_ws.argtypes = [vp, vp, vp, vp, i64, i64, f32, f32, f32, vp, vp, vp, vp, sz, vp]
        lib.espo_advantages_terminal_ws.restype = C.c_int
        lib.espo_advantages_terminal_ws.argtypes = [vp, vp, vp, vp, i64, i64, f32, f32, f32, i32, vp, vp, vp, vp, vp, sz, vp]
        lib.espo_length_order.restype = C.c_int
        lib.espo_length_order.argtypes = [vp, i64, i64, vp, vp]
        lib.espo_advantages_ws_bytes.restype = sz
        lib.espo_advantages_ws_bytes.argtypes = [i64]
        lib.espo_whiten_from_ws.restype = C.c_int
        lib.espo_whiten_from_ws.argtypes = [vp, vp, i64, i64, f32, i32, i32, vp, vp, vp, sz, vp]
        lib.espo_strerror.restype = C.c_char_p
        lib.espo_strerror.argtypes = [C.c_int]
        lib.espo_version.restype = C.c_int
        lib.espo_debug_step.restype = C.c_int
        lib.espo_debug_step.argtypes = lib.espo_step.argtypes + [f32, i32, i32]
        lib.espo_debug_step_workspace_bytes.restype = sz
        lib.espo_debug_step_workspace_bytes.argtypes = [i64, i32]
        lib.espo_debug_read.restype = C.c_int
        lib.espo_debug_read.argtypes = [vp, sz, vp, vp]
        lib.espo_debug_sweep.restype = C.c_int
        lib.espo_debug_sweep.argtypes = [vp, sz, vp, sz, vp]
        lib.espo_debug_sweep_padded.restype = C.c_int
        lib.espo_debug_sweep_padded.argtypes = [vp, vp, vp, i64, i64, vp, vp, vp]
        lib.espo_debug_math_errors.restype = C.c_int
        lib.espo_debug_math_errors.argtypes = [C.c_void_p, C.c_void_p]
        lib.espo_batch_stats.restype = C.c_int
        lib.espo_batch_stats.argtypes = [vp, vp, vp, i64, i64, f32, f32, f32, C.POINTER(_BatchCtrl), vp, vp, sz, vp]
        lib.espo_batch_stats_static.restype = C.c_int
        lib.espo_batch_stats_static.argtypes = [vp, vp, vp, i64, i64, f32, f32, f32, C.POINTER(_BatchCtrl), vp, vp]
        lib.espo_batch_stats_workspace_bytes.restype = sz
        lib.espo_batch_stats_workspace_bytes.argtypes = [i64, i64]
        lib.espo_debug_copy.restype = C.c_int
        lib.espo_debug_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        _lib = lib
    return _lib


def _check(rc: int):
    if rc != 0:
        raise EspoError(rc, load_library().espo_strerror(rc).decode())


def _on_gpu(t: torch.Tensor) -> bool:
    return t.is_cuda


def _dev(t: torch.Tensor, dtype, name: str, numel: int | None = None, shape: tuple | None = None):
    """Device pointer of a tensor after checking what the C ABI cannot: placement, type, layout and size.
    The library takes bare pointers, so a tensor that is too short would become an out-of-bounds access
    on the GPU; it is refused here instead (`numel`: at least that many elements; `shape`: exactly that)."""
    if t is None:
        return None
    if not _on_gpu(t) or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name}: need a contiguous GPU tensor of {dtype}")
    if numel is not None and t.numel() < numel:
        raise ValueError(f"{name}: need at least {numel} elements, got {t.numel()}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: need shape {tuple(shape)}, got {tuple(t.shape)}")
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def espo_debug_math_errors(out: torch.Tensor, stream=None) -> None:
    """Diagnostics: accuracy of the hardware ln / exp on this device (see include/espo_debug.h); `out` = 3 zeroed floats."""
    _check(load_library().espo_debug_math_errors(_dev(out, torch.float32, "out", numel=3), _stream(stream)))


def espo_debug_read(src: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    """Diagnostics: bare streaming read of `src` (see include/espo_debug.h); `sink`: at least 4 bytes on the GPU."""
    if not src.is_cuda or not src.is_contiguous() or not sink.is_cuda or sink.numel() * sink.element_size() < 4:
        raise TypeError("src: contiguous GPU tensor; sink: GPU tensor of at least 4 bytes")
    _check(load_library().espo_debug_read(C.c_void_p(src.data_ptr()), src.numel() * src.element_size(),
                                          C.c_void_p(sink.data_ptr()), _stream(stream)))


def espo_debug_sweep(src: torch.Tensor, read_bytes: int, dst: torch.Tensor, write_bytes: int, stream=None) -> None:
    """Diagnostics: flat sweep that reads `read_bytes` of src and writes `write_bytes` of dst (see include/espo_debug.h)."""
    for name, t, n in (("src", src, read_bytes), ("dst", dst, write_bytes)):
        if not t.is_cuda or not t.is_contiguous() or t.numel() * t.element_size() < n:
            raise ValueError(f"{name}: need a contiguous GPU tensor of at least {n} bytes")
    _check(load_library().espo_debug_sweep(C.c_void_p(src.data_ptr()), int(read_bytes), C.c_void_p(dst.data_ptr()),
                                           int(write_bytes), _stream(stream)))


def espo_debug_sweep_padded(rewards: torch.Tensor, values: torch.Tensor, lengths: torch.Tensor, td: torch.Tensor,
                            adv: torch.Tensor, stream=None) -> None:
    """Diagnostics: the memory traffic of espo_advantages in its own layout, no dependency (see include/espo_debug.h)."""
    B, T = rewards.shape
    _check(load_library().espo_debug_sweep_padded(
        _dev(rewards, torch.float32, "rewards"), _dev(values, torch.float32, "values", shape=(B, T)),
        _dev(lengths, torch.int32, "lengths", numel=B), B, T, _dev(td, torch.float32, "td", shape=(B, T)),
        _dev(adv, torch.float32, "adv", shape=(B, T)), _stream(stream)))


def espo_batch_stats_workspace_bytes(B: int, T: int) -> int:
    return int(load_library().espo_batch_stats_workspace_bytes(B, T))


def espo_batch_stats(regret: torch.Tensor, lengths: torch.Tensor, stopped: torch.Tensor, mu_g: float, var_g: float,
                     beta: float, out: torch.Tensor, workspace: torch.Tensor, alpha_ema: float = 0.99,
                     eta_beta: float = 0.1, target_rate: float = 0.25, beta_min: float = 0.0, beta_max: float = 7.0,
                     stream=None) -> None:
    """Batch-boundary update (Section 4.2, Eq. beta_update).  `out`: uint8 GPU tensor of BATCH_RESULT_BYTES bytes
    (decode a host copy with `read_batch_result`); `workspace`: uint8 GPU tensor of the size the library asks for."""
    if regret.dim() != 2:
        raise ValueError("regret must be [B, T]")
    B, T = regret.shape
    ctrl = _BatchCtrl(alpha_ema, eta_beta, target_rate, beta_min, beta_max)
    _check(load_library().espo_batch_stats(
        _dev(regret, torch.float32, "regret"), _dev(lengths, torch.int32, "lengths", numel=B),
        _dev(stopped, torch.uint8, "stopped", numel=B),
        B, T, float(mu_g), float(var_g), float(beta), C.byref(ctrl), _dev(out, torch.uint8, "out", numel=BATCH_RESULT_BYTES),
        _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream)))


def espo_batch_stats_static(regret: torch.Tensor, lengths: torch.Tensor, stopped: torch.Tensor, mu_g: float, var_g: float,
                            beta: float, out: torch.Tensor, alpha_ema: float = 0.99, eta_beta: float = 0.1,
                            target_rate: float = 0.25, beta_min: float = 0.0, beta_max: float = 7.0, stream=None) -> None:
    """`espo_batch_stats` on the library's own scratch (no workspace argument, nothing allocated)."""
    if regret.dim() != 2:
        raise ValueError("regret must be [B, T]")
    B, T = regret.shape
    ctrl = _BatchCtrl(alpha_ema, eta_beta, target_rate, beta_min, beta_max)
    _check(load_library().espo_batch_stats_static(
        _dev(regret, torch.float32, "regret"), _dev(lengths, torch.int32, "lengths", numel=B),
        _dev(stopped, torch.uint8, "stopped", numel=B),
        B, T, float(mu_g), float(var_g), float(beta), C.byref(ctrl), _dev(out, torch.uint8, "out", numel=BATCH_RESULT_BYTES),
        _stream(stream)))


def read_batch_result(out: torch.Tensor) -> dict:
    """Host view of an espo_batch_result that `espo_batch_stats` wrote (synchronises through the copy)."""
    raw = bytes(out.cpu().numpy().tobytes()[:BATCH_RESULT_BYTES])
    r = _BatchResult.from_buffer_copy(raw)
    return {name: getattr(r, name) for name, _ in _BatchResult._fields_}


def espo_debug_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    """Diagnostics: plain copy kernel of known traffic, for calibrating hardware counters (see include/espo.h)."""
    if dst.dtype != src.dtype or dst.numel() != src.numel():
        raise ValueError("dst and src must match")
    nbytes = src.numel() * src.element_size()
    _check(load_library().espo_debug_copy(_dev(dst, dst.dtype, "dst"), _dev(src, src.dtype, "src"), nbytes, _stream(stream)))


def espo_step_workspace_bytes(B: int, V: int, dtype: torch.dtype) -> int:
    dt = ESPO_BF16 if dtype == torch.bfloat16 else ESPO_F32
    return int(load_library().espo_step_workspace_bytes(B, V, dt))


def espo_debug_step_workspace_bytes(B: int, chunks: int) -> int:
    return int(load_library().espo_debug_step_workspace_bytes(B, chunks))


def espo_step(logits: torch.Tensor, temperature: float, seed: int, step: int, values: torch.Tensor,
              params: EspoParams, z: torch.Tensor, alive: torch.Tensor, stop_step: torch.Tensor,
              tokens: torch.Tensor, regret: torch.Tensor, logprob: torch.Tensor | None = None,
              V: int | None = None, workspace: torch.Tensor | None = None, stream=None,
              entropy: torch.Tensor | None = None, margin_scale: float | None = None, waves: int | None = None,
              chunks: int | None = None) -> None:
    """One decode step; see `espo_step` in include/espo.h.  `logits` is [B, row_stride].  `workspace`: a
    zero-initialised uint8 GPU tensor of `espo_step_workspace_bytes` bytes (rows are then split over several
    workgroups) or None.  With any of `margin_scale`, `waves`, `chunks` the call goes through
    `espo_debug_step` (include/espo_debug.h), which exposes those choices for this call."""
    lib = load_library()
    if logits.dtype == torch.bfloat16:
        dt = ESPO_BF16
    elif logits.dtype == torch.float32:
        dt = ESPO_F32
    else:
        raise TypeError("logits must be bfloat16 or float32")
    if logits.dim() != 2 or logits.stride(1) != 1 or not _on_gpu(logits):
        raise TypeError("logits: need a 2-D GPU tensor with unit stride along the vocabulary")
    B, width = logits.shape
    row_stride = logits.stride(0) if B > 1 else width
    V = width if V is None else int(V)
    if V > width:
        raise EspoError(-1, "V exceeds the width of logits")
    ws_ptr, ws_bytes = None, 0
    if workspace is not None:
        ws_ptr, ws_bytes = _dev(workspace, torch.uint8, "workspace"), workspace.numel()
    p = params._c()
    args = [C.c_void_p(logits.data_ptr()), dt, B, V, row_stride, float(temperature), int(seed),
            int(step), _dev(values, torch.float32, "values", numel=B), C.byref(p),
            _dev(z, torch.float32, "z", numel=B), _dev(alive, torch.uint8, "alive", numel=B),
            _dev(stop_step, torch.int32, "stop_step", numel=B), _dev(tokens, torch.int32, "tokens", numel=B),
            _dev(regret, torch.float32, "regret", numel=B), _dev(logprob, torch.float32, "logprob", numel=B),
            _dev(entropy, torch.float32, "entropy", numel=B), ws_ptr, ws_bytes, _stream(stream)]
    if margin_scale is None and waves is None and chunks is None:
        rc = lib.espo_step(*args)
    else:
        rc = lib.espo_debug_step(*args, 1.0 if margin_scale is None else float(margin_scale), int(waves or 0), int(chunks or 0))
    _check(rc)


def espo_advantages(rewards: torch.Tensor, values: torch.Tensor, lengths: torch.Tensor,
                    stopped: torch.Tensor, r_fail: float, gamma: float, lam: float,
                    td: torch.Tensor, adv: torch.Tensor, stream=None) -> None:
    """TD errors and GAE on truncated trajectories; see `espo_advantages` in include/espo.h."""
    lib = load_library()
    if rewards.dim() != 2:
        raise TypeError("rewards: need [B, T]")
    B, T = rewards.shape
    rc = lib.espo_advantages(_dev(rewards, torch.float32, "rewards"), _dev(values, torch.float32, "values", shape=(B, T)),
                             _dev(lengths, torch.int32, "lengths", numel=B), _dev(stopped, torch.uint8, "stopped", numel=B),
                             B, T, float(r_fail), float(gamma), float(lam),
                             _dev(td, torch.float32, "td", shape=(B, T)), _dev(adv, torch.float32, "adv", shape=(B, T)),
                             _stream(stream))
    _check(rc)


def espo_advantages_ws_bytes(B: int) -> int:
    return int(load_library().espo_advantages_ws_bytes(B))


def espo_length_order(lengths: torch.Tensor, T: int, order: torch.Tensor, stream=None) -> None:
    """The rows by length, longest first; see `espo_length_order` in include/espo.h."""
    lib = load_library()
    B = lengths.numel()
    _check(lib.espo_length_order(_dev(lengths, torch.int32, "lengths"), B, int(T), _dev(order, torch.int32, "order", numel=B),
                                 _stream(stream)))


def espo_advantages_ws(rewards: torch.Tensor, values: torch.Tensor, lengths: torch.Tensor,
                       stopped: torch.Tensor, r_fail: float, gamma: float, lam: float,
                       td: torch.Tensor, adv: torch.Tensor, workspace: torch.Tensor, order: torch.Tensor | None = None,
                       stream=None) -> None:
    """espo_advantages with the rows' sums left in `workspace` and, optionally, the rows taken in a
    given order; see `espo_advantages_ws` in include/espo.h."""
    lib = load_library()
    if rewards.dim() != 2:
        raise TypeError("rewards: need [B, T]")
    B, T = rewards.shape
    rc = lib.espo_advantages_ws(_dev(rewards, torch.float32, "rewards"), _dev(values, torch.float32, "values", shape=(B, T)),
                                _dev(lengths, torch.int32, "lengths", numel=B), _dev(stopped, torch.uint8, "stopped", numel=B),
                                B, T, float(r_fail), float(gamma), float(lam),
                                _dev(td, torch.float32, "td", shape=(B, T)), _dev(adv, torch.float32, "adv", shape=(B, T)),
                                _dev(order, torch.int32, "order", numel=B),
                                _dev(workspace, torch.uint8, "workspace"), workspace.numel() if workspace is not None else 0,
                                _stream(stream))
    _check(rc)


def espo_whiten_from_ws(adv: torch.Tensor, lengths: torch.Tensor, out: torch.Tensor, workspace: torch.Tensor,
                        eps: float = 1e-8, shift_mean: bool = True, unbiased: bool = False,
                        stats: torch.Tensor | None = None, stream=None) -> None:
    """espo_whiten from the sums that espo_advantages_ws left in `workspace`; see
    `espo_whiten_from_ws` in include/espo.h."""
    lib = load_library()
    if adv.dim() != 2:
        raise TypeError("adv: need [B, T]")
    B, T = adv.shape
    if out.shape != adv.shape or lengths.numel() != B:
        raise TypeError("out: need the shape of adv; lengths: need [B]")
    if stats is not None and stats.numel() < 3:
        raise TypeError("stats: need 3 doubles")
    rc = lib.espo_whiten_from_ws(_dev(adv, torch.float32, "adv"), _dev(lengths, torch.int32, "lengths", numel=B), B, T,
                                 float(eps), int(bool(shift_mean)), int(bool(unbiased)), _dev(out, torch.float32, "out"),
                                 _dev(stats, torch.float64, "stats", numel=3), _dev(workspace, torch.uint8, "workspace"),
                                 workspace.numel() if workspace is not None else 0, _stream(stream))
    _check(rc)


def espo_whiten_workspace_bytes(B: int, T: int) -> int:
    return int(load_library().espo_whiten_workspace_bytes(B, T))


def espo_whiten(adv: torch.Tensor, lengths: torch.Tensor, out: torch.Tensor, workspace: torch.Tensor, eps: float = 1e-8,
                shift_mean: bool = True, unbiased: bool = False, stats: torch.Tensor | None = None, stream=None) -> None:
    """Whitening of the advantages over the valid tokens; see `espo_whiten` in include/espo.h.
    `adv` is [B, T] (or [N] with `lengths` = [N] for a packed batch); `out` may be `adv`."""
    lib = load_library()
    if adv.dim() == 1:
        B, T = 1, adv.numel()
    elif adv.dim() == 2:
        B, T = adv.shape
    else:
        raise TypeError("adv: need [B, T] or [N]")
    if out.shape != adv.shape or lengths.numel() != B:
        raise TypeError("out: need the shape of adv; lengths: need [B]")
    if stats is not None and stats.numel() < 3:
        raise TypeError("stats: need 3 doubles")
    rc = lib.espo_whiten(_dev(adv, torch.float32, "adv"), _dev(lengths, torch.int32, "lengths", numel=B), B, T, float(eps),
                         int(bool(shift_mean)), int(bool(unbiased)), _dev(out, torch.float32, "out"),
                         _dev(stats, torch.float64, "stats", numel=3), _dev(workspace, torch.uint8, "workspace"),
                         workspace.numel() if workspace is not None else 0, _stream(stream))
    _check(rc)


def espo_advantages_packed(values: torch.Tensor, cu_seqlens: torch.Tensor, stopped: torch.Tensor,
                           r_fail: float, gamma: float, lam: float, td: torch.Tensor, adv: torch.Tensor,
                           rewards: torch.Tensor | None = None, terminal_reward: torch.Tensor | None = None,
                           returns: torch.Tensor | None = None, stream=None) -> None:
    """The advantage pass over trajectories stored back to back; see `espo_advantages_packed`
    in include/espo.h.  Exactly one of `rewards` [N] and `terminal_reward` [B]."""
    lib = load_library()
    if values.dim() != 1 or cu_seqlens.dim() != 1 or cu_seqlens.numel() != stopped.numel() + 1:
        raise TypeError("values: need [N]; cu_seqlens: need [B + 1]")
    N, B = values.numel(), stopped.numel()
    for name, t in (("td", td), ("adv", adv), ("returns", returns), ("rewards", rewards)):
        if t is not None and t.numel() != N:
            raise TypeError(f"{name}: need [N]")
    if terminal_reward is not None and terminal_reward.numel() != B:
        raise TypeError("terminal_reward: need [B]")
    rc = lib.espo_advantages_packed(_dev(rewards, torch.float32, "rewards"),
                                    _dev(terminal_reward, torch.float32, "terminal_reward"),
                                    _dev(values, torch.float32, "values"), _dev(cu_seqlens, torch.int64, "cu_seqlens"),
                                    _dev(stopped, torch.uint8, "stopped"), B, N, float(r_fail), float(gamma), float(lam),
                                    _dev(td, torch.float32, "td"), _dev(adv, torch.float32, "adv"),
                                    _dev(returns, torch.float32, "returns"), _stream(stream))
    _check(rc)


def espo_advantages_terminal(values: torch.Tensor, lengths: torch.Tensor, stopped: torch.Tensor,
                             terminal_reward: torch.Tensor, r_fail: float, gamma: float, lam: float,
                             td: torch.Tensor, adv: torch.Tensor, returns: torch.Tensor | None = None,
                             zero_padding: bool = True, stream=None) -> None:
    """The advantage pass when only the last reward of a row is non-zero; see
    `espo_advantages_terminal` in include/espo.h."""
    lib = load_library()
    if values.dim() != 2:
        raise TypeError("values: need [B, T]")
    B, T = values.shape
    rc = lib.espo_advantages_terminal(_dev(values, torch.float32, "values"), _dev(lengths, torch.int32, "lengths", numel=B),
                                      _dev(stopped, torch.uint8, "stopped", numel=B),
                                      _dev(terminal_reward, torch.float32, "terminal_reward", numel=B), B, T,
                                      float(r_fail), float(gamma), float(lam), int(bool(zero_padding)),
                                      _dev(td, torch.float32, "td", shape=(B, T)), _dev(adv, torch.float32, "adv", shape=(B, T)),
                                      _dev(returns, torch.float32, "returns", shape=(B, T)), _stream(stream))
    _check(rc)


def espo_advantages_terminal_ws(values: torch.Tensor, lengths: torch.Tensor, stopped: torch.Tensor,
                                terminal_reward: torch.Tensor, r_fail: float, gamma: float, lam: float,
                                td: torch.Tensor, adv: torch.Tensor, workspace: torch.Tensor,
                                returns: torch.Tensor | None = None, zero_padding: bool = True,
                                order: torch.Tensor | None = None, stream=None) -> None:
    """espo_advantages_terminal with the later rows taken longest first and the rows' sums left in
    `workspace`; see `espo_advantages_terminal_ws` in include/espo.h."""
    lib = load_library()
    if values.dim() != 2:
        raise TypeError("values: need [B, T]")
    B, T = values.shape
    rc = lib.espo_advantages_terminal_ws(_dev(values, torch.float32, "values"), _dev(lengths, torch.int32, "lengths", numel=B),
                                         _dev(stopped, torch.uint8, "stopped", numel=B),
                                         _dev(terminal_reward, torch.float32, "terminal_reward", numel=B), B, T,
                                         float(r_fail), float(gamma), float(lam), int(bool(zero_padding)),
                                         _dev(td, torch.float32, "td", shape=(B, T)), _dev(adv, torch.float32, "adv", shape=(B, T)),
                                         _dev(returns, torch.float32, "returns", shape=(B, T)),
                                         _dev(order, torch.int32, "order", numel=B),
                                         _dev(workspace, torch.uint8, "workspace"), workspace.numel() if workspace is not None else 0,
                                         _stream(stream))
    _check(rc)
