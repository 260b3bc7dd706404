"""The C-ABI library loads and exports every symbol that include/espo.h and include/espo_debug.h declare.

Runs without a GPU: nothing is launched, only argument checking is exercised.
"""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2605_29860_amd import binding
    if not os.path.exists(binding.library_path()):
        from paper_2605_29860_amd import build
        build.build_library()
    return binding.load_library()


def _declared_functions(header="espo.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(espo_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert {"espo_step", "espo_advantages", "espo_advantages_terminal", "espo_advantages_packed", "espo_whiten", "espo_whiten_workspace_bytes", "espo_step_workspace_bytes", "espo_strerror", "espo_version",
            "espo_batch_stats", "espo_batch_stats_workspace_bytes", "espo_batch_stats_static"} <= set(names)
    assert not any(n.startswith("espo_debug") for n in names)       # diagnostics live in their own header
    debug = _declared_functions("espo_debug.h")
    assert {"espo_debug_step", "espo_debug_step_workspace_bytes", "espo_debug_math_errors", "espo_debug_copy",
            "espo_debug_read", "espo_debug_sweep", "espo_debug_sweep_padded"} <= set(debug)
    for n in names + debug:
        assert hasattr(lib, n), n


def test_status_strings_and_version(lib):
    assert lib.espo_version() >= 100
    seen = set()
    for code in (0, -1, -2, -3, -4, -5, -99):
        s = lib.espo_strerror(code)
        assert s and len(s) > 3
        seen.add(s)
    assert len(seen) == 7


def test_argument_checks_need_no_gpu(lib):
    from paper_2605_29860_amd.binding import _Params
    p = _Params(0, 1, 1e-8, 10, 0.9, 7, 0.2, 1, -1)
    fake = ctypes.c_void_p(0x1000)
    def step(B=1, V=8, stride=8, tau=1.0, logits=fake, params=ctypes.byref(p), dt=1, stepno=0):
        return lib.espo_step(logits, dt, B, V, stride, tau, 0, stepno, fake, params, fake, fake, fake, fake, fake,
                             None, None, None, 0, None)
    assert step(B=0) == 0                                   # empty batch is a no-op
    assert step(tau=0.0) == -1 and step(tau=float("nan")) == -1
    assert step(V=0) == -1 and step(stride=4) == -1 and step(B=-1) == -1 and step(stepno=-1) == -1
    assert step(dt=7) == -1 and step(params=None) == -1 and step(logits=None) == -1
    assert step(logits=ctypes.c_void_p(0x1008)) == -2       # misaligned base
    assert step(V=3, stride=3) == -2                        # row pitch of 6 bytes
    assert step(V=5_000_000, stride=5_000_000) == -5        # beyond the supported vocabulary
    adv = lambda B=1, T=8, g=1.0: lib.espo_advantages(fake, fake, fake, fake, B, T, -1.0, g, 0.95, fake, fake, None)
    assert adv(B=0) == 0 and adv(T=0) == 0
    assert adv(B=-1) == -1 and adv(g=float("inf")) == -1
    term = lambda B=1, T=8, g=1.0, ret=None, values=fake: lib.espo_advantages_terminal(
        values, fake, fake, fake, B, T, -1.0, g, 0.95, 1, fake, fake, ret, None)
    assert term(B=0) == 0 and term(T=0) == 0
    assert term(B=-1) == -1 and term(g=float("nan")) == -1 and term(values=None) == -1
    assert term(ret=ctypes.c_void_p(0x1004)) == -2          # misaligned optional output
    lib.espo_advantages_packed.argtypes = [ctypes.c_void_p] * 5 + [ctypes.c_int64] * 2 + [ctypes.c_float] * 3 + [ctypes.c_void_p] * 4
    packed = lambda r=None, term=fake, B=1, N=8, g=1.0, cu=fake, ret=None: lib.espo_advantages_packed(
        r, term, fake, cu, fake, B, N, -1.0, g, 0.95, fake, fake, ret, None)
    assert packed(B=0) == 0 and packed(N=0) == 0
    assert packed(B=-1) == -1 and packed(N=-1) == -1 and packed(g=float("nan")) == -1 and packed(cu=None) == -1
    assert packed(r=fake, term=fake) == -1 and packed(r=None, term=None) == -1   # exactly one reward form
    assert packed(ret=ctypes.c_void_p(0x1004)) == -2 and packed(r=ctypes.c_void_p(0x1008), term=None) == -2
    lib.espo_whiten.argtypes = [ctypes.c_void_p] * 2 + [ctypes.c_int64] * 2 + [ctypes.c_float] + [ctypes.c_int32] * 2 + \
        [ctypes.c_void_p] * 3 + [ctypes.c_size_t, ctypes.c_void_p]
    lib.espo_whiten_workspace_bytes.restype = ctypes.c_size_t
    lib.espo_whiten_workspace_bytes.argtypes = [ctypes.c_int64] * 2
    need = lib.espo_whiten_workspace_bytes(4, 100)
    assert 0 < need <= 32768 and lib.espo_whiten_workspace_bytes(1024, 16384) <= 32768 and lib.espo_whiten_workspace_bytes(0, 5) == 0
    wh = lambda B=4, T=100, eps=1e-8, adv=fake, out=fake, stats=None, ws=fake, nws=need: lib.espo_whiten(
        adv, fake, B, T, eps, 1, 0, out, stats, ws, nws, None)
    assert wh(B=0) == 0 and wh(T=0) == 0
    assert wh(B=-1) == -1 and wh(eps=-1.0) == -1 and wh(eps=float("nan")) == -1 and wh(adv=None) == -1
    assert wh(out=ctypes.c_void_p(0x1004)) == -2 and wh(stats=ctypes.c_void_p(0x1004)) == -2
    assert wh(ws=None) == -3 and wh(nws=need - 1) == -3
    assert lib.espo_step_workspace_bytes(1024, 152064, 1) == 0 and lib.espo_step_workspace_bytes(0, 152064, 1) == 0
    lib.espo_debug_step.argtypes = lib.espo_step.argtypes + [ctypes.c_float, ctypes.c_int32, ctypes.c_int32]
    dbg = lambda scale=1.0, waves=0, chunks=0: lib.espo_debug_step(fake, 1, 4, 4096, 4096, 1.0, 0, 0, fake, ctypes.byref(p), fake, fake,
                                                                   fake, fake, fake, None, None, None, 0, None, scale, waves, chunks)
    assert dbg(scale=0.5) == -1 and dbg(scale=float("nan")) == -1 and dbg(waves=5) == -1 and dbg(chunks=-1) == -1
    assert dbg(chunks=4) == -3                                # a split without a workspace
    need = 4 * 4 * 32 + 256
    wsd = lambda ws, nws: lib.espo_debug_step(fake, 1, 4, 4096, 4096, 1.0, 0, 0, fake, ctypes.byref(p), fake, fake, fake, fake, fake,
                                              None, None, ws, nws, None, 1.0, 0, 4)
    assert wsd(fake, need - 1) == -3 and wsd(ctypes.c_void_p(0x1004), need) == -3   # too small; misaligned
    lib.espo_debug_step_workspace_bytes.restype = ctypes.c_size_t
    lib.espo_debug_step_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int32]
    assert lib.espo_debug_step_workspace_bytes(4, 1) == 0 and lib.espo_debug_step_workspace_bytes(4, 4) >= 4 * 4 * 32
