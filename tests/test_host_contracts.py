"""Host-side contracts that need no GPU: the benchmark's one-GPU rule, the product path's
refusal to run without its HIP library, the separation between the oracle and the GPU path,
and the determinism of the seeded input generators."""
import ast
import os
import subprocess
import sys

import numpy as np
import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    for argv, env in ((["--gpus", "2"], {}), ([], {"WORLD_SIZE": "4"})):
        res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *argv], capture_output=True, text=True,
                             env={**os.environ, **env}, timeout=120)
        assert res.returncode != 0
        assert "one GPU" in res.stderr and res.stdout.strip() == ""


def test_product_path_fails_loudly_without_its_library(monkeypatch, tmp_path):
    from paper_2605_29860_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "libespo.so"))
    with pytest.raises(FileNotFoundError, match="no fallback"):
        binding.load_library()
    with pytest.raises(FileNotFoundError):
        binding.espo_step_workspace_bytes(1, 8, torch.float32)


def _imports(path):
    tree = ast.parse(open(path).read())
    names = set()
    for node in ast.walk(tree):
        if isinstance(node, ast.Import):
            names.update(a.name.split(".")[0] for a in node.names)
        elif isinstance(node, ast.ImportFrom) and node.level == 0 and node.module:
            names.add(node.module.split(".")[0])
    return names


def test_oracle_and_gpu_path_do_not_import_each_other():
    pkg = os.path.join(ROOT, "paper_2605_29860_amd")
    for f in os.listdir(pkg):
        if f.endswith(".py"):
            assert "oracle" not in _imports(os.path.join(pkg, f)), f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            assert "paper_2605_29860_amd" not in _imports(os.path.join(ROOT, "oracle", f)), f
    # no shared sources either: the GPU sources include nothing from oracle/ and the oracle nothing from csrc/
    for d, banned in ((os.path.join(pkg, "csrc"), "oracle"), (os.path.join(ROOT, "oracle"), "csrc")):
        for f in os.listdir(d):
            if f.endswith((".hip", ".h", ".c")):
                for line in open(os.path.join(d, f)):
                    if line.lstrip().startswith("#include"):
                        assert banned not in line, (f, line)
    # nothing that ships reads the working folder or the paper's text at run time
    for f in ("bench.py", "__graft_entry__.py"):
        text = open(os.path.join(ROOT, f)).read()
        assert "_work/" not in text and '"_work"' not in text and "/root/reference" not in text


def test_input_generators_are_seeded_and_hold_no_method_arithmetic():
    from paper_2605_29860_amd import workloads as W
    a = W.ZipfLogits(V=4096, seed=5).rows(3, step=2)
    b = W.ZipfLogits(V=4096, seed=5).rows(3, step=2)
    c = W.ZipfLogits(V=4096, seed=6).rows(3, step=2)
    assert torch.equal(a, b) and not torch.equal(a, c) and a.dtype == torch.bfloat16
    r1 = W.advantage_batch(B=8, T=64, len_lo=4, seed=1)
    r2 = W.advantage_batch(B=8, T=64, len_lo=4, seed=1)
    assert all(torch.equal(x, y) for x, y in zip(r1, r2))
    rewards, values, lengths, stopped = r1
    last = rewards[torch.arange(8), (lengths - 1).long()]
    assert ((rewards != 0).sum(1) <= 1).all() and set(last.tolist()) <= {0.0, 1.0}      # terminal reward only
    assert (last[stopped > 0] == 0).all() and float(values.abs().max()) <= 1.0
    g1 = W.regret_batch(4, 32, seed=3)
    g2 = W.regret_batch(4, 32, seed=3)
    assert all(torch.equal(x, y) for x, y in zip(g1, g2))
    bits = W.to_host_bits(a)
    assert bits.dtype == np.uint16 and bits.shape == (3, 4096)


def test_parameter_structs_of_both_sides_have_the_same_layout():
    # The two sides define their parameter structs separately (they share no code); the fields, their
    # order, types and defaults must still agree, and both must match the C header's declaration order.
    import dataclasses
    import re
    import oracle.espo_oracle as o
    from paper_2605_29860_amd import binding as b
    assert [(n, t) for n, t in b._Params._fields_] == [(n, t) for n, t in o._Params._fields_]
    gd = {f.name: f.default for f in dataclasses.fields(b.EspoParams)}
    od = {f.name: f.default for f in dataclasses.fields(o.OracleParams)}
    assert gd == od and list(gd) == [n for n, _ in b._Params._fields_]
    header = open(os.path.join(ROOT, "include", "espo.h")).read()
    body = header[header.index("typedef struct {", header.index("frozen for a whole rollout batch")):header.index("} espo_params;")]
    declared = re.findall(r"^\s*(?:float|int32_t)\s+(\w+);", body, flags=re.M)
    assert declared == list(gd)


def test_binding_refuses_tensors_that_are_too_short(monkeypatch):
    # The C ABI takes bare pointers and cannot know sizes: a short tensor would be an out-of-bounds access on
    # the GPU.  The binding therefore checks every tensor against B, T and N before the call.  Here the library
    # is replaced by a recorder and host tensors stand in for device memory, so that nothing is launched.
    from paper_2605_29860_amd import binding as b

    class Recorder:
        calls = 0

        def __getattr__(self, name):
            def call(*args):
                Recorder.calls += 1
                return 0
            return call

    monkeypatch.setattr(b, "load_library", lambda: Recorder())
    monkeypatch.setattr(b, "_on_gpu", lambda t: True)
    monkeypatch.setattr(b, "_stream", lambda s: None)
    B, V, T = 4, 64, 16
    f32, i32, u8 = torch.float32, torch.int32, torch.uint8
    mk = lambda n, dt: torch.zeros(n, dtype=dt)
    step_args = lambda **short: dict(
        logits=torch.zeros(B, V), temperature=1.0, seed=0, step=0, values=mk(short.get("values", B), f32), params=b.EspoParams(),
        z=mk(short.get("z", B), f32), alive=mk(short.get("alive", B), u8), stop_step=mk(short.get("stop_step", B), i32),
        tokens=mk(short.get("tokens", B), i32), regret=mk(short.get("regret", B), f32),
        logprob=mk(short.get("logprob", B), f32), entropy=mk(short.get("entropy", B), f32))
    b.espo_step(**step_args())
    assert Recorder.calls == 1
    for name in ("values", "z", "alive", "stop_step", "tokens", "regret", "logprob", "entropy"):
        with pytest.raises(ValueError, match=name):
            b.espo_step(**step_args(**{name: B - 1}))
    with pytest.raises(b.EspoError):
        b.espo_step(**{**step_args(), "V": V + 1})
    assert Recorder.calls == 1

    adv_args = lambda **o: dict(rewards=torch.zeros(B, T), values=torch.zeros(*o.get("values", (B, T))),
                                lengths=mk(o.get("lengths", B), i32), stopped=mk(o.get("stopped", B), u8), r_fail=-1.0, gamma=1.0,
                                lam=0.95, td=torch.zeros(*o.get("td", (B, T))), adv=torch.zeros(*o.get("adv", (B, T))))
    b.espo_advantages(**adv_args())
    assert Recorder.calls == 2
    for name, bad in (("values", (B, T - 1)), ("td", (B - 1, T)), ("adv", (B, T + 1)), ("lengths", B - 1), ("stopped", B - 1)):
        with pytest.raises(ValueError, match=name):
            b.espo_advantages(**adv_args(**{name: bad}))
    term_args = lambda **o: dict(values=torch.zeros(B, T), lengths=mk(o.get("lengths", B), i32), stopped=mk(o.get("stopped", B), u8),
                                 terminal_reward=mk(o.get("terminal_reward", B), f32), r_fail=-1.0, gamma=1.0, lam=0.95,
                                 td=torch.zeros(*o.get("td", (B, T))), adv=torch.zeros(B, T), returns=torch.zeros(*o.get("returns", (B, T))))
    b.espo_advantages_terminal(**term_args())
    for name, bad in (("lengths", B - 1), ("stopped", 1), ("terminal_reward", B - 1), ("td", (B, T - 4)), ("returns", (B + 1, T))):
        with pytest.raises(ValueError, match=name):
            b.espo_advantages_terminal(**term_args(**{name: bad}))
    out, ws = mk(b.BATCH_RESULT_BYTES, u8), mk(64, u8)
    b.espo_batch_stats(torch.zeros(B, T), mk(B, i32), mk(B, u8), 1.0, 1.0, 1.0, out, ws)
    b.espo_batch_stats_static(torch.zeros(B, T), mk(B, i32), mk(B, u8), 1.0, 1.0, 1.0, out)
    calls = Recorder.calls
    for fn, extra in ((b.espo_batch_stats, (ws,)), (b.espo_batch_stats_static, ())):
        with pytest.raises(ValueError, match="lengths"):
            fn(torch.zeros(B, T), mk(B - 1, i32), mk(B, u8), 1.0, 1.0, 1.0, out, *extra)
        with pytest.raises(ValueError, match="stopped"):
            fn(torch.zeros(B, T), mk(B, i32), mk(B - 2, u8), 1.0, 1.0, 1.0, out, *extra)
        with pytest.raises(ValueError, match="out"):
            fn(torch.zeros(B, T), mk(B, i32), mk(B, u8), 1.0, 1.0, 1.0, mk(8, u8), *extra)
    assert Recorder.calls == calls
    # the pair with a workspace between them, and the order by length
    wsp = mk(256 + 32 * B, u8)
    b.espo_advantages_ws(**adv_args(), workspace=wsp, order=mk(B, i32))
    b.espo_whiten_from_ws(torch.zeros(B, T), mk(B, i32), torch.zeros(B, T), wsp)
    b.espo_length_order(mk(B, i32), T, mk(B, i32))
    calls = Recorder.calls
    for name, bad in (("values", (B, T - 1)), ("td", (B - 1, T)), ("adv", (B, T + 1)), ("lengths", B - 1), ("stopped", B - 1)):
        with pytest.raises(ValueError, match=name):
            b.espo_advantages_ws(**adv_args(**{name: bad}), workspace=wsp)
    with pytest.raises(ValueError, match="order"):
        b.espo_advantages_ws(**adv_args(), workspace=wsp, order=mk(B - 1, i32))
    with pytest.raises(ValueError, match="order"):
        b.espo_length_order(mk(B, i32), T, mk(B - 1, i32))
    with pytest.raises(TypeError):
        b.espo_whiten_from_ws(torch.zeros(B, T), mk(B - 1, i32), torch.zeros(B, T), wsp)
    with pytest.raises(TypeError):
        b.espo_whiten_from_ws(torch.zeros(B, T), mk(B, i32), torch.zeros(B, T + 1), wsp)
    assert Recorder.calls == calls
    b.espo_advantages_terminal_ws(**term_args(), workspace=wsp, order=mk(B, i32))
    calls = Recorder.calls
    for name, bad in (("lengths", B - 1), ("stopped", 1), ("terminal_reward", B - 1), ("td", (B, T - 4)), ("returns", (B + 1, T))):
        with pytest.raises(ValueError, match=name):
            b.espo_advantages_terminal_ws(**term_args(**{name: bad}), workspace=wsp)
    with pytest.raises(ValueError, match="order"):
        b.espo_advantages_terminal_ws(**term_args(), workspace=wsp, order=mk(B - 2, i32))
    assert Recorder.calls == calls
