"""The C ABI driven from a plain HIP host program (no Python binding, no PyTorch in that process),
checked against the CPU oracle (needs an MI355X)."""
import ctypes as C
import os
import subprocess

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle  # noqa: E402
from paper_2605_29860_amd import binding, build  # noqa: E402


def test_native_program_matches_the_oracle(tmp_path):
    print("[case] native ABI check", flush=True)
    if not os.path.exists(build.ABI_CHECK):
        build.build_abi_check()
    rng = np.random.default_rng(7)
    B, V, T, step, seed, tau = 516, 5003, 300, 4, 123456789012345, 0.8   # more rows than resident workgroups
    V_pad = 5004                              # a pitch of 5003 floats is not a multiple of 16 bytes: pad the rows
    logits = (rng.standard_normal((B, V_pad)) * 3).astype(np.float32)
    logits[:, V:] = 1e4
    values = rng.random(B).astype(np.float32)
    z = (rng.random(B) * 2 - 1).astype(np.float32)
    alive = (np.arange(B) % 6 != 2).astype(np.uint8)
    stop_step = np.full(B, -1, np.int32)
    rewards = rng.standard_normal((B, T)).astype(np.float32)
    vals2 = (rng.random((B, T)) * 2 - 1).astype(np.float32)
    lengths = rng.integers(0, T + 1, B).astype(np.int32)
    stopped = (rng.random(B) < 0.5).astype(np.uint8)
    op = oracle.OracleParams(mu_g=1.0, var_g=2.0, beta=1.0)
    gp = binding.EspoParams(mu_g=1.0, var_g=2.0, beta=1.0)._c()

    # the program takes V as the row pitch too, so hand it the padded width and mask the pad away
    logits_in = logits.copy()
    logits_in[:, V:] = -np.inf
    fin, fout = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(fin, "wb") as f:
        f.write(np.array([B, V_pad, T], np.int32).tobytes())
        f.write(np.float32(tau).tobytes())
        f.write(np.uint64(seed).tobytes())
        f.write(np.int32(step).tobytes())
        f.write(bytes(gp))
        for a in (logits_in, values, z, alive, stop_step, rewards, vals2, lengths, stopped):
            f.write(a.tobytes())
    res = subprocess.run([build.ABI_CHECK, str(fin), str(fout)], capture_output=True, text=True, timeout=120)
    print(res.stdout, res.stderr, flush=True)
    assert res.returncode == 0

    raw = open(fout, "rb").read()
    off = 0
    def take(dtype, n):
        nonlocal off
        a = np.frombuffer(raw, dtype, n, off)
        off += a.nbytes
        return a
    tokens, regret, z_g, alive_g, ss_g, logprob = (take(np.int32, B), take(np.float32, B), take(np.float32, B),
                                                   take(np.uint8, B), take(np.int32, B), take(np.float32, B))
    entropy = take(np.float32, B)
    td, adv = take(np.float32, B * T).reshape(B, T), take(np.float32, B * T).reshape(B, T)
    wh, td_p, adv_p = take(np.float32, B * T).reshape(B, T), take(np.float32, B * T), take(np.float32, B * T)
    order, adv_ws, wh_ws = take(np.int32, B), take(np.float32, B * T).reshape(B, T), take(np.float32, B * T).reshape(B, T)

    z_o, alive_o, ss_o = z.copy(), alive.copy(), stop_step.copy()
    ref = oracle.step(logits_in, tau, seed, step, values, op, z_o, alive_o, ss_o, want_entropy=True)
    np.testing.assert_array_equal(tokens, ref["tokens"])
    np.testing.assert_array_equal(regret.view(np.uint32), ref["regret"].view(np.uint32))
    np.testing.assert_array_equal(z_g.view(np.uint32), z_o.view(np.uint32))
    np.testing.assert_array_equal(alive_g, alive_o)
    np.testing.assert_array_equal(ss_g, ss_o)
    live = alive == 1
    assert np.abs(logprob[live] - ref["logprob"][live]).max() <= 1e-5 * np.maximum(np.abs(ref["logprob"][live]), 1).max()
    assert (np.abs(entropy - ref["entropy"]) <= 1e-5 * np.maximum(ref["entropy"], 1)).all() and (entropy[~live] == 0).all()
    td_o, adv_o, scale = oracle.advantages(rewards, vals2, lengths, stopped, -1.0, 1.0, 0.95)
    assert np.abs(td - td_o).max() <= 2e-7 * (max(np.abs(rewards).max(), 1.0) + 2 * np.abs(vals2).max())
    assert (np.abs(adv - adv_o) <= 2e-6 * np.maximum(np.abs(adv_o), scale)).all()
    # whitening of the advantages the program itself produced (its fp32 output is the oracle's input)
    wh_o, _ = oracle.whiten(adv, lengths)
    mask = np.arange(T)[None, :] < np.clip(lengths, 0, T)[:, None]
    assert (np.abs(wh[mask] - wh_o[mask]) <= 2e-7 * np.maximum(np.abs(wh_o[mask]), 1)).all() and (wh[~mask] == 0).all()
    # the [B, T] values as B full trajectories stored back to back, terminal reward values[b]
    cu = (np.arange(B + 1) * T).astype(np.int64)
    tdp_o, advp_o, _, scale_p = oracle.advantages_packed(None, values, vals2.reshape(-1), cu, stopped, -1.0, 1.0, 0.95)
    assert np.abs(td_p - tdp_o).max() <= 2e-7 * (max(np.abs(values).max(), 1.0) + 2 * np.abs(vals2).max())
    assert (np.abs(adv_p - advp_o) <= 2e-6 * np.maximum(np.abs(advp_o), scale_p)).all()
    # the pair with a workspace between them: a permutation with the longest rows first, the same advantages,
    # and the whitening from the rows' sums against the oracle
    assert sorted(order.tolist()) == list(range(B))
    cls = (np.clip(lengths, 0, T)[order].astype(np.int64) * 256) // (T + 1)
    assert (np.diff(cls) <= 0).all()
    np.testing.assert_array_equal(adv_ws[mask].view(np.uint32), adv[mask].view(np.uint32))
    assert (np.abs(wh_ws[mask] - wh_o[mask]) <= 2e-7 * np.maximum(np.abs(wh_o[mask]), 1)).all() and (wh_ws[~mask] == 0).all()
