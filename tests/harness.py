"""Shared helpers of the GPU parity tests: run the HIP path and the CPU oracle on the same
bits and compare them to the stated bar.

Bar (from the build's target): stop steps, masks, the smoothed state and the regret are
bit-exact; tokens are bit-exact except where the oracle's two largest perturbed scores
lie within 1e-6 relative, in which case the runner-up is accepted and forced into the
oracle so that the rest of the trajectory stays comparable; log-probabilities agree
within rtol * max(|ref|, 1) with rtol 1e-5 for fp32 logits and 2e-3 for bf16 logits.
The entropy output agrees within 1e-5 * max(ref, 1) for both types (bf16 logits are exact
inputs to both sides; what differs is fp32 summation and the hardware exp2/log2, a few 1e-7
relative on each of the two sums the entropy is formed from).
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2605_29860_amd as espo
from paper_2605_29860_amd.workloads import to_host_bits

RTOL_F32 = 1e-5
RTOL_BF16 = 2e-3
NEAR_TIE = 1e-6
# Advantages: |err| <= ADV_RTOL * scale, scale = sum_l c^l (|r| + |gamma V'| + |V|) being the magnitude of the
# terms that fp32 rounding and reassociation act on.  The target states 1e-5 relative; the scan achieves a few
# 1e-7 of that scale (the tests print the worst case), so the bar is held five times tighter than the target.
ADV_RTOL = 2e-6
# TD errors: delta = (r + gamma V') - V is three fp32 roundings on exact inputs, each at most 2^-24 of a partial
# result no larger than |r| + |gamma V'| + |V|: at most 1.8e-7 of that sum.  No additive floor: where all three
# terms vanish the result must be exactly 0.
TD_RTOL = 2e-7


def td_bound(r_eff, v, v_next, gamma):
    """The bound on |delta_gpu - delta_oracle| from the sizes of the three terms (arrays of the same shape;
    r_eff is the reward the step really uses, i.e. the failure reward at the last token of a stopped row)."""
    return TD_RTOL * (np.abs(r_eff) + abs(gamma) * np.abs(v_next) + np.abs(v))


def params_pair(**kw):
    """The same frozen parameters for the GPU binding and for the oracle."""
    return espo.EspoParams(**kw), oracle.OracleParams(**kw)


class GpuState:
    """Per-row state and per-step outputs as GPU tensors."""

    def __init__(self, B, device="cuda", z=None, alive=None, stop_step=None):
        self.z = torch.zeros(B, dtype=torch.float32, device=device) if z is None else z.to(device).clone()
        self.alive = torch.ones(B, dtype=torch.uint8, device=device) if alive is None else alive.to(device).clone()
        self.stop_step = (torch.full((B,), -1, dtype=torch.int32, device=device)
                          if stop_step is None else stop_step.to(device).clone())
        self.tokens = torch.full((B,), -7, dtype=torch.int32, device=device)
        self.regret = torch.full((B,), -7.0, dtype=torch.float32, device=device)
        self.logprob = torch.full((B,), -7.0, dtype=torch.float32, device=device)
        self.entropy = torch.full((B,), -7.0, dtype=torch.float32, device=device)

    def host(self):
        return {k: getattr(self, k).cpu().numpy()
                for k in ("z", "alive", "stop_step", "tokens", "regret", "logprob", "entropy")}


_workspaces = {}


def step_workspace(nbytes, device="cuda"):
    """A zero-initialised workspace of at least `nbytes` bytes.  espo_step leaves its workspace zero again,
    so one buffer per size serves every call of a test run (calls here never overlap)."""
    if nbytes <= 0:
        return None
    size = 1 << (int(nbytes) - 1).bit_length()
    if size not in _workspaces:
        _workspaces[size] = torch.zeros(size, dtype=torch.uint8, device=device)
    return _workspaces[size]


def gpu_step(logits, tau, seed, step, values, gparams, st: GpuState, V=None, entropy=False, logprob=True,
             workspace=True, margin_scale=None, waves=None, chunks=None):
    """One espo_step call.  By default it gets a workspace, i.e. the library splits rows over workgroups
    wherever it sees fit (the production layout); `workspace=False` gives the one-workgroup-per-row layout.
    `margin_scale`, `waves`, `chunks` force those choices through the diagnostics entry point."""
    B, width = logits.shape
    ws = None
    if chunks is not None and chunks > 1:
        ws = step_workspace(espo.espo_debug_step_workspace_bytes(B, chunks))
    elif workspace and chunks is None:
        ws = step_workspace(espo.espo_step_workspace_bytes(B, width if V is None else V, logits.dtype))
    espo.espo_step(logits, tau, seed, step, values, gparams, st.z, st.alive, st.stop_step,
                   st.tokens, st.regret, st.logprob if logprob else None, V=V, entropy=st.entropy if entropy else None,
                   workspace=ws, margin_scale=margin_scale, waves=waves, chunks=chunks)


def compare_step(logits, tau, seed, step, values, gparams, oparams, st: GpuState, V=None, rows=None,
                 stats=None, entropy=False, **layout):
    """Runs one step on both sides from the GPU's current state and compares all outputs.

    `rows` restricts the oracle to a subset of rows (the GPU always runs the whole batch).
    With `entropy` the step is asked for its entropy output as well (the kernel's other
    instantiation) and that is compared too.  Returns the GPU's host-side outputs of the step.
    """
    B = logits.shape[0]
    rows = np.arange(B) if rows is None else np.asarray(rows)
    ridx = torch.as_tensor(rows, device=logits.device, dtype=torch.long)
    before = {"z": st.z[ridx].cpu().numpy(), "alive": st.alive[ridx].cpu().numpy(),
              "stop_step": st.stop_step[ridx].cpu().numpy()}
    vals_h = values[ridx].cpu().numpy()
    bits = np.ascontiguousarray(to_host_bits(logits[ridx]))
    gpu_step(logits, tau, seed, step, values, gparams, st, V=V, entropy=entropy, **layout)
    torch.cuda.synchronize()
    got = st.host()
    for ws in _workspaces.values():                          # the call must hand its workspace back as it got it
        assert not bool(ws.any()), "espo_step left its workspace non-zero"

    # the oracle keys its stream by the row id in the full batch: give it a batch in which
    # the subset sits at its real positions (other rows dead)
    nfull = int(rows.max()) + 1 if len(rows) else 0
    full_bits = np.zeros((nfull, bits.shape[1]), bits.dtype)
    full_bits[rows] = bits
    z = np.zeros(nfull, np.float32); z[rows] = before["z"]
    alive = np.zeros(nfull, np.uint8); alive[rows] = before["alive"]
    ss = np.full(nfull, -1, np.int32); ss[rows] = before["stop_step"]
    vals = np.zeros(nfull, np.float32); vals[rows] = vals_h
    z0, alive0, ss0 = z.copy(), alive.copy(), ss.copy()
    ref = oracle.step(full_bits, tau, seed, step, vals, oparams, z, alive, ss, V=V, want_entropy=entropy)

    tok_g = got["tokens"][rows]
    tok_o = ref["tokens"][rows]
    mism = rows[tok_g != tok_o]
    if len(mism):
        forced = np.full(nfull, -1, np.int32)
        for b in mism:
            s1, s2 = ref["best_score"][b], ref["second_score"][b]
            ok = got["tokens"][b] == ref["second_token"][b] and (s1 - s2) <= NEAR_TIE * abs(s1)
            assert ok, (f"step {step} row {b}: token {got['tokens'][b]} != oracle {ref['tokens'][b]} "
                        f"(runner-up {ref['second_token'][b]}, scores {s1!r} {s2!r})")
            forced[b] = got["tokens"][b]
        if stats is not None:
            stats["near_ties"] = stats.get("near_ties", 0) + len(mism)
        z, alive, ss = z0, alive0, ss0
        ref = oracle.step(full_bits, tau, seed, step, vals, oparams, z, alive, ss, V=V, forced_tokens=forced,
                          want_entropy=entropy)

    where = f"step {step}"
    np.testing.assert_array_equal(got["tokens"][rows], ref["tokens"][rows], err_msg=where)
    np.testing.assert_array_equal(got["regret"][rows].view(np.uint32), ref["regret"][rows].view(np.uint32), err_msg=where)
    np.testing.assert_array_equal(got["z"][rows].view(np.uint32), z[rows].view(np.uint32), err_msg=where)
    np.testing.assert_array_equal(got["alive"][rows], alive[rows], err_msg=where)
    np.testing.assert_array_equal(got["stop_step"][rows], ss[rows], err_msg=where)
    rtol = RTOL_BF16 if logits.dtype == torch.bfloat16 else RTOL_F32
    lp_g, lp_o = got["logprob"][rows].astype(np.float64), ref["logprob"][rows].astype(np.float64)
    err = np.abs(lp_g - lp_o)
    assert (err <= rtol * np.maximum(np.abs(lp_o), 1.0)).all(), (where, err.max(), lp_g[err.argmax()], lp_o[err.argmax()])
    if entropy:
        h_g, h_o = got["entropy"][rows].astype(np.float64), ref["entropy"][rows].astype(np.float64)
        herr = np.abs(h_g - h_o)
        assert (herr <= RTOL_F32 * np.maximum(h_o, 1.0)).all(), (where, herr.max(), h_g[herr.argmax()], h_o[herr.argmax()])
        if stats is not None:
            stats["max_entropy_err"] = max(stats.get("max_entropy_err", 0.0), float(herr.max()) if len(herr) else 0.0)
    if stats is not None:
        stats["max_logprob_err"] = max(stats.get("max_logprob_err", 0.0), float(err.max()) if len(err) else 0.0)
        stats["rows_checked"] = stats.get("rows_checked", 0) + int(before["alive"].sum())
    return got


def _padded_terms(r_h, v_h, L_h, s_h, r_fail, T):
    """|r_eff|, |V| and |V'| of a padded batch as the kernels must see them: the failure reward at the last
    token of a stopped row, nothing at or beyond the length, V := 0 after the last token."""
    B = v_h.shape[0]
    Lc = np.clip(L_h, 0, T)
    pad = np.arange(T)[None, :] >= Lc[:, None]
    r_eff = np.where(pad, 0.0, np.nan_to_num(r_h.astype(np.float64)))
    rows = np.nonzero((Lc > 0) & (s_h != 0))[0]
    r_eff[rows, Lc[rows] - 1] = r_fail
    v_abs = np.where(pad, 0.0, np.abs(np.nan_to_num(v_h.astype(np.float64))))
    v_next = np.concatenate([v_abs[:, 1:], np.zeros((B, 1))], axis=1)
    return pad, np.abs(r_eff), v_abs, v_next


def check_advantages(rewards, values, lengths, stopped, r_fail, gamma, lam, rtol=ADV_RTOL):
    """GPU TD errors / GAE against the double-precision oracle on the same inputs.

    Tolerance: |err| <= rtol * scale with scale = sum_l c^l (|r| + |gamma V'| + |V|) >= |ref|,
    the magnitude of the terms that fp32 rounding and reassociation act on (delta itself
    may cancel to almost nothing); padding must be exactly zero.
    """
    B, T = rewards.shape
    td = torch.full((B, T), 7.0, dtype=torch.float32, device=rewards.device)
    adv = torch.full((B, T), 7.0, dtype=torch.float32, device=rewards.device)
    espo.espo_advantages(rewards, values, lengths, stopped, r_fail, gamma, lam, td, adv)
    torch.cuda.synchronize()
    r_h, v_h = rewards.cpu().numpy(), values.cpu().numpy()
    L_h, s_h = lengths.cpu().numpy(), stopped.cpu().numpy()
    td_o, adv_o, scale = oracle.advantages(r_h, v_h, L_h, s_h, r_fail, gamma, lam)
    td_g, adv_g = td.cpu().numpy().astype(np.float64), adv.cpu().numpy().astype(np.float64)
    pad, r_abs, v_abs, v_next = _padded_terms(r_h, v_h, L_h, s_h, r_fail, T)
    assert (td_g[pad] == 0).all() and (adv_g[pad] == 0).all(), "padding must be exactly zero"
    assert np.isfinite(td_g).all() and np.isfinite(adv_g).all()
    e_td = np.abs(td_g - td_o)
    assert (e_td <= td_bound(r_abs, v_abs, v_next, gamma)).all(), e_td.max()
    e_adv = np.abs(adv_g - adv_o)
    tol = rtol * np.maximum(np.abs(adv_o), scale)
    assert (e_adv <= tol).all(), (e_adv.max(), np.unravel_index((e_adv - tol).argmax(), e_adv.shape))
    return float((e_adv / np.maximum(scale, 1e-30))[~pad].max()) if (~pad).any() else 0.0


def check_advantages_terminal(values, lengths, stopped, term, r_fail, gamma, lam, zero_padding=True, want_returns=True,
                              rtol=ADV_RTOL):
    """The terminal-reward form against its oracle.  Same tolerances as `check_advantages`; the
    value targets carry one more fp32 addition.  Without zero padding every position at or
    beyond a row's length must be either untouched or zero, and nothing else is required of it.
    """
    B, T = values.shape
    FILL = 7.0
    td = torch.full((B, T), FILL, dtype=torch.float32, device=values.device)
    adv = torch.full((B, T), FILL, dtype=torch.float32, device=values.device)
    ret = torch.full((B, T), FILL, dtype=torch.float32, device=values.device) if want_returns else None
    espo.espo_advantages_terminal(values, lengths, stopped, term, r_fail, gamma, lam, td, adv, returns=ret,
                                  zero_padding=zero_padding)
    torch.cuda.synchronize()
    v_h, L_h, s_h, t_h = values.cpu().numpy(), lengths.cpu().numpy(), stopped.cpu().numpy(), term.cpu().numpy()
    td_o, adv_o, ret_o = oracle.advantages_terminal(v_h, L_h, s_h, t_h, r_fail, gamma, lam)
    Lc = np.clip(L_h, 0, T)
    pad = np.arange(T)[None, :] >= Lc[:, None]
    # magnitude of the terms: the dense-form oracle's scale on the same rewards spelled out
    dense = np.zeros((B, T), np.float32)
    rows = np.nonzero(Lc > 0)[0]
    dense[rows, Lc[rows] - 1] = t_h[rows]
    v_clean = np.where(pad, 0, v_h).astype(np.float32)
    _, _, scale = oracle.advantages(dense, v_clean, L_h, s_h, r_fail, gamma, lam)
    outs = [("td", td, td_o), ("adv", adv, adv_o)] + ([("returns", ret, ret_o)] if want_returns else [])
    worst = 0.0
    for name, g, o in outs:
        g = g.cpu().numpy().astype(np.float64)
        if zero_padding:
            assert (g[pad] == 0).all(), f"{name}: padding must be exactly zero"
        else:
            assert ((g[pad] == 0) | (g[pad] == FILL)).all(), f"{name}: padding is neither untouched nor zero"
        assert np.isfinite(g[~pad]).all()
        err = np.abs(g - o)[~pad]
        if name == "td":
            _, r_abs, v_abs, v_next = _padded_terms(dense, v_clean, L_h, s_h, r_fail, T)
            assert (err <= td_bound(r_abs, v_abs, v_next, gamma)[~pad]).all(), (name, err.max())
        else:
            tol = (rtol * np.maximum(np.abs(o), scale))[~pad]
            assert (err <= tol).all(), (name, err.max())
            if len(err):
                worst = max(worst, float((err / np.maximum(scale[~pad], 1e-30)).max()))
    return worst


def check_advantages_packed(values, cu, stopped, r_fail, gamma, lam, rewards=None, term=None, want_returns=True,
                            rtol=ADV_RTOL):
    """The packed layout against its oracle.  Tolerances as in `check_advantages`; positions that
    no trajectory owns must keep what they held, bit for bit."""
    N = values.numel()
    FILL = 7.0
    td = torch.full((N,), FILL, dtype=torch.float32, device=values.device)
    adv = torch.full((N,), FILL, dtype=torch.float32, device=values.device)
    ret = torch.full((N,), FILL, dtype=torch.float32, device=values.device) if want_returns else None
    espo.espo_advantages_packed(values, cu, stopped, r_fail, gamma, lam, td, adv, rewards=rewards, terminal_reward=term,
                                returns=ret)
    torch.cuda.synchronize()
    v_h, cu_h, s_h = values.cpu().numpy(), cu.cpu().numpy(), stopped.cpu().numpy()
    r_h = rewards.cpu().numpy() if rewards is not None else None
    t_h = term.cpu().numpy() if term is not None else None
    td_o, adv_o, ret_o, scale = oracle.advantages_packed(r_h, t_h, v_h, cu_h, s_h, r_fail, gamma, lam)
    owned = ~np.isnan(td_o)                                  # the oracle writes only what a trajectory owns
    outs = [("td", td, td_o), ("adv", adv, adv_o)] + ([("returns", ret, ret_o)] if want_returns else [])
    worst = 0.0
    for name, g, o in outs:
        g = g.cpu().numpy().astype(np.float64)
        assert (g[~owned] == FILL).all(), f"{name}: a position that no trajectory owns was written"
        assert np.isfinite(g[owned]).all(), name
        err = np.abs(g - o)[owned]
        if name == "td":
            # delta_t is three fp32 operations on exact inputs, judged against the size of its terms: the reward
            # the step really uses (at a trajectory's last token r_fail or the terminal reward, zero before it
            # in the terminal form) and the two values (V := 0 after the last token)
            v_abs = np.abs(np.nan_to_num(v_h.astype(np.float64)))
            v_next = np.append(v_abs[1:], 0.0)
            r_abs = np.abs(np.nan_to_num(r_h.astype(np.float64))) if r_h is not None else np.zeros(N)
            for b in range(len(s_h)):                        # extents as the library clips them
                first, end = min(max(int(cu_h[b]), 0), N), min(int(cu_h[b + 1]), N)
                if end > first:
                    v_next[end - 1] = 0.0
                    if s_h[b]:
                        r_abs[end - 1] = abs(r_fail)
                    elif t_h is not None:
                        r_abs[end - 1] = abs(float(t_h[b]))
            assert (err <= td_bound(r_abs, v_abs, v_next, gamma)[owned]).all(), (name, err.max())
        else:
            tol = (rtol * np.maximum(np.abs(o), scale))[owned]
            assert (err <= tol).all(), (name, err.max(), int((err - tol).argmax()))
            if len(err):
                worst = max(worst, float((err / np.maximum(scale[owned], 1e-30)).max()))
    return worst
