"""Pins of the CPU oracle's TD-error / GAE pass (Section 3, Eq. gae; Section 4.4).

CPU only.  The backward recursion is checked against hand-worked numbers, the explicit
double sum of Eq. gae, textbook special cases and the truncation rules.
"""
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_batch(rng, B, T, stop_p=0.4):
    rewards = rng.normal(0, 1, (B, T)).astype(np.float32)
    values = rng.uniform(-1, 1, (B, T)).astype(np.float32)
    lengths = rng.integers(0, T + 1, B).astype(np.int32)
    stopped = (rng.random(B) < stop_p).astype(np.uint8)
    return rewards, values, lengths, stopped


def test_hand_worked_examples(oracle):
    rows = [l.split() for l in open(os.path.join(GOLDEN, "gae_hand_example.txt"))
            if l.strip() and not l.startswith("#")]
    exp = {}
    for case, t, td, adv in rows:
        exp.setdefault(case, []).append((int(t), float(td), float(adv)))
    v = np.array([[0.5, 0.2, -0.1]], np.float32)
    cases = {
        "A": (np.array([[0, 0, 1]], np.float32), v, [3], [0], -1.0, 1.0, 0.95),
        "B": (np.array([[0, 7, 1]], np.float32), v, [2], [1], -1.0, 1.0, 0.95),   # stored 7 is replaced
        "C": (np.array([[0, 0, 2]], np.float32), np.array([[1, 2, 4]], np.float32), [3], [0], -1.0, 0.5, 0.5),
    }
    for name, (r, val, L, st, rf, gam, lam) in cases.items():
        td, adv, _ = oracle.advantages(r, val, np.array(L, np.int32), np.array(st, np.uint8), rf, gam, lam)
        for t, e_td, e_adv in exp[name]:
            assert abs(td[0, t] - e_td) < 1e-6, (name, t)          # inputs are fp32-rounded decimals
            assert abs(adv[0, t] - e_adv) < 1e-6, (name, t)


@pytest.mark.parametrize("gamma,lam", [(1.0, 0.95), (0.99, 0.9), (0.5, 1.0), (1.0, 1.0), (0.9, 0.0)])
def test_recursion_equals_explicit_sum(oracle, gamma, lam):
    rng = np.random.default_rng(7)
    for T in (1, 2, 5, 16):
        r, v, L, st = _rand_batch(rng, 12, T)
        td, adv, _ = oracle.advantages(r, v, L, st, -1.0, gamma, lam)
        brute = oracle.gae_bruteforce(r, v, L, st, -1.0, gamma, lam)
        np.testing.assert_allclose(adv, brute, rtol=1e-12, atol=1e-12)


def test_td_error_definition_and_truncation(oracle):
    rng = np.random.default_rng(8)
    B, T = 20, 11
    r, v, L, st = _rand_batch(rng, B, T)
    L[0], L[1], L[2] = 0, T, 1
    gamma, lam, rf = 0.97, 0.9, -1.0
    td, adv, scale = oracle.advantages(r, v, L, st, rf, gamma, lam)
    g = float(np.float32(gamma))
    for b in range(B):
        n = int(L[b])
        assert (td[b, n:] == 0).all() and (adv[b, n:] == 0).all() and (scale[b, n:] == 0).all()
        for t in range(n):
            last = t == n - 1
            r_t = rf if (last and st[b]) else float(r[b, t])          # Eq. failure_reward: overwrite
            v_next = 0.0 if last else float(v[b, t + 1])               # no bootstrap past the end
            assert abs(td[b, t] - (r_t + g * v_next - float(v[b, t]))) < 1e-12
        if n:
            assert abs(adv[b, n - 1] - td[b, n - 1]) < 1e-15           # A_{L-1} = delta_{L-1}
    assert (scale >= np.abs(adv) - 1e-12).all()


def test_lambda_zero_gives_td_and_ones_give_telescoping_return(oracle):
    rng = np.random.default_rng(9)
    B, T = 10, 40
    r, v, L, st = _rand_batch(rng, B, T)
    td, adv, _ = oracle.advantages(r, v, L, st, -2.0, 0.9, 0.0)
    np.testing.assert_array_equal(adv, td)                            # lambda = 0: A = delta
    td, adv, _ = oracle.advantages(r, v, L, st, -2.0, 1.0, 1.0)
    for b in range(B):
        n = int(L[b])
        rr = r[b, :n].astype(np.float64).copy()
        if n and st[b]:
            rr[n - 1] = -2.0
        ret = np.cumsum(rr[::-1])[::-1]                               # Monte-Carlo return-to-go
        np.testing.assert_allclose(adv[b, :n], ret - v[b, :n], rtol=1e-12, atol=1e-12)


def test_failure_penalty_propagates_geometrically(oracle):
    # zero values and rewards, stopped at L: A_t = r_fail * (gamma*lambda)^(L-1-t)
    B, T = 3, 64
    r = np.zeros((B, T), np.float32)
    v = np.zeros((B, T), np.float32)
    L = np.array([64, 10, 1], np.int32)
    st = np.array([1, 1, 1], np.uint8)
    td, adv, _ = oracle.advantages(r, v, L, st, -1.0, 1.0, 0.95)
    c = float(np.float32(0.95))
    for b in range(B):
        n = int(L[b])
        t = np.arange(n)
        np.testing.assert_allclose(adv[b, :n], -1.0 * c ** (n - 1 - t), rtol=1e-12)
        assert td[b, n - 1] == -1.0 and (td[b, : n - 1] == 0).all()
    # a survivor with the same inputs gets nothing
    td, adv, _ = oracle.advantages(r, v, L, np.zeros(B, np.uint8), -1.0, 1.0, 0.95)
    assert (adv == 0).all() and (td == 0).all()


def test_padding_is_never_read_and_lengths_are_clamped(oracle):
    rng = np.random.default_rng(10)
    B, T = 8, 30
    r, v, L, st = _rand_batch(rng, B, T)
    L[:] = rng.integers(1, T, B)
    ref = oracle.advantages(r, v, L, st, -1.0, 1.0, 0.95)
    r2, v2 = r.copy(), v.copy()
    for b in range(B):
        r2[b, L[b]:] = np.nan
        v2[b, L[b]:] = np.nan
    got = oracle.advantages(r2, v2, L, st, -1.0, 1.0, 0.95)
    for a, b_ in zip(ref, got):
        np.testing.assert_array_equal(a, b_)
    # out-of-range lengths behave like 0 and T
    Lc = L.copy()
    Lc[0], Lc[1] = -5, T + 100
    a = oracle.advantages(r, v, Lc, st, -1.0, 1.0, 0.95)
    Lc[0], Lc[1] = 0, T
    b_ = oracle.advantages(r, v, Lc, st, -1.0, 1.0, 0.95)
    np.testing.assert_array_equal(a[1], b_[1])
    assert (a[1][0] == 0).all()


def test_empty_shapes(oracle):
    e = np.zeros((0, 5), np.float32)
    td, adv, _ = oracle.advantages(e, e, np.zeros(0, np.int32), np.zeros(0, np.uint8), -1.0, 1.0, 0.95)
    assert td.shape == (0, 5)
    e = np.zeros((3, 0), np.float32)
    td, adv, _ = oracle.advantages(e, e, np.zeros(3, np.int32), np.zeros(3, np.uint8), -1.0, 1.0, 0.95)
    assert adv.shape == (3, 0)


# ------------------------------------------------------------------ terminal-reward form (Algorithm 1's rewards)
def _terminal_batch(rng, B, T, stop_p=0.4):
    values = rng.uniform(-1, 1, (B, T)).astype(np.float32)
    lengths = rng.integers(0, T + 1, B).astype(np.int32)
    stopped = (rng.random(B) < stop_p).astype(np.uint8)
    term = rng.integers(0, 2, B).astype(np.float32) + rng.normal(0, 0.1, B).astype(np.float32)
    return values, lengths, stopped, term


def test_terminal_form_hand_examples(oracle):
    rows = [l.split() for l in open(os.path.join(GOLDEN, "gae_terminal_hand_example.txt"))
            if l.strip() and not l.startswith("#")]
    v = np.array([[0.5, 0.2, -0.1]], np.float32)
    cases = {"A": (v, [3], [0], [1.0], -1.0, 1.0, 0.95), "B": (v, [2], [1], [9.0], -1.0, 1.0, 0.95),
             "C": (np.array([[1, 2, 4]], np.float32), [3], [0], [2.0], -1.0, 0.5, 0.5)}
    assert len(rows) == 9
    for name, t, e_td, e_adv, e_ret in rows:
        val, L, st, term, rf, gam, lam = cases[name]
        td, adv, ret = oracle.advantages_terminal(val, np.array(L, np.int32), np.array(st, np.uint8),
                                                  np.array(term, np.float32), rf, gam, lam)
        t = int(t)
        assert abs(td[0, t] - float(e_td)) < 1e-6 and abs(adv[0, t] - float(e_adv)) < 1e-6, (name, t)
        assert abs(ret[0, t] - float(e_ret)) < 1e-6, (name, t)


def test_terminal_form_equals_dense_form_and_bruteforce(oracle):
    rng = np.random.default_rng(31)
    B, T = 24, 41
    values, lengths, stopped, term = _terminal_batch(rng, B, T)
    lengths[:3] = [0, 1, T]
    dense = np.zeros((B, T), np.float32)                    # the same rewards, spelled out per token
    for b in range(B):
        if lengths[b] > 0:
            dense[b, lengths[b] - 1] = term[b]
    for gam, lam in [(1.0, 0.95), (0.9, 0.8), (1.0, 1.0), (0.7, 0.0)]:
        td, adv, ret = oracle.advantages_terminal(values, lengths, stopped, term, -1.0, gam, lam)
        td_d, adv_d, _ = oracle.advantages(dense, values, lengths, stopped, -1.0, gam, lam)
        brute = oracle.gae_bruteforce(dense, values, lengths, stopped, -1.0, gam, lam)
        np.testing.assert_allclose(td, td_d, rtol=0, atol=1e-15)
        np.testing.assert_allclose(adv, adv_d, rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(adv, brute, rtol=1e-11, atol=1e-12)
        mask = np.arange(T)[None, :] < lengths[:, None]
        np.testing.assert_allclose(ret, np.where(mask, adv + values, 0.0), rtol=1e-15, atol=0)
        assert (td[~mask] == 0).all() and (adv[~mask] == 0).all() and (ret[~mask] == 0).all()


def test_terminal_form_textbook_targets(oracle):
    rng = np.random.default_rng(32)
    B, T = 16, 30
    values, lengths, stopped, term = _terminal_batch(rng, B, T)
    lengths = np.maximum(lengths, 1).astype(np.int32)
    r_fail, gam = -1.0, 0.9
    r_end = np.where(stopped == 1, np.float64(r_fail), term.astype(np.float64))
    t = np.arange(T)[None, :]
    mask = t < lengths[:, None]
    # lambda = 1: the target is the discounted Monte-Carlo return, whatever the critic says
    _, _, ret = oracle.advantages_terminal(values, lengths, stopped, term, r_fail, gam, 1.0)
    mc = np.where(mask, r_end[:, None] * np.float64(np.float32(gam)) ** (lengths[:, None] - 1 - t).clip(0), 0.0)
    np.testing.assert_allclose(ret, mc, rtol=1e-12, atol=1e-13)
    # lambda = 0: the one-step TD target gamma V(s_{t+1}), and the terminal reward at the end
    _, adv0, ret0 = oracle.advantages_terminal(values, lengths, stopped, term, r_fail, gam, 0.0)
    nxt = np.concatenate([values[:, 1:], np.zeros((B, 1), np.float32)], axis=1).astype(np.float64)
    want = np.where(t == lengths[:, None] - 1, r_end[:, None], np.float64(np.float32(gam)) * nxt)
    np.testing.assert_allclose(ret0, np.where(mask, want, 0.0), rtol=1e-13, atol=1e-15)
    # zero critic: A_t = r_end (gamma lambda)^(L-1-t), so early stopping reaches back geometrically
    zero = np.zeros_like(values)
    _, adv, _ = oracle.advantages_terminal(zero, lengths, stopped, term, r_fail, 1.0, 0.95)
    geo = np.where(mask, r_end[:, None] * np.float64(np.float32(0.95)) ** (lengths[:, None] - 1 - t).clip(0), 0.0)
    np.testing.assert_allclose(adv, geo, rtol=1e-12, atol=0)
    # NaN beyond the lengths is never read
    poisoned = values.copy()
    poisoned[~mask] = np.nan
    a, b, c = oracle.advantages_terminal(poisoned, lengths, stopped, term, r_fail, gam, 0.95)
    a2, b2, c2 = oracle.advantages_terminal(values, lengths, stopped, term, r_fail, gam, 0.95)
    assert np.array_equal(a, a2) and np.array_equal(b, b2) and np.array_equal(c, c2)


# ------------------------------------------------------------------ trajectories stored back to back

def _packed_batch(rng, B, max_len, gap=0):
    """Random extents (some empty), optional unowned gaps between them."""
    lens = rng.integers(0, max_len + 1, B)
    lens[rng.random(B) < 0.15] = 0
    cu = np.zeros(B + 1, np.int64)
    starts = np.zeros(B, np.int64)
    pos = 0
    for b in range(B):
        pos += int(rng.integers(0, gap + 1))
        starts[b] = pos
        pos += int(lens[b])
    N = pos + gap
    values = rng.uniform(-1, 1, N).astype(np.float32)
    rewards = rng.normal(0, 1, N).astype(np.float32)
    stopped = (rng.random(B) < 0.4).astype(np.uint8)
    term = rng.choice(np.array([0.0, 1.0, -0.5], np.float32), B)
    return lens.astype(np.int64), starts, values, rewards, stopped, term


def test_packed_hand_worked_examples(oracle):
    """The three worked examples of the padded layout, laid end to end (case B keeps 2 of its 3 tokens)."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "gae_hand_example.txt"))
            if l.strip() and not l.startswith("#")]
    exp = {}
    for case, t, td, adv in rows:
        exp.setdefault(case, []).append((int(t), float(td), float(adv)))
    v = [0.5, 0.2, -0.1]
    for gam, lam, names in ((1.0, 0.95, "AB"), (0.5, 0.5, "C")):
        if names == "AB":
            values = np.array(v + v[:2], np.float32)
            rewards = np.array([0, 0, 1, 0, 7], np.float32)          # the stored 7 is replaced by r_fail
            cu = np.array([0, 3, 5], np.int64)
            stopped = np.array([0, 1], np.uint8)
        else:
            values = np.array([1, 2, 4], np.float32)
            rewards = np.array([0, 0, 2], np.float32)
            cu = np.array([0, 3], np.int64)
            stopped = np.array([0], np.uint8)
        td, adv, ret, _ = oracle.advantages_packed(rewards, None, values, cu, stopped, -1.0, gam, lam)
        for k, name in enumerate(names):
            for t, e_td, e_adv in exp[name]:
                if cu[k] + t < cu[k + 1]:
                    assert abs(td[cu[k] + t] - e_td) < 1e-6 and abs(adv[cu[k] + t] - e_adv) < 1e-6, (name, t)
                    assert abs(ret[cu[k] + t] - (e_adv + float(values[cu[k] + t]))) < 1e-6


@pytest.mark.parametrize("gamma,lam", [(1.0, 0.95), (0.99, 0.9), (1.0, 1.0), (0.9, 0.0)])
def test_packed_equals_explicit_sum_per_slice(oracle, gamma, lam):
    """Eq. gae written out as a double sum over each slice, both reward forms."""
    rng = np.random.default_rng(41)
    B = 20
    lens, starts, values, rewards, stopped, term = _packed_batch(rng, B, 17)
    cu = np.concatenate([starts, [starts[-1] + lens[-1]]]).astype(np.int64)
    g, c = np.float64(np.float32(gamma)), np.float64(np.float32(gamma)) * np.float64(np.float32(lam))
    for dense in (True, False):
        td, adv, ret, _ = oracle.advantages_packed(rewards if dense else None, None if dense else term, values, cu,
                                                   stopped, -1.0, gamma, lam)
        for b in range(B):
            s, L = int(cu[b]), int(lens[b])
            v = values[s:s + L].astype(np.float64)
            r = rewards[s:s + L].astype(np.float64) if dense else np.zeros(L)
            if L and not dense:
                r[-1] = term[b]
            if L and stopped[b]:
                r[-1] = -1.0
            delta = r + g * np.append(v[1:], 0.0) - v if L else np.zeros(0)
            for t in range(L):
                want = sum(c ** l * delta[t + l] for l in range(L - t))
                assert abs(adv[s + t] - want) <= 1e-12 * max(1.0, abs(want))
                assert td[s + t] == delta[t] and ret[s + t] == adv[s + t] + v[t]


def test_packed_agrees_with_the_padded_layout(oracle):
    rng = np.random.default_rng(42)
    B, T = 16, 33
    lens, starts, values, rewards, stopped, term = _packed_batch(rng, B, T)
    cu = np.concatenate([starts, [starts[-1] + lens[-1]]]).astype(np.int64)
    pad_r, pad_v = np.zeros((B, T), np.float32), np.zeros((B, T), np.float32)
    for b in range(B):
        pad_r[b, :lens[b]] = rewards[cu[b]:cu[b + 1]]
        pad_v[b, :lens[b]] = values[cu[b]:cu[b + 1]]
    td_p, adv_p, sc_p = oracle.advantages(pad_r, pad_v, lens.astype(np.int32), stopped, -1.0, 1.0, 0.95)
    td, adv, ret, sc = oracle.advantages_packed(rewards, None, values, cu, stopped, -1.0, 1.0, 0.95)
    td_t, adv_t, ret_t = oracle.advantages_terminal(pad_v, lens.astype(np.int32), stopped, term, -1.0, 1.0, 0.95)
    td2, adv2, ret2, _ = oracle.advantages_packed(None, term, values, cu, stopped, -1.0, 1.0, 0.95)
    for b in range(B):
        sl, L = slice(int(cu[b]), int(cu[b + 1])), int(lens[b])
        assert np.array_equal(td[sl], td_p[b, :L]) and np.array_equal(adv[sl], adv_p[b, :L])
        assert np.array_equal(sc[sl], sc_p[b, :L])
        assert np.array_equal(td2[sl], td_t[b, :L]) and np.array_equal(adv2[sl], adv_t[b, :L])
        assert np.array_equal(ret2[sl], ret_t[b, :L])


def test_packed_extents_gaps_and_neighbours(oracle):
    """Unowned positions are neither read nor written, a trajectory never sees its neighbour,
    extents are clipped to the arrays and reversed ones are empty."""
    rng = np.random.default_rng(43)
    B = 12
    lens, starts, values, rewards, stopped, term = _packed_batch(rng, B, 9, gap=3)
    N = values.shape[0]
    owned = np.zeros(N, bool)
    for b in range(B):
        owned[starts[b]:starts[b] + lens[b]] = True
    values[~owned] = np.nan
    # with gaps the extents are not a running sum: one call per trajectory, its own two offsets
    for b in range(B):
        cu = np.array([starts[b], starts[b] + lens[b]], np.int64)
        td, adv, ret, _ = oracle.advantages_packed(None, term[b:b + 1], values, cu, stopped[b:b + 1], -1.0, 0.9, 0.95)
        mine = np.zeros(N, bool)
        mine[cu[0]:cu[1]] = True
        assert np.isfinite(td[mine]).all() and np.isfinite(adv[mine]).all() and np.isnan(td[~mine]).all()
        # the same trajectory on its own gives the same numbers: nothing leaks in from either side
        alone = oracle.advantages_packed(None, term[b:b + 1], values[cu[0]:cu[1]].copy(), np.array([0, lens[b]], np.int64),
                                         stopped[b:b + 1], -1.0, 0.9, 0.95)
        assert np.array_equal(adv[mine], alone[1]) and np.array_equal(ret[mine], alone[2])
    # clipping: an extent that runs past N ends at N, a negative start begins at 0, a reversed one is empty
    v = rng.uniform(-1, 1, 10).astype(np.float32)
    one = np.array([0], np.uint8)
    ref = oracle.advantages_packed(None, np.ones(1, np.float32), v, np.array([4, 10], np.int64), one, -1.0, 1.0, 0.95)
    got = oracle.advantages_packed(None, np.ones(1, np.float32), v, np.array([4, 99], np.int64), one, -1.0, 1.0, 0.95)
    assert np.array_equal(ref[1][4:], got[1][4:])
    got = oracle.advantages_packed(None, np.ones(1, np.float32), v, np.array([-5, 10], np.int64), one, -1.0, 1.0, 0.95)
    ref = oracle.advantages_packed(None, np.ones(1, np.float32), v, np.array([0, 10], np.int64), one, -1.0, 1.0, 0.95)
    assert np.array_equal(ref[1], got[1])
    got = oracle.advantages_packed(None, np.ones(1, np.float32), v, np.array([7, 3], np.int64), one, -1.0, 1.0, 0.95)
    assert np.isnan(got[0]).all() and np.isnan(got[1]).all()


def test_packed_monte_carlo_return(oracle):
    """lambda = 1 with the rewards of Algorithm 1: the target is r_end gamma^(L-1-t), whatever the critic says."""
    rng = np.random.default_rng(44)
    B = 10
    lens, starts, values, rewards, stopped, term = _packed_batch(rng, B, 25)
    cu = np.concatenate([starts, [starts[-1] + lens[-1]]]).astype(np.int64)
    _, _, ret, _ = oracle.advantages_packed(None, term, values, cu, stopped, -2.0, 0.9, 1.0)
    g = np.float64(np.float32(0.9))
    for b in range(B):
        r_end = -2.0 if stopped[b] else float(term[b])
        want = r_end * g ** (lens[b] - 1 - np.arange(lens[b]))
        np.testing.assert_allclose(ret[cu[b]:cu[b + 1]], want, rtol=1e-12, atol=1e-13)
