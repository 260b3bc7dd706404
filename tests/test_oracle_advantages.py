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
