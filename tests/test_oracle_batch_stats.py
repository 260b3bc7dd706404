"""Pins of the oracle's batch-boundary update (Section 4.2, Eq. beta_update) against hand
values, closed forms and numpy's textbook routines."""
import os

import numpy as np
import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))
CTRL = dict(alpha_ema=0.99, eta_beta=0.1, target_rate=0.25, beta_min=0.0, beta_max=7.0)


def _golden(name):
    out = {}
    for line in open(os.path.join(HERE, "golden", name)):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            out[k] = float(v)
    return out


def test_hand_example():
    want = _golden("batch_stats_hand_example.txt")
    g = np.array([[1, 2, 3, 9], [4, 0, 9, 9]], np.float32)
    got = oracle.batch_stats(g, np.array([3, 1], np.int32), np.array([1, 0], np.uint8), 1.0, 2.0, 3.0, **CTRL)
    for k, v in want.items():
        assert got[k] == pytest.approx(v, rel=1e-6), k
    assert got["tokens"] == 4


def test_matches_numpy_on_valid_tokens_and_never_reads_beyond_length():
    rng = np.random.default_rng(0)
    B, T = 37, 211
    g = rng.gamma(2.0, 1.5, (B, T)).astype(np.float32)
    L = rng.integers(0, T + 1, B).astype(np.int32)
    L[3], L[4] = 0, T
    stopped = (rng.random(B) < 0.3).astype(np.uint8)
    mask = np.arange(T)[None, :] < L[:, None]
    valid = g[mask].astype(np.float64)
    poisoned = g.copy()
    poisoned[~mask] = np.nan
    got = oracle.batch_stats(poisoned, L, stopped, 0.7, 1.3, 5.0, **CTRL)
    assert got["tokens"] == int(L.sum())
    assert got["mean"] == pytest.approx(valid.mean(), rel=1e-12)
    assert got["var"] == pytest.approx(valid.var(), rel=1e-12)           # numpy's default: divisor n
    assert got["stop_rate"] == stopped.mean()
    a, mu0, var0 = (float(np.float32(x)) for x in (0.99, 0.7, 1.3))   # the parameters are floats
    assert got["mu_g"] == np.float32(a * mu0 + (1 - a) * valid.mean())
    assert got["var_g"] == np.float32(a * var0 + (1 - a) * valid.var())
    # lengths outside [0, T] are clamped
    L2 = L.copy(); L2[3], L2[4] = -5, T + 9
    again = oracle.batch_stats(poisoned, L2, stopped, 0.7, 1.3, 5.0, **CTRL)
    assert again == got


def test_constant_regret_and_ema_fixed_point():
    g = np.full((5, 9), 2.25, np.float32)
    L = np.array([9, 1, 0, 4, 9], np.int32)
    s = np.zeros(5, np.uint8)
    got = oracle.batch_stats(g, L, s, 2.25, 0.0, 1.0, **CTRL)
    assert got["mean"] == 2.25 and got["var"] == 0.0
    assert got["mu_g"] == np.float32(2.25) and got["var_g"] == np.float32(0.0)   # already at the fixed point
    # repeated updates move the statistics geometrically towards the batch values: after k
    # updates the distance has shrunk by alpha^k
    mu, var = 0.0, 5.0
    for k in range(1, 6):
        r = oracle.batch_stats(g, L, s, mu, var, 1.0, **CTRL)
        mu, var = float(r["mu_g"]), float(r["var_g"])
        assert mu == pytest.approx(2.25 * (1 - 0.99 ** k), rel=1e-5)
        assert var == pytest.approx(5.0 * 0.99 ** k, rel=1e-5)


def test_beta_controller_direction_and_clipping():
    g = np.ones((8, 4), np.float32)
    L = np.full(8, 4, np.int32)
    def beta_after(nstop, beta, **kw):
        s = np.zeros(8, np.uint8); s[:nstop] = 1
        c = dict(CTRL); c.update(kw)
        return float(oracle.batch_stats(g, L, s, 1.0, 1.0, beta, **c)["beta"])
    assert beta_after(2, 3.0) == np.float32(3.0)                      # at the target rate: unchanged
    assert beta_after(8, 3.0) == pytest.approx(3.075, rel=1e-6)       # too many stops: threshold goes up
    assert beta_after(0, 3.0) == pytest.approx(2.975, rel=1e-6)       # too few: it comes down
    assert beta_after(8, 6.99) == 7.0                                 # clipped at beta_max
    assert beta_after(0, 0.01) == 0.0                                 # and at beta_min
    assert beta_after(0, 3.0, eta_beta=0.0) == 3.0


def test_empty_batches_leave_the_state_alone():
    g = np.zeros((3, 5), np.float32)
    none = oracle.batch_stats(g, np.zeros(3, np.int32), np.array([1, 1, 1], np.uint8), 0.4, 0.6, 2.0, **CTRL)
    assert none["tokens"] == 0 and none["mu_g"] == np.float32(0.4) and none["var_g"] == np.float32(0.6)
    assert none["beta"] == pytest.approx(2.075, rel=1e-6)             # the stop rate is still defined
    empty = oracle.batch_stats(np.zeros((0, 5), np.float32), np.zeros(0, np.int32), np.zeros(0, np.uint8),
                               0.4, 0.6, 2.0, **CTRL)
    assert empty["mu_g"] == np.float32(0.4) and empty["beta"] == np.float32(2.0) and empty["stop_rate"] == 0.0
