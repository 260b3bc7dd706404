"""Pins of the CPU oracle's advantage whitening (the normalisation standard PPO applies to the
GAE output; Section 3 keeps the standard PPO update).  CPU only: a hand-worked case, numpy's
mean / var on full rows, the moments of the result, affine invariance and the masking rules."""
import numpy as np
import pytest


def test_hand_worked_case(oracle):
    # 1, 2, 3, 4: mean 5/2, squared deviations 9/4, 1/4, 1/4, 9/4 -> variance 5/4 (divisor 4) or 5/3 (divisor 3)
    a = np.array([[1, 2, 3, 4]], np.float32)
    L = np.array([4], np.int32)
    out, st = oracle.whiten(a, L, eps=0.0)
    assert st[0] == 2.5 and st[1] == 1.25 and st[2] == 4
    np.testing.assert_allclose(out[0], np.array([-1.5, -0.5, 0.5, 1.5]) / np.sqrt(1.25), rtol=1e-15)
    out, st = oracle.whiten(a, L, eps=0.0, unbiased=True)
    assert abs(st[1] - 5.0 / 3.0) < 1e-15
    np.testing.assert_allclose(out[0], np.array([-1.5, -0.5, 0.5, 1.5]) / np.sqrt(5.0 / 3.0), rtol=1e-15)
    out, _ = oracle.whiten(a, L, eps=0.0, shift_mean=False)                  # scaled only
    np.testing.assert_allclose(out[0], np.array([1, 2, 3, 4]) / np.sqrt(1.25), rtol=1e-15)
    out, _ = oracle.whiten(a, L, eps=0.75)                                   # eps joins the variance: sqrt(2)
    np.testing.assert_allclose(out[0], np.array([-1.5, -0.5, 0.5, 1.5]) / np.sqrt(2.0), rtol=1e-15)
    # two rows that hold the same four tokens between them: the batch is the unit, not the row
    b = np.array([[1, 2, 9], [3, 4, 9]], np.float32)
    out2, st2 = oracle.whiten(b, np.array([2, 2], np.int32), eps=0.0)
    assert st2[0] == 2.5 and st2[1] == 1.25
    np.testing.assert_allclose(np.concatenate([out2[0, :2], out2[1, :2]]), np.array([-1.5, -0.5, 0.5, 1.5]) / np.sqrt(1.25))


@pytest.mark.parametrize("unbiased", [False, True])
def test_full_rows_are_numpy_mean_and_var(oracle, unbiased):
    rng = np.random.default_rng(3)
    a = (rng.normal(0.7, 2.5, (7, 33))).astype(np.float32)
    L = np.full(7, 33, np.int32)
    out, st = oracle.whiten(a, L, eps=1e-8, unbiased=unbiased)
    a64 = a.astype(np.float64)
    assert abs(st[0] - a64.mean()) < 1e-13 and abs(st[1] - a64.var(ddof=int(unbiased))) < 1e-12 and st[2] == a.size
    np.testing.assert_allclose(out, (a64 - a64.mean()) / np.sqrt(a64.var(ddof=int(unbiased)) + np.float64(np.float32(1e-8))),
                               rtol=1e-12, atol=1e-13)


def test_moments_invariance_and_masking(oracle):
    rng = np.random.default_rng(4)
    B, T = 9, 40
    a = rng.normal(-0.3, 1.7, (B, T)).astype(np.float32)
    L = rng.integers(0, T + 1, B).astype(np.int32)
    L[:3] = [0, T, 1]
    mask = np.arange(T)[None, :] < L[:, None]
    out, st = oracle.whiten(a, L, eps=0.0)
    assert np.isnan(out[~mask]).all() and np.isfinite(out[mask]).all()       # padding is not written
    w = out[mask]
    assert abs(w.mean()) < 1e-14 and abs(w.var() - 1.0) < 1e-13 and st[2] == mask.sum()
    # padding is never read
    poisoned = a.copy()
    poisoned[~mask] = np.nan
    out_p, _ = oracle.whiten(poisoned, L, eps=0.0)
    assert np.array_equal(out_p[mask], out[mask])
    # a positive affine map of the advantages leaves the whitened values alone (eps = 0)
    a2 = (a.astype(np.float64) * 4.0 + 8.0).astype(np.float32)             # rounded to fp32 again, hence the two checks
    out2, _ = oracle.whiten(a2, L, eps=0.0)
    ref2 = (a2.astype(np.float64) - a2.astype(np.float64)[mask].mean()) / a2.astype(np.float64)[mask].std()
    np.testing.assert_allclose(out2[mask], ref2[mask], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(out2[mask], out[mask], rtol=0, atol=1e-5)     # a2 was rounded to fp32
    # lengths are clamped
    out_c, st_c = oracle.whiten(a, np.array([-4] + [T + 9] * (B - 1), np.int32), eps=0.0)
    assert np.isnan(out_c[0]).all() and st_c[2] == (B - 1) * T


def test_degenerate_batches(oracle):
    a = np.full((2, 5), 3.0, np.float32)
    out, st = oracle.whiten(a, np.array([0, 0], np.int32))
    assert np.isnan(out).all() and st[2] == 0                                # no valid token: nothing is written
    out, st = oracle.whiten(a, np.array([5, 2], np.int32), eps=1e-8)
    assert st[1] == 0 and (out[0] == 0).all() and (out[1, :2] == 0).all()    # constant batch: zero after the shift
    out, st = oracle.whiten(a, np.array([1, 0], np.int32), eps=1e-8, unbiased=True)
    assert st[1] == 0 and out[0, 0] == 0                                     # n - 1 = 0: variance taken as 0
    out, _ = oracle.whiten(a, np.array([1, 0], np.int32), eps=0.25, shift_mean=False)
    assert out[0, 0] == 6.0                                                  # 3 / sqrt(0 + 1/4)
    out, _ = oracle.whiten(a, np.array([5, 2], np.int32), eps=0.0)          # var + eps = 0: zeros, not 0/0
    assert (out[0] == 0).all() and (out[1, :2] == 0).all()
    out, _ = oracle.whiten(a, np.array([1, 0], np.int32), eps=0.0, shift_mean=False, unbiased=True)
    assert out[0, 0] == 0
    e = np.zeros((0, 4), np.float32)
    out, st = oracle.whiten(e, np.zeros(0, np.int32))
    assert out.shape == (0, 4) and st[2] == 0
