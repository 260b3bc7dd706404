"""Parity of the HIP espo_whiten with the CPU oracle, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import oracle  # noqa: E402
import paper_2605_29860_amd as espo  # noqa: E402
from paper_2605_29860_amd import workloads as W  # noqa: E402

FILL = 7.0


def _say(msg):
    print(msg, flush=True)


def _check(adv, lengths, eps=1e-8, shift_mean=True, unbiased=False, in_place=False):
    """Element by element against the oracle.  Each output is one subtraction and one product in
    double, rounded to float once, on a mean and a variance that carry ~1e-13 of relative error:
    the rounding to float is 6e-8 |ref|; 2e-7 * max(|ref|, 1)
    is what is asserted.  Padding must keep what it held."""
    B, T = adv.shape
    a_h, L_h = adv.cpu().numpy(), lengths.cpu().numpy()
    ref, st = oracle.whiten(a_h, L_h, eps, shift_mean, unbiased)
    ws = torch.empty(espo.espo_whiten_workspace_bytes(B, T), dtype=torch.uint8, device="cuda")
    stats = torch.full((3,), -1.0, dtype=torch.float64, device="cuda")
    mask = np.arange(T)[None, :] < np.clip(L_h, 0, T)[:, None]
    if in_place:
        out = adv.clone()
        espo.espo_whiten(out, lengths, out, ws, eps, shift_mean, unbiased, stats)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        keep = a_h[~mask]
        assert np.array_equal(got[~mask].view(np.uint32), keep.view(np.uint32)), "padding was written"
    else:
        out = torch.full((B, T), FILL, dtype=torch.float32, device="cuda")
        espo.espo_whiten(adv, lengths, out, ws, eps, shift_mean, unbiased, stats)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert (got[~mask] == FILL).all(), "padding was written"
    s = stats.cpu().numpy()
    if st[2] > 0:
        assert s[2] == st[2]
        assert abs(s[0] - st[0]) <= 1e-12 * max(abs(st[0]), np.sqrt(st[1]), 1e-30)
        assert abs(s[1] - st[1]) <= 1e-11 * max(st[1], 1e-300)
    else:
        assert (s == 0).all()
    g, r = got[mask].astype(np.float64), ref[mask]
    assert np.isfinite(g).all()
    err = np.abs(g - r)
    assert (err <= 2e-7 * np.maximum(np.abs(r), 1.0)).all(), (err.max(), int(err.argmax()))
    return float(err.max()) if len(err) else 0.0


def _batch(B, T, seed, lengths=None, mean=0.0, std=1.0):
    g = torch.Generator().manual_seed(seed)
    a = torch.randn(B, T, generator=g) * std + mean
    L = torch.randint(0, T + 1, (B,), generator=g) if lengths is None else torch.as_tensor(lengths)
    a[torch.arange(T)[None, :] >= L.clamp(0, T)[:, None]] = float("nan")      # padding must never be read
    return a.cuda(), L.to(torch.int32).cuda()


@pytest.mark.parametrize("T", [1, 3, 4, 7, 64, 1023, 1024, 4095, 4096, 4097, 8192, 9001, 16384])
def test_shapes_lengths_and_options(T):
    _say(f"[case] whiten T={T}")
    L = [0, T, 1, max(T - 1, 0), T // 2, min(T, 4096), min(T, 4097), min(T, 513), T]
    a, Lt = _batch(len(L), T, seed=T, lengths=L, mean=-0.4, std=1.3)
    _check(a, Lt)
    _check(a, Lt, unbiased=True)
    _check(a, Lt, shift_mean=False, eps=0.0)
    _check(a, Lt, eps=0.5, in_place=True)


def test_mean_far_from_zero_and_tiny_spread():
    _say("[case] whiten, mean far from zero")
    # values 1000 +- 0.01: a one-pass variance about zero would lose every digit in fp32 and ten in double
    a, L = _batch(40, 5000, seed=3, mean=1000.0, std=0.01)
    _check(a, L, eps=0.0)
    a, L = _batch(40, 5000, seed=4, mean=-3.0e4, std=2.0)
    _check(a, L, eps=1e-8, unbiased=True)


def test_degenerate_batches_and_errors():
    _say("[case] whiten, degenerate batches")
    a, L = _batch(3, 100, seed=5, lengths=[0, 0, 0])
    _check(a, L)                                              # no valid token: nothing written, stats zero
    a, L = _batch(3, 100, seed=6, lengths=[0, 1, 0])
    _check(a, L, eps=0.25, unbiased=True)                     # one token, n - 1 = 0: variance 0
    _check(a, L, eps=0.25, shift_mean=False)
    c = torch.full((4, 300), 2.5, device="cuda")
    _check(c, torch.tensor([300, 7, 0, 150], dtype=torch.int32, device="cuda"))   # constant: zeros
    _check(c, torch.tensor([300, 7, 0, 150], dtype=torch.int32, device="cuda"), eps=0.0)   # var + eps = 0: zeros too
    _check(c, torch.tensor([0, 1, 0, 0], dtype=torch.int32, device="cuda"), eps=0.0, shift_mean=False, unbiased=True)
    a, _ = _batch(4, 100, seed=7, lengths=[100] * 4)
    _check(a, torch.tensor([-3, 150, 0, 17], dtype=torch.int32, device="cuda"))   # lengths are clamped
    ws = torch.empty(espo.espo_whiten_workspace_bytes(4, 100), dtype=torch.uint8, device="cuda")
    e = torch.zeros(0, 5, device="cuda")
    espo.espo_whiten(e, torch.zeros(0, dtype=torch.int32, device="cuda"), e.clone(), ws)
    with pytest.raises(espo.EspoError):
        espo.espo_whiten(a, torch.zeros(4, dtype=torch.int32, device="cuda"), a.clone(), ws[:8])
    with pytest.raises(espo.EspoError):
        espo.espo_whiten(a, torch.zeros(4, dtype=torch.int32, device="cuda"), a.clone(), ws, eps=-1.0)


def test_packed_batch_is_one_long_row():
    _say("[case] whiten, packed batch")
    g = torch.Generator().manual_seed(8)
    N = 1_000_003
    a = (torch.randn(N, generator=g) * 0.7 - 0.2).cuda()
    L = torch.tensor([N], dtype=torch.int32, device="cuda")
    ws = torch.empty(espo.espo_whiten_workspace_bytes(1, N), dtype=torch.uint8, device="cuda")
    out = torch.empty_like(a)
    espo.espo_whiten(a, L, out, ws)
    torch.cuda.synchronize()
    ref, _ = oracle.whiten(a.cpu().numpy()[None, :], L.cpu().numpy())
    err = np.abs(out.cpu().numpy().astype(np.float64) - ref[0])
    assert (err <= 2e-7 * np.maximum(np.abs(ref[0]), 1.0)).all(), err.max()


def test_same_bits_on_every_run():
    _say("[case] whiten, run-to-run")
    a, L = _batch(64, 9001, seed=9)
    ws = torch.empty(espo.espo_whiten_workspace_bytes(64, 9001), dtype=torch.uint8, device="cuda")
    outs = []
    for _ in range(3):
        o = torch.zeros_like(a)
        espo.espo_whiten(a, L, o, ws)
        torch.cuda.synchronize()
        outs.append(o)
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


def test_config5_full_size_after_the_advantage_pass():
    _say("[case] whiten on the advantages of config 5 (B=1024, T=16384)")
    r, v, L, s = W.advantage_batch(device="cuda", poison=True, seed=5)
    td, adv = torch.empty_like(r), torch.empty_like(r)
    espo.espo_advantages(r, v, L, s, -1.0, 1.0, 0.95, td, adv)
    torch.cuda.synchronize()
    worst = _check(adv, L)
    _say(f"  worst error {worst:.2e}")
    worst = _check(adv, L, unbiased=True, in_place=True)
    _say(f"  worst error {worst:.2e}")


def test_seeded_sweep():
    _say("[case] whiten, seeded sweep")
    rng = np.random.default_rng(6262)
    worst = 0.0
    for case in range(100):
        T = int(rng.choice([rng.integers(1, 64), rng.integers(64, 5000), rng.integers(5000, 20000)]))
        B = int(rng.integers(1, 40))
        a, L = _batch(B, T, seed=11000 + case, mean=float(rng.choice([0.0, -0.5, 30.0])), std=float(rng.choice([1.0, 0.05, 20.0])))
        try:
            worst = max(worst, _check(a, L, eps=float(rng.choice([1e-8, 0.0, 0.1])), shift_mean=bool(rng.random() < 0.7),
                                      unbiased=bool(rng.random() < 0.5), in_place=bool(rng.random() < 0.5)))
        except AssertionError as err:
            raise AssertionError(f"case {case}: B={B} T={T}: {err}")
    _say(f"  worst error {worst:.2e}")
