"""Parity of the HIP espo_advantages with the CPU oracle, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2605_29860_amd as espo  # noqa: E402
from paper_2605_29860_amd import workloads as W  # noqa: E402
import harness as H  # noqa: E402


def _say(msg):
    print(msg, flush=True)


def _batch(B, T, seed, lengths=None, stop_p=0.4, poison=True):
    g = torch.Generator().manual_seed(seed)
    rewards = torch.randn(B, T, generator=g)
    values = torch.rand(B, T, generator=g) * 2 - 1
    L = torch.randint(0, T + 1, (B,), generator=g) if lengths is None else torch.as_tensor(lengths)
    stopped = (torch.rand(B, generator=g) < stop_p).to(torch.uint8)
    if poison:
        pad = torch.arange(T)[None, :] >= L.clamp(0, T)[:, None]
        rewards[pad] = float("nan")
        values[pad] = float("nan")
    return rewards.cuda(), values.cuda(), L.to(torch.int32).cuda(), stopped.cuda()


@pytest.mark.parametrize("T", [1, 3, 4, 7, 8, 9, 64, 511, 512, 2047, 2048, 2049, 4100, 6151])
def test_shapes_and_ragged_lengths(T):
    _say(f"[case] advantages T={T}")
    B = 9
    L = [0, T, 1, max(T - 1, 0), T // 2, min(T, 2048), min(T, 2049), min(T, 513), T]
    for gamma, lam in ((1.0, 0.95), (0.99, 0.9), (1.0, 1.0), (0.9, 0.0)):
        r, v, Lt, s = _batch(B, T, seed=T, lengths=L)
        H.check_advantages(r, v, Lt, s, -1.0, gamma, lam)


def test_out_of_range_lengths_and_empty():
    _say("[case] advantages clamping / empty")
    B, T = 4, 100
    r, v, _, s = _batch(B, T, seed=1, lengths=[T, T, T, T], poison=False)
    L = torch.tensor([-3, T + 50, 0, 17], dtype=torch.int32).cuda()
    H.check_advantages(r, v, L, s, -1.0, 1.0, 0.95)
    e = torch.zeros(0, 5, device="cuda")
    espo.espo_advantages(e, e, torch.zeros(0, dtype=torch.int32, device="cuda"),
                         torch.zeros(0, dtype=torch.uint8, device="cuda"), -1.0, 1.0, 0.95, e.clone(), e.clone())
    with pytest.raises(espo.EspoError):
        espo.espo_advantages(r, v, L, s, -1.0, float("nan"), 0.95, torch.empty_like(r), torch.empty_like(r))


def test_closed_forms_on_device():
    _say("[case] advantages closed forms")
    # zero values, stopped: A_t = r_fail c^(L-1-t); gamma = lambda = 1: A_t = return-to-go - V_t
    B, T = 3, 5000
    z = torch.zeros(B, T, device="cuda")
    L = torch.tensor([5000, 3000, 1], dtype=torch.int32, device="cuda")
    st = torch.ones(B, dtype=torch.uint8, device="cuda")
    td, adv = torch.empty_like(z), torch.empty_like(z)
    espo.espo_advantages(z, z, L, st, -1.0, 1.0, 0.95, td, adv)
    a = adv.cpu().numpy().astype(np.float64)
    c = float(np.float32(0.95))
    for b, n in enumerate([5000, 3000, 1]):
        ref = -1.0 * c ** (n - 1 - np.arange(n))
        np.testing.assert_allclose(a[b, :n], ref, rtol=2e-5, atol=1e-30)
        assert (a[b, n:] == 0).all()
    r, v, Lr, s = _batch(6, 3000, seed=5)
    H.check_advantages(r, v, Lr, s, -2.0, 1.0, 1.0)


def test_config5_full_size():
    _say("[case] config 5 (B=1024, T=16384)")
    r, v, L, s = W.advantage_batch(device="cuda", poison=True, seed=5)
    assert r.shape == (1024, 16384)
    worst = H.check_advantages(r, v, L, s, -1.0, 1.0, 0.95)
    frac = float(s.float().mean())
    _say(f"  config 5: valid tokens {int(L.sum())}, stopped fraction {frac:.2f}, worst scaled error {worst:.2e}")
    assert 0.2 < frac < 0.4
    # a second call on the same inputs gives the same bits
    td1, adv1 = torch.empty_like(r), torch.empty_like(r)
    td2, adv2 = torch.empty_like(r), torch.empty_like(r)
    espo.espo_advantages(r, v, L, s, -1.0, 1.0, 0.95, td1, adv1)
    espo.espo_advantages(r, v, L, s, -1.0, 1.0, 0.95, td2, adv2)
    torch.cuda.synchronize()
    assert torch.equal(td1, td2) and torch.equal(adv1, adv2)


def test_ablation_variant_without_the_failure_penalty():
    _say("[case] advantages, variant C (no terminal penalty)")
    # Section 6, variant C: trajectories are truncated by the stop rule but get no failure reward.  That is this
    # call with every `stopped` flag zero: the truncated row keeps its stored last reward (0 in Algorithm 1).
    # Checked against the oracle, and against the full method on the same rows: only the rows that the rule had
    # stopped change, by r_fail (gamma lambda)^(L-1-t).
    r, v, L, s = W.advantage_batch(B=64, T=3000, len_lo=1, seed=31, device="cuda", poison=True)
    none = torch.zeros_like(s)
    H.check_advantages(r, v, L, none, -1.0, 1.0, 0.95)
    td_c, adv_c = torch.empty_like(r), torch.empty_like(r)
    td_a, adv_a = torch.empty_like(r), torch.empty_like(r)
    espo.espo_advantages(r, v, L, none, -1.0, 1.0, 0.95, td_c, adv_c)
    espo.espo_advantages(r, v, L, s, -1.0, 1.0, 0.95, td_a, adv_a)
    torch.cuda.synchronize()
    diff = (adv_a - adv_c).cpu().numpy().astype(np.float64)
    L_h, s_h = L.cpu().numpy(), s.cpu().numpy()
    assert s_h.any() and not s_h.all()
    c = float(np.float32(0.95))
    for b in range(64):
        n = int(L_h[b])
        want = -1.0 * c ** (n - 1 - np.arange(n)) if s_h[b] else np.zeros(n)   # the stored last reward of a stopped row is 0
        np.testing.assert_allclose(diff[b, :n], want, rtol=0, atol=1e-4)    # two fp32 scans of sums of size ~30
        assert (diff[b, n:] == 0).all()


@pytest.mark.parametrize("B", [513, 1025, 2500, 4096, 4097])
def test_many_rows(B):
    _say(f"[case] advantages B={B}")
    # More rows than workgroups fit on the chip at once: every row must still be processed
    # exactly once (outputs are pre-filled with a sentinel by the check), also with many equal
    # lengths, empty rows and lengths out of range.
    T = 260
    g = torch.Generator().manual_seed(B)
    L = torch.randint(0, T + 1, (B,), generator=g)
    L[::7] = T
    L[3::11] = 0
    L[5::13] = 17
    r, v, Lt, s = _batch(B, T, seed=B, lengths=L.tolist())
    H.check_advantages(r, v, Lt, s, -1.0, 1.0, 0.95)
    Lt[1] = -4
    Lt[2] = T + 100
    r = torch.nan_to_num(r, nan=0.0)
    v = torch.nan_to_num(v, nan=0.0)
    H.check_advantages(r, v, Lt, s, -0.5, 0.97, 0.9)
    # all rows of one length: the scans after the first 512 look their rows up by class of length and,
    # inside a class, by index; here that is one class, over several chunks of 1024 rows for the larger B
    r, v, Lt, s = _batch(B, T, seed=B + 1, lengths=[T - 1] * B)
    H.check_advantages(r, v, Lt, s, -1.0, 1.0, 0.95)


# --------------------------------------------------------------------------- terminal-reward form
def _terminal_batch(B, T, seed, lengths=None, stop_p=0.4):
    g = torch.Generator().manual_seed(seed)
    values = torch.rand(B, T, generator=g) * 2 - 1
    L = torch.randint(0, T + 1, (B,), generator=g) if lengths is None else torch.as_tensor(lengths)
    stopped = (torch.rand(B, generator=g) < stop_p).to(torch.uint8)
    term = torch.randint(0, 2, (B,), generator=g).float() + 0.25 * torch.randn(B, generator=g)
    values[torch.arange(T)[None, :] >= L.clamp(0, T)[:, None]] = float("nan")   # never to be read
    return values.cuda(), L.to(torch.int32).cuda(), stopped.cuda(), term.cuda()


@pytest.mark.parametrize("T", [1, 3, 4, 7, 8, 9, 64, 511, 512, 2047, 2048, 2049, 4100, 6151, 8192, 9000])
def test_terminal_form_shapes_and_options(T):
    _say(f"[case] advantages, terminal form T={T}")
    L = [0, T, 1, max(T - 1, 0), T // 2, min(T, 2048), min(T, 2049), min(T, 513), T, min(T, 4096), min(T, 4097)]
    v, Lt, s, term = _terminal_batch(len(L), T, seed=T, lengths=L)
    for gamma, lam in ((1.0, 0.95), (0.99, 0.9), (1.0, 1.0), (0.9, 0.0)):
        H.check_advantages_terminal(v, Lt, s, term, -1.0, gamma, lam, zero_padding=True, want_returns=True)
    H.check_advantages_terminal(v, Lt, s, term, -1.0, 1.0, 0.95, zero_padding=False, want_returns=True)
    H.check_advantages_terminal(v, Lt, s, term, -0.5, 1.0, 0.95, zero_padding=False, want_returns=False)
    H.check_advantages_terminal(v, Lt, s, term, -0.5, 1.0, 0.95, zero_padding=True, want_returns=False)


def test_terminal_form_equals_dense_form_bit_for_bit():
    _say("[case] advantages, terminal form vs dense form")
    B, T = 64, 9001
    v, L, s, term = _terminal_batch(B, T, seed=77)
    dense = torch.zeros(B, T, device="cuda")
    rows = torch.nonzero(L > 0).flatten()
    dense[rows, (L[rows] - 1).long()] = term[rows]
    td_d, adv_d = torch.empty_like(dense), torch.empty_like(dense)
    td_t, adv_t, ret = torch.empty_like(dense), torch.empty_like(dense), torch.empty_like(dense)
    espo.espo_advantages(dense, v, L, s, -1.0, 0.99, 0.95, td_d, adv_d)
    espo.espo_advantages_terminal(v, L, s, term, -1.0, 0.99, 0.95, td_t, adv_t, returns=ret)
    torch.cuda.synchronize()
    assert torch.equal(td_d, td_t) and torch.equal(adv_d, adv_t)
    valid = torch.arange(T, device="cuda")[None, :] < L[:, None]
    assert torch.equal(ret[valid], (adv_t + torch.nan_to_num(v))[valid]) and (ret[~valid] == 0).all()
    # lambda = 1: the value target is the discounted terminal reward, whatever the critic says
    espo.espo_advantages_terminal(v, L, s, term, -1.0, 0.999, 1.0, td_t, adv_t, returns=ret)
    torch.cuda.synchronize()
    r_end = torch.where(s > 0, torch.full_like(term, -1.0), term).double()
    dist = (L[:, None] - 1 - torch.arange(T, device="cuda")[None, :]).clamp(min=0).double()
    want = r_end[:, None] * float(np.float32(0.999)) ** dist
    err = (ret.double() - want).abs()[valid]
    assert float(err.max()) < 2e-4, float(err.max())     # ~9000 fp32 steps through values of size 1


def test_terminal_form_config5_full_size():
    _say("[case] config 5 in the terminal form (B=1024, T=16384)")
    r, v, L, s = W.advantage_batch(device="cuda", poison=True, seed=5)
    rows = torch.arange(r.shape[0], device="cuda")
    term = torch.nan_to_num(r[rows, (L - 1).clamp(min=0).long()])    # the survivors' terminal reward in {0, 1}
    worst = H.check_advantages_terminal(v, L, s, term, -1.0, 1.0, 0.95, zero_padding=False, want_returns=True)
    _say(f"  worst scaled error {worst:.2e}")
    worst = H.check_advantages_terminal(v, L, s, term, -1.0, 1.0, 0.95, zero_padding=True, want_returns=False)
    _say(f"  worst scaled error {worst:.2e}")


@pytest.mark.parametrize("part", range(5))
def test_seeded_sweep_of_both_forms(part):
    _say(f"[case] advantages, seeded sweep, part {part} (140 cases, both reward forms each)")
    rng = np.random.default_rng(4242 + part)
    worst = 0.0
    for case in range(part * 140, part * 140 + 140):
        T = int(rng.choice([rng.integers(1, 64), rng.integers(64, 5000), rng.integers(5000, 20000)]))
        B = int(rng.integers(1, 12))
        g = torch.Generator().manual_seed(7000 + case)
        v = (torch.rand(B, T, generator=g) * 2 - 1) * float(rng.choice([1.0, 30.0]))
        r = torch.randn(B, T, generator=g)
        L = torch.randint(0, T + 1, (B,), generator=g)
        pad = torch.arange(T)[None, :] >= L[:, None]
        v[pad] = float("nan")
        r[pad] = float("nan")
        s = (torch.rand(B, generator=g) < 0.4).to(torch.uint8)
        term = torch.randn(B, generator=g)
        gamma, lam = float(rng.choice([1.0, 0.99, 0.9])), float(rng.choice([0.95, 1.0, 0.0, 0.5]))
        r_fail = float(rng.choice([-1.0, -0.25, 0.0]))
        args = (v.cuda(), L.to(torch.int32).cuda(), s.cuda())
        try:
            worst = max(worst, H.check_advantages(r.cuda(), *args, r_fail, gamma, lam))
            worst = max(worst, H.check_advantages_terminal(*args, term.cuda(), r_fail, gamma, lam,
                                                           zero_padding=bool(rng.random() < 0.5),
                                                           want_returns=bool(rng.random() < 0.5)))
        except AssertionError as err:
            raise AssertionError(f"case {case}: T={T} B={B} gamma={gamma} lambda={lam} r_fail={r_fail}: {err}")
    _say(f"  worst scaled error {worst:.2e}")


# ------------------------------------------------------------------ trajectories stored back to back

def _packed(lens, seed, gaps=None, scale=1.0, stop_p=0.4):
    """Values, rewards, extents for the given lengths; `gaps[b]` unowned tokens (NaN) before trajectory b."""
    g = torch.Generator().manual_seed(seed)
    B = len(lens)
    gaps = [0] * B if gaps is None else gaps
    starts, pos = [], 0
    for b in range(B):
        pos += gaps[b]
        starts.append(pos)
        pos += lens[b]
    N = pos
    values = (torch.rand(N, generator=g) * 2 - 1) * scale
    rewards = torch.randn(N, generator=g)
    owned = torch.zeros(N, dtype=torch.bool)
    for b in range(B):
        owned[starts[b]:starts[b] + lens[b]] = True
    values[~owned] = float("nan")
    rewards[~owned] = float("nan")
    stopped = (torch.rand(B, generator=g) < stop_p).to(torch.uint8)
    term = torch.randn(B, generator=g)
    return values.cuda(), rewards.cuda(), starts, stopped.cuda(), term.cuda()


def _check_packed_both_forms(lens, seed, gaps=None, gamma=1.0, lam=0.95, r_fail=-1.0, scale=1.0):
    """With gaps the extents are not one running sum, so gapped layouts go one call per extent pair:
    cu = [start_b, end_b] is a valid one-trajectory call into the same arrays."""
    v, r, starts, s, term = _packed(lens, seed, gaps, scale)
    worst = 0.0
    if gaps is None:
        cu = torch.tensor(starts + [starts[-1] + lens[-1]] if lens else [0], dtype=torch.int64).cuda()
        worst = max(worst, H.check_advantages_packed(v, cu, s, r_fail, gamma, lam, rewards=r, want_returns=False))
        worst = max(worst, H.check_advantages_packed(v, cu, s, r_fail, gamma, lam, term=term, want_returns=True))
    else:
        for b in range(len(lens)):
            cu = torch.tensor([starts[b], starts[b] + lens[b]], dtype=torch.int64).cuda()
            worst = max(worst, H.check_advantages_packed(v, cu, s[b:b + 1], r_fail, gamma, lam, rewards=r, want_returns=True))
            worst = max(worst, H.check_advantages_packed(v, cu, s[b:b + 1], r_fail, gamma, lam, term=term[b:b + 1], want_returns=False))
    return worst


@pytest.mark.parametrize("L", [1, 2, 3, 4, 5, 7, 8, 63, 64, 257, 4093, 4096, 4097, 8191, 8200, 12289])
def test_packed_every_alignment_of_start_and_end(L):
    _say(f"[case] packed advantages, L={L}")
    # neighbours of 1..3 tokens shift the start through all four alignments; each one is a trajectory itself
    lens = [L, 1, L, 2, L, 3, L, 0, L, 5, 0, 0, L]
    for gamma, lam in ((1.0, 0.95), (0.99, 0.9), (1.0, 1.0), (0.9, 0.0)):
        _check_packed_both_forms(lens, seed=L, gamma=gamma, lam=lam)


def test_packed_gaps_are_neither_read_nor_written():
    _say("[case] packed advantages, unowned gaps")
    lens = [5, 4096, 1, 300, 4099, 2, 8193]
    gaps = [3, 1, 2, 5, 0, 7, 1]
    _check_packed_both_forms(lens, seed=11, gaps=gaps)


def test_packed_extents_are_clipped_and_empty_batches():
    _say("[case] packed advantages, clipping / empty")
    v, r, starts, s, term = _packed([100, 50], seed=12)
    N = v.numel()
    td, adv = torch.full((N,), 7.0, device="cuda"), torch.full((N,), 7.0, device="cuda")
    ref_td, ref_adv = torch.full((N,), 7.0, device="cuda"), torch.full((N,), 7.0, device="cuda")
    espo.espo_advantages_packed(v, torch.tensor([0, 100, 150]).cuda(), s, -1.0, 1.0, 0.95, ref_td, ref_adv, terminal_reward=term)
    espo.espo_advantages_packed(v, torch.tensor([-9, 100, 10**12]).cuda(), s, -1.0, 1.0, 0.95, td, adv, terminal_reward=term)
    torch.cuda.synchronize()
    assert torch.equal(td, ref_td) and torch.equal(adv, ref_adv)
    td.fill_(7.0)
    espo.espo_advantages_packed(v, torch.tensor([120, 30, 10]).cuda(), s, -1.0, 1.0, 0.95, td, adv, terminal_reward=term)
    torch.cuda.synchronize()
    assert (td == 7.0).all()                                  # reversed extents hold no token
    H.check_advantages_packed(v, torch.tensor([-9, 100, 10**12]).cuda(), s, -1.0, 1.0, 0.95, rewards=r)
    e = torch.zeros(0, device="cuda")
    espo.espo_advantages_packed(e, torch.zeros(1, dtype=torch.int64, device="cuda"), torch.zeros(0, dtype=torch.uint8, device="cuda"),
                                -1.0, 1.0, 0.95, e.clone(), e.clone(), terminal_reward=e.clone())
    with pytest.raises(espo.EspoError):                       # both reward forms at once
        espo.espo_advantages_packed(v, torch.tensor([0, 100, 150]).cuda(), s, -1.0, 1.0, 0.95, td, adv, rewards=r, terminal_reward=term)
    with pytest.raises(espo.EspoError):                       # a view that starts 4 bytes into an allocation
        espo.espo_advantages_packed(v[1:], torch.tensor([0, 100, 149]).cuda(), s, -1.0, 1.0, 0.95, td[1:], adv[1:], terminal_reward=term)


def test_packed_config5_full_size():
    _say("[case] config 5 stored back to back (B=1024, lengths as in the padded workload)")
    r, v, L, s = W.advantage_batch(device="cuda", poison=False, seed=5)
    B, T = v.shape
    valid = torch.arange(T, device="cuda")[None, :] < L[:, None]
    cu = torch.zeros(B + 1, dtype=torch.int64, device="cuda")
    cu[1:] = torch.cumsum(L.long(), 0)
    vp, rp = v[valid].contiguous(), r[valid].contiguous()
    rows = torch.arange(B, device="cuda")
    term = r[rows, (L - 1).clamp(min=0).long()].contiguous()
    _say(f"  N = {vp.numel()} of {B * T}")
    worst = H.check_advantages_packed(vp, cu, s, -1.0, 1.0, 0.95, rewards=rp, want_returns=False)
    _say(f"  dense form: worst scaled error {worst:.2e}")
    worst = H.check_advantages_packed(vp, cu, s, -1.0, 1.0, 0.95, term=term, want_returns=True)
    _say(f"  terminal form: worst scaled error {worst:.2e}")


@pytest.mark.parametrize("part", range(4))
def test_packed_seeded_sweep(part):
    _say(f"[case] packed advantages, seeded sweep, part {part} (100 cases, both reward forms each)")
    rng = np.random.default_rng(5151 + part)
    worst = 0.0
    for case in range(part * 100, part * 100 + 100):
        B = int(rng.integers(1, 24))
        top = int(rng.choice([8, 200, 5000, 14000]))
        lens = [int(x) for x in rng.integers(0, top + 1, B)]
        for b in range(B):
            if rng.random() < 0.15:
                lens[b] = 0
        gamma, lam = float(rng.choice([1.0, 0.99, 0.9])), float(rng.choice([0.95, 1.0, 0.0, 0.5]))
        r_fail = float(rng.choice([-1.0, -0.25, 0.0]))
        try:
            worst = max(worst, _check_packed_both_forms(lens, 9000 + case, gamma=gamma, lam=lam, r_fail=r_fail,
                                                        scale=float(rng.choice([1.0, 30.0]))))
        except AssertionError as err:
            raise AssertionError(f"case {case}: lens={lens[:8]}... gamma={gamma} lambda={lam} r_fail={r_fail}: {err}")
    _say(f"  worst scaled error {worst:.2e}")
