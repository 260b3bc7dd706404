"""espo_advantages_ws, espo_length_order and espo_whiten_from_ws through the C ABI (needs an MI355X):
the advantage pass that takes its rows in a given order and leaves their sums in a workspace, the
order by length, and the whitening that starts from those sums.  td and adv must be the bits of espo_advantages (which the other tests hold against
the oracle); the whitened output is held against the oracle's."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import oracle  # noqa: E402
import paper_2605_29860_amd as espo  # noqa: E402
from paper_2605_29860_amd import workloads as W  # noqa: E402
import harness as H  # noqa: E402

FILL = 7.0
CLASSES = 256  # classes of the counting sort (rows of one class come in any order)


def _say(msg):
    print(msg, flush=True)


def _batch(B, T, seed, lengths=None, stop_p=0.4, offset=0.0):
    g = torch.Generator().manual_seed(seed)
    rewards = torch.randn(B, T, generator=g) + offset
    values = torch.rand(B, T, generator=g) * 2 - 1
    L = torch.randint(0, T + 1, (B,), generator=g) if lengths is None else torch.as_tensor(lengths)
    stopped = (torch.rand(B, generator=g) < stop_p).to(torch.uint8)
    pad = torch.arange(T)[None, :] >= L.clamp(0, T)[:, None]
    rewards[pad] = float("nan")                                   # padding must never be read
    values[pad] = float("nan")
    return rewards.cuda(), values.cuda(), L.to(torch.int32).cuda(), stopped.cuda()


FIRST = 512  # rows that are scanned in index order when the launch sorts the rest itself
HEAD = 256   # bytes at the start of the workspace that must be zero before its first use


def _workspace(B):
    n = espo.espo_advantages_ws_bytes(B)
    assert n == HEAD + 32 * B + (4 * max(B - FIRST, 0) + 15) // 16 * 16
    ws = torch.full((n,), 0xA5, dtype=torch.uint8, device="cuda")      # contents are irrelevant ...
    ws[:HEAD] = 0                                                     # ... but for the first 256 bytes
    return ws


def _run(r, v, L, s, r_fail=-1.0, gamma=1.0, lam=0.95, eps=1e-8, shift_mean=True, unbiased=False, oracle_pass=True,
         ordered=True):
    """Both advantage passes, the order, the workspace's contents, and both whitenings.  Returns the
    worst whitening error against the oracle."""
    B, T = r.shape
    td0, adv0 = torch.full_like(r, FILL), torch.full_like(r, FILL)
    td1, adv1 = torch.full_like(r, FILL), torch.full_like(r, FILL)
    ws = _workspace(B)
    Lc = np.clip(L.cpu().numpy().astype(np.int64), 0, T)
    order = None
    if ordered:  # the order: a permutation of the rows, classes of length never growing
        order = torch.full((B,), -7, dtype=torch.int32, device="cuda")
        espo.espo_length_order(L, T, order)
        o_h = order.cpu().numpy()
        assert sorted(o_h.tolist()) == list(range(B)), "the order is not a permutation of the rows"
        cls = (Lc[o_h] * CLASSES) // (T + 1)
        assert (np.diff(cls) <= 0).all(), "rows are not ordered by class of length, longest first"
    espo.espo_advantages(r, v, L, s, r_fail, gamma, lam, td0, adv0)
    espo.espo_advantages_ws(r, v, L, s, r_fail, gamma, lam, td1, adv1, ws, order)
    torch.cuda.synchronize()
    assert torch.equal(td0.view(torch.int32), td1.view(torch.int32)), "td differs from espo_advantages"
    assert torch.equal(adv0.view(torch.int32), adv1.view(torch.int32)), "adv differs from espo_advantages"

    assert not bool(ws[:HEAD].any()), "the first 256 bytes of the workspace must be zero again after the call"
    if not ordered and B > FIRST:  # the launch sorted rows FIRST.. itself: a permutation of them, longest first
        srt = ws[HEAD + 32 * B:HEAD + 32 * B + 4 * (B - FIRST)].view(torch.int32).cpu().numpy()
        assert sorted(srt.tolist()) == list(range(FIRST, B)), "the launch's own order is not a permutation of the later rows"
        assert (np.diff((Lc[srt] * CLASSES) // (T + 1)) <= 0).all()

    # the rows' sums: n, and mean and squared deviations as numpy forms them in double from adv
    rows = ws[HEAD:HEAD + 32 * B].view(torch.float64).cpu().numpy().reshape(B, 4)
    n = ws[HEAD:HEAD + 32 * B].view(torch.int64).cpu().numpy().reshape(B, 4)[:, 3]
    assert (n == Lc).all()
    a_h = adv1.cpu().numpy().astype(np.float64)
    for b in range(B):
        if Lc[b] == 0:
            continue
        x = a_h[b, :Lc[b]]
        mean = rows[b, 2] + rows[b, 0] / Lc[b]
        m2 = rows[b, 1] - rows[b, 0] ** 2 / Lc[b]
        scale = max(np.abs(x).max(), 1e-30)
        assert abs(mean - x.mean()) <= 1e-12 * scale, (b, mean, x.mean())
        assert abs(m2 - ((x - x.mean()) ** 2).sum()) <= 1e-9 * Lc[b] * scale ** 2, (b, m2)

    # whitening from the sums: against the oracle and against espo_whiten on the same advantages
    mask = np.arange(T)[None, :] < Lc[:, None]
    out1 = torch.full_like(r, FILL)
    st1 = torch.full((3,), -1.0, dtype=torch.float64, device="cuda")
    espo.espo_whiten_from_ws(adv1, L, out1, ws, eps, shift_mean, unbiased, st1)
    out0 = torch.full_like(r, FILL)
    st0 = torch.full((3,), -1.0, dtype=torch.float64, device="cuda")
    w0 = torch.empty(espo.espo_whiten_workspace_bytes(B, T), dtype=torch.uint8, device="cuda")
    espo.espo_whiten(adv1, L, out0, w0, eps, shift_mean, unbiased, st0)
    torch.cuda.synchronize()
    g1, g0 = out1.cpu().numpy(), out0.cpu().numpy()
    assert (g1[~mask] == FILL).all(), "padding was written"
    s1, s0 = st1.cpu().numpy(), st0.cpu().numpy()
    assert s1[2] == s0[2] == Lc.sum()
    worst = 0.0
    if Lc.sum() > 0:
        sd = np.sqrt(max(s0[1], 0.0))
        assert abs(s1[0] - s0[0]) <= 1e-12 * max(abs(s0[0]), sd, 1e-30), (s1, s0)
        assert abs(s1[1] - s0[1]) <= 1e-11 * max(s0[1], 1e-300), (s1, s0)
        # one unit in the last place of float at most between the two ways of summing
        ulp = np.spacing(np.abs(g0[mask]).astype(np.float32)).astype(np.float64)
        assert (np.abs(g1[mask].astype(np.float64) - g0[mask].astype(np.float64)) <= ulp + 1e-11).all()
        if oracle_pass:
            ref, st = oracle.whiten(adv1.cpu().numpy(), L.cpu().numpy(), eps, shift_mean, unbiased)
            assert abs(s1[0] - st[0]) <= 1e-12 * max(abs(st[0]), np.sqrt(st[1]), 1e-30)
            assert abs(s1[1] - st[1]) <= 1e-11 * max(st[1], 1e-300)
            err = np.abs(g1[mask].astype(np.float64) - ref[mask])
            assert (err <= 2e-7 * np.maximum(np.abs(ref[mask]), 1.0)).all(), err.max()
            worst = float(err.max())
    else:
        assert (s1 == 0).all()
    return worst


@pytest.mark.parametrize("T", [1, 3, 4, 7, 64, 1023, 4096, 4097, 9001])
def test_shapes_and_ragged_lengths(T):
    _say(f"[case] advantages_ws T={T}")
    L = [0, T, 1, max(T - 1, 0), T // 2, min(T, 4096), min(T, 4097), min(T, 513), T]
    r, v, Lt, s = _batch(len(L), T, seed=T, lengths=L)
    for gamma, lam in ((1.0, 0.95), (0.99, 0.9)):
        _run(r, v, Lt, s, gamma=gamma, lam=lam)
    _run(r, v, Lt, s, ordered=False)
    _run(r, v, Lt, s, unbiased=True, eps=0.0, shift_mean=False)
    # against the oracle's advantages as well, once per shape
    H.check_advantages(r, v, Lt, s, -1.0, 1.0, 0.95)


@pytest.mark.parametrize("B", [1, 9, 255, 256, 257, 300, 512, 513, 514, 1025, 2600])
def test_row_counts_around_the_class_count(B):
    _say(f"[case] advantages_ws B={B}")
    T = 700
    r, v, L, s = _batch(B, T, seed=B)
    _run(r, v, L, s, oracle_pass=B <= 300)
    _run(r, v, L, s, oracle_pass=False, ordered=False)
    # all rows equally long (one class), and no valid token at all
    r, v, L, s = _batch(B, T, seed=B + 1, lengths=[T // 3] * B)
    _run(r, v, L, s, oracle_pass=B <= 300)
    r, v, L, s = _batch(B, T, seed=B + 2, lengths=[0] * B)
    _run(r, v, L, s)


def test_lengths_out_of_range_and_rows_already_sorted():
    _say("[case] advantages_ws, clamped lengths, sorted and reversed rows")
    B, T = 64, 3000
    r, v, _, s = _batch(B, T, seed=3, lengths=[T] * B)
    L = torch.tensor([-3, T + 50, 0, 17] * 16, dtype=torch.int32).cuda()
    _run(r, v, L, s)
    for order in (np.arange(B), np.arange(B)[::-1]):
        L = torch.tensor((order * (T // B)).copy(), dtype=torch.int32).cuda()
        _run(r, v, L, s)


def test_mean_far_from_zero():
    _say("[case] advantages_ws, advantages far from zero")
    # rewards around 1000 with gamma = lambda = 1: advantages grow to millions along a row, so a row's
    # sums about any one value of its own lose digits; the bars of _run must still hold
    r, v, L, s = _batch(40, 5000, seed=4, offset=1000.0, stop_p=0.0)
    _run(r, v, L, s, gamma=1.0, lam=1.0, eps=0.0)
    _run(r, v, L, s, gamma=1.0, lam=0.0, eps=0.0, unbiased=True)     # lam = 0: adv = td, about 1000 +- 1


def test_workspace_contract_and_same_bits_on_every_run():
    _say("[case] advantages_ws, workspace contract")
    B, T = 33, 1000
    r, v, L, s = _batch(B, T, seed=6)
    td, adv = torch.empty_like(r), torch.empty_like(r)
    ws = _workspace(B)
    with pytest.raises(espo.EspoError) as e:
        espo.espo_advantages_ws(r, v, L, s, -1.0, 1.0, 0.95, td, adv, ws[:-1])
    assert e.value.code == -3
    big = torch.empty(ws.numel() + 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(espo.EspoError) as e:
        espo.espo_advantages_ws(r, v, L, s, -1.0, 1.0, 0.95, td, adv, big[8:8 + ws.numel()].zero_())   # not 16-byte aligned
    assert e.value.code == -3
    with pytest.raises(ValueError):
        espo.espo_advantages_ws(r, v, L, s, -1.0, 1.0, 0.95, td, adv, ws, torch.zeros(B - 1, dtype=torch.int32, device="cuda"))
    # an order with entries that name no row: those workgroups do nothing, the named rows are as ever
    td.fill_(FILL); adv.fill_(FILL)
    bad = torch.arange(B, dtype=torch.int32, device="cuda")
    bad[3], bad[7] = -1, B + 5
    espo.espo_advantages_ws(r, v, L, s, -1.0, 1.0, 0.95, td, adv, ws, bad)
    td_ref, adv_ref = torch.empty_like(r), torch.empty_like(r)
    espo.espo_advantages(r, v, L, s, -1.0, 1.0, 0.95, td_ref, adv_ref)
    torch.cuda.synchronize()
    named = torch.ones(B, dtype=torch.bool, device="cuda")
    named[3] = named[7] = False
    assert torch.equal(adv[named], adv_ref[named]) and (adv[~named] == FILL).all() and (td[~named] == FILL).all()
    with pytest.raises(espo.EspoError) as e:
        espo.espo_whiten_from_ws(adv, L, adv.clone(), ws[:-1])
    assert e.value.code == -3
    assert espo.espo_advantages_ws_bytes(0) == 0
    e0 = torch.zeros(0, 5, device="cuda")
    espo.espo_advantages_ws(e0, e0, torch.zeros(0, dtype=torch.int32, device="cuda"),
                            torch.zeros(0, dtype=torch.uint8, device="cuda"), -1.0, 1.0, 0.95, e0.clone(), e0.clone(), ws)
    espo.espo_length_order(torch.zeros(0, dtype=torch.int32, device="cuda"), 5, torch.zeros(0, dtype=torch.int32, device="cuda"))
    outs = []
    for _ in range(3):
        ws[HEAD:].fill_(0x5A)
        espo.espo_advantages_ws(r, v, L, s, -1.0, 1.0, 0.95, td, adv, ws)
        o = torch.zeros_like(adv)
        espo.espo_whiten_from_ws(adv, L, o, ws)
        torch.cuda.synchronize()
        outs.append(o)
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
    # in place
    o = adv.clone()
    espo.espo_whiten_from_ws(o, L, o, ws)
    torch.cuda.synchronize()
    mask = (torch.arange(T, device="cuda")[None, :] < L.clamp(0, T)[:, None])
    assert torch.equal(o[mask], outs[0][mask]) and torch.equal(o[~mask].view(torch.int32), adv[~mask].view(torch.int32))


def test_config5_full_size():
    _say("[case] advantages_ws + whiten_from_ws on config 5 (B=1024, T=16384)")
    r, v, L, s = W.advantage_batch(device="cuda", poison=True, seed=5)
    worst = _run(r, v, L, s)
    _say(f"  worst whitening error {worst:.2e}")
    _run(r, v, L, s, ordered=False, oracle_pass=False)      # the launch sorts rows 512.. itself
    # a workspace that served another batch size, and the same call twice: the first 256 bytes are all that has to be zero
    ws = _workspace(2600)
    td, adv = torch.empty_like(r), torch.empty_like(r)
    td_ref, adv_ref = torch.empty_like(r), torch.empty_like(r)
    espo.espo_advantages(r, v, L, s, -1.0, 1.0, 0.95, td_ref, adv_ref)
    for _ in range(3):
        td.fill_(FILL); adv.fill_(FILL)
        espo.espo_advantages_ws(r, v, L, s, -1.0, 1.0, 0.95, td, adv, ws)
        torch.cuda.synchronize()
        assert torch.equal(td, td_ref) and torch.equal(adv, adv_ref) and not bool(ws[:HEAD].any())


def test_seeded_sweep():
    _say("[case] advantages_ws, seeded sweep")
    rng = np.random.default_rng(7171)
    worst = 0.0
    for case in range(120):
        T = int(rng.choice([rng.integers(1, 64), rng.integers(64, 5000), rng.integers(5000, 20000)]))
        B = int(rng.choice([rng.integers(1, 40), rng.integers(40, 600), rng.integers(500, 1400)])) if T < 5000 else int(rng.integers(1, 40))
        r, v, L, s = _batch(B, T, seed=21000 + case, stop_p=float(rng.random()))
        try:
            worst = max(worst, _run(r, v, L, s, r_fail=float(rng.choice([-1.0, -5.0, 0.0])), gamma=float(rng.choice([1.0, 0.99])),
                                    lam=float(rng.choice([0.95, 1.0, 0.0])), eps=float(rng.choice([1e-8, 0.0, 0.1])),
                                    shift_mean=bool(rng.random() < 0.7), unbiased=bool(rng.random() < 0.5), oracle_pass=B * T < 4e6,
                                    ordered=bool(rng.random() < 0.5)))
        except AssertionError as err:
            raise AssertionError(f"case {case}: B={B} T={T}: {err}")
    _say(f"  worst whitening error {worst:.2e}")


# --------------------------------------------------------------------------- the terminal-reward form
def _run_terminal(v, L, s, term, zero_padding, want_returns, ordered, gamma=1.0, lam=0.95):
    """espo_advantages_terminal_ws against espo_advantages_terminal (bits, wherever that call defines the result),
    then the whitening from the rows' sums against espo_whiten on the same advantages."""
    B, T = v.shape
    Lc = np.clip(L.cpu().numpy().astype(np.int64), 0, T)
    mask = torch.arange(T, device="cuda")[None, :] < L.clamp(0, T)[:, None]
    outs = []
    ws = _workspace(B)
    for k in range(2):
        td, adv = torch.full_like(v, FILL), torch.full_like(v, FILL)
        ret = torch.full_like(v, FILL) if want_returns else None
        if k == 0:
            espo.espo_advantages_terminal(v, L, s, term, -1.0, gamma, lam, td, adv, returns=ret, zero_padding=zero_padding)
        else:
            order = None
            if ordered:
                order = torch.empty(B, dtype=torch.int32, device="cuda")
                espo.espo_length_order(L, T, order)
            espo.espo_advantages_terminal_ws(v, L, s, term, -1.0, gamma, lam, td, adv, ws, returns=ret,
                                             zero_padding=zero_padding, order=order)
        torch.cuda.synchronize()
        outs.append((td, adv, ret))
    for a, b in zip(outs[0], outs[1]):
        if a is None:
            continue
        assert torch.equal(a[mask].view(torch.int32), b[mask].view(torch.int32))
        if zero_padding:
            assert torch.equal(a, b)
        else:   # beyond the lengths every position is either untouched or zero
            pad = b[~mask]
            assert bool(((pad == FILL) | (pad == 0)).all())
    assert not bool(ws[:HEAD].any())
    n = ws[HEAD:HEAD + 32 * B].view(torch.int64).cpu().numpy().reshape(B, 4)[:, 3]
    assert (n == Lc).all()
    adv = outs[1][1]
    out1, out0 = torch.full_like(v, FILL), torch.full_like(v, FILL)
    espo.espo_whiten_from_ws(adv, L, out1, ws)
    espo.espo_whiten(adv, L, out0, torch.empty(espo.espo_whiten_workspace_bytes(B, T), dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()
    g1, g0 = out1[mask].cpu().numpy(), out0[mask].cpu().numpy()
    ulp = np.spacing(np.abs(g0)).astype(np.float64)
    assert (np.abs(g1.astype(np.float64) - g0.astype(np.float64)) <= ulp + 1e-11).all()
    assert bool((out1[~mask] == FILL).all())


@pytest.mark.parametrize("B,T", [(9, 700), (300, 1023), (513, 64), (1100, 2049)])
def test_terminal_form(B, T):
    _say(f"[case] advantages_terminal_ws B={B} T={T}")
    g = torch.Generator().manual_seed(B + T)
    values = torch.rand(B, T, generator=g) * 2 - 1
    L = torch.randint(0, T + 1, (B,), generator=g)
    values[torch.arange(T)[None, :] >= L[:, None]] = float("nan")
    stopped = (torch.rand(B, generator=g) < 0.4).to(torch.uint8)
    term = torch.rand(B, generator=g)
    v, Lt, s, tr = values.cuda(), L.to(torch.int32).cuda(), stopped.cuda(), term.cuda()
    for zero_padding, want_returns, ordered in ((True, True, False), (False, False, False), (False, True, True), (True, False, True)):
        _run_terminal(v, Lt, s, tr, zero_padding, want_returns, ordered)
    # and against the oracle once per shape (the plain call is what the other tests hold against it)
    H.check_advantages_terminal(v, Lt, s, tr, -1.0, 1.0, 0.95)


def test_terminal_form_config5_full_size():
    _say("[case] advantages_terminal_ws on config 5 (B=1024, T=16384)")
    r, v, L, s = W.advantage_batch(device="cuda", poison=True, seed=5)
    term = torch.rand(r.shape[0], device="cuda")
    _run_terminal(v, L, s, term, False, True, False)
    _run_terminal(v, L, s, term, True, False, False)
