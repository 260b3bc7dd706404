"""Pins of the CPU oracle's decode step against what the paper and mathematics fix.

None of these tests needs a GPU.  They check the oracle against hand values, closed
forms, library routines on special cases and statistical laws, so that a dropped term,
a wrong sign or a shifted index somewhere in it fails at least one of them.
"""
import math
import os

import numpy as np
import pytest
from scipy import special, stats

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _state(B):
    return (np.zeros(B, np.float32), np.ones(B, np.uint8), np.full(B, -1, np.int32))


def _params(oracle, **kw):
    base = dict(mu_g=0.0, var_g=1.0, delta=0.0, clip_c=10.0, alpha_s=0.9, beta=7.0, eps=0.2,
                stop_enabled=1, eos_id=-1)
    base.update(kw)
    return oracle.OracleParams(**base)


def _two_token_logits(g, tau=1.0):
    """A row whose token 1 has regret exactly g (token 0 is the mode)."""
    return np.array([[0.0, -g * tau]], np.float32)


# ------------------------------------------------------------------ regret (Eq. step_gap)
def test_regret_hand_values(oracle):
    rows = [l.split() for l in open(os.path.join(GOLDEN, "regret_three_token.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 12
    for x0, x1, x2, tau, tok, g in rows:
        logits = np.array([[float(x0), float(x1), float(x2)]], np.float32)
        z, alive, ss = _state(1)
        out = oracle.step(logits, float(tau), 1, 0, np.zeros(1, np.float32), _params(oracle),
                          z, alive, ss, forced_tokens=np.array([int(tok)], np.int32))
        assert out["regret"][0] == np.float32(g)
        assert out["tokens"][0] == int(tok)


def test_regret_nonnegative_zero_iff_mode_and_shift_invariant(oracle):
    rng = np.random.default_rng(5)
    B, V = 64, 37
    logits = rng.normal(0, 3, (B, V)).astype(np.float32)
    vals = np.zeros(B, np.float32)
    z, alive, ss = _state(B)
    out = oracle.step(logits, 0.7, 11, 3, vals, _params(oracle, stop_enabled=0), z, alive, ss)
    g, tok = out["regret"], out["tokens"]
    assert (g >= 0).all()                                   # "by construction g_t >= 0"
    mode = logits.argmax(1)
    assert ((g == 0) == (tok == mode)).all()
    assert (tok != mode).any() and (tok == mode).any()
    # definition through log-softmax computed by a library routine
    inv = np.float64(np.float32(1.0) / np.float32(0.7))          # the step divides once in fp32
    lsm = special.log_softmax(logits.astype(np.float64) * inv, axis=1)
    g_def = lsm.max(1) - lsm[np.arange(B), tok]
    np.testing.assert_allclose(g, g_def, rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(out["logprob"], lsm[np.arange(B), tok], rtol=1e-6, atol=1e-6)
    # adding a constant to a row changes neither token nor regret (a 2^-10 grid keeps fp32 exact)
    grid = (np.round(logits * 1024) / 1024).astype(np.float32)
    shifted = (grid + np.float32(4.0)).astype(np.float32)
    assert ((shifted - np.float32(4.0)) == grid).all()
    za, aa, sa = _state(B)
    zb, ab, sb = _state(B)
    oa = oracle.step(grid, 0.7, 11, 3, vals, _params(oracle, stop_enabled=0), za, aa, sa)
    ob = oracle.step(shifted, 0.7, 11, 3, vals, _params(oracle, stop_enabled=0), zb, ab, sb)
    assert (oa["tokens"] == ob["tokens"]).all()
    assert (oa["regret"] == ob["regret"]).all()
    np.testing.assert_allclose(oa["logprob"], ob["logprob"], rtol=1e-6, atol=1e-6)


def test_uniform_logits_logprob_is_minus_log_V(oracle):
    for V in (1, 2, 5, 1000):
        logits = np.full((3, V), 1.25, np.float32)
        z, alive, ss = _state(3)
        out = oracle.step(logits, 1.3, 2, 0, np.zeros(3, np.float32), _params(oracle), z, alive, ss)
        np.testing.assert_allclose(out["logprob"], -math.log(V), rtol=1e-6, atol=1e-7)
        assert (out["regret"] == 0).all()
        np.testing.assert_allclose(out["sum_exp"], V, rtol=1e-12)


def test_temperature_scales_regret_and_softmax(oracle):
    rng = np.random.default_rng(9)
    logits = rng.normal(0, 2, (8, 50)).astype(np.float32)
    for tau in (0.25, 0.6, 1.0, 2.0):
        z, alive, ss = _state(8)
        forced = np.arange(8, dtype=np.int32)
        out = oracle.step(logits, tau, 0, 0, np.zeros(8, np.float32), _params(oracle), z, alive, ss,
                          forced_tokens=forced)
        inv = np.float64(np.float32(1.0) / np.float32(tau))
        lsm = special.log_softmax(logits.astype(np.float64) * inv, axis=1)
        np.testing.assert_allclose(out["logprob"], lsm[np.arange(8), forced], rtol=2e-6, atol=2e-6)
        np.testing.assert_allclose(out["regret"], (logits.max(1) - logits[np.arange(8), forced]) * inv,
                                   rtol=2e-7)


def test_masked_vocabulary_minus_inf(oracle):
    rng = np.random.default_rng(2)
    B, V = 32, 64
    logits = rng.normal(0, 1, (B, V)).astype(np.float32)
    logits[:, ::3] = -np.inf
    z, alive, ss = _state(B)
    out = oracle.step(logits, 1.0, 4, 1, np.zeros(B, np.float32), _params(oracle), z, alive, ss)
    assert (out["tokens"] % 3 != 0).all()
    assert np.isfinite(out["logprob"]).all() and np.isfinite(out["regret"]).all()
    lsm = special.log_softmax(logits.astype(np.float64), axis=1)
    np.testing.assert_allclose(out["logprob"], lsm[np.arange(B), out["tokens"]], rtol=1e-6, atol=1e-6)


def test_bf16_rows_equal_their_fp32_upcast(oracle):
    rng = np.random.default_rng(3)
    x = rng.normal(0, 3, (16, 300)).astype(np.float32)
    bits = (x.view(np.uint32) >> 16).astype(np.uint16)           # truncate to bf16 bit patterns
    up = (bits.astype(np.uint32) << 16).view(np.float32)
    p = _params(oracle)
    za, aa, sa = _state(16)
    zb, ab, sb = _state(16)
    vals = np.full(16, 0.5, np.float32)
    oa = oracle.step(bits, 0.6, 7, 2, vals, p, za, aa, sa)
    ob = oracle.step(np.ascontiguousarray(up), 0.6, 7, 2, vals, p, zb, ab, sb)
    for k in ("tokens", "regret", "logprob", "best_score"):
        assert (oa[k] == ob[k]).all()
    assert (za == zb).all()


def test_row_stride_and_batch_independence(oracle):
    rng = np.random.default_rng(4)
    B, V, stride = 6, 40, 48
    buf = rng.normal(0, 2, (B, stride)).astype(np.float32)
    p = _params(oracle)
    vals = np.zeros(B, np.float32)
    z, a, s = _state(B)
    o1 = oracle.step(buf, 1.0, 5, 9, vals, p, z, a, s, V=V)
    z2, a2, s2 = _state(B)
    o2 = oracle.step(np.ascontiguousarray(buf[:, :V]), 1.0, 5, 9, vals, p, z2, a2, s2)
    assert (o1["tokens"] == o2["tokens"]).all() and (o1["regret"] == o2["regret"]).all()
    # a row's result depends on its row id, not on how many rows are in the batch
    z3, a3, s3 = _state(3)
    o3 = oracle.step(np.ascontiguousarray(buf[:3, :V]), 1.0, 5, 9, vals[:3], p, z3, a3, s3)
    assert (o3["tokens"] == o2["tokens"][:3]).all()


# ------------------------------------------------------------------ sampler (a_t ~ pi)
def test_gumbel_max_matches_softmax_frequencies(oracle):
    """Empirical token frequencies over many (row, step) streams follow softmax(x/tau)."""
    x = np.array([1.5, 0.0, -1.0, 2.0, 0.5, -3.0, 1.0, 0.25], np.float32)
    B, steps, tau = 2048, 48, 0.8
    logits = np.tile(x, (B, 1))
    counts = np.zeros(8, np.int64)
    p = _params(oracle, stop_enabled=0)
    vals = np.zeros(B, np.float32)
    for t in range(steps):
        z, alive, ss = _state(B)
        out = oracle.step(logits, tau, 1234, t, vals, p, z, alive, ss)
        counts += np.bincount(out["tokens"], minlength=8)
    n = B * steps
    probs = special.softmax(x.astype(np.float64) / tau)
    chi2 = ((counts - n * probs) ** 2 / (n * probs)).sum()
    assert chi2 < stats.chi2.ppf(1 - 1e-4, df=7), (chi2, counts / n, probs)
    # the rarest token (p ~ 0.3 %) is hit at a rate within 5 sigma of its probability
    k = int(np.argmin(probs))
    assert abs(counts[k] - n * probs[k]) < 5 * math.sqrt(n * probs[k])


def test_sampler_seed_row_step_all_matter(oracle):
    x = np.zeros((256, 16), np.float32)                          # uniform: pure RNG
    p = _params(oracle, stop_enabled=0)
    vals = np.zeros(256, np.float32)

    def draw(seed, step):
        z, a, s = _state(256)
        return oracle.step(x, 1.0, seed, step, vals, p, z, a, s)["tokens"]

    base = draw(1, 0)
    assert (base == draw(1, 0)).all()                            # deterministic
    assert (base != draw(2, 0)).mean() > 0.8                     # seed (low word)
    assert (base != draw(1 + (1 << 32), 0)).mean() > 0.8         # seed (high word)
    assert (base != draw(1, 1)).mean() > 0.8                     # step
    assert len(set(base.tolist())) > 8                           # rows differ
    cnt = np.bincount(base, minlength=16)
    assert stats.chisquare(cnt).pvalue > 1e-4


def test_low_temperature_is_greedy(oracle):
    rng = np.random.default_rng(8)
    logits = rng.normal(0, 1, (32, 100)).astype(np.float32)
    z, a, s = _state(32)
    out = oracle.step(logits, 1e-3, 3, 0, np.zeros(32, np.float32), _params(oracle), z, a, s)
    # gaps between the top two logits exceed 20 * tau in all but a negligible fraction of rows
    srt = np.sort(logits, 1)
    clear = (srt[:, -1] - srt[:, -2]) > 0.03
    assert clear.sum() > 20
    assert (out["tokens"][clear] == logits.argmax(1)[clear]).all()
    assert (out["regret"][clear] == 0).all()


def test_ties_break_to_lowest_index_and_runner_up(oracle):
    # two identical dominant logits: their scores differ only through the stream;
    # best/second diagnostics are ordered and the runner-up differs from the token
    logits = np.full((64, 12), -50.0, np.float32)
    logits[:, 3] = 5.0
    logits[:, 7] = 5.0
    z, a, s = _state(64)
    out = oracle.step(logits, 1.0, 99, 0, np.zeros(64, np.float32), _params(oracle), z, a, s)
    assert set(out["tokens"].tolist()) == {3, 7}
    assert (out["best_score"] >= out["second_score"]).all()
    assert (out["second_token"] != out["tokens"]).all()
    assert set(out["second_token"].tolist()) <= {3, 7}
    # recompute the two scores from the stream definition: y + G
    for b in range(64):
        s3 = 5.0 + oracle.gumbel_at(99, b, 0, 3, 12)
        s7 = 5.0 + oracle.gumbel_at(99, b, 0, 7, 12)
        assert out["tokens"][b] == (3 if s3 >= s7 else 7)
        assert out["best_score"][b] == max(s3, s7) and out["second_score"][b] == min(s3, s7)


# ------------------------------------------------------------------ random stream
def _philox_py(ctr, key):
    """Philox4x32-10 restated in Python integers (guards the C arithmetic, e.g. overflow)."""
    c = list(ctr)
    k = list(key)
    for _ in range(10):
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & 0xFFFFFFFF, p1 & 0xFFFFFFFF,
             ((p0 >> 32) ^ c[3] ^ k[1]) & 0xFFFFFFFF, p0 & 0xFFFFFFFF]
        k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
    return c


def test_philox_weyl_constants_are_the_published_irrationals():
    # key schedule increments: golden ratio and sqrt(3) - 1 scaled to 32 bits
    assert int((math.sqrt(5) - 1) / 2 * 2 ** 32) == 0x9E3779B9
    assert int((math.sqrt(3) - 1) * 2 ** 32) == 0xBB67AE85


def test_philox_known_answers(oracle):
    # the identity of the oracle's generator with the published Philox4x32-10: its authors' known-answer inputs
    # (zeros, ones, digits of pi); a wrong multiplier, Weyl constant, round count or word order fails all three
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_known_answers.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        got = oracle.philox4x32_10(np.array(w[:4], np.uint32), np.array(w[4:6], np.uint32)).tolist()
        assert got == w[6:], ([hex(x) for x in got], r)
        assert _philox_py(w[:4], w[4:6]) == w[6:]


def test_philox_c_matches_integer_restatement(oracle):
    rng = np.random.default_rng(0)
    for _ in range(200):
        ctr = rng.integers(0, 2 ** 32, 4, dtype=np.uint64).astype(np.uint32)
        key = rng.integers(0, 2 ** 32, 2, dtype=np.uint64).astype(np.uint32)
        assert oracle.philox4x32_10(ctr, key).tolist() == _philox_py([int(x) for x in ctr], [int(x) for x in key])
    edge = np.array([0xFFFFFFFF] * 4, np.uint32)
    assert oracle.philox4x32_10(edge, edge[:2]).tolist() == _philox_py([0xFFFFFFFF] * 4, [0xFFFFFFFF] * 2)


def test_philox_avalanche_and_bijection(oracle):
    """Flipping any single input bit flips about half of the 128 output bits; distinct
    counters under one key give distinct blocks (the round function is a permutation)."""
    rng = np.random.default_rng(1)
    flips = []
    for _ in range(40):
        ctr = rng.integers(0, 2 ** 32, 4, dtype=np.uint64).astype(np.uint32)
        key = rng.integers(0, 2 ** 32, 2, dtype=np.uint64).astype(np.uint32)
        ref = oracle.philox4x32_10(ctr, key)
        for word in range(6):
            bit = int(rng.integers(0, 32))
            c2, k2 = ctr.copy(), key.copy()
            if word < 4:
                c2[word] ^= np.uint32(1 << bit)
            else:
                k2[word - 4] ^= np.uint32(1 << bit)
            diff = oracle.philox4x32_10(c2, k2) ^ ref
            flips.append(sum(bin(int(d)).count("1") for d in diff))
    flips = np.array(flips)
    assert 60 < flips.mean() < 68 and flips.min() > 35 and flips.max() < 93
    key = np.array([7, 9], np.uint32)
    seen = set()
    for i in range(4096):
        seen.add(tuple(oracle.philox4x32_10(np.array([i, 0, 0, 0], np.uint32), key).tolist()))
    assert len(seen) == 4096


def test_stream_word_layout(oracle):
    """word(v) is lane v & 3 of the Philox block whose counter is (v >> 2, step, row, tag)."""
    seed = (0xABCDEF01 << 32) | 0x12345678
    for v in (0, 1, 2, 3, 4, 5, 152063, 2 ** 31 - 9):
        for row, step in ((0, 0), (5, 17), (511, 1023)):
            blk = _philox_py([v >> 2, step, row, 0x6573706F], [0x12345678, 0xABCDEF01])
            assert oracle.stream_word(seed, row, step, v) == blk[v & 3]


def test_uniform_and_gumbel_ranges(oracle):
    assert oracle.uniform(0) == 2.0 ** -24
    assert oracle.uniform(0xFFFFFFFF) == 1.0 - 2.0 ** -24
    assert oracle.uniform(0x1FF) == 2.0 ** -24                  # low 9 bits are unused
    assert oracle.uniform(0x200) == 3 * 2.0 ** -24
    assert oracle.uniform(0x80000000) == 0.5 + 2.0 ** -24
    g_lo, g_hi = oracle.gumbel(0), oracle.gumbel(0xFFFFFFFF)
    assert abs(g_lo - (-math.log(24 * math.log(2)))) < 1e-12     # -ln(-ln 2^-24)
    assert abs(g_hi - (-math.log(-math.log1p(-2.0 ** -24)))) < 1e-9
    assert -2.8116 < g_lo < -2.8114 and 16.635 < g_hi < 16.636


def test_stream_moments(oracle):
    """u is uniform on (0,1) and G = -ln(-ln u) has mean Euler-gamma and variance pi^2/6."""
    n = 200_000
    words = np.array([oracle.stream_word(42, v % 7, v % 3, v) for v in range(n)], dtype=np.uint64)
    u = ((2 * (words >> 9) + 1) / 2.0 ** 24)
    assert abs(u.mean() - 0.5) < 5 * math.sqrt(1 / 12 / n)
    assert abs(u.var() - 1 / 12) < 5 * math.sqrt(1 / 180 / n)
    cnt = np.bincount((words >> 24).astype(np.int64), minlength=256)
    assert stats.chisquare(cnt).pvalue > 1e-4
    low = np.bincount(((words >> 9) & 0xFF).astype(np.int64), minlength=256)
    assert stats.chisquare(low).pvalue > 1e-4
    G = -np.log(-np.log(u))
    assert abs(G.mean() - 0.5772156649015329) < 5 * math.sqrt((math.pi ** 2 / 6) / n)
    assert abs(G.var() - math.pi ** 2 / 6) < 0.03
    lag = np.corrcoef(u[:-1], u[1:])[0, 1]
    assert abs(lag) < 5 / math.sqrt(n)


def test_block_draw_layout_and_law(oracle):
    """M_q and pos_q come from one word of a Philox call shared by four blocks (own call if ragged)."""
    seed = (0x0BADF00D << 32) | 0x00C0FFEE
    for q, n, row, step in ((0, 64, 0, 0), (2375, 64, 511, 1023), (6, 64, 1, 1), (3, 12, 7, 5), (1, 1, 2, 2)):
        w = _philox_py([q >> 2, step, row, 0x4553504F], [0x00C0FFEE, 0x0BADF00D])[q & 3]
        u = (2 * (w >> 9) + 1) / 2.0 ** 24
        M, pos = oracle.block_draw(seed, row, step, q, n)
        assert abs(M - (math.log(n) - math.log(-math.log(u)))) < 1e-12
        if n == 64:
            assert pos == (w >> 3) & 63
        else:
            w2 = _philox_py([q, step, row, 0x52414747], [0x00C0FFEE, 0x0BADF00D])[0]
            assert pos == (w2 * n) >> 32 and 0 <= pos < n
    # M - ln n is standard Gumbel, pos is uniform, and the two are independent
    n = 64
    draws = [oracle.block_draw(77, r, s, q, n) for r in range(20) for s in range(20) for q in range(50)]
    M = np.array([d[0] for d in draws]) - math.log(n)
    pos = np.array([d[1] for d in draws])
    assert stats.kstest(M, lambda g: np.exp(-np.exp(-g))).pvalue > 1e-4
    assert stats.chisquare(np.bincount(pos // 4, minlength=16)).pvalue > 1e-4
    assert abs(np.corrcoef(M, pos)[0, 1]) < 5 / math.sqrt(len(M))


def test_blockwise_variates_are_iid_standard_gumbel(oracle):
    """The top-down construction (block maximum, its position, truncated rest) must have
    the joint law of iid standard Gumbels: checked on the marginal cdf, on the block
    maximum, on the second largest value and on independence across neighbours."""
    V = 1100                                                      # 17 blocks of 64 and one of 12
    rows = 160
    G = np.array([[oracle.gumbel_at(5, r, 3, v, V) for v in range(V)] for r in range(rows)])
    cdf = lambda g: np.exp(-np.exp(-g))
    assert stats.kstest(G.ravel(), cdf).pvalue > 1e-4             # marginal law
    assert abs(G.mean() - 0.5772156649015329) < 5 * math.sqrt((math.pi ** 2 / 6) / G.size)
    assert abs(G.var() - math.pi ** 2 / 6) < 0.03
    for lo, hi in ((0, 64), (64, 128), (1024, 1088), (1088, 1100)):
        blk = G[:, lo:hi]
        n = hi - lo
        for r in range(rows):
            M, pos = oracle.block_draw(5, r, 3, lo // 64, n)
            assert blk[r].argmax() == pos and blk[r, pos] == M    # the drawn maximum is the maximum
            assert (np.delete(blk[r], pos) < M).all()
        # maximum of n iid Gumbels ~ Gumbel(ln n); second largest has cdf F^n + n F^(n-1) (1 - F)
        assert stats.kstest(blk.max(1) - math.log(n), cdf).pvalue > 1e-4
        second = np.sort(blk, 1)[:, -2] if n > 1 else None
        F2 = lambda g: cdf(g) ** n + n * cdf(g) ** (n - 1) * (1 - cdf(g))
        assert stats.kstest(second, F2).pvalue > 1e-4
    # the argmax over the whole row is uniform over indices (no block is favoured)
    big = np.array([[oracle.gumbel_at(6, r, 0, v, V) for v in range(V)] for r in range(600)])
    which = np.digitize(big.argmax(1), [512, 1088])
    exp = 600 * np.array([512, 576, 12]) / V
    assert stats.chisquare(np.bincount(which, minlength=3), exp).pvalue > 1e-4
    assert abs(np.corrcoef(G[:, :-1].ravel(), G[:, 1:].ravel())[0, 1]) < 5 / math.sqrt(G.size)


def test_sampler_frequencies_across_blocks(oracle):
    """Softmax frequencies on a vocabulary that spans 18 blocks (one ragged): heavy tokens
    in several blocks plus a flat background, so block maxima, positions and truncated variates
    all take part in the argmax."""
    V, tau = 1100, 0.9
    x = np.full(V, -2.0, np.float32)
    heavy = {5: 3.0, 63: 2.0, 64: 2.5, 300: 1.5, 512: 1.5, 900: 3.5, 1087: 1.0, 1088: 2.0, 1099: 3.0}
    for k, val in heavy.items():
        x[k] = val
    B, steps = 1024, 40
    logits = np.tile(x, (B, 1))
    p = _params(oracle, stop_enabled=0)
    vals = np.zeros(B, np.float32)
    keys = sorted(heavy)
    counts = np.zeros(len(keys) + 3, np.int64)
    for t in range(steps):
        z, alive, ss = _state(B)
        tok = oracle.step(logits, tau, 4321, t, vals, p, z, alive, ss)["tokens"]
        for i, k in enumerate(keys):
            counts[i] += (tok == k).sum()
        bg = ~np.isin(tok, keys)
        counts[len(keys):] += np.bincount(np.digitize(tok[bg], [512, 1024]), minlength=3)
    probs = special.softmax(x.astype(np.float64) * np.float64(np.float32(1.0) / np.float32(tau)))
    bgmask = np.ones(V, bool)
    bgmask[keys] = False
    blk = np.digitize(np.arange(V), [512, 1024])
    exp = np.array([probs[k] for k in keys] + [probs[bgmask & (blk == j)].sum() for j in range(3)])
    n = B * steps
    assert counts.sum() == n and abs(exp.sum() - 1) < 1e-12
    chi2 = ((counts - n * exp) ** 2 / (n * exp)).sum()
    assert chi2 < stats.chi2.ppf(1 - 1e-4, df=len(exp) - 1), (chi2, counts / n, exp)


# ------------------------------------------------------------------ normalise, smooth (Eq. normalized_gap, smoothed_score)
def _run_forced(oracle, g_seq, p, values=None, tau=1.0):
    """Feed a prescribed regret sequence through the step (token 1 of a 2-token row)."""
    z, alive, ss = _state(1)
    zs, al = [], []
    for t, g in enumerate(g_seq):
        v = np.array([0.5 if values is None else values[t]], np.float32)
        out = oracle.step(_two_token_logits(g, tau), tau, 0, t, v, p, z, alive, ss,
                          forced_tokens=np.array([1], np.int32))
        assert out is not None
        zs.append(float(z[0]))
        al.append(int(alive[0]))
    return np.array(zs), np.array(al), int(ss[0])


def test_constant_signal_closed_form(oracle):
    # g~ = (g - mu)/sqrt(var + delta) = (3 - 1)/2 = 1; z_n = 1 - alpha^n  (z_0 = 0)
    p = _params(oracle, mu_g=1.0, var_g=3.0, delta=1.0, alpha_s=0.9, stop_enabled=0)
    zs, _, _ = _run_forced(oracle, [3.0] * 60, p)
    n = np.arange(1, 61)
    np.testing.assert_allclose(zs, 1 - 0.9 ** n, rtol=3e-6)
    # first step already applies the update (Algorithm 1 starts at t = 0 with z = 0)
    assert abs(zs[0] - 0.1) < 1e-7


def test_general_sequence_closed_form_and_alpha_extremes(oracle):
    rng = np.random.default_rng(12)
    g = rng.uniform(0, 6, 40)
    p = _params(oracle, mu_g=2.0, var_g=4.0, delta=0.0, alpha_s=0.75, stop_enabled=0)
    zs, _, _ = _run_forced(oracle, g, p)
    gt = (g.astype(np.float32).astype(np.float64) - 2.0) / 2.0
    for n in range(1, 41):
        ref = 0.25 * sum(0.75 ** (n - k) * gt[k - 1] for k in range(1, n + 1))
        assert abs(zs[n - 1] - ref) < 5e-6
    z1, _, _ = _run_forced(oracle, g, _params(oracle, mu_g=2.0, var_g=4.0, alpha_s=0.0, stop_enabled=0))
    np.testing.assert_allclose(z1, gt, rtol=1e-6, atol=1e-7)      # alpha = 0: z = g~
    z2, _, _ = _run_forced(oracle, g, _params(oracle, mu_g=2.0, var_g=4.0, alpha_s=1.0, stop_enabled=0))
    assert (z2 == 0).all()                                        # alpha = 1: z stays at z_0 = 0


def test_signal_equal_to_mean_keeps_state_zero_and_clip_saturates(oracle):
    p = _params(oracle, mu_g=1.5, var_g=0.25, stop_enabled=0)
    zs, _, _ = _run_forced(oracle, [1.5] * 20, p)
    assert (zs == 0).all()
    # (g - mu)/sd = (100 - 0)/1 = 100 -> clipped to c = 2.5; z_n = 2.5 (1 - 0.9^n)
    p = _params(oracle, clip_c=2.5, stop_enabled=0)
    zs, _, _ = _run_forced(oracle, [100.0] * 30, p)
    np.testing.assert_allclose(zs, 2.5 * (1 - 0.9 ** np.arange(1, 31)), rtol=3e-6)
    # lower clip: g = 0, mu = 50 -> -50 -> clipped to -2.5
    p = _params(oracle, mu_g=50.0, clip_c=2.5, stop_enabled=0)
    zs, _, _ = _run_forced(oracle, [0.0] * 30, p)
    np.testing.assert_allclose(zs, -2.5 * (1 - 0.9 ** np.arange(1, 31)), rtol=3e-6)
    # variance and stabiliser enter as sqrt(var + delta)
    p = _params(oracle, var_g=5.0, delta=4.0, alpha_s=0.0, stop_enabled=0)
    zs, _, _ = _run_forced(oracle, [6.0], p)
    assert abs(zs[0] - 2.0) < 1e-6


# ------------------------------------------------------------------ stop rule (Eq. stop_rule, Eq. failure_reward)
def test_stop_never_fires_with_zero_regret(oracle):
    rng = np.random.default_rng(1)
    for mu in (0.0, 0.7):
        for beta in (0.0, 0.5, 7.0):
            p = _params(oracle, mu_g=mu, beta=beta)
            vals = rng.uniform(-1, 1, 300)
            zs, al, ss = _run_forced(oracle, [0.0] * 300, p, values=vals)
            assert al.all() and ss == -1 and (zs <= 0).all()


def test_stop_never_fires_during_warmup(oracle):
    p = _params(oracle, stop_enabled=0)
    zs, al, ss = _run_forced(oracle, [50.0] * 100, p, values=[-1.0] * 100)
    assert al.all() and ss == -1
    assert zs[-1] > 9.9                                           # the state is still updated


def test_stop_fires_at_closed_form_step_under_constant_drift(oracle):
    # g~ = kappa constant, z_0 = 0: z_n = kappa (1 - alpha^n) first exceeds theta at
    # n* = floor(ln(1 - theta/kappa)/ln(alpha)) + 1  (smallest n with alpha^n < 1 - theta/kappa)
    for kappa, value, beta in ((4.0, 0.3, 7.0), (2.0, 0.05, 7.0), (9.0, 1.0, 7.0), (1.0, 0.5, 1.0)):
        theta = beta * max(value, 0.2)
        n_star = math.floor(math.log(1 - theta / kappa) / math.log(0.9)) + 1
        p = _params(oracle, beta=beta)
        zs, al, ss = _run_forced(oracle, [kappa] * (n_star + 20), p, values=[value] * (n_star + 20))
        assert ss == n_star - 1, (kappa, value, ss, n_star)       # steps are 0-based
        assert al[: n_star - 1].all() and not al[n_star - 1:].any()
        assert zs[n_star - 1] > theta >= zs[n_star - 2]
        assert (zs[n_star - 1:] == zs[n_star - 1]).all()          # absorbing: state frozen


def test_stop_always_fires_under_monotone_drift(oracle):
    # g~_t nondecreasing and eventually >= kappa > theta: fires no later than n* steps after
    # the drift reaches kappa
    theta = 7.0 * 0.2
    kappa = 3.0
    t0 = 25
    g = np.concatenate([np.linspace(0, kappa, t0), kappa + 0.05 * np.arange(60)])
    p = _params(oracle)
    zs, al, ss = _run_forced(oracle, g, p, values=[0.0] * len(g))
    n_star = math.floor(math.log(1 - theta / kappa) / math.log(0.9)) + 1
    assert 0 <= ss <= t0 + n_star
    assert (np.diff(al) <= 0).all()                               # never revived


def test_stop_rule_is_strict_and_floors_the_value(oracle):
    # alpha = 0 makes z = g~ = g (mu 0, var 1, delta 0); beta = 1: stop iff g > max(value, eps)
    p = _params(oracle, alpha_s=0.0, beta=1.0, eps=0.2)
    for g, value, expect in ((0.75, 0.75, False), (0.75, 0.7499999, True), (0.75, 0.8, False),
                             (0.25, -5.0, True), (0.2, -5.0, False), (0.15, -5.0, False),
                             (0.25, 0.1, True)):
        g32 = float(np.float32(g))
        zs, al, ss = _run_forced(oracle, [g32], p, values=[value])
        assert (ss == 0) == expect, (g, value)
        assert bool(al[0]) == (not expect)


def test_stopped_rows_are_skipped_and_written_once(oracle):
    B, V = 4, 16
    rng = np.random.default_rng(3)
    logits = rng.normal(0, 1, (B, V)).astype(np.float32)
    z = np.array([0.3, -0.2, 5.0, 0.1], np.float32)
    alive = np.array([1, 0, 1, 1], np.uint8)
    ss = np.array([-1, 4, -1, -1], np.int32)
    vals = np.array([1.0, 1.0, 0.0, 1.0], np.float32)
    p = _params(oracle)
    out = oracle.step(logits, 1.0, 0, 9, vals, p, z, alive, ss)
    assert out["tokens"][1] == -1 and out["regret"][1] == 0 and out["logprob"][1] == 0
    assert z[1] == np.float32(-0.2) and ss[1] == 4 and alive[1] == 0   # untouched
    assert alive[2] == 0 and ss[2] == 9                                 # z = 4.5+ > 1.4
    assert alive[0] == 1 and alive[3] == 1 and ss[0] == -1
    z_before = z.copy()
    out = oracle.step(logits, 1.0, 0, 10, vals, p, z, alive, ss)
    assert ss[2] == 9 and z[2] == z_before[2] and out["tokens"][2] == -1


def test_eos_ends_row_without_failure(oracle):
    logits = np.full((2, 8), -30.0, np.float32)
    logits[:, 5] = 10.0                                           # token 5 is certain
    z = np.array([9.0, 9.0], np.float32)                          # would trip the stop rule
    alive = np.ones(2, np.uint8)
    ss = np.full(2, -1, np.int32)
    p = _params(oracle, eos_id=5)
    out = oracle.step(logits, 1.0, 0, 3, np.zeros(2, np.float32), p, z, alive, ss)
    assert (out["tokens"] == 5).all() and (alive == 0).all() and (ss == -1).all()
    p = _params(oracle, eos_id=6)
    alive[:] = 1
    z[:] = 9.0
    oracle.step(logits, 1.0, 0, 3, np.zeros(2, np.float32), p, z, alive, ss)
    assert (alive == 0).all() and (ss == 3).all()


def test_state_update_replays_step(oracle):
    rng = np.random.default_rng(21)
    B, V = 24, 33
    p = _params(oracle, mu_g=1.0, var_g=2.0, beta=1.0)
    z, alive, ss = _state(B)
    z2, alive2, ss2 = _state(B)
    for t in range(40):
        logits = rng.normal(0, 3, (B, V)).astype(np.float32)
        vals = rng.uniform(-0.5, 1, B).astype(np.float32)
        alive_before = alive.copy()
        out = oracle.step(logits, 0.6, 3, t, vals, p, z, alive, ss)
        oracle.state_update(out["regret"], out["tokens"], vals, p, t, z2, alive2, ss2)
        assert (z == z2).all() and (alive == alive2).all() and (ss == ss2).all()
        assert (out["tokens"][alive_before == 0] == -1).all()
    assert 0 < alive.sum() < B                                    # some rows stopped, some did not


def test_invalid_arguments_are_rejected(oracle):
    logits = np.zeros((1, 4), np.float32)
    z, a, s = _state(1)
    for tau in (0.0, -1.0, float("inf"), float("nan")):
        with pytest.raises(ValueError):
            oracle.step(logits, tau, 0, 0, np.zeros(1, np.float32), _params(oracle), z, a, s)
    with pytest.raises(ValueError):
        oracle.step(logits, 1.0, 0, 0, np.zeros(1, np.float32), _params(oracle), z, a, s, V=5)


# --------------------------------------------------------------------------- stop modes of the ablations, simulate mode
def _one_step(oracle, p, z0, value, seed=0, step=0, B=1):
    """One oracle step on a row whose single dominant token makes the regret 0."""
    x = np.full((B, 8), -40.0, np.float32)
    x[:, 3] = 10.0
    z = np.full(B, z0, np.float32)
    alive = np.ones(B, np.uint8)
    ss = np.full(B, -1, np.int32)
    out = oracle.step(x, 1.0, seed, step, np.full(B, value, np.float32), p, z, alive, ss)
    return out, z, alive, ss


def test_value_only_and_regret_only_stop_modes(oracle):
    # Section 6: variant D stops when V < threshold whatever the regret, variant E when z > threshold
    # whatever the value.  With g = 0 and mu_g = 0 the state just decays: z' = 0.9 z.
    base = dict(mu_g=0.0, var_g=1.0, alpha_s=0.9, beta=7.0, eps=0.2)
    d = oracle.OracleParams(stop_mode=1, stop_threshold=0.3, **base)
    for value, want in ((0.29, 0), (0.3, 1), (0.31, 1), (-5.0, 0)):
        _, z, alive, ss = _one_step(oracle, d, 100.0, value)       # a huge z does not matter
        assert alive[0] == want and (ss[0] == 0) == (want == 0), value
    e = oracle.OracleParams(stop_mode=2, stop_threshold=0.9, **base)
    for z0, want in ((1.0, 1), (1.01, 0), (0.5, 1)):        # z' = 0.9 z0 against 0.9, strict
        _, z, alive, ss = _one_step(oracle, e, z0, -100.0)          # a hopeless value does not matter
        assert alive[0] == want, z0
    # the gate still applies
    _, _, alive, _ = _one_step(oracle, oracle.OracleParams(stop_mode=1, stop_threshold=0.3, stop_enabled=0, **base), 0.0, 0.0)
    assert alive[0] == 1


def test_random_stop_mode_rate_and_independence(oracle):
    # variant F: a coin per (row, step) with the given probability, keyed like the rest of the stream
    base = dict(mu_g=0.0, var_g=1.0)
    B, steps, prob = 4000, 3, 0.2
    p = oracle.OracleParams(stop_mode=3, stop_threshold=prob, **base)
    stops = []
    for t in range(steps):
        _, _, alive, ss = _one_step(oracle, p, 0.0, 0.5, seed=5, step=t, B=B)
        stops.append(alive == 0)
        assert (ss[alive == 0] == t).all() and (ss[alive == 1] == -1).all()
    rate = np.mean(stops)
    assert abs(rate - prob) < 4 * np.sqrt(prob * (1 - prob) / (B * steps))
    assert 0.1 < np.mean(stops[0] ^ stops[1]) < 0.5          # different steps, different coins
    _, _, again, _ = _one_step(oracle, p, 0.0, 0.5, seed=5, step=0, B=B)
    assert ((again == 0) == stops[0]).all()                   # same key, same coins
    _, _, other, _ = _one_step(oracle, p, 0.0, 0.5, seed=6, step=0, B=B)
    assert ((other == 0) != stops[0]).any()
    for prob_edge, want in ((0.0, 1), (1.0, 0)):              # never / always
        _, _, alive, _ = _one_step(oracle, oracle.OracleParams(stop_mode=3, stop_threshold=prob_edge, **base), 0.0, 0.5, B=64)
        assert (alive == want).all()


def test_simulate_mode_records_the_first_stop_and_keeps_decoding(oracle):
    # Section 7 ("ESPO/Original"): the first position that satisfies the rule is recorded, the
    # sequence is not truncated.  Regret-only rule on a decaying state: z = 2, 1.8, 1.62, ...
    p = oracle.OracleParams(mu_g=0.0, var_g=1.0, alpha_s=0.9, stop_mode=2, stop_threshold=1.5, simulate=1)
    x = np.full((1, 8), -40.0, np.float32); x[:, 3] = 10.0
    z = np.array([2.0 / 0.9], np.float32); alive = np.ones(1, np.uint8); ss = np.full(1, -1, np.int32)
    for t in range(5):
        out = oracle.step(x, 1.0, 0, t + 4, np.zeros(1, np.float32), p, z, alive, ss)
        assert alive[0] == 1 and out["tokens"][0] == 3       # still decoding
        assert ss[0] == 4                                     # the first step that fired, not the later ones
    assert z[0] == pytest.approx(2.0 * 0.9 ** 4, rel=1e-6)
    # end of sequence still ends the row
    p2 = oracle.OracleParams(mu_g=0.0, var_g=1.0, stop_mode=2, stop_threshold=-1.0, simulate=1, eos_id=3)
    alive = np.ones(1, np.uint8); ss = np.full(1, -1, np.int32)
    oracle.step(x, 1.0, 0, 0, np.zeros(1, np.float32), p2, np.zeros(1, np.float32), alive, ss)
    assert alive[0] == 0 and ss[0] == -1


# ------------------------------------------------------------------ policy entropy (Fig. 2b)
def _entropy(oracle, logits, tau, **kw):
    B = logits.shape[0]
    z, alive, ss = _state(B)
    out = oracle.step(logits, tau, 3, 0, np.zeros(B, np.float32), _params(oracle, stop_enabled=0),
                      z, alive, ss, want_entropy=True, **kw)
    return out["entropy"].astype(np.float64)


def test_entropy_closed_forms(oracle):
    # uniform row: ln V, at any temperature
    for V in (1, 2, 7, 64, 1000):
        H = _entropy(oracle, np.full((1, V), 1.25, np.float32), 0.6)
        assert H[0] == pytest.approx(math.log(V), abs=1e-6)
    # two tokens with logit gap d at temperature tau: binary entropy of sigmoid(d / tau)
    for d, tau in [(0.0, 1.0), (1.0, 1.0), (3.0, 0.5), (0.25, 2.0), (40.0, 1.0)]:
        H = _entropy(oracle, np.array([[d, 0.0]], np.float32), tau)
        p = special.expit(np.float64(np.float32(d)) * np.float64(np.float32(1.0) / np.float32(tau)))
        want = -(p * math.log(p) + (1 - p) * math.log1p(-p)) if p < 1 else 0.0
        assert H[0] == pytest.approx(want, rel=1e-6, abs=1e-7)
    # k equal modes and the rest masked out: ln k, and a single finite entry gives exactly 0
    row = np.full((1, 50), -np.inf, np.float32)
    row[0, [3, 17, 44]] = 2.0
    assert _entropy(oracle, row, 1.0)[0] == pytest.approx(math.log(3), abs=1e-6)
    row[0, [3, 44]] = -np.inf
    assert _entropy(oracle, row, 1.0)[0] == 0.0


def test_entropy_matches_library_and_identities(oracle):
    rng = np.random.default_rng(12)
    B, V, tau = 16, 301, 0.6
    logits = (rng.normal(0, 3, (B, V)) + 6.0 * (rng.random((B, V)) < 0.01)).astype(np.float32)
    H = _entropy(oracle, logits, tau)
    inv = np.float64(np.float32(1.0) / np.float32(tau))
    y = logits.astype(np.float64) * inv
    want = stats.entropy(special.softmax(y, axis=1), axis=1)            # library routine, nats
    np.testing.assert_allclose(H, want, rtol=2e-6)
    # H = -E_pi[ln pi]: the same number from the log-softmax the regret test uses
    lsm = special.log_softmax(y, axis=1)
    np.testing.assert_allclose(H, -(np.exp(lsm) * lsm).sum(1), rtol=2e-6)
    # bounds, invariance under a shift of the row, and monotone growth with the temperature
    assert (H > 0).all() and (H < math.log(V)).all()
    np.testing.assert_allclose(_entropy(oracle, logits + np.float32(8.0), tau), H, rtol=1e-5)
    assert (_entropy(oracle, logits, 1.5) > H).all()
    # rows that are done report 0 and padding beyond V is not read
    z, alive, ss = _state(B)
    alive[::2] = 0
    padded = np.concatenate([logits, np.full((B, 11), 50.0, np.float32)], axis=1)
    out = oracle.step(padded, tau, 3, 0, np.zeros(B, np.float32), _params(oracle, stop_enabled=0),
                      z, alive, ss, V=V, want_entropy=True)
    assert (out["entropy"][::2] == 0).all()
    np.testing.assert_allclose(out["entropy"][1::2], H[1::2], rtol=1e-6)


# ------------------------------------------------------------------ filtered sampling (top-p, top-k)
def _filtered(oracle, logits, tau, seed=5, step=0, **kw):
    B = logits.shape[0]
    z, alive, ss = _state(B)
    return oracle.step(logits, tau, seed, step, np.zeros(B, np.float32), _params(oracle, stop_enabled=0, **kw), z, alive, ss)


def _kept_by_definition(y, p=None, k=None):
    """v is kept iff the mass (count) of strictly larger logits is below p (k): O(V^2), no sort."""
    pi = special.softmax(y)
    keep = np.zeros(len(y), bool)
    for v in range(len(y)):
        above = y > y[v]
        keep[v] = (pi[above].sum() < p) if p is not None else (above.sum() < k)
    return keep


def test_kept_set_matches_its_definition_and_a_sorted_cumsum(oracle):
    rng = np.random.default_rng(41)
    for trial in range(30):
        V = int(rng.integers(2, 90))
        tau = float(rng.choice([0.6, 1.0, 2.0]))
        x = rng.normal(0, 2.5, (1, V)).astype(np.float32)
        if trial % 3 == 0:
            x = np.round(x * 2) / 2                           # many exact ties
        y = x[0].astype(np.float64) * np.float64(np.float32(1.0) / np.float32(tau))
        for p in (0.05, 0.5, 0.7, 0.95):
            out = _filtered(oracle, x, tau, top_p=p)
            keep = _kept_by_definition(y, p=np.float64(np.float32(p)))
            assert out["kept"][0] == keep.sum() and keep[out["tokens"][0]]
            # the same set from a library sort: shortest prefix of the sorted probabilities that reaches p,
            # extended over the ties of its last element
            order = np.argsort(-y, kind="stable")
            cum = np.cumsum(special.softmax(y)[order])
            n = int(np.searchsorted(cum, np.float64(np.float32(p)), side="left")) + 1
            n = min(n, V)
            thr = y[order[n - 1]]
            assert (y >= thr).sum() == keep.sum() or abs(cum[n - 1] - p) < 1e-12
        for k in (1, 2, 5, V, V + 3):
            out = _filtered(oracle, x, tau, top_k=k)
            keep = _kept_by_definition(y, k=k)
            assert out["kept"][0] == keep.sum() and keep[out["tokens"][0]]
            assert keep.sum() >= min(k, V)                    # ties at the k-th value are all kept


def test_filters_that_keep_everything_or_only_the_mode(oracle):
    rng = np.random.default_rng(42)
    B, V = 32, 300
    x = rng.normal(0, 3, (B, V)).astype(np.float32)
    plain = _filtered(oracle, x, 0.8)
    assert (plain["kept"] == V).all()
    for kw in (dict(top_p=1.0), dict(top_p=0.0), dict(top_k=V), dict(top_k=0), dict(top_k=10 * V)):
        out = _filtered(oracle, x, 0.8, **kw)
        np.testing.assert_array_equal(out["tokens"], plain["tokens"])
        np.testing.assert_array_equal(out["regret"], plain["regret"])
    mode = x.argmax(1)
    for kw in (dict(top_k=1), dict(top_p=1e-6)):
        out = _filtered(oracle, x, 0.8, **kw)
        np.testing.assert_array_equal(out["tokens"], mode)
        assert (out["regret"] == 0).all() and (out["kept"] == 1).all()
    # tied modes are kept together and the draw chooses among them
    x[:, 7] = x[:, 99] = 50.0
    toks = np.concatenate([_filtered(oracle, x, 0.8, seed=s, top_k=1)["tokens"] for s in range(8)])
    assert set(toks.tolist()) == {7, 99}
    # the statistics of the unfiltered distribution are not touched by the filter
    a, b = _filtered(oracle, x, 0.8, top_p=0.7), _filtered(oracle, x, 0.8)
    np.testing.assert_array_equal(a["sum_exp"], b["sum_exp"])
    np.testing.assert_array_equal(a["row_max"], b["row_max"])
    with pytest.raises(ValueError):
        _filtered(oracle, x, 0.8, top_p=0.7, top_k=5)
    with pytest.raises(ValueError):
        _filtered(oracle, x, 0.8, top_p=1.5)


def test_filtered_draws_follow_the_renormalised_distribution(oracle):
    V, tau, p = 12, 1.0, 0.7
    x = np.array([[2.0, 1.5, 1.5, 0.5, 0.0, -0.5, 3.0, -1.0, 1.0, 0.2, -2.0, 0.8]], np.float32)
    y = x[0].astype(np.float64)
    keep = _kept_by_definition(y, p=np.float64(np.float32(p)))
    assert 1 < keep.sum() < V
    n = 6000
    rows = np.repeat(x, n, axis=0)
    z, alive, ss = _state(n)
    out = oracle.step(rows, tau, 123, 0, np.zeros(n, np.float32), _params(oracle, stop_enabled=0, top_p=p), z, alive, ss)
    counts = np.bincount(out["tokens"], minlength=V)
    assert counts[~keep].sum() == 0                           # nothing outside the kept set is ever drawn
    want = special.softmax(y[keep])
    chi2 = stats.chisquare(counts[keep], want * n)
    assert chi2.pvalue > 1e-4
    # the kept set grows with p
    sizes = [_filtered(oracle, x, tau, top_p=q)["kept"][0] for q in (0.1, 0.3, 0.5, 0.7, 0.9, 0.999)]
    assert sizes == sorted(sizes) and sizes[-1] >= sizes[0]
