"""Parity of the HIP espo_step with the CPU oracle, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2605_29860_amd as espo  # noqa: E402
from paper_2605_29860_amd import workloads as W  # noqa: E402
import harness as H  # noqa: E402


def _say(msg):
    print(msg, flush=True)


def _rand_logits(B, V, stride, dtype, seed, sigma=3.0):
    g = torch.Generator().manual_seed(seed)
    x = torch.randn(B, stride, generator=g) * sigma
    return x.to(dtype).cuda()


# --------------------------------------------------------------------------- small shapes, edge cases
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("V", [1, 3, 8, 37, 511, 512, 513, 1100, 8192, 8200, 16391, 40000])
def test_shapes_and_ragged_tails(V, dtype):
    _say(f"[case] shapes V={V} dtype={dtype}")
    B = 5
    stride = ((V + 7) // 8) * 8 + 8                         # padded rows: pitch is a multiple of 16 bytes
    logits = _rand_logits(B, V, stride, dtype, seed=V)
    logits[:, V:] = 1e4                                      # beyond V must never be looked at
    gp, op = H.params_pair(mu_g=1.0, var_g=2.0, beta=1.0)
    st = H.GpuState(B, z=torch.tensor([0.0, 0.5, -0.3, 2.0, 0.1]), alive=torch.tensor([1, 1, 0, 1, 1], dtype=torch.uint8))
    vals = torch.tensor([0.5, -1.0, 0.3, 0.0, 1.0], device="cuda")
    for step in range(3):
        got = H.compare_step(logits, 0.8, 17, step, vals, gp, op, st, V=V)
        assert got["tokens"][2] == -1 and got["regret"][2] == 0 and got["logprob"][2] == 0
        assert ((got["tokens"] < V) & (got["tokens"] >= -1)).all()


def test_masked_vocabulary_and_ties():
    _say("[case] masked vocabulary, exact ties")
    B, V = 8, 3000
    x = torch.randn(B, V, generator=torch.Generator().manual_seed(1)) * 2
    x[:, ::2] = float("-inf")
    x[:, 1001] = 6.0
    x[:, 2001] = 6.0                                         # two exactly equal modes in different blocks
    for dtype in (torch.float32, torch.bfloat16):
        logits = x.to(dtype).cuda()
        gp, op = H.params_pair()
        st = H.GpuState(B)
        vals = torch.zeros(B, device="cuda")
        for step in range(4):
            got = H.compare_step(logits, 1.0, 5, step, vals, gp, op, st)
            live = got["tokens"] >= 0
            assert (got["tokens"][live] % 2 == 1).all()


def test_flat_rows_visit_many_blocks():
    _say("[case] flat rows")
    # uniform logits: no block stands out, so the bound-based pruning has the least to work with
    B, V = 4, 20000
    for dtype in (torch.float32, torch.bfloat16):
        logits = torch.full((B, V), 0.75, dtype=dtype).cuda()
        gp, op = H.params_pair(stop_enabled=0)
        st = H.GpuState(B)
        vals = torch.zeros(B, device="cuda")
        for step in range(6):
            got = H.compare_step(logits, 1.0, 99, step, vals, gp, op, st)
            assert (got["regret"] == 0).all()
            np.testing.assert_allclose(got["logprob"], -np.log(V), rtol=1e-5)


def test_extreme_temperatures_and_large_logits():
    _say("[case] temperatures")
    B, V = 6, 5000
    logits = _rand_logits(B, V, V, torch.float32, seed=3, sigma=30.0)
    for tau in (0.05, 0.6, 1.0, 4.0):
        gp, op = H.params_pair(stop_enabled=0)
        st = H.GpuState(B)
        H.compare_step(logits, tau, 11, 0, torch.zeros(B, device="cuda"), gp, op, st)


def test_eos_and_warmup_gate():
    _say("[case] eos / warmup")
    B, V = 4, 600
    x = torch.full((B, V), -30.0)
    x[:, 77] = 10.0
    logits = x.cuda()
    vals = torch.zeros(B, device="cuda")
    gp, op = H.params_pair(eos_id=77)
    st = H.GpuState(B, z=torch.full((B,), 9.0))
    got = H.compare_step(logits, 1.0, 0, 3, vals, gp, op, st)
    assert (got["alive"] == 0).all() and (got["stop_step"] == -1).all()
    gp, op = H.params_pair(stop_enabled=0)
    st = H.GpuState(B, z=torch.full((B,), 9.0))
    got = H.compare_step(logits, 1.0, 0, 3, vals, gp, op, st)
    assert (got["alive"] == 1).all()
    gp, op = H.params_pair()
    st = H.GpuState(B, z=torch.full((B,), 9.0))
    got = H.compare_step(logits, 1.0, 0, 3, vals, gp, op, st)
    assert (got["alive"] == 0).all() and (got["stop_step"] == 3).all()


def test_empty_batch_and_argument_errors():
    _say("[case] errors")
    gp, _ = H.params_pair()
    B, V = 2, 64
    logits = torch.zeros(B, V, dtype=torch.bfloat16, device="cuda")
    st = H.GpuState(B)
    vals = torch.zeros(B, device="cuda")
    espo.espo_step(logits[:0], 1.0, 0, 0, vals[:0], gp, st.z[:0], st.alive[:0], st.stop_step[:0],
                   st.tokens[:0], st.regret[:0], st.logprob[:0])
    for tau in (0.0, -1.0, float("nan"), float("inf")):
        with pytest.raises(espo.EspoError) as e:
            H.gpu_step(logits, tau, 0, 0, vals, gp, st)
        assert e.value.code == -1
    with pytest.raises(espo.EspoError) as e:                 # V beyond the row pitch
        H.gpu_step(logits, 1.0, 0, 0, vals, gp, st, V=V + 1)
    assert e.value.code == -1
    odd = torch.zeros(B, 72, dtype=torch.bfloat16, device="cuda")[:, 4:68]   # base not 16-byte aligned
    with pytest.raises(espo.EspoError) as e:
        H.gpu_step(odd, 1.0, 0, 0, vals, gp, st)
    assert e.value.code == -2
    bad, _ = H.params_pair(alpha_s=1.5)
    with pytest.raises(espo.EspoError):
        H.gpu_step(logits, 1.0, 0, 0, vals, bad, st)
    torch.cuda.synchronize()
    assert (st.tokens.cpu().numpy() == -7).all()              # nothing was launched


# --------------------------------------------------------------------------- config 1: small reference rollout
def test_config1_small_reference_rollout():
    _say("[case] config 1 rollout")
    cfg = W.SmallReference()
    gp, op = H.params_pair(**cfg.params.as_dict())
    vals_all = cfg.values("cuda")
    st = H.GpuState(cfg.B)
    stats = {}
    tokens = np.zeros((cfg.B, cfg.T), np.int32)
    for t in range(cfg.T):
        got = H.compare_step(cfg.logits(t, "cuda"), cfg.temperature, cfg.seed, t,
                             vals_all[:, t].contiguous(), gp, op, st, stats=stats)
        tokens[:, t] = got["tokens"]
    end = st.host()
    assert end["alive"].tolist() == [1, 1, 0, 0]              # rows 0-1 survive, rows 2-3 must stop
    assert (end["stop_step"][:2] == -1).all() and (end["stop_step"][2:] > 0).all()
    for b in (2, 3):
        assert (tokens[b, end["stop_step"][b] + 1:] == -1).all()
    # advantages on the resulting truncated trajectories
    lengths = np.where(end["stop_step"] >= 0, end["stop_step"] + 1, cfg.T).astype(np.int32)
    stopped = (end["stop_step"] >= 0).astype(np.uint8)
    rewards = torch.zeros(cfg.B, cfg.T)
    for b in range(cfg.B):
        if not stopped[b]:
            rewards[b, lengths[b] - 1] = 1.0
    H.check_advantages(rewards.cuda(), vals_all, torch.as_tensor(lengths).cuda(),
                       torch.as_tensor(stopped).cuda(), cfg.r_fail, cfg.gamma, cfg.lam)
    _say(f"  config 1: stop steps {end['stop_step'].tolist()} stats {stats}")


# --------------------------------------------------------------------------- config 2: one fused step, Qwen vocabulary
def test_config2_single_fused_step():
    _say("[case] config 2")
    B, V = 64, W.QWEN_VOCAB
    gen = W.ZipfLogits(V=V, seed=2, device="cuda")
    logits = gen.rows(B, step=0)
    z, alive, ss = W.seeded_state(B, seed=2, device="cuda")
    vals = W.step_values(B, 2, 0, -0.2, 1.0, device="cuda")
    gp, op = H.params_pair(**W.RolloutParams().as_dict())
    st = H.GpuState(B, z=z, alive=alive, stop_step=ss)
    stats = {}
    got = H.compare_step(logits, 0.6, 2, 0, vals, gp, op, st, stats=stats)
    assert (got["tokens"][7::8] == -1).all() and (got["tokens"][got["alive"] == 1] >= 0).all()
    assert (got["z"][7::8] == z.cpu().numpy()[7::8]).all()   # dead rows untouched
    _say(f"  config 2: mean regret {got['regret'][got['tokens'] >= 0].mean():.3f} stats {stats}")


# --------------------------------------------------------------------------- configs 3, 4: rollout loops at full batch size
def _rollout(B, steps, plant_fraction, onset_lo, onset_hi, seed, oracle_rows, val_lo, val_hi):
    """The rollout loop at full batch size.  At EVERY step the oracle runs on `oracle_rows` (tokens, regret,
    z, masks, stop steps and log-probabilities compared as in every other test), and for ALL rows the scalar
    chain is replayed on the host from the GPU's own regret and tokens and must give the GPU's z, alive and
    stop_step bit for bit."""
    V = W.QWEN_VOCAB
    gen = W.ZipfLogits(V=V, seed=seed, device="cuda")
    plant = W.RegretPlant.make(B, V, plant_fraction, onset_lo, onset_hi, seed)
    gp, op = H.params_pair(**W.RolloutParams().as_dict())
    st = H.GpuState(B)
    import oracle
    z_r, alive_r, ss_r = np.zeros(B, np.float32), np.ones(B, np.uint8), np.full(B, -1, np.int32)
    buf = torch.empty(B, V, dtype=torch.bfloat16, device="cuda")
    stats = {}
    live_curve = []
    for t in range(steps):
        x = gen.rows(B, step=t, out=None)
        x = plant.apply(x.float(), t).to(torch.bfloat16)
        buf.copy_(x)
        vals = W.step_values(B, seed, t, val_lo, val_hi, device="cuda")
        alive_before = st.alive.cpu().numpy().copy()
        got = H.compare_step(buf, 0.6, seed, t, vals, gp, op, st, rows=oracle_rows, stats=stats)
        # invariants on all rows
        dead = alive_before == 0
        assert (got["tokens"][dead] == -1).all() and (got["regret"][dead] == 0).all()
        live = ~dead
        assert ((got["tokens"][live] >= 0) & (got["tokens"][live] < V)).all()
        assert (got["regret"][live] >= 0).all()
        assert (got["alive"] <= alive_before).all()          # never revived
        oracle.state_update(got["regret"], got["tokens"], vals.cpu().numpy(), op, t, z_r, alive_r, ss_r)
        np.testing.assert_array_equal(got["z"].view(np.uint32), z_r.view(np.uint32), err_msg=f"step {t}")
        np.testing.assert_array_equal(got["alive"], alive_r, err_msg=f"step {t}")
        np.testing.assert_array_equal(got["stop_step"], ss_r, err_msg=f"step {t}")
        live_curve.append(int(alive_r.sum()))
        if t % 64 == 0:
            _say(f"  step {t}: live {live_curve[-1]}/{B}, oracle rows checked so far {stats.get('rows_checked', 0)}")
    return plant, st.host(), live_curve, stats


def _oracle_subset(plant, B, n_each=32):
    """`n_each` planted rows (spread over the onset steps) and as many that are not planted."""
    order = np.argsort(plant.onset, kind="stable")
    planted = plant.rows[order[np.linspace(0, len(order) - 1, n_each).astype(int)]].tolist()
    free = np.setdiff1d(np.arange(B), plant.rows)
    others = free[np.linspace(0, len(free) - 1, n_each).astype(int)].tolist()
    return sorted(set(planted) | set(others))


def test_config3_sustained_rollout():
    _say("[case] config 3 (B=512, 1024 steps, oracle on 64 rows at every step)")
    B, steps, seed = 512, 1024, 3
    rows = _oracle_subset(W.RegretPlant.make(B, W.QWEN_VOCAB, 0.25, 8, 1000, seed), B)
    assert len(rows) >= 64
    plant, end, curve, stats = _rollout(B, steps, 0.25, 8, 1000, seed, rows, 0.2, 1.0)
    stopped_planted = (end["stop_step"][plant.rows] >= 0).mean()
    _say(f"  config 3: live at end {curve[-1]}, planted rows stopped {stopped_planted:.2f}, stats {stats}")
    assert stats["rows_checked"] > 0.6 * len(rows) * steps   # the oracle followed its rows for as long as they lived
    assert stopped_planted > 0.9
    assert 0.6 * B < curve[-1] < 0.8 * B                      # about a quarter of the batch stops
    on = end["stop_step"][plant.rows]
    assert (on[on >= 0] >= plant.onset[on >= 0]).all()        # never before the drift starts


def test_config4_heavy_termination():
    _say("[case] config 4 (B=1024, 256 steps, oracle on 64 rows at every step)")
    B, steps, seed = 1024, 256, 4
    # onsets in [14, 150]: the smoothed regret needs at least three steps to cross the lowest threshold and
    # crosses a typical one within a dozen, so the stops land in the stated window [16, 200]
    rows = _oracle_subset(W.RegretPlant.make(B, W.QWEN_VOCAB, 0.6, 14, 150, seed), B)
    assert len(rows) >= 64
    plant, end, curve, stats = _rollout(B, steps, 0.6, 14, 150, seed, rows, 0.2, 1.0)
    ss = end["stop_step"][plant.rows]
    _say(f"  config 4: live at end {curve[-1]}, planted stop steps in [{ss[ss >= 0].min()}, {ss.max()}], stats {stats}")
    assert (ss >= 0).mean() > 0.95
    assert ((ss[ss >= 0] >= 16) & (ss[ss >= 0] <= 200)).all()
    assert 0.3 * B < curve[-1] < 0.5 * B


# --------------------------------------------------------------------------- replay / resume / batch independence
def test_determinism_resume_and_batch_independence():
    _say("[case] determinism")
    B, V, steps = 24, 9000, 12
    gen = W.ZipfLogits(V=V, seed=9, device="cuda")
    gp, _ = H.params_pair(mu_g=1.0, var_g=2.0, beta=2.0)

    def run(rows, start, stop, st):
        outs = []
        for t in range(start, stop):
            x = gen.rows(B, step=t)[rows].contiguous()
            vals = W.step_values(B, 9, t, 0.0, 1.0, device="cuda")[rows].contiguous()
            H.gpu_step(x, 0.6, 9, t, vals, gp, st)
            torch.cuda.synchronize()
            outs.append(st.host())
        return outs

    allrows = torch.arange(B, device="cuda")
    a = run(allrows, 0, steps, H.GpuState(B))
    b = run(allrows, 0, steps, H.GpuState(B))
    for x, y in zip(a, b):
        for k in x:
            np.testing.assert_array_equal(x[k].view(np.uint8), y[k].view(np.uint8))
    # resume: copy the state out after 5 steps, continue in a fresh state object
    st = H.GpuState(B)
    run(allrows, 0, 5, st)
    st2 = H.GpuState(B, z=st.z.cpu(), alive=st.alive.cpu(), stop_step=st.stop_step.cpu())
    c = run(allrows, 5, steps, st2)
    for k in c[-1]:
        np.testing.assert_array_equal(c[-1][k].view(np.uint8), a[-1][k].view(np.uint8))
    # a row's stream is keyed by its index in the batch: the first rows of a larger batch
    # behave exactly like a smaller batch made of them
    d = run(allrows[:7], 0, steps, H.GpuState(7))
    for k in d[-1]:
        np.testing.assert_array_equal(d[-1][k].view(np.uint8), a[-1][k][:7].view(np.uint8))


# --------------------------------------------------------------------------- fp32 scores: margin and exact fallback
def test_hardware_ln_exp_within_the_margin_assumptions():
    _say("[case] hardware ln / exp accuracy")
    # The fp32 scores of espo_step are built from the hardware log2 / exp2; their margin assumes
    # relative errors of at most 1.7e-7 (ln, also of every u(w)) and 2e-6 (exp).  Measured here
    # on the device against the double-precision functions.
    out = torch.zeros(3, dtype=torch.float32, device="cuda")
    espo.espo_debug_math_errors(out)
    torch.cuda.synchronize()
    e_u, e_ln, e_exp = out.cpu().tolist()
    _say(f"  max relative error: ln u(w) {e_u:.3e}, ln x {e_ln:.3e}, exp x {e_exp:.3e}")
    assert 0 < e_u <= 1.7e-7 and 0 < e_ln <= 1.7e-7 and 0 < e_exp <= 2e-6


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_exact_fallback_decides_every_row_like_the_oracle(dtype):
    _say(f"[case] double-precision fallback forced, dtype={dtype}")
    # A huge margin makes the fp32 search "uncertain" for every row, so every token below is
    # decided by the double-precision search; it must agree with the oracle, and with the
    # tokens the default margin gives.
    B = 6
    gp, op = H.params_pair(stop_enabled=0)
    for V, tau in ((37, 1.0), (8200, 0.6), (40000, 1.3)):
        stride = ((V + 7) // 8) * 8
        logits = _rand_logits(B, V, stride, dtype, seed=100 + V)
        vals = torch.zeros(B, device="cuda")
        tokens = {}
        for scale in (1.0, 3e4, 1e12):  # 3e4: a few candidates per row, decided in double one by one; 1e12: block by block
            st = H.GpuState(B)
            for step in range(3):
                got = H.compare_step(logits, tau, 23, step, vals, gp, op, st, V=V, margin_scale=scale)
                tokens[(scale, step)] = got["tokens"].copy()
        for step in range(3):
            np.testing.assert_array_equal(tokens[(1.0, step)], tokens[(3e4, step)])
            np.testing.assert_array_equal(tokens[(1.0, step)], tokens[(1e12, step)])


def test_exact_fallback_at_full_width_matches_default_margin():
    _say("[case] double-precision fallback forced, B=512 x V=152064")
    B, V = 512, W.QWEN_VOCAB
    gen = W.ZipfLogits(V=V, seed=11, device="cuda")
    logits = gen.rows(B, step=0)
    plant = W.RegretPlant.make(B, V, 0.25, 0, 0, 11)     # flat, tie-heavy rows among them
    plant.apply(logits, 0)
    vals = torch.zeros(B, device="cuda")
    gp, op = H.params_pair(stop_enabled=0)
    res = {}
    for layout in (dict(), dict(workspace=False)):            # rows split over workgroups, and one workgroup per row
        for scale in (1.0, 3e4, 1e12):
            st = H.GpuState(B)
            H.gpu_step(logits, 0.6, 11, 0, vals, gp, st, margin_scale=scale, **layout)
            torch.cuda.synchronize()
            res[scale] = st.host()
        for scale in (3e4, 1e12):
            for k in ("tokens", "regret", "z"):
                np.testing.assert_array_equal(res[1.0][k].view(np.uint32), res[scale][k].view(np.uint32))
            assert np.abs(res[1.0]["logprob"] - res[scale]["logprob"]).max() == 0
    with pytest.raises(espo.EspoError):
        H.gpu_step(logits, 0.6, 11, 0, vals, gp, H.GpuState(B), margin_scale=0.5)


# --------------------------------------------------------------------------- largest supported vocabulary
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_largest_vocabulary_and_range_error(dtype):
    _say(f"[case] V = 400000 (more than 64 KB of LDS per workgroup), dtype={dtype}")
    B, V = 3, 400000
    logits = _rand_logits(B, V, V, dtype, seed=77)
    logits[1, 399999] = 25.0                                  # the mode in the very last block
    gp, op = H.params_pair(stop_enabled=0)
    st = H.GpuState(B)
    vals = torch.zeros(B, device="cuda")
    for step in range(2):
        got = H.compare_step(logits, 1.0, 31, step, vals, gp, op, st)
        assert ((got["tokens"] >= 0) & (got["tokens"] < V)).all()
    big = torch.zeros(1, 400008, dtype=dtype, device="cuda")
    with pytest.raises(espo.EspoError) as e:
        H.gpu_step(big, 1.0, 0, 0, vals[:1], gp, H.GpuState(1), V=400001)
    assert e.value.code == -5


# --------------------------------------------------------------------------- ablation stop modes, simulate mode
@pytest.mark.parametrize("mode,thr", [(1, 0.03), (2, 0.35), (3, 0.05)])
def test_ablation_stop_modes_match_the_oracle(mode, thr):
    _say(f"[case] stop mode {mode}")
    B, V, steps = 48, 6000, 24
    gen = W.ZipfLogits(V=V, seed=40 + mode, device="cuda")
    gp, op = H.params_pair(mu_g=1.0, var_g=2.0, stop_mode=mode, stop_threshold=thr)
    st = H.GpuState(B)
    for t in range(steps):
        vals = W.step_values(B, 40 + mode, t, 0.0, 1.0, device="cuda")
        H.compare_step(gen.rows(B, step=t), 0.6, 40 + mode, t, vals, gp, op, st)
    end = st.host()
    stopped = end["stop_step"] >= 0
    assert 0 < stopped.sum() < B                              # the rule fired for some rows, not for all
    assert (end["alive"][stopped] == 0).all() and (end["alive"][~stopped] == 1).all()
    bad, _ = H.params_pair(stop_mode=7)
    with pytest.raises(espo.EspoError):
        H.gpu_step(gen.rows(B, step=0), 0.6, 0, 0, vals, bad, H.GpuState(B))


def test_simulate_mode_keeps_rows_alive_and_records_first_stop():
    _say("[case] simulate mode")
    B, V, steps = 32, 5000, 30
    gen = W.ZipfLogits(V=V, seed=50, device="cuda")
    kw = dict(mu_g=1.0, var_g=2.0, beta=1.0, eps=0.2)
    gp, op = H.params_pair(simulate=1, **kw)
    gp0, op0 = H.params_pair(**kw)
    st, st0 = H.GpuState(B), H.GpuState(B)
    for t in range(steps):
        vals = W.step_values(B, 50, t, 0.0, 1.0, device="cuda")
        x = gen.rows(B, step=t)
        got = H.compare_step(x, 0.6, 50, t, vals, gp, op, st)
        assert (got["alive"] == 1).all() and (got["tokens"] >= 0).all()     # nobody is truncated
        H.gpu_step(x, 0.6, 50, t, vals, gp0, st0)
    torch.cuda.synchronize()
    sim, real = st.host(), st0.host()
    # until a row's first stop both runs see the same stream, so the recorded step is the step
    # at which the real run truncated the row
    np.testing.assert_array_equal(sim["stop_step"], real["stop_step"])
    assert (sim["stop_step"] >= 0).sum() > 0


# --------------------------------------------------------------------------- seeded sweep over shapes, structures and search paths
def _structured_logits(rng, g, B, V, stride, kind):
    x = torch.randn(B, stride, generator=g) * float(rng.choice([0.5, 3.0, 12.0]))
    if kind == "flat":
        x[:] = float(rng.choice([1.5, -3.0, 0.0]))
    elif kind == "plateau":                               # half of the vocabulary tied just below one peak
        x[:, 0::2] = 20.0
        x[:, min(V - 1, 7)] = 22.0
    elif kind == "masked":
        x[:, torch.rand(stride, generator=g) < 0.7] = float("-inf")
        x[:, V // 2] = 0.25                                # at least one finite entry
    elif kind == "peaked":
        x[:, V - 1] = 40.0
    elif kind == "twopeak":                               # two equal modes, first and last index
        x[:, 0] = 30.0
        x[:, V - 1] = 30.0
    elif kind == "ramp":
        x[:] = torch.arange(stride).float()[None, :] * (10.0 / V)
    x[:, V:] = 1e4                                         # beyond V must never matter
    return x


@pytest.mark.parametrize("part", range(5))
def test_seeded_sweep_of_shapes_structures_and_margins(part):
    _say(f"[case] seeded sweep, part {part} (400 cases)")
    # Random shapes, logit structures, temperatures, margin scales (1 = production; larger ones send
    # more rows through the long-list and the double-precision paths), stop modes, simulate mode,
    # end-of-sequence ids, partly dead batches, with and without the entropy output, and every layout:
    # the library's own choice with a workspace, one workgroup of 16 waves per row, and forced numbers of
    # chunks per row and waves per workgroup.
    rng = np.random.default_rng(2024 + part)
    paths, layouts, stats = {1.0: 0, 3e4: 0, 1e12: 0}, {}, {}
    for case in range(part * 400, part * 400 + 400):
        V = int(rng.choice([rng.integers(1, 600), rng.integers(600, 9000), rng.integers(9000, 70000),
                            rng.integers(70000, 200000)], p=[0.3, 0.3, 0.3, 0.1]))
        B = int(rng.integers(1, 7))
        dtype = torch.bfloat16 if rng.random() < 0.5 else torch.float32
        tau = float(rng.choice([0.05, 0.3, 0.6, 1.0, 2.5, 8.0]))
        kind = str(rng.choice(["gauss", "flat", "plateau", "masked", "peaked", "twopeak", "ramp"]))
        stride = ((V + 7) // 8) * 8 + int(rng.choice([0, 8, 64]))
        g = torch.Generator().manual_seed(1000 + case)
        logits = _structured_logits(rng, g, B, V, stride, kind).to(dtype).cuda()
        scale = float(rng.choice([1.0, 1.0, 1.0, 3e4, 1e12]))
        paths[scale] += 1
        mode, simulate = int(rng.choice([0, 0, 0, 1, 2, 3])), int(rng.random() < 0.15)
        filt = [dict(), dict(), dict(top_p=float(rng.choice([0.3, 0.7, 0.95]))), dict(top_k=int(rng.choice([1, 3, 40])))][int(rng.integers(0, 4))]
        if filt:                                             # a filtered draw has one layout
            layout = dict()
        else:
            layout = [dict(), dict(), dict(workspace=False), dict(chunks=int(rng.choice([1, 2, 3, 5, 8, 13, 64]))),
                      dict(chunks=int(rng.choice([2, 4, 7])), waves=int(rng.choice([4, 8, 16]))),
                      dict(waves=int(rng.choice([4, 8, 16])))][int(rng.integers(0, 6))]
        layouts[str(layout)] = layouts.get(str(layout), 0) + 1
        gp, op = H.params_pair(mu_g=1.0, var_g=2.0, beta=float(rng.choice([0.5, 7.0])), stop_mode=mode,
                               stop_threshold=float(rng.choice([0.05, 0.3, 1.0])), simulate=simulate,
                               eos_id=int(rng.choice([-1, -1, 0, V - 1])), **filt)
        st = H.GpuState(B, z=torch.rand(B, generator=g) * 2 - 1, alive=(torch.rand(B, generator=g) < 0.85).to(torch.uint8))
        vals = torch.rand(B, generator=g).cuda()
        entropy = bool(rng.random() < 0.4)
        # where nothing needs the softmax sum, the same steps also run without the log-probability output
        bare = H.GpuState(B, z=st.z, alive=st.alive) if not filt and not entropy else None
        try:
            for step in range(2):
                got = H.compare_step(logits, tau, 900 + case, step, vals, gp, op, st, V=V, stats=stats, entropy=entropy,
                                     margin_scale=scale, **layout)
                if bare is not None:
                    H.gpu_step(logits, tau, 900 + case, step, vals, gp, bare, V=V, logprob=False, margin_scale=scale, **layout)
                    torch.cuda.synchronize()
                    other = bare.host()
                    for k in ("tokens", "regret", "z", "alive", "stop_step"):
                        np.testing.assert_array_equal(got[k].view(np.uint8), other[k].view(np.uint8), err_msg=f"no logprob: {k}")
        except AssertionError as err:
            raise AssertionError(f"case {case}: V={V} B={B} {dtype} tau={tau} {kind} scale={scale} mode={mode} "
                                 f"simulate={simulate} entropy={entropy} {filt} {layout}: {err}")
    _say(f"  cases per margin scale: {paths}; per layout: {layouts}; {stats}")


# --------------------------------------------------------------------------- rows split over workgroups
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_every_split_of_a_row_gives_the_bits_of_the_whole_row(dtype):
    _say(f"[case] rows split over workgroups {dtype}")
    # The row is cut at multiples of 512 indices (8 draw blocks).  Cases: a vocabulary of one tile (no split
    # possible), ragged last tiles of 1 and 511 indices, a last chunk that holds only the ragged tile, more
    # chunks asked for than there are tiles, the winner in the first and in the last chunk, rows whose chunks
    # are mostly masked, and the Qwen vocabulary at the split the library itself picks for B = 512.
    cases = [(300, "gauss"), (512, "gauss"), (513, "gauss"), (1023, "peaked_last"), (1537, "peaked_first"),
             (5000, "masked"), (20481, "gauss"), (40000, "flat"), (70001, "twopeak"), (152064, "zipf")]
    for case, (V, kind) in enumerate(cases):
        B = 4
        stride = ((V + 7) // 8) * 8 + 8
        g = torch.Generator().manual_seed(4000 + case)
        x = torch.randn(B, stride, generator=g) * 3.0
        if kind == "peaked_last":
            x[:, V - 1] = 30.0
        elif kind == "peaked_first":
            x[:, 0] = 30.0
        elif kind == "masked":
            x[:, :] = float("-inf")
            x[:, 4700:4710] = torch.randn(B, 10, generator=g)     # every chunk but one is empty
        elif kind == "flat":
            x[:] = -1.25
        elif kind == "twopeak":
            x[:, 3] = 25.0
            x[:, V - 2] = 25.0                                   # equal modes in the first and the last chunk
        elif kind == "zipf":
            x[:, :V] += W.ZipfLogits(V=V, seed=case, device="cpu").boost
        x[:, V:] = 1e4
        logits = x.to(dtype).cuda()
        vals = torch.rand(B, generator=g).cuda()
        gp, op = H.params_pair(mu_g=1.0, var_g=2.0, beta=0.8)
        alive0 = torch.tensor([1, 1, 0, 1], dtype=torch.uint8)
        whole = H.GpuState(B, alive=alive0)
        for step in range(2):
            H.compare_step(logits, 0.7, 57, step, vals, gp, op, whole, V=V, entropy=True, workspace=False)
        ref = whole.host()
        ntiles = (V + 511) // 512
        for layout in (dict(), dict(chunks=2), dict(chunks=3, waves=8), dict(chunks=ntiles), dict(chunks=ntiles + 5, waves=4),
                       dict(chunks=7, waves=16), dict(chunks=64), dict(chunks=1, waves=4), dict(chunks=8, margin_scale=1e12)):
            st = H.GpuState(B, alive=alive0)
            for step in range(2):
                H.compare_step(logits, 0.7, 57, step, vals, gp, op, st, V=V, entropy=True, **layout)
            got = st.host()
            for k in ("tokens", "regret", "z", "alive", "stop_step"):
                np.testing.assert_array_equal(got[k].view(np.uint8), ref[k].view(np.uint8), err_msg=f"V={V} {kind} {layout} {k}")
            # the sums are added in another order: last bits only
            np.testing.assert_allclose(got["logprob"], ref["logprob"], rtol=0, atol=4e-6 * max(1.0, float(np.abs(ref["logprob"]).max())))
            np.testing.assert_allclose(got["entropy"], ref["entropy"], rtol=0, atol=1e-5 * max(1.0, float(ref["entropy"].max())))


def test_workspace_contract():
    _say("[case] workspace contract of espo_step and of a forced split")
    B, V = 600, 3000
    logits = _rand_logits(B, V, V, torch.bfloat16, seed=9)
    vals = torch.zeros(B, device="cuda")
    gp, _ = H.params_pair(stop_enabled=0)
    assert espo.espo_step_workspace_bytes(B, V, torch.bfloat16) == 0       # one workgroup per row: no scratch needed
    need = espo.espo_debug_step_workspace_bytes(B, 3)
    assert need >= B * 3 * 32
    st = H.GpuState(B)
    call = lambda **kw: espo.espo_step(logits, 1.0, 0, 0, vals, gp, st.z, st.alive, st.stop_step, st.tokens, st.regret, st.logprob, **kw)
    with pytest.raises(espo.EspoError) as e:                  # given but too small
        call(workspace=torch.zeros(need - 16, dtype=torch.uint8, device="cuda"), chunks=3)
    assert e.value.code == -3
    with pytest.raises(espo.EspoError) as e:                  # misaligned
        call(workspace=torch.zeros(need + 16, dtype=torch.uint8, device="cuda")[4:], chunks=3)
    assert e.value.code == -3
    with pytest.raises(espo.EspoError) as e:                  # a forced split without a workspace
        call(chunks=4)
    assert e.value.code == -3
    with pytest.raises(espo.EspoError) as e:
        call(waves=5)
    assert e.value.code == -1
    torch.cuda.synchronize()
    assert (st.tokens.cpu().numpy() == -7).all()              # nothing was launched
    # one buffer serves split calls of different shapes one after the other, and comes back zero every time
    ws = torch.zeros(max(need, espo.espo_debug_step_workspace_bytes(700, 2)), dtype=torch.uint8, device="cuda")
    a, b, o3 = H.GpuState(B), H.GpuState(B), H.GpuState(B)
    for step in range(3):
        espo.espo_step(logits, 1.0, 4, step, vals, gp, a.z, a.alive, a.stop_step, a.tokens, a.regret, a.logprob, workspace=ws)
        other = _rand_logits(700, 1600, 1600, torch.float32, seed=step)
        o = H.GpuState(700)
        espo.espo_step(other, 1.0, 4, step, torch.zeros(700, device="cuda"), gp, o.z, o.alive, o.stop_step, o.tokens, o.regret,
                       o.logprob, workspace=ws, chunks=2)
        espo.espo_step(logits, 1.0, 4, step, vals, gp, o3.z, o3.alive, o3.stop_step, o3.tokens, o3.regret, o3.logprob,
                       workspace=ws, chunks=3)
        espo.espo_step(logits, 1.0, 4, step, vals, gp, b.z, b.alive, b.stop_step, b.tokens, b.regret, b.logprob)
        torch.cuda.synchronize()
        assert not bool(ws.any())
        for k in ("tokens", "regret", "z"):
            np.testing.assert_array_equal(a.host()[k].view(np.uint8), b.host()[k].view(np.uint8))
            np.testing.assert_array_equal(o3.host()[k].view(np.uint8), b.host()[k].view(np.uint8))


@pytest.mark.parametrize("B", [513, 600, 1024, 1500, 2600])
def test_more_rows_than_resident_workgroups(B):
    _say(f"[case] more rows than resident workgroups, B={B}")
    # More rows than the GPU holds workgroups at once.  Every row must be handled exactly once whatever the pattern
    # of rows that are done (none, most, runs of them, all), with the oracle's results; a row split three ways
    # through the workspace must give the same bits.
    V = 2504                                                  # a pitch of 16-byte multiples
    g = torch.Generator().manual_seed(B)
    logits = (torch.randn(B, V, generator=g) * 3).to(torch.bfloat16).cuda()
    vals = torch.rand(B, generator=g).cuda()
    gp, op = H.params_pair(mu_g=1.0, var_g=2.0, beta=1.5)
    patterns = {"none": torch.ones(B), "most": (torch.rand(B, generator=g) < 0.3).float(), "all": torch.zeros(B),
                "runs": ((torch.arange(B) // 97) % 2).float(), "first512": (torch.arange(B) >= 512).float()}
    for name, alive in patterns.items():
        st = H.GpuState(B, alive=alive.to(torch.uint8), z=torch.rand(B, generator=g))
        ref = H.GpuState(B, alive=alive.to(torch.uint8), z=st.z.cpu())
        for step in range(3):
            H.compare_step(logits, 0.8, 71, step, vals, gp, op, st)
            H.gpu_step(logits, 0.8, 71, step, vals, gp, ref, chunks=3, waves=8)
            torch.cuda.synchronize()
            got, want = st.host(), ref.host()
            for k in ("tokens", "regret", "z", "alive", "stop_step"):      # the split adds the softmax sum in another order
                np.testing.assert_array_equal(got[k].view(np.uint8), want[k].view(np.uint8), err_msg=f"{name} step {step} {k}")


# --------------------------------------------------------------------------- entropy output
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_entropy_output_matches_the_oracle(dtype):
    _say(f"[case] entropy {dtype}")
    stats = {}
    rng = np.random.default_rng(77)
    for case, (V, kind, tau) in enumerate([(1, "gauss", 1.0), (5, "gauss", 0.6), (513, "gauss", 0.6), (4099, "flat", 1.0),
                                           (9000, "masked", 0.8), (20000, "peaked", 0.6), (33000, "gauss", 0.05),
                                           (33000, "gauss", 4.0), (70001, "zipf", 0.6), (152064, "zipf", 0.6)]):
        B = 4
        stride = ((V + 7) // 8) * 8 + 8
        g = torch.Generator().manual_seed(500 + case)
        x = torch.randn(B, stride, generator=g) * 3.0
        if kind == "flat":
            x[:] = -2.0
        elif kind == "masked":
            x[:, torch.rand(stride, generator=g) < 0.8] = float("-inf")
            x[:, V // 3] = 1.0
        elif kind == "peaked":
            x[:, V - 2] = 60.0                                  # far beyond the rest: entropy next to 0
        elif kind == "zipf":
            x[:, :V] += W.ZipfLogits(V=V, seed=case, device="cpu").boost   # the shape of the benchmark rows
        x[:, V:] = 1e4
        logits = x.to(dtype).cuda()
        gp, op = H.params_pair(mu_g=1.0, var_g=2.0, beta=3.0)
        st = H.GpuState(B, alive=torch.tensor([1, 1, 0, 1], dtype=torch.uint8))
        vals = torch.rand(B, generator=g).cuda()
        # the same step without the entropy output: every other output must be the same bits
        plain = H.GpuState(B, alive=torch.tensor([1, 1, 0, 1], dtype=torch.uint8))
        H.gpu_step(logits, tau, 41, 0, vals, gp, plain, V=V)
        got = H.compare_step(logits, tau, 41, 0, vals, gp, op, st, V=V, entropy=True, stats=stats)
        ref = plain.host()
        for k in ("tokens", "regret", "z", "alive", "stop_step", "logprob"):
            np.testing.assert_array_equal(got[k].view(np.uint8), ref[k].view(np.uint8), err_msg=f"case {case} {k}")
        assert got["entropy"][2] == 0 and (got["entropy"] >= 0).all() and (got["entropy"] <= np.log(V) * (1 + 1e-6) + 1e-6).all()
        if kind == "flat":
            np.testing.assert_allclose(got["entropy"][[0, 1, 3]], np.log(V), rtol=1e-6)
    _say(f"  largest entropy error {stats.get('max_entropy_err', 0):.2e}")


# --------------------------------------------------------------------------- concurrent streams
def test_two_streams_do_not_interfere():
    _say("[case] two streams")
    # The library keeps no state between calls: rollouts interleaved on two streams give the bits
    # of the same rollouts run one after the other.
    B, V, steps = 640, 9000, 10                              # more rows than resident workgroups
    gens = [W.ZipfLogits(V=V, seed=60 + i, device="cuda") for i in range(2)]
    data = [[g.rows(B, step=t) for t in range(steps)] for g in gens]
    vals = [[W.step_values(B, 60 + i, t, 0.0, 1.0, device="cuda") for t in range(steps)] for i in range(2)]
    gp, _ = H.params_pair(mu_g=1.0, var_g=2.0, beta=1.0)
    # rollout 1 runs with every row split in two (calls that may overlap must not share a workspace: it has its own)
    wss = [None, torch.zeros(espo.espo_debug_step_workspace_bytes(B, 2), dtype=torch.uint8, device="cuda")]
    lay = [dict(), dict(chunks=2, workspace=wss[1])]

    def one(i, st, stream=None):
        for t in range(steps):
            espo.espo_step(data[i][t], 0.6, 60 + i, t, vals[i][t], gp, st.z, st.alive, st.stop_step,
                           st.tokens, st.regret, st.logprob, stream=stream, **lay[i])

    serial = [H.GpuState(B), H.GpuState(B)]
    for i in range(2):
        one(i, serial[i])
    torch.cuda.synchronize()
    inter = [H.GpuState(B), H.GpuState(B)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for t in range(steps):
        for i in range(2):
            st = inter[i]
            espo.espo_step(data[i][t], 0.6, 60 + i, t, vals[i][t], gp, st.z, st.alive, st.stop_step,
                           st.tokens, st.regret, st.logprob, stream=streams[i], **lay[i])
    torch.cuda.synchronize()
    assert not bool(wss[1].any())
    for i in range(2):
        a, b = serial[i].host(), inter[i].host()
        for k in a:
            np.testing.assert_array_equal(a[k].view(np.uint8), b[k].view(np.uint8), err_msg=f"stream {i} {k}")


# --------------------------------------------------------------------------- no log-probability asked for
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_step_without_logprob_gives_the_same_token_and_state(dtype):
    _say(f"[case] no logprob output {dtype}")
    # Without the log-probability (and without entropy or a filter) the softmax sum is not formed at all:
    # another instantiation of the kernel.  Everything else must be the same bits, and the oracle's.
    import oracle
    for case, (V, kind, tau) in enumerate([(1, "gauss", 1.0), (37, "gauss", 0.6), (513, "masked", 0.8), (8200, "flat", 1.0),
                                           (40000, "gauss", 0.05), (152064, "zipf", 0.6)]):
        B = 5
        stride = ((V + 7) // 8) * 8 + 8
        g = torch.Generator().manual_seed(300 + case)
        x = torch.randn(B, stride, generator=g) * 3.0
        if kind == "flat":
            x[:] = 0.25
        elif kind == "masked":
            x[:, torch.rand(stride, generator=g) < 0.7] = float("-inf")
            x[:, V // 2] = 1.0
        elif kind == "zipf":
            x[:, :V] += W.ZipfLogits(V=V, seed=case, device="cpu").boost
        x[:, V:] = 1e4
        logits = x.to(dtype).cuda()
        vals = torch.rand(B, generator=g).cuda()
        gp, op = H.params_pair(mu_g=1.0, var_g=2.0, beta=0.8)
        alive0 = torch.tensor([1, 0, 1, 1, 1], dtype=torch.uint8)
        full, bare = H.GpuState(B, alive=alive0), H.GpuState(B, alive=alive0)
        for step in range(3):
            H.compare_step(logits, tau, 19, step, vals, gp, op, full, V=V)
            H.gpu_step(logits, tau, 19, step, vals, gp, bare, V=V, logprob=False)
            torch.cuda.synchronize()
            a, b = full.host(), bare.host()
            for k in ("tokens", "regret", "z", "alive", "stop_step"):
                np.testing.assert_array_equal(a[k].view(np.uint8), b[k].view(np.uint8), err_msg=f"case {case} step {step} {k}")
            assert (b["logprob"] == -7.0).all()                  # not written


# --------------------------------------------------------------------------- filtered draws
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_top_p_and_top_k_draws_match_the_oracle(dtype):
    _say(f"[case] filtered draws {dtype}")
    import oracle
    stats = {}
    cases = [(7, "gauss", 1.0), (513, "gauss", 0.6), (4099, "flat", 1.0), (9000, "masked", 0.8), (20000, "peaked", 1.0),
             (33000, "gauss", 2.5), (40000, "ties", 1.0), (152064, "zipf", 1.0), (152064, "zipf", 0.6)]
    filters = [dict(top_p=0.7), dict(top_p=0.1), dict(top_p=0.97), dict(top_k=1), dict(top_k=5), dict(top_k=50)]
    for case, (V, kind, tau) in enumerate(cases):
        B = 6
        stride = ((V + 7) // 8) * 8 + 8
        g = torch.Generator().manual_seed(800 + case)
        x = torch.randn(B, stride, generator=g) * 3.0
        if kind == "flat":
            x[:] = 0.5
        elif kind == "masked":
            x[:, torch.rand(stride, generator=g) < 0.8] = float("-inf")
            x[:, V // 3] = 1.0
        elif kind == "peaked":
            x[:, V - 2] = 30.0
        elif kind == "ties":
            x = torch.round(x)                                   # a handful of distinct values, huge tie groups
        elif kind == "zipf":
            x[:, :V] += W.ZipfLogits(V=V, seed=case, device="cpu").boost
        x[:, V:] = 1e4
        logits = x.to(dtype).cuda()
        vals = torch.rand(B, generator=g).cuda()
        for f in filters:
            gp, op = H.params_pair(mu_g=1.0, var_g=2.0, beta=3.0, **f)
            st = H.GpuState(B, alive=torch.tensor([1, 1, 0, 1, 1, 1], dtype=torch.uint8))
            for step in range(3):
                try:
                    got = H.compare_step(logits, tau, 61, step, vals, gp, op, st, V=V, stats=stats, entropy=(step == 1))
                except AssertionError as err:
                    raise AssertionError(f"case {case} V={V} {kind} tau={tau} {f} step {step}: {err}")
            if f.get("top_k") == 1:
                live = got["tokens"] >= 0
                assert (got["regret"][live] == 0).all()          # only modes are kept
    # a filter that keeps everything gives the bits of the plain step
    V, B = 5000, 4
    logits = _rand_logits(B, V, V, dtype, seed=3)
    vals = torch.zeros(B, device="cuda")
    outs = []
    for f in (dict(), dict(top_p=1.0), dict(top_k=V), dict(top_p=0.999999)):
        gp, _ = H.params_pair(stop_enabled=0, **f)
        st = H.GpuState(B)
        H.gpu_step(logits, 0.9, 8, 0, vals, gp, st)
        outs.append(st.host())
    for o in outs[1:3]:
        for k in ("tokens", "regret", "z"):
            np.testing.assert_array_equal(o[k].view(np.uint8), outs[0][k].view(np.uint8))
        # the filtered draw streams the row with 8 waves instead of 16: the softmax sum is associated differently
        np.testing.assert_allclose(o["logprob"], outs[0]["logprob"], rtol=2e-6, atol=2e-6)
    with pytest.raises(espo.EspoError):
        gp, _ = H.params_pair(top_p=0.5, top_k=3)
        H.gpu_step(logits, 0.9, 8, 0, vals, gp, H.GpuState(B))
    _say(f"  {stats}")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_filtered_draws_on_flat_rows_match_the_oracle(dtype):
    _say(f"[case] filtered draws, nuclei of hundreds of tokens {dtype}")
    # At temperature 1 and above the synthetic rows are flat: the kept set has from a few dozen to a few
    # thousand tokens, below the first trial floor on many rows.  These rows take the second trial floor,
    # the selection of the edge through bins (several hundred collected logits) and, for the widest
    # filters, the loop over successive winners.  V = 30000 has too few blocks for the bins and compares
    # all collected logits with each other instead.
    stats = {}
    for case, (V, B, tau, filters) in enumerate([
            (152064, 40, 1.0, [dict(top_p=0.7), dict(top_p=0.5), dict(top_p=0.85), dict(top_k=96), dict(top_k=400)]),
            (152064, 12, 1.3, [dict(top_p=0.7), dict(top_p=0.3), dict(top_k=1000)]),
            (30000, 12, 1.0, [dict(top_p=0.7), dict(top_p=0.9), dict(top_k=200)]),
            (100003, 12, 1.0, [dict(top_p=0.7), dict(top_k=150)])]):
        stride = ((V + 7) // 8) * 8 + 8
        g = torch.Generator().manual_seed(900 + case)
        x = torch.randn(B, stride, generator=g) * 3.0
        x[:, :V] += W.ZipfLogits(V=V, seed=40 + case, device="cpu").boost
        x[:, V:] = 1e4
        logits = x.to(dtype).cuda()
        vals = torch.rand(B, generator=g).cuda()
        for f in filters:
            gp, op = H.params_pair(mu_g=1.0, var_g=2.0, beta=3.0, stop_enabled=0, **f)
            st = H.GpuState(B)
            for step in range(2):
                try:
                    H.compare_step(logits, tau, 67, step, vals, gp, op, st, V=V, stats=stats)
                except AssertionError as err:
                    raise AssertionError(f"case {case} V={V} tau={tau} {f} step {step}: {err}")
    _say(f"  {stats}")


def test_top_p_at_the_edge_of_the_kept_set_is_decided_like_the_oracle():
    _say("[case] filtered draws, mass next to p")
    # One tall token and many equal ones: the equal ones are kept iff the tall one's probability is below p.
    # p is set to that probability rounded to fp32, so the comparison is closer than fp32 sums can tell
    # and the kernel has to repeat it in double.
    B = 16
    for V, a, tau in [(1000, 5.0, 1.0), (30000, 9.5, 1.0), (152064, 11.0, 0.6)]:
        x = torch.zeros(B, V)
        x[:, 17] = a
        inv = np.float64(np.float32(1.0) / np.float32(tau))
        pa = 1.0 / (1.0 + (V - 1) * np.exp(-np.float64(np.float32(a)) * inv))
        for p_val in (float(np.float32(pa)), float(np.nextafter(np.float32(pa), np.float32(1))),
                      float(np.nextafter(np.float32(pa), np.float32(0)))):
            if not 0.0 < p_val < 1.0:
                continue
            gp, op = H.params_pair(stop_enabled=0, top_p=p_val)
            st = H.GpuState(B)
            for step in range(2):
                H.compare_step(x.cuda(), tau, 99, step, torch.zeros(B, device="cuda"), gp, op, st)


# --------------------------------------------------------------------------- HIP graph capture
def test_steps_captured_in_a_graph_replay_like_eager_launches():
    _say("[case] graph capture and replay")
    # The library allocates nothing and synchronises nothing, so its launches can be captured.
    # A graph of three consecutive steps plus the advantage pass (padded and packed) and the whitening
    # of its result is replayed several times, with
    # eager work and synchronisations in between, from a restored state; every replay must give
    # the bits of the eager run.
    B, V, T = 560, 6000, 700                                 # more rows than resident workgroups
    gen = W.ZipfLogits(V=V, seed=21, device="cuda")
    logits = [gen.rows(B, step=s) for s in range(3)]
    vals = [W.step_values(B, 21, s, 0.2, 1.0, device="cuda") for s in range(3)]
    gp, _ = H.params_pair(mu_g=1.0, var_g=2.0, beta=0.6)
    r, v, L, stp = W.advantage_batch(B=B, T=T, len_lo=1, seed=8, device="cuda")
    z0 = torch.rand(B, device="cuda") - 0.5
    cu = torch.zeros(B + 1, dtype=torch.int64, device="cuda")
    cu[1:] = torch.cumsum(L.long(), 0)
    vp = v[torch.arange(T, device="cuda")[None, :] < L[:, None]].contiguous()
    term = torch.rand(B, device="cuda")
    ws = torch.empty(espo.espo_whiten_workspace_bytes(B, T), dtype=torch.uint8, device="cuda")
    # the last step runs with every row split in three: the tickets in its workspace must be back at zero after every replay
    step_ws = torch.zeros(espo.espo_debug_step_workspace_bytes(B, 3), dtype=torch.uint8, device="cuda")
    # the advantage pass that sorts its later rows itself (B > 512) and the whitening from its rows' sums: the
    # two words at the head of their workspace must be back at zero after every replay, too
    adv_ws = torch.zeros(espo.espo_advantages_ws_bytes(B), dtype=torch.uint8, device="cuda")

    def fresh():
        st = H.GpuState(B, z=z0)
        st.out = [torch.empty(B, dtype=torch.int32, device="cuda") for _ in range(3)]
        st.td, st.adv = torch.empty(B, T, device="cuda"), torch.empty(B, T, device="cuda")
        st.wh = torch.full((B, T), 7.0, device="cuda")
        st.tdp, st.advp = torch.empty_like(vp), torch.empty_like(vp)
        st.td2, st.adv2 = torch.empty(B, T, device="cuda"), torch.empty(B, T, device="cuda")
        st.wh2 = torch.full((B, T), 7.0, device="cuda")
        return st

    def work(st):
        for s in range(3):
            espo.espo_step(logits[s], 0.6, 77, s, vals[s], gp, st.z, st.alive, st.stop_step, st.out[s], st.regret,
                           st.logprob, entropy=st.entropy, **(dict(workspace=step_ws, chunks=3) if s == 2 else dict()))
        espo.espo_advantages(r, v, L, stp, -1.0, 1.0, 0.95, st.td, st.adv)
        espo.espo_whiten(st.adv, L, st.wh, ws)
        espo.espo_advantages_packed(vp, cu, stp, -1.0, 1.0, 0.95, st.tdp, st.advp, terminal_reward=term)
        espo.espo_advantages_ws(r, v, L, stp, -1.0, 1.0, 0.95, st.td2, st.adv2, adv_ws)
        espo.espo_whiten_from_ws(st.adv2, L, st.wh2, adv_ws)

    eager = fresh()
    work(eager)
    torch.cuda.synchronize()
    want = {k: getattr(eager, k).clone() for k in ("z", "alive", "stop_step", "regret", "logprob", "entropy", "td", "adv", "wh", "tdp", "advp", "td2", "adv2", "wh2")}
    assert torch.equal(want["adv2"], want["adv"]) and torch.equal(want["td2"], want["td"])
    want_tok = [t.clone() for t in eager.out]
    assert int(want["alive"].sum()) < B                      # some rows stop inside the graph

    st = fresh()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        work(st)                                             # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        work(st)
    for replay in range(4):
        st.z.copy_(z0); st.alive.fill_(1); st.stop_step.fill_(-1)       # restore the state the graph starts from
        st.td.fill_(7.0); st.adv.fill_(7.0); st.regret.fill_(-7.0)
        st.wh.fill_(7.0); st.tdp.fill_(7.0); st.advp.fill_(7.0); ws.fill_(0x5a)
        st.td2.fill_(7.0); st.adv2.fill_(7.0); st.wh2.fill_(7.0); adv_ws[256:].fill_(0x5a)
        for t in st.out:
            t.fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert not bool(step_ws.any()) and not bool(adv_ws[:256].any()), replay
        for k, w in want.items():
            assert torch.equal(getattr(st, k), w), (replay, k)
        for a, b in zip(st.out, want_tok):
            assert torch.equal(a, b), replay
        H.gpu_step(logits[0], 0.6, 5, replay, vals[0], gp, fresh())      # unrelated eager work between replays
        torch.cuda.synchronize()
