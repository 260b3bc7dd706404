#!/usr/bin/env python3
"""Benchmark of the ESPO per-step hot path on one MI355X.

A "step" is one `espo_step` call over a batch of 512 trajectories with Qwen-vocabulary
bf16 logits (the sustained-rollout workload: state carried from step to step, about a
quarter of the rows driven over the stop threshold at seeded steps, dead rows skipped).
Every step reads its own logit buffer, all of them generated on the device before the
timed region (288 GB of HBM hold hundreds of 156 MB steps), so no step can be served
from a cache.  The companion `espo_advantages` pass is timed on the B=1024, T=16384 batch
and reported in the same JSON line, as are two bare kernels of the same memory traffic
(the ceilings this GPU's memory system sets for kernels of these shapes), the launch
duration against the number of live rows on the heavy-termination rollout, and the CPU
oracle on a bounded sample, whose tokens and state are compared with the GPU's for the
same steps.

    python bench.py [--gpus 1] [--steps K] [--warmup W]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
STEP_SCALAR_BYTES = 34         # per live row: value, z in/out, alive in/out, stop step, token, regret, logprob
B_STEP, V_STEP = 512, 152064
B_ADV, T_ADV = 1024, 16384
NEAR_TIE = 1e-6                # relative gap of the oracle's two best scores below which its runner-up is accepted


def _traffic_from_profiles(kernel: str):
    """HBM bytes per launch measured with rocprofv3 counters, and the run they were measured on, if a
    summary was committed (counters cannot be read from inside this process)."""
    path = os.path.join(ROOT, "profiles", f"traffic_{kernel}.txt")
    val, where = None, None
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                val = float(line.split(":")[1])
            if line.startswith("measured_on:"):
                where = line.split(":", 1)[1].strip()
    except OSError:
        pass
    return val, where


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--adv-reps", type=int, default=60)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copies", type=int, default=0,
                    help="also launch this many plain 1 GiB copies (known traffic, for counter calibration; untimed)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="oracle time to spend on the CPU baseline")
    ap.add_argument("--no-live-curve", action="store_true",
                    help="skip the heavy-termination rollout (B=1024, 256 steps, 60%% of rows planted to stop) that "
                         "reports the launch duration against the number of live rows")
    ap.add_argument("--only-step", action="store_true", help="time the headline step loop only (for profiler runs)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU; rows shard over GPUs without any exchange, "
              "so a multi-GPU figure would be N independent copies of this run. Use --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2605_29860_amd as espo
    from paper_2605_29860_amd import workloads as W

    if not os.path.exists(espo.library_path()):
        from paper_2605_29860_amd import build
        build.build_library()
    espo.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    K, Wm = args.steps, args.warmup
    total = K + Wm
    seed, tau = 3, 0.6

    def timer():
        return torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(n, call, warm=0):
        """Microseconds per call of n back-to-back calls between two events on the launch stream."""
        for i in range(warm):
            call(i)
        torch.cuda.synchronize()
        ev = timer()
        ev[0].record()
        for i in range(n):
            call(i)
        ev[1].record()
        torch.cuda.synchronize()
        return ev[0].elapsed_time(ev[1]) / n * 1e3

    # ------------------------------------------------------------------ inputs, resident in HBM (untimed)
    gen = W.ZipfLogits(V=V_STEP, seed=seed, device=dev)
    plant = W.RegretPlant.make(B_STEP, V_STEP, 0.25, Wm, max(Wm, total - 24), seed)
    logits = torch.empty(total, B_STEP, V_STEP, dtype=torch.bfloat16, device=dev)
    values = torch.empty(total, B_STEP, dtype=torch.float32, device=dev)
    for s in range(total):
        gen.rows(B_STEP, step=s, out=logits[s])
        plant.apply(logits[s], s)
        values[s] = W.step_values(B_STEP, seed, s, 0.2, 1.0, device=dev)
    params = espo.EspoParams(**W.RolloutParams().as_dict())
    tokens = torch.empty(B_STEP, dtype=torch.int32, device=dev)
    regret = torch.empty(B_STEP, dtype=torch.float32, device=dev)
    logprob = torch.empty(B_STEP, dtype=torch.float32, device=dev)
    nws = espo.espo_step_workspace_bytes(B_STEP, V_STEP, torch.bfloat16)      # 0 in this version: one workgroup per row
    step_ws = torch.zeros(nws, dtype=torch.uint8, device=dev) if nws else None

    def run(first, last, z, alive, ss, events=None, entropy=None, params=params, lp=logprob, temperature=tau, ws=step_ws, **layout):
        for s in range(first, last):
            if events is not None:
                events[s - first][0].record()
            espo.espo_step(logits[s], temperature, seed, s, values[s], params, z, alive, ss, tokens, regret, lp,
                           entropy=entropy, workspace=ws, **layout)
            if events is not None:
                events[s - first][1].record()

    def fresh_state(**kw):
        z, alive, ss = W.initial_state(B_STEP, device=dev)
        run(0, Wm, z, alive, ss, **kw)            # warmup steps are the first steps of the trajectory
        torch.cuda.synchronize()
        return z, alive, ss

    if args.calibration_copies:
        src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(args.calibration_copies):
            espo.espo_debug_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    # ------------------------------------------------------------------ the first steps once more, kept for the parity check
    # tokens, regret and state after each of the first steps of the same trajectory (untimed): what the CPU oracle
    # is compared with further down
    keep = 0 if args.no_cpu_baseline or args.only_step else min(total, 160)
    hist = {"tokens": torch.empty(keep, B_STEP, dtype=torch.int32, device=dev),
            "regret": torch.empty(keep, B_STEP, dtype=torch.float32, device=dev),
            "z": torch.empty(keep, B_STEP, dtype=torch.float32, device=dev),
            "alive": torch.empty(keep, B_STEP, dtype=torch.uint8, device=dev),
            "stop_step": torch.empty(keep, B_STEP, dtype=torch.int32, device=dev)}
    zp, ap_, sp = W.initial_state(B_STEP, device=dev)
    for s in range(keep):
        run(s, s + 1, zp, ap_, sp)
        for k, t in (("tokens", tokens), ("regret", regret), ("z", zp), ("alive", ap_), ("stop_step", sp)):
            hist[k][s].copy_(t)
    torch.cuda.synchronize()

    # ------------------------------------------------------------------ timed region: exactly K steps
    z, alive, ss = fresh_state()
    region = timer()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    region[0].record()                           # on the stream the kernels are launched on (torch's current one)
    run(Wm, total, z, alive, ss)
    region[1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    region_ms = region[0].elapsed_time(region[1])
    ss_h = ss.cpu().numpy()
    steps_idx = np.arange(Wm, total)
    live = ((ss_h[None, :] < 0) | (ss_h[None, :] >= steps_idx[:, None])).sum(1)   # rows decoded at each timed step
    live_rows = int(live.sum())
    step_bytes = live * (V_STEP * 2 + STEP_SCALAR_BYTES) + (B_STEP - live) * 1
    step_gbs = float(step_bytes.sum() / (region_ms * 1e-3) / 1e9)   # events around the K back-to-back launches
    step_us = region_ms / K * 1e3
    step_traffic, step_traffic_on = _traffic_from_profiles("espo_step")

    out = {
        "metric": "logit rows/sec & HBM GB/s (fused step, V=152064 bf16); advantages tokens/sec",
        "value": live_rows / wall, "unit": "rows/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": wall / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "sustained rollout step loop: B=512, V=152064 bf16, state carried, "
                               "~25% of rows planted to stop, one resident logit buffer per step",
                   "B": B_STEP, "V": V_STEP, "logits_dtype": "bf16", "temperature": tau, "live_rows_mean": float(live.mean()),
                   "live_rows_last": int(live[-1])},
        "step_hbm_gbs_wall": float(step_bytes.sum() / wall / 1e9),
        "roofline": {"kernel": "espo_step_kernel<bf16>", "bound": "hbm", "achieved": step_gbs,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": step_gbs / HBM_PEAK_GBS,
                     "avg_launch_us": step_us,
                     "algorithmic_bytes_per_launch": float(step_bytes.mean()),
                     "traffic": step_traffic, "traffic_measured_on": step_traffic_on},
    }
    if args.only_step:
        print(json.dumps(out))
        return 0

    # same K steps again with an event pair around every launch (each pair adds a few microseconds of its own)
    z2, alive2, ss2 = fresh_state()
    ev = [timer() for _ in range(K)]
    run(Wm, total, z2, alive2, ss2, events=ev)
    torch.cuda.synchronize()
    assert torch.equal(ss2, ss) and torch.equal(z2, z), "replay of the timed steps is not deterministic"
    kern_ms = np.array([a.elapsed_time(b) for a, b in ev])
    out["roofline"]["avg_launch_us_event_pair_each"] = float(kern_ms.mean() * 1e3)

    def variant(name, **kw):
        """The same K steps through another form of the call; the trajectory must not change unless said so."""
        zz, aa, sz = fresh_state(**kw)
        r = timer()
        r[0].record()
        run(Wm, total, zz, aa, sz, **kw)
        r[1].record()
        torch.cuda.synchronize()
        return r[0].elapsed_time(r[1]) / K * 1e3, zz, aa, sz

    # every row split over several workgroups that combine through a workspace (diagnostics entry point): the finer
    # grain that was meant to fill the GPU better at this batch size, measured here beside the layout espo_step uses
    split = {}
    for waves, chunks in ((16, 2), (8, 2), (4, 8)):
        ws_split = torch.zeros(espo.espo_debug_step_workspace_bytes(B_STEP, chunks), dtype=torch.uint8, device=dev)
        us6, z6, _, ss6 = variant("split", ws=ws_split, waves=waves, chunks=chunks)
        assert torch.equal(ss6, ss) and torch.equal(z6, z), "the layout changed the trajectory"
        assert not bool(ws_split.any()), "a split step left its workspace non-zero"
        split[f"{chunks}_chunks_of_{waves}_waves"] = us6
    # with the optional entropy output (the kernel's other instantiation)
    entropy = torch.empty(B_STEP, dtype=torch.float32, device=dev)
    ent_us, z3, alive3, ss3 = variant("entropy", entropy=entropy)
    assert torch.equal(ss3, ss) and torch.equal(z3, z), "the entropy output changed the trajectory"
    # without the log-probability output (no softmax sum is formed then)
    nolp_us, z5, _, ss5 = variant("nolp", lp=None)
    assert torch.equal(ss5, ss) and torch.equal(z5, z), "dropping the log-probability output changed the trajectory"
    # with the nucleus filter of the paper's evaluation set-up (top-p 0.7), at the rollout temperature and at 1.0
    params_p = espo.EspoParams(**{**W.RolloutParams().as_dict(), "top_p": 0.7})
    topp_us, _, alive4, _ = variant("top_p", params=params_p)
    # at temperature 1 the regrets of these rows are large and most rows would stop within a few steps: the
    # comparison with the plain step is made with the stop rule switched off, all 512 rows live in both runs
    off = {**W.RolloutParams().as_dict(), "stop_enabled": 0}
    topp1_us, _, alive7, _ = variant("top_p_tau1", params=espo.EspoParams(**{**off, "top_p": 0.7}), temperature=1.0)
    plain1_us, _, _, _ = variant("tau1", params=espo.EspoParams(**off), temperature=1.0)
    frac_of = lambda us: step_gbs / HBM_PEAK_GBS * step_us / us
    out["step_rows_split_over_workgroups"] = {"avg_launch_us": split, "one_workgroup_per_row_us": step_us,
                                              "note": "espo_debug_step with forced chunks; same tokens, regret, state and masks"}
    out["step_with_entropy"] = {"avg_launch_us": ent_us, "frac": frac_of(ent_us),
                                "mean_entropy_last_step": float(entropy[alive3 > 0].mean()) if bool((alive3 > 0).any()) else None}
    out["step_without_logprob"] = {"avg_launch_us": nolp_us, "frac": frac_of(nolp_us),
                                   "note": "logprob = NULL: token, regret, state and masks only, no softmax sum"}
    out["step_top_p_0.7"] = {"avg_launch_us": topp_us, "live_rows_last": float((alive4 > 0).sum()),
                             "note": "filtered draw: own kernel instantiation, reads parts of the row again"}
    out["step_top_p_0.7_tau1"] = {"avg_launch_us": topp1_us, "plain_step_at_tau1_us": plain1_us,
                                  "ratio_to_plain": topp1_us / plain1_us, "live_rows_last": float((alive7 > 0).sum()),
                                  "note": "the paper's evaluation sampling (temperature 1.0, nucleus 0.7) on the same rows, stop rule "
                                          "off in both runs (all rows live)"}

    # ------------------------------------------------------------------ ceiling: a bare streaming read of the same buffers
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    read_us = timed(K, lambda i: espo.espo_debug_read(logits[Wm + i], sink), warm=4)
    read_gbs = B_STEP * V_STEP * 2 / read_us / 1e3
    out["roofline"]["ceiling_gbs"] = read_gbs
    out["roofline"]["frac_of_ceiling"] = step_gbs / read_gbs
    out["roofline"]["ceiling"] = {"kernel": "espo_debug_read: nontemporal 16-byte loads of a [512,152064] bf16 buffer, nothing else",
                                  "bytes_per_launch": B_STEP * V_STEP * 2, "avg_launch_us": read_us,
                                  "frac_of_peak": read_gbs / HBM_PEAK_GBS}

    # ------------------------------------------------------------------ advantages (B=1024, T=16384), rotated buffers
    nbuf = 8   # 2.1 GB of inputs and outputs in rotation: a re-read can never come from the 256 MB Infinity Cache
    adv_in = [W.advantage_batch(B=B_ADV, T=T_ADV, seed=50 + i, device=dev) for i in range(nbuf)]
    adv_out = [(torch.empty(B_ADV, T_ADV, device=dev), torch.empty(B_ADV, T_ADV, device=dev)) for _ in range(nbuf)]
    def adv_call(i):
        r, v, L, s = adv_in[i % nbuf]
        td, ad = adv_out[i % nbuf]
        espo.espo_advantages(r, v, L, s, -1.0, 1.0, 0.95, td, ad)
    for i in range(nbuf):
        adv_call(i)
    torch.cuda.synchronize()
    aev = [timer() for _ in range(args.adv_reps)]
    aregion = timer()
    ta = time.perf_counter()
    aregion[0].record()
    for i in range(args.adv_reps):
        adv_call(i)
    aregion[1].record()
    torch.cuda.synchronize()
    adv_wall = time.perf_counter() - ta
    adv_region_ms = aregion[0].elapsed_time(aregion[1])
    for i in range(args.adv_reps):               # again, one event pair per launch
        aev[i][0].record()
        adv_call(i)
        aev[i][1].record()
    torch.cuda.synchronize()
    adv_ms = np.array([a.elapsed_time(b) for a, b in aev])
    valid = np.array([int(adv_in[i % nbuf][2].sum()) for i in range(args.adv_reps)])
    adv_bytes = valid * 16 + (B_ADV * T_ADV - valid) * 8 + B_ADV * 5
    adv_gbs = float(adv_bytes.sum() / (adv_region_ms * 1e-3) / 1e9)
    adv_traffic, adv_traffic_on = _traffic_from_profiles("espo_advantages")

    # ceiling: a flat sweep with the same read / write mix (8 bytes read per valid token, 8 written per position)
    rd_bytes = int(valid.mean()) * 8 // 16 * 16
    wr_bytes = B_ADV * T_ADV * 8
    sw_src = [torch.empty(rd_bytes // 4, device=dev).normal_() for _ in range(nbuf)]
    sw_dst = [torch.empty(wr_bytes // 4, device=dev) for _ in range(nbuf)]
    sweep_us = timed(args.adv_reps, lambda i: espo.espo_debug_sweep(sw_src[i % nbuf], rd_bytes, sw_dst[i % nbuf], wr_bytes), warm=nbuf)
    sweep_gbs = (rd_bytes + wr_bytes) / sweep_us / 1e3
    del sw_src, sw_dst
    # and the same traffic in the pass's own layout (four [B, T] arrays, inputs read below the lengths), no dependency
    def padded_call(i):
        r, v, L, s = adv_in[i % nbuf]
        td, ad = adv_out[i % nbuf]
        espo.espo_debug_sweep_padded(r, v, L, td, ad)
    padded_us = timed(args.adv_reps, padded_call, warm=nbuf)
    padded_gbs = float(adv_bytes.mean()) / padded_us / 1e3

    # the same batches in the terminal-reward form (no reward array, padding left to the caller's mask)
    rows_all = torch.arange(B_ADV, device=dev)
    adv_term = [r[rows_all, (L - 1).clamp(min=0).long()].contiguous() for r, v, L, s in adv_in]
    def advt_call(i):
        r, v, L, s = adv_in[i % nbuf]
        td, ad = adv_out[i % nbuf]
        espo.espo_advantages_terminal(v, L, s, adv_term[i % nbuf], -1.0, 1.0, 0.95, td, ad, zero_padding=False)
    advt_us = timed(args.adv_reps, advt_call, warm=nbuf)
    advt_bytes = float(np.mean(valid * 12 + B_ADV * 9))

    # the same trajectories stored back to back: nothing but the valid tokens is read or written
    pk = []
    for r, v, L, s in adv_in:
        mask = torch.arange(T_ADV, device=dev)[None, :] < L[:, None]
        cu = torch.zeros(B_ADV + 1, dtype=torch.int64, device=dev)
        cu[1:] = torch.cumsum(L.long(), 0)
        vp, rp = v[mask].contiguous(), r[mask].contiguous()
        pk.append((vp, rp, cu, torch.empty_like(vp), torch.empty_like(vp)))
    del mask
    def pk_call(i, dense):
        vp, rp, cu, td, ad = pk[i % nbuf]
        s = adv_in[i % nbuf][3]
        if dense:
            espo.espo_advantages_packed(vp, cu, s, -1.0, 1.0, 0.95, td, ad, rewards=rp)
        else:
            espo.espo_advantages_packed(vp, cu, s, -1.0, 1.0, 0.95, td, ad, terminal_reward=adv_term[i % nbuf])
    pk_us = {dense: timed(args.adv_reps, lambda i, d=dense: pk_call(i, d), warm=nbuf) for dense in (True, False)}
    pk_bytes = {True: float(np.mean(valid * 16 + B_ADV * 9)), False: float(np.mean(valid * 12 + B_ADV * 13))}
    del pk

    # whitening of the advantages over the valid tokens (two passes over A, one store)
    wh_ws = torch.empty(espo.espo_whiten_workspace_bytes(B_ADV, T_ADV), dtype=torch.uint8, device=dev)
    def wh_call(i):
        td, ad = adv_out[i % nbuf]
        espo.espo_whiten(ad, adv_in[i % nbuf][2], td, wh_ws)      # td serves as the output buffer here
    for i in range(nbuf):
        adv_call(i)                                               # the advantages these whiten
    wh_us = timed(args.adv_reps, wh_call, warm=nbuf)
    wh_bytes = float(np.mean(valid * 12 + B_ADV * 8))

    # the pair with a workspace between them: the advantage pass sorts its later rows by length inside the launch and
    # leaves every row's sums, the whitening starts from those; and the same pass with an order from the caller,
    # written beforehand or in the region
    aw_ws = [torch.zeros(espo.espo_advantages_ws_bytes(B_ADV), dtype=torch.uint8, device=dev) for _ in range(nbuf)]
    aw_order = [torch.empty(B_ADV, dtype=torch.int32, device=dev) for _ in range(nbuf)]
    def aw_call(i, ordered=False, order_now=False):
        r, v, L, s = adv_in[i % nbuf]
        td, ad = adv_out[i % nbuf]
        if order_now:
            espo.espo_length_order(L, T_ADV, aw_order[i % nbuf])
        espo.espo_advantages_ws(r, v, L, s, -1.0, 1.0, 0.95, td, ad, aw_ws[i % nbuf], aw_order[i % nbuf] if ordered else None)
    for i in range(nbuf):
        espo.espo_length_order(adv_in[i][2], T_ADV, aw_order[i])
    aw_us = timed(args.adv_reps, aw_call, warm=nbuf)
    aw_ord_us = timed(args.adv_reps, lambda i: aw_call(i, ordered=True), warm=nbuf)
    aw_ord_now_us = timed(args.adv_reps, lambda i: aw_call(i, ordered=True, order_now=True), warm=nbuf)
    order_us = timed(args.adv_reps, lambda i: espo.espo_length_order(adv_in[i % nbuf][2], T_ADV, aw_order[i % nbuf]), warm=nbuf)
    wh_tmp = torch.empty(B_ADV, T_ADV, device=dev)
    def whw_call(i):
        td, ad = adv_out[i % nbuf]
        espo.espo_whiten_from_ws(ad, adv_in[i % nbuf][2], wh_tmp, aw_ws[i % nbuf])
    whw_us = timed(args.adv_reps, whw_call, warm=nbuf)
    def pair_call(i, fused):
        td, ad = adv_out[i % nbuf]
        if fused:
            aw_call(i)
            espo.espo_whiten_from_ws(ad, adv_in[i % nbuf][2], wh_tmp, aw_ws[i % nbuf])
        else:
            adv_call(i)
            espo.espo_whiten(ad, adv_in[i % nbuf][2], wh_tmp, wh_ws)
    pair_us = {f: timed(args.adv_reps, lambda i, f=f: pair_call(i, f), warm=nbuf) for f in (False, True)}
    # the terminal-reward form of the same pair (no reward array, no zero fill)
    def awt_call(i):
        r, v, L, s = adv_in[i % nbuf]
        td, ad = adv_out[i % nbuf]
        espo.espo_advantages_terminal_ws(v, L, s, adv_term[i % nbuf], -1.0, 1.0, 0.95, td, ad, aw_ws[i % nbuf], zero_padding=False)
    awt_us = timed(args.adv_reps, awt_call, warm=nbuf)
    def pair_t_call(i, fused):
        td, ad = adv_out[i % nbuf]
        if fused:
            awt_call(i)
            espo.espo_whiten_from_ws(ad, adv_in[i % nbuf][2], wh_tmp, aw_ws[i % nbuf])
        else:
            advt_call(i)
            espo.espo_whiten(ad, adv_in[i % nbuf][2], wh_tmp, wh_ws)
    pair_t_us = {f: timed(args.adv_reps, lambda i, f=f: pair_t_call(i, f), warm=nbuf) for f in (False, True)}
    del wh_tmp

    # ------------------------------------------------------------------ batch-boundary statistics (B=512, T=8192)
    bs_sets = [W.regret_batch(512, 8192, seed=70 + i, device=dev) for i in range(nbuf)]   # 134 MB in rotation
    bs_out = torch.zeros(espo.BATCH_RESULT_BYTES, dtype=torch.uint8, device=dev)
    bs_ws = torch.zeros(espo.espo_batch_stats_workspace_bytes(512, 8192), dtype=torch.uint8, device=dev)
    def bs_call(i):
        g, L, s = bs_sets[i % nbuf]
        espo.espo_batch_stats(g, L, s, 1.0, 2.0, 7.0, bs_out, bs_ws)
    bs_us = timed(args.adv_reps, bs_call, warm=nbuf)
    bs_bytes = float(np.mean([int(bs_sets[i % nbuf][1].sum()) * 4 + 512 * 5 for i in range(args.adv_reps)]))
    bs_res = espo.read_batch_result(bs_out)
    del bs_sets

    # ------------------------------------------------------------------ launch duration vs live rows (B=1024)
    curve = None
    if not args.no_live_curve:
        Bc, Sc, seed_c, blk = 1024, 256, 4, 8
        plant_c = W.RegretPlant.make(Bc, V_STEP, 0.6, 14, 150, seed_c)
        gen_c = W.ZipfLogits(V=V_STEP, seed=seed_c, device=dev)
        logits_c = torch.empty(Sc, Bc, V_STEP, dtype=torch.bfloat16, device=dev)   # 80 GB, all steps resident
        values_c = torch.empty(Sc, Bc, dtype=torch.float32, device=dev)
        for t in range(Sc):                                                # generation: untimed
            gen_c.rows(Bc, step=t, out=logits_c[t])
            plant_c.apply(logits_c[t], t)
            values_c[t] = W.step_values(Bc, seed_c, t, 0.2, 1.0, device=dev)
        torch.cuda.synchronize()
        zc_, ac_, sc_ = W.initial_state(Bc, device=dev)
        tok_c = torch.empty(Bc, dtype=torch.int32, device=dev)
        reg_c = torch.empty(Bc, dtype=torch.float32, device=dev)
        lp_c = torch.empty(Bc, dtype=torch.float32, device=dev)   # with the log-probability, as in the headline figure
        cev = [timer() for _ in range(Sc // blk)]                 # one event pair per block of 8 consecutive launches
        for t in range(Sc):
            if t % blk == 0:
                cev[t // blk][0].record()
            espo.espo_step(logits_c[t], tau, seed_c, t, values_c[t], params, zc_, ac_, sc_, tok_c, reg_c, lp_c)
            if t % blk == blk - 1:
                cev[t // blk][1].record()
        torch.cuda.synchronize()
        ss_c = sc_.cpu().numpy()
        live_c = ((ss_c[None, :] < 0) | (ss_c[None, :] >= np.arange(Sc)[:, None])).sum(1)   # rows decoded at each step
        live_b = live_c.reshape(-1, blk).mean(1)
        cus = np.array([a.elapsed_time(b) * 1e3 / blk for a, b in cev])
        curve = []
        for lo in range(400, 1025, 104):                                   # six bins of live rows
            sel = (live_b > lo - 104) & (live_b <= lo)
            if sel.any():
                rows_m, us_m = float(live_b[sel].mean()), float(cus[sel].mean())
                curve.append({"live_rows": rows_m, "launches": int(sel.sum()) * blk, "us_per_launch": us_m,
                              "rows_per_s": rows_m / us_m * 1e6,
                              "gbs": (rows_m * (V_STEP * 2 + STEP_SCALAR_BYTES) + (Bc - rows_m)) / us_m / 1e3})
        if curve:
            top = curve[-1]
            for c in curve:       # 1.0 = time falls in proportion to the live rows, measured from the fullest bin
                c["us_over_proportional"] = c["us_per_launch"] / (top["us_per_launch"] * c["live_rows"] / top["live_rows"])
        # What the position of the done rows in the batch costs: the mask the rollout ended with, as it is
        # and with the same number of live rows moved to the front (what a caller gets who keeps the batch
        # compacted), stop rule and end-of-sequence off so that the mask stays as it is.
        fixed = espo.EspoParams(**{**W.RolloutParams().as_dict(), "stop_enabled": 0, "eos_id": -1})
        n_live_end = int((ac_ > 0).sum())
        masks = {"as_the_rollout_left_them": ac_.clone(),
                 "live_rows_first": (torch.arange(Bc, device=dev) < n_live_end).to(torch.uint8)}
        position = {"live_rows": n_live_end}
        for name, mask in masks.items():
            zz_ = torch.zeros(Bc, dtype=torch.float32, device=dev)
            for t in range(Sc - 72, Sc - 64):                                  # warm-up
                espo.espo_step(logits_c[t], tau, seed_c, t, values_c[t], fixed, zz_, mask, sc_, tok_c, reg_c, lp_c)
            r = timer()
            r[0].record()
            for t in range(Sc - 64, Sc):
                espo.espo_step(logits_c[t], tau, seed_c, t, values_c[t], fixed, zz_, mask, sc_, tok_c, reg_c, lp_c)
            r[1].record()
            torch.cuda.synchronize()
            assert int((mask > 0).sum()) == n_live_end
            position[name + "_us"] = r[0].elapsed_time(r[1]) / 64 * 1e3
        del logits_c

    # ------------------------------------------------------------------ CPU oracle on a bounded sample, compared with the GPU
    cpu, parity = None, None
    if not args.no_cpu_baseline:
        import oracle
        oracle.build_oracle()
        op = oracle.OracleParams(**W.RolloutParams().as_dict())
        zc, ac, sc = (np.zeros(B_STEP, np.float32), np.ones(B_STEP, np.uint8), np.full(B_STEP, -1, np.int32))
        cpu_s, cpu_rows, cpu_steps = 0.0, 0, 0
        hist_h = {k: v.cpu().numpy() for k, v in hist.items()}
        parity = {"parity_checked_steps": 0, "parity_checked_rows": 0, "parity_near_ties": 0, "parity_ok": True}
        while cpu_s < args.cpu_seconds and cpu_steps < keep:       # the first steps of the same trajectory
            bits = W.to_host_bits(logits[cpu_steps])               # copy to the host: untimed
            vals_h = values[cpu_steps].cpu().numpy()
            if cpu_steps == 0:
                cpu_first_bits, cpu_first_vals = bits, vals_h
            live_before = int(ac.sum())
            cpu_rows += live_before
            z0, a0, s0 = zc.copy(), ac.copy(), sc.copy()
            tc = time.perf_counter()
            ref = oracle.step(bits, tau, seed, cpu_steps, vals_h, op, zc, ac, sc)
            cpu_s += time.perf_counter() - tc
            # the GPU's tokens, regret and state after the same step (untimed)
            g_tok = hist_h["tokens"][cpu_steps]
            mism = np.nonzero(g_tok != ref["tokens"])[0]
            if len(mism):                                          # the oracle's runner-up is accepted in a near tie
                forced = np.full(B_STEP, -1, np.int32)
                for b in mism:
                    s1, s2 = ref["best_score"][b], ref["second_score"][b]
                    if g_tok[b] == ref["second_token"][b] and (s1 - s2) <= NEAR_TIE * abs(s1):
                        forced[b] = g_tok[b]
                    else:
                        parity["parity_ok"] = False
                        parity["first_mismatch"] = {"step": cpu_steps, "row": int(b), "gpu": int(g_tok[b]), "oracle": int(ref["tokens"][b])}
                if not parity["parity_ok"]:
                    break
                parity["parity_near_ties"] += len(mism)
                zc, ac, sc = z0, a0, s0
                ref = oracle.step(bits, tau, seed, cpu_steps, vals_h, op, zc, ac, sc, forced_tokens=forced)
            same = (np.array_equal(g_tok, ref["tokens"])
                    and np.array_equal(hist_h["regret"][cpu_steps].view(np.uint32), ref["regret"].view(np.uint32))
                    and np.array_equal(hist_h["z"][cpu_steps].view(np.uint32), zc.view(np.uint32))
                    and np.array_equal(hist_h["alive"][cpu_steps], ac)
                    and np.array_equal(hist_h["stop_step"][cpu_steps], sc))
            if not same:
                parity["parity_ok"] = False
                parity["first_mismatch"] = {"step": cpu_steps, "what": "regret, state or masks"}
                break
            parity["parity_checked_steps"] += 1
            parity["parity_checked_rows"] += live_before
            cpu_steps += 1
        r, v, L, s = [x.cpu().numpy() for x in adv_in[0]]
        tc = time.perf_counter()
        oracle.advantages(r, v, L, s, -1.0, 1.0, 0.95, want_scale=False)
        cpu_adv_s = time.perf_counter() - tc
        # the advantage pass on that batch against the oracle (untimed): errors against the scale of the terms summed
        td_o, adv_o, scale = oracle.advantages(r, v, L, s, -1.0, 1.0, 0.95)
        adv_call(0)
        torch.cuda.synchronize()
        e_adv = np.abs(adv_out[0][1].cpu().numpy().astype(np.float64) - adv_o)
        e_td = np.abs(adv_out[0][0].cpu().numpy().astype(np.float64) - td_o)
        parity["advantages_worst_scaled_error"] = float((e_adv / np.maximum(scale, 1e-30)).max())
        parity["advantages_worst_td_error"] = float(e_td.max())
        parity["advantages_parity_ok"] = bool((e_adv <= 2e-6 * np.maximum(scale, 1e-30)).all() and e_td.max() <= 1e-6)
        # the same oracle on one thread, on a slice of the first step (it is deliberately plain code)
        nthreads = oracle.num_threads()
        oracle.set_threads(1)
        n1 = 96
        z1, a1, s1 = (np.zeros(n1, np.float32), np.ones(n1, np.uint8), np.full(n1, -1, np.int32))
        tc = time.perf_counter()
        oracle.step(np.ascontiguousarray(cpu_first_bits[:n1]), tau, seed, 0, cpu_first_vals[:n1], op, z1, a1, s1)
        cpu_1t_rows = n1 / (time.perf_counter() - tc)
        tc = time.perf_counter()
        oracle.advantages(r[:64], v[:64], L[:64], s[:64], -1.0, 1.0, 0.95, want_scale=False)
        cpu_1t_adv = float(L[:64].clip(0, T_ADV).sum() / (time.perf_counter() - tc))
        oracle.set_threads(nthreads)
        cpu = {"value": cpu_rows / max(cpu_s, 1e-9), "unit": "rows/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"the first {cpu_steps} steps of the same workload ({cpu_rows} live rows x 152064 bf16 "
                         f"logits), {cpu_s:.1f} s of oracle time",
               "advantages_tokens_per_s": float(L.clip(0, T_ADV).sum() / cpu_adv_s),
               "one_thread": {"rows_per_s": cpu_1t_rows, "advantages_tokens_per_s": cpu_1t_adv,
                              "sample": f"{n1} rows of the first step; 64 rows of the advantage batch"}}

    out.update({
        "advantages": {"workload": "B=1024, T=16384 fp32, lengths U[512,16384], 30% stopped, 8 rotated buffer sets",
                       "tokens_per_s": float(valid.sum() / adv_wall), "ms_per_call": adv_wall / args.adv_reps * 1e3,
                       "roofline": {"kernel": "espo_advantages_kernel", "bound": "hbm", "achieved": adv_gbs,
                                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": adv_gbs / HBM_PEAK_GBS,
                                    "avg_launch_us": adv_region_ms / args.adv_reps * 1e3,
                                    "avg_launch_us_event_pair_each": float(adv_ms.mean() * 1e3),
                                    "algorithmic_bytes_per_launch": float(adv_bytes.mean()),
                                    "traffic": adv_traffic, "traffic_measured_on": adv_traffic_on,
                                    "ceiling_gbs": padded_gbs, "frac_of_ceiling": adv_gbs / padded_gbs,
                                    "ceiling": {"kernel": "espo_debug_sweep_padded: the same four [B, T] arrays, inputs read below the "
                                                          "lengths, outputs written everywhere, no dependency between elements",
                                                "avg_launch_us": padded_us, "frac_of_peak": padded_gbs / HBM_PEAK_GBS},
                                    "ceiling_contiguous": {"kernel": "espo_debug_sweep: the same bytes read (8 per valid token) and written "
                                                                     "(8 per position) on two contiguous buffers",
                                                           "read_bytes": rd_bytes, "write_bytes": wr_bytes, "avg_launch_us": sweep_us,
                                                           "gbs": sweep_gbs, "frac_of_peak": sweep_gbs / HBM_PEAK_GBS}}},
        "advantages_terminal": {"workload": "the same batches, terminal-reward form: reads V, writes td and A at t < L only",
                                "us_per_call": advt_us, "tokens_per_s": float(valid.mean() / advt_us * 1e6),
                                "algorithmic_bytes_per_call": advt_bytes, "gbs": advt_bytes / advt_us / 1e3,
                                "frac": advt_bytes / advt_us / 1e3 / HBM_PEAK_GBS},
        "advantages_packed": {"workload": "the same trajectories stored back to back (cu_seqlens), no padding",
                              "dense": {"us_per_call": pk_us[True], "algorithmic_bytes_per_call": pk_bytes[True],
                                        "gbs": pk_bytes[True] / pk_us[True] / 1e3,
                                        "frac": pk_bytes[True] / pk_us[True] / 1e3 / HBM_PEAK_GBS},
                              "terminal": {"us_per_call": pk_us[False], "algorithmic_bytes_per_call": pk_bytes[False],
                                           "gbs": pk_bytes[False] / pk_us[False] / 1e3,
                                           "frac": pk_bytes[False] / pk_us[False] / 1e3 / HBM_PEAK_GBS}},
        "whiten": {"workload": "whitening of the advantages of the same batches over their valid tokens",
                   "us_per_call": wh_us, "launches_per_call": 2, "algorithmic_bytes_per_call": wh_bytes,
                   "gbs": wh_bytes / wh_us / 1e3, "frac": wh_bytes / wh_us / 1e3 / HBM_PEAK_GBS},
        "advantages_ws": {"workload": "the same batches through espo_advantages_ws: rows 513.. sorted by length by the launch's "
                                      "first workgroup, every row's sums left in the workspace; same td and adv",
                          "us_per_call": aw_us, "gbs": float(adv_bytes.mean()) / aw_us / 1e3,
                          "frac": float(adv_bytes.mean()) / aw_us / 1e3 / HBM_PEAK_GBS,
                          "frac_of_ceiling": float(adv_bytes.mean()) / aw_us / 1e3 / padded_gbs,
                          "order_from_the_caller": {"us_per_call": aw_ord_us,
                                                 "frac": float(adv_bytes.mean()) / aw_ord_us / 1e3 / HBM_PEAK_GBS,
                                                 "order": "written by espo_length_order before the timed region",
                                                 "us_per_call_with_the_order_written_in_the_region": aw_ord_now_us,
                                                 "espo_length_order_us_per_call": order_us}},
        "whiten_from_ws": {"workload": "the whitening of the same advantages from the rows' sums: the rewrite only",
                           "us_per_call": whw_us, "launches_per_call": 1, "algorithmic_bytes_per_call": float(np.mean(valid * 8 + B_ADV * 36)),
                           "frac": float(np.mean(valid * 8 + B_ADV * 36)) / whw_us / 1e3 / HBM_PEAK_GBS},
        "advantages_then_whiten": {"workload": "both calls back to back on the same batches",
                                   "espo_advantages_and_espo_whiten_us": pair_us[False],
                                   "espo_advantages_ws_and_espo_whiten_from_ws_us": pair_us[True],
                                   "espo_advantages_terminal_and_espo_whiten_us": pair_t_us[False],
                                   "espo_advantages_terminal_ws_and_espo_whiten_from_ws_us": pair_t_us[True]},
        "advantages_terminal_ws": {"workload": "the terminal-reward form without zero fill through espo_advantages_terminal_ws",
                                   "us_per_call": awt_us, "frac": advt_bytes / awt_us / 1e3 / HBM_PEAK_GBS},
        "batch_stats": {"workload": "B=512, T=8192 fp32 regrets, lengths U[64,8192], 25% stopped, 8 rotated sets",
                        "us_per_call": bs_us, "algorithmic_bytes_per_call": bs_bytes,
                        "gbs": bs_bytes / bs_us / 1e3, "launches_per_call": 2,
                        "mu_g": bs_res["mu_g"], "var_g": bs_res["var_g"], "beta": bs_res["beta"]},
        "cpu_baseline": cpu,
    })
    if parity is not None:
        out.update(parity)
    if curve is not None:
        out["live_curve"] = {"workload": "heavy termination: B=1024, V=152064 bf16, 256 steps, 60% of rows planted to stop in "
                                         "[16,200]; every step's logits resident, one event pair per 8 consecutive launches",
                             "bins": curve,
                             "done_rows_by_position": {**position, "note": "64 launches each on the last 64 steps' logits, mask held "
                                                       "fixed; the second figure is what a compacted batch costs"}}
    print(json.dumps(out))
    if parity is not None and not (parity["parity_ok"] and parity["advantages_parity_ok"]):
        print("bench.py: the GPU's results differ from the oracle's", file=sys.stderr)
        return 1
    return 0


if __name__ == "__main__":
    sys.exit(main())
