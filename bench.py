#!/usr/bin/env python3
"""Benchmark of the ESPO per-step hot path on one MI355X.

A "step" is one `espo_step` call over a batch of 512 trajectories with Qwen-vocabulary
bf16 logits (the sustained-rollout workload: state carried from step to step, about a
quarter of the rows driven over the stop threshold at seeded steps, dead rows skipped).
Every step reads its own logit buffer, all of them generated on the device before the
timed region (288 GB of HBM hold hundreds of 156 MB steps), so no step can be served
from a cache.  The companion `espo_advantages` pass is timed on the B=1024, T=16384 batch
and reported in the same JSON line, as is the CPU oracle on a bounded sample.

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


def _traffic_from_profiles(kernel: str):
    """HBM bytes per launch measured with rocprofv3 counters, if a summary was committed."""
    path = os.path.join(ROOT, "profiles", f"traffic_{kernel}.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


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
    ap.add_argument("--live-curve", action="store_true",
                    help="also run the heavy-termination rollout (B=1024, 256 steps, 60%% of rows planted to stop) "
                         "and report the launch duration against the number of live rows")
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

    def run(first, last, z, alive, ss, events=None, entropy=None, params=params):
        for s in range(first, last):
            if events is not None:
                events[s - first][0].record()
            espo.espo_step(logits[s], tau, seed, s, values[s], params, z, alive, ss, tokens, regret, logprob,
                           entropy=entropy)
            if events is not None:
                events[s - first][1].record()

    def fresh_state():
        z, alive, ss = W.initial_state(B_STEP, device=dev)
        run(0, Wm, z, alive, ss)                 # warmup steps are the first steps of the trajectory
        torch.cuda.synchronize()
        return z, alive, ss

    if args.calibration_copies:
        src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(args.calibration_copies):
            espo.espo_debug_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    # ------------------------------------------------------------------ timed region: exactly K steps
    z, alive, ss = fresh_state()
    region = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
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

    # same K steps again with an event pair around every launch (each pair adds a few microseconds of its own)
    z2, alive2, ss2 = fresh_state()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(K)]
    run(Wm, total, z2, alive2, ss2, events=ev)
    torch.cuda.synchronize()
    assert torch.equal(ss2, ss) and torch.equal(z2, z), "replay of the timed steps is not deterministic"
    kern_ms = np.array([a.elapsed_time(b) for a, b in ev])

    # and once more with the optional entropy output (the kernel's other instantiation)
    z3, alive3, ss3 = fresh_state()
    entropy = torch.empty(B_STEP, dtype=torch.float32, device=dev)
    eregion = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
    eregion[0].record()
    run(Wm, total, z3, alive3, ss3, entropy=entropy)
    eregion[1].record()
    torch.cuda.synchronize()
    assert torch.equal(ss3, ss) and torch.equal(z3, z), "the entropy output changed the trajectory"
    ent_us = eregion[0].elapsed_time(eregion[1]) / K * 1e3

    # and without the log-probability output (no softmax sum is formed then)
    z5, alive5, ss5 = fresh_state()
    nregion = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
    nregion[0].record()
    for s in range(Wm, total):
        espo.espo_step(logits[s], tau, seed, s, values[s], params, z5, alive5, ss5, tokens, regret, None)
    nregion[1].record()
    torch.cuda.synchronize()
    assert torch.equal(ss5, ss) and torch.equal(z5, z), "dropping the log-probability output changed the trajectory"
    nolp_us = nregion[0].elapsed_time(nregion[1]) / K * 1e3

    # and with the nucleus filter of the paper's evaluation set-up (top-p 0.7) on the same logits
    params_p = espo.EspoParams(**{**W.RolloutParams().as_dict(), "top_p": 0.7})
    z4, alive4, ss4 = W.initial_state(B_STEP, device=dev)
    run(0, Wm, z4, alive4, ss4, params=params_p)
    torch.cuda.synchronize()
    pregion = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
    pregion[0].record()
    run(Wm, total, z4, alive4, ss4, params=params_p)
    pregion[1].record()
    torch.cuda.synchronize()
    topp_us = pregion[0].elapsed_time(pregion[1]) / K * 1e3
    topp_live = float((alive4 > 0).sum())
    step_bytes = live * (V_STEP * 2 + STEP_SCALAR_BYTES) + (B_STEP - live) * 1
    step_gbs = float(step_bytes.sum() / (region_ms * 1e-3) / 1e9)   # events around the K back-to-back launches

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
    aev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.adv_reps)]
    aregion = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
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

    # the same batches in the terminal-reward form (no reward array, padding left to the caller's mask)
    rows_all = torch.arange(B_ADV, device=dev)
    adv_term = [r[rows_all, (L - 1).clamp(min=0).long()].contiguous() for r, v, L, s in adv_in]
    def advt_call(i):
        r, v, L, s = adv_in[i % nbuf]
        td, ad = adv_out[i % nbuf]
        espo.espo_advantages_terminal(v, L, s, adv_term[i % nbuf], -1.0, 1.0, 0.95, td, ad, zero_padding=False)
    for i in range(nbuf):
        advt_call(i)
    torch.cuda.synchronize()
    tregion = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
    tregion[0].record()
    for i in range(args.adv_reps):
        advt_call(i)
    tregion[1].record()
    torch.cuda.synchronize()
    advt_us = tregion[0].elapsed_time(tregion[1]) / args.adv_reps * 1e3
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
    pk_us = {}
    for dense in (True, False):
        for i in range(nbuf):
            pk_call(i, dense)
        torch.cuda.synchronize()
        kregion = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
        kregion[0].record()
        for i in range(args.adv_reps):
            pk_call(i, dense)
        kregion[1].record()
        torch.cuda.synchronize()
        pk_us[dense] = kregion[0].elapsed_time(kregion[1]) / args.adv_reps * 1e3
    pk_bytes = {True: float(np.mean(valid * 16 + B_ADV * 9)), False: float(np.mean(valid * 12 + B_ADV * 13))}
    del pk

    # whitening of the advantages over the valid tokens (two passes over A, one store)
    wh_ws = torch.empty(espo.espo_whiten_workspace_bytes(B_ADV, T_ADV), dtype=torch.uint8, device=dev)
    def wh_call(i):
        td, ad = adv_out[i % nbuf]
        espo.espo_whiten(ad, adv_in[i % nbuf][2], td, wh_ws)      # td serves as the output buffer here
    for i in range(nbuf):
        adv_call(i)                                               # the advantages these whiten
    for i in range(nbuf):
        wh_call(i)
    torch.cuda.synchronize()
    wregion = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
    wregion[0].record()
    for i in range(args.adv_reps):
        wh_call(i)
    wregion[1].record()
    torch.cuda.synchronize()
    wh_us = wregion[0].elapsed_time(wregion[1]) / args.adv_reps * 1e3
    wh_bytes = float(np.mean(valid * 12 + B_ADV * 8))

    # ------------------------------------------------------------------ batch-boundary statistics (B=512, T=8192)
    bs_sets = [W.regret_batch(512, 8192, seed=70 + i, device=dev) for i in range(nbuf)]   # 134 MB in rotation
    bs_out = torch.zeros(espo.BATCH_RESULT_BYTES, dtype=torch.uint8, device=dev)
    bs_ws = torch.zeros(espo.espo_batch_stats_workspace_bytes(512, 8192), dtype=torch.uint8, device=dev)
    def bs_call(i):
        g, L, s = bs_sets[i % nbuf]
        espo.espo_batch_stats(g, L, s, 1.0, 2.0, 7.0, bs_out, bs_ws)
    for i in range(nbuf):
        bs_call(i)
    torch.cuda.synchronize()
    bregion = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
    bregion[0].record()
    for i in range(args.adv_reps):
        bs_call(i)
    bregion[1].record()
    torch.cuda.synchronize()
    bs_us = bregion[0].elapsed_time(bregion[1]) / args.adv_reps * 1e3
    bs_bytes = float(np.mean([int(bs_sets[i % nbuf][1].sum()) * 4 + 512 * 5 for i in range(args.adv_reps)]))
    bs_res = espo.read_batch_result(bs_out)

    # ------------------------------------------------------------------ optional: launch duration vs live rows (B=1024)
    curve = None
    if args.live_curve:
        Bc, Sc, seed_c = 1024, 256, 4
        plant_c = W.RegretPlant.make(Bc, V_STEP, 0.6, 12, 190, seed_c)
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
        cev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(Sc)]
        for t in range(Sc):
            cev[t][0].record()
            espo.espo_step(logits_c[t], tau, seed_c, t, values_c[t], params, zc_, ac_, sc_, tok_c, reg_c, lp_c)
            cev[t][1].record()
        torch.cuda.synchronize()
        ss_c = sc_.cpu().numpy()
        live_c = ((ss_c[None, :] < 0) | (ss_c[None, :] >= np.arange(Sc)[:, None])).sum(1)   # rows decoded at each step
        cus = np.array([a.elapsed_time(b) * 1e3 for a, b in cev])
        curve = []
        for lo in range(400, 1025, 104):                                   # six bins of live rows
            sel = (live_c > lo - 104) & (live_c <= lo)
            if sel.any():
                rows_m, us_m = float(live_c[sel].mean()), float(cus[sel].mean())
                curve.append({"live_rows": rows_m, "steps": int(sel.sum()), "us_per_launch_event_pair": us_m,
                              "rows_per_s": rows_m / us_m * 1e6,
                              "gbs": (rows_m * (V_STEP * 2 + STEP_SCALAR_BYTES) + (Bc - rows_m)) / us_m / 1e3})
        del logits_c

    # ------------------------------------------------------------------ CPU oracle on a bounded sample (context only)
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        oracle.build_oracle()
        op = oracle.OracleParams(**W.RolloutParams().as_dict())
        zc, ac, sc = (np.zeros(B_STEP, np.float32), np.ones(B_STEP, np.uint8), np.full(B_STEP, -1, np.int32))
        cpu_s, cpu_rows, cpu_steps = 0.0, 0, 0
        while cpu_s < args.cpu_seconds and cpu_steps < total:      # the first steps of the same trajectory
            bits = W.to_host_bits(logits[cpu_steps])               # copy to the host: untimed
            vals_h = values[cpu_steps].cpu().numpy()
            if cpu_steps == 0:
                cpu_first_bits, cpu_first_vals = bits, vals_h
            cpu_rows += int(ac.sum())
            tc = time.perf_counter()
            oracle.step(bits, tau, seed, cpu_steps, vals_h, op, zc, ac, sc)
            cpu_s += time.perf_counter() - tc
            cpu_steps += 1
        r, v, L, s = [x.cpu().numpy() for x in adv_in[0]]
        tc = time.perf_counter()
        oracle.advantages(r, v, L, s, -1.0, 1.0, 0.95, want_scale=False)
        cpu_adv_s = time.perf_counter() - tc
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
        cpu = {"value": cpu_rows / cpu_s, "unit": "rows/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"the first {cpu_steps} steps of the same workload ({cpu_rows} live rows x 152064 bf16 "
                         f"logits), {cpu_s:.1f} s of oracle time",
               "advantages_tokens_per_s": float(L.clip(0, T_ADV).sum() / cpu_adv_s),
               "one_thread": {"rows_per_s": cpu_1t_rows, "advantages_tokens_per_s": cpu_1t_adv,
                              "sample": f"{n1} rows of the first step; 64 rows of the advantage batch"}}

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
                     "avg_launch_us": region_ms / K * 1e3,
                     "avg_launch_us_event_pair_each": float(kern_ms.mean() * 1e3),
                     "algorithmic_bytes_per_launch": float(step_bytes.mean()),
                     "traffic": _traffic_from_profiles("espo_step")},
        "step_with_entropy": {"avg_launch_us": ent_us, "frac": step_gbs / HBM_PEAK_GBS * (region_ms / K * 1e3) / ent_us,
                              "mean_entropy_last_step": float(entropy[alive3 > 0].mean()) if bool((alive3 > 0).any()) else None},
        "step_without_logprob": {"avg_launch_us": nolp_us, "frac": step_gbs / HBM_PEAK_GBS * (region_ms / K * 1e3) / nolp_us,
                                 "note": "logprob = NULL: token, regret, state and masks only, no softmax sum"},
        "step_top_p_0.7": {"avg_launch_us": topp_us, "live_rows_last": topp_live,
                           "note": "filtered draw: own kernel instantiation, reads parts of the row again"},
        "advantages": {"workload": "B=1024, T=16384 fp32, lengths U[512,16384], 30% stopped, 8 rotated buffer sets",
                       "tokens_per_s": float(valid.sum() / adv_wall), "ms_per_call": adv_wall / args.adv_reps * 1e3,
                       "roofline": {"kernel": "espo_advantages_kernel", "bound": "hbm", "achieved": adv_gbs,
                                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": adv_gbs / HBM_PEAK_GBS,
                                    "avg_launch_us": adv_region_ms / args.adv_reps * 1e3,
                                    "avg_launch_us_event_pair_each": float(adv_ms.mean() * 1e3),
                                    "algorithmic_bytes_per_launch": float(adv_bytes.mean()),
                                    "traffic": _traffic_from_profiles("espo_advantages")}},
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
        "batch_stats": {"workload": "B=512, T=8192 fp32 regrets, lengths U[64,8192], 25% stopped, 8 rotated sets",
                        "us_per_call": bs_us, "algorithmic_bytes_per_call": bs_bytes,
                        "gbs": bs_bytes / bs_us / 1e3, "launches_per_call": 2,
                        "mu_g": bs_res["mu_g"], "var_g": bs_res["var_g"], "beta": bs_res["beta"]},
        "cpu_baseline": cpu,
    }
    if curve is not None:
        out["live_curve"] = {"workload": "heavy termination: B=1024, V=152064 bf16, 256 steps, 60% of rows planted to stop in "
                                         "[16,200]; every step's logits resident, one event pair per launch",
                             "bins": curve}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
