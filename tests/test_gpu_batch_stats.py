"""Parity of the HIP espo_batch_stats with the CPU oracle, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import oracle  # noqa: E402
import paper_2605_29860_amd as espo  # noqa: E402
from paper_2605_29860_amd import workloads as W  # noqa: E402

CTRL = dict(alpha_ema=0.99, eta_beta=0.1, target_rate=0.25, beta_min=0.0, beta_max=7.0)


def _run(regret, lengths, stopped, mu_g, var_g, beta, **ctrl):
    c = dict(CTRL); c.update(ctrl)
    B, T = regret.shape
    out = torch.full((espo.BATCH_RESULT_BYTES,), 0xAB, dtype=torch.uint8, device="cuda")
    ws = torch.full((max(espo.espo_batch_stats_workspace_bytes(B, T), 8),), 0xCD, dtype=torch.uint8, device="cuda")
    espo.espo_batch_stats(regret, lengths, stopped, mu_g, var_g, beta, out, ws, **c)
    got = espo.read_batch_result(out)
    ref = oracle.batch_stats(regret.cpu().numpy(), lengths.cpu().numpy(), stopped.cpu().numpy(), mu_g, var_g, beta, **c)
    # counts and everything derived from counts alone: exact
    assert got["tokens"] == ref["tokens"] and got["stopped"] == int(stopped.sum())
    assert got["stop_rate"] == ref["stop_rate"]
    assert np.float32(got["beta"]).view(np.uint32) == np.float32(ref["beta"]).view(np.uint32)
    # sums in double, in another order than the oracle's: 1e-12; the float parameters may differ
    # by one rounding where the double lands next to a tie
    assert got["mean_g"] == pytest.approx(ref["mean"], rel=1e-12, abs=1e-300)
    assert got["var_g_batch"] == pytest.approx(ref["var"], rel=1e-10, abs=1e-300)
    assert abs(np.float32(got["mu_g"]) - ref["mu_g"]) <= np.spacing(np.float32(abs(ref["mu_g"])))
    assert abs(np.float32(got["var_g"]) - ref["var_g"]) <= np.spacing(np.float32(abs(ref["var_g"])))
    return got


@pytest.mark.parametrize("B,T", [(1, 1), (3, 7), (5, 64), (17, 1000), (64, 4099), (1500, 260)])
def test_shapes_ragged_lengths_and_poisoned_padding(B, T):
    print(f"[case] batch stats B={B} T={T}", flush=True)
    regret, lengths, stopped = W.regret_batch(B, T, len_lo=0, seed=B * 31 + T, device="cuda", poison=True)
    _run(regret, lengths, stopped, 1.0, 2.0, 7.0)
    lengths[0] = -3
    lengths[-1] = T + 11                                       # clamped on the device
    regret = torch.nan_to_num(regret, nan=0.5)
    _run(regret, lengths, stopped, 0.3, 0.1, 2.0, beta_max=3.0)


def test_rollout_sized_batch_and_determinism():
    print("[case] batch stats B=512 T=8192", flush=True)
    regret, lengths, stopped = W.regret_batch(512, 8192, seed=5, device="cuda", poison=True)
    a = _run(regret, lengths, stopped, 1.0, 2.0, 7.0)
    b = _run(regret, lengths, stopped, 1.0, 2.0, 7.0)
    assert a == b                                              # fixed reduction order: identical bits
    assert 0.9 < a["mean_g"] < 1.1 and 0.15 < a["stop_rate"] < 0.35


def test_degenerate_batches_and_argument_errors():
    print("[case] batch stats degenerate", flush=True)
    B, T = 4, 16
    regret = torch.full((B, T), 2.25, device="cuda")
    stopped = torch.ones(B, dtype=torch.uint8, device="cuda")
    got = _run(regret, torch.zeros(B, dtype=torch.int32, device="cuda"), stopped, 0.4, 0.6, 2.0)
    assert got["tokens"] == 0 and np.float32(got["mu_g"]) == np.float32(0.4) and np.float32(got["var_g"]) == np.float32(0.6)
    got = _run(regret, torch.full((B,), T, dtype=torch.int32, device="cuda"), stopped, 2.25, 0.0, 2.0)
    assert got["var_g_batch"] == 0.0 and got["mean_g"] == 2.25
    got = _run(regret[:0], torch.zeros(0, dtype=torch.int32, device="cuda"), stopped[:0], 0.4, 0.6, 2.0)
    assert got["tokens"] == 0 and np.float32(got["beta"]) == np.float32(2.0)
    out = torch.zeros(espo.BATCH_RESULT_BYTES, dtype=torch.uint8, device="cuda")
    ws = torch.zeros(8, dtype=torch.uint8, device="cuda")
    L = torch.full((B,), T, dtype=torch.int32, device="cuda")
    with pytest.raises(espo.EspoError) as e:                   # workspace too small
        espo.espo_batch_stats(regret, L, stopped, 1.0, 1.0, 1.0, out, ws)
    assert e.value.code == -3
    ws = torch.zeros(espo.espo_batch_stats_workspace_bytes(B, T), dtype=torch.uint8, device="cuda")
    with pytest.raises(espo.EspoError) as e:
        espo.espo_batch_stats(regret, L, stopped, 1.0, 1.0, 1.0, out, ws, alpha_ema=1.5)
    assert e.value.code == -1
    with pytest.raises(espo.EspoError) as e:
        espo.espo_batch_stats(regret, L, stopped, 1.0, 1.0, 1.0, out, ws, beta_min=2.0, beta_max=1.0)
    assert e.value.code == -1
