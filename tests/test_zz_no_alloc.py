"""The entry point that allocates nothing, `espo_batch_stats_static`, against `espo_batch_stats`
through the C ABI (needs an MI355X).  Both run the same kernels, so every field of the result
must be the same bits; the calls come in a row on the library's one scratch array, the second on
a smaller batch, and the array is filled with junk in between by a larger batch.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2605_29860_amd as espo  # noqa: E402
from paper_2605_29860_amd import workloads as W  # noqa: E402

CTRL = dict(alpha_ema=0.99, eta_beta=0.1, target_rate=0.25, beta_min=0.0, beta_max=7.0)


def _both(B, T, seed, mu_g, var_g, beta):
    regret, lengths, stopped = W.regret_batch(B, T, len_lo=0, seed=seed, device="cuda", poison=True)
    ref_out = torch.full((espo.BATCH_RESULT_BYTES,), 0xAB, dtype=torch.uint8, device="cuda")
    ws = torch.full((max(espo.espo_batch_stats_workspace_bytes(B, T), 8),), 0xCD, dtype=torch.uint8, device="cuda")
    espo.espo_batch_stats(regret, lengths, stopped, mu_g, var_g, beta, ref_out, ws, **CTRL)
    got_out = torch.full((espo.BATCH_RESULT_BYTES,), 0x5A, dtype=torch.uint8, device="cuda")
    espo.espo_batch_stats_static(regret, lengths, stopped, mu_g, var_g, beta, got_out, **CTRL)
    torch.cuda.synchronize()
    return ref_out.cpu().numpy(), got_out.cpu().numpy(), espo.read_batch_result(got_out)


def test_static_scratch_matches_the_workspace_call_on_two_calls_in_a_row():
    print("[case] espo_batch_stats_static B=1500 then B=37", flush=True)
    ref, got, res = _both(1500, 260, seed=11, mu_g=1.0, var_g=2.0, beta=7.0)       # fills all 1024 partial sums
    np.testing.assert_array_equal(got, ref)
    assert res["tokens"] > 0
    print("[case] second call, smaller batch", flush=True)
    ref, got, res = _both(37, 1000, seed=12, mu_g=0.3, var_g=0.1, beta=2.0)        # 37 partial sums, the rest is stale
    np.testing.assert_array_equal(got, ref)
    assert res["tokens"] > 0
    ref, got, res = _both(1, 5, seed=13, mu_g=0.3, var_g=0.1, beta=2.0)
    np.testing.assert_array_equal(got, ref)


def test_static_scratch_argument_errors_enqueue_nothing():
    print("[case] espo_batch_stats_static errors", flush=True)
    regret, lengths, stopped = W.regret_batch(4, 16, len_lo=0, seed=1, device="cuda")
    out = torch.full((espo.BATCH_RESULT_BYTES,), 0x5A, dtype=torch.uint8, device="cuda")
    with pytest.raises(espo.EspoError) as e:
        espo.espo_batch_stats_static(regret, lengths, stopped, 1.0, 1.0, 1.0, out, alpha_ema=1.5)
    assert e.value.code == -1
    with pytest.raises(espo.EspoError) as e:
        espo.espo_batch_stats_static(regret, lengths, stopped, float("nan"), 1.0, 1.0, out)
    assert e.value.code == -1
    torch.cuda.synchronize()
    assert (out.cpu().numpy() == 0x5A).all()
    # an empty batch is a valid call: the parameters come back unchanged
    espo.espo_batch_stats_static(regret[:0], lengths[:0], stopped[:0], 0.4, 0.6, 2.0, out)
    res = espo.read_batch_result(out)
    assert res["tokens"] == 0 and np.float32(res["beta"]) == np.float32(2.0)
