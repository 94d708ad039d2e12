"""vla_decode_step_static (staging in the library's own device array, nothing allocated) against
vla_decode_step, through the C ABI: same bits, on two calls in a row, the second with a smaller batch."""
from dataclasses import replace

import numpy as np
import pytest

import workloads as W
from tests import parity as P
from tests.test_gpu_parity import make_policy, ragged_obs

pytestmark = pytest.mark.gpu


def _decode_logits(pol, wl, obs, static):
    """prefill, then two decode steps fed with fixed tokens; returns the logits of the two steps."""
    import torch
    dev = P.device_inputs(pol, obs)
    first = pol.prefill(dev["patch_emb"], obs["cu_patch"], dev["instr_ids"], obs["cu_instr"])
    B = len(obs["cu_patch"]) - 1
    outs = [first.cpu().numpy()]
    for step in range(2):
        ids = torch.full((B,), wl.shape.action_id0 + 3 + 5 * step, dtype=torch.int32, device=pol.device)
        ids += torch.arange(B, dtype=torch.int32, device=pol.device)
        outs.append(pol.decode_step(ids, static=static).cpu().numpy())
    return outs


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_static_decode_step_matches_decode_step_twice_in_a_row(dtype):
    import torch
    shape = W.PolicyShape(2, 256, 2, 128, 704, 1024, dtype=dtype)
    wl = W.Workload("Ts", 31, shape, batch=7, n_patches=40, instr_len=(0, 12), n_tokens=4)
    weights = W.make_weights(wl.shape, wl.seed)
    big = ragged_obs(wl, [40, 40, 1, 40, 33, 40, 40], [0, 3, 0, 12, 9, 5, 1], seed=91)
    small = ragged_obs(replace(wl, batch=3), [40, 2, 17], [4, 0, 12], seed=92)
    ref = make_policy(wl, weights)
    want_big = _decode_logits(ref, wl, big, static=False)
    want_small = _decode_logits(ref, wl, small, static=False)
    ref.close()
    pol = make_policy(wl, weights)
    got_big = _decode_logits(pol, wl, big, static=True)       # first call(s) on this GPU
    got_small = _decode_logits(pol, wl, small, static=True)   # right after, smaller batch: stale staging rows present
    torch.cuda.synchronize()
    for want, got in ((want_big, got_big), (want_small, got_small)):
        for w, g in zip(want, got):
            assert np.isfinite(g).all()
            assert np.array_equal(w, g)
    # against the oracle as well (teacher-forced on the same fed tokens), at the parity tolerance
    tol = P.tolerances(wl)
    B = 3
    feed = np.stack([np.arange(B) + 3, np.arange(B) + 8, np.zeros(B, dtype=np.int64)], axis=1)
    from oracle import vla_oracle as O
    pes, ids = P.split_obs(small, range(B))
    ora = O.OraclePolicy(wl.shape, weights).policy_step(pes, ids, 3, mode="cached", forced_tokens=feed)
    err = max(float(np.abs(got_small[k] - ora["logits"][:, k]).max()) for k in range(3))
    assert err <= tol["logit"], err
    pol.close()


def test_static_decode_step_rejects_what_does_not_fit():
    from paper_2603_18464_amd import VlaError
    import torch
    # 4 planes x 128 rows x max(3d, 2f) x 4 bytes = 46 MiB > 32 MiB
    shape = W.PolicyShape(1, 4096, 32, 128, 11264, 1024, dtype="bf16")
    wl = W.Workload("Tb", 33, shape, batch=128, n_patches=1, instr_len=(0, 0), n_tokens=2)
    weights = W.make_weights(wl.shape, wl.seed)
    pol = make_policy(wl, weights)
    obs = W.make_observations(wl)
    dev = P.device_inputs(pol, obs)
    pol.prefill(dev["patch_emb"], obs["cu_patch"], dev["instr_ids"], obs["cu_instr"])
    ids = torch.full((wl.batch,), shape.action_id0, dtype=torch.int32, device=pol.device)
    with pytest.raises(VlaError) as e:
        pol.decode_step(ids, static=True)
    assert e.value.code == -4 and "static" in str(e.value)
    pol.decode_step(ids)                                      # the ordinary entry point still takes it
    torch.cuda.synchronize()
    pol.close()
