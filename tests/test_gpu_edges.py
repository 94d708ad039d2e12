"""GPU edge cases of the 16-bit path against the fp64 oracle: batches above one decode chunk (every row
compared), value ranges at the edges of half precision, sharp attention, exact ties, non-finite logits, fewer
bins than lanes."""
from dataclasses import replace

import numpy as np
import pytest

import workloads as W
from tests import parity as P
from tests.test_gpu_parity import make_policy, ragged_obs, run_both

pytestmark = pytest.mark.gpu

SMALL = W.PolicyShape(2, 256, 2, 128, 704, 1024, dtype="bf16")
# every matrix a multiple of 256 columns and of 64 in depth: what the tiled split-K decode GEMM of batches above
# 128 rows takes (with SMALL, the gate/up projection of such a batch stays on the weight-streaming kernel)
TILED = W.PolicyShape(2, 512, 4, 128, 1024, 1024, dtype="bf16")


def bf16(x):
    return W.bf16_bits_from_f32(np.asarray(x, dtype=np.float32))


def as_f32(bits):
    return W.f32_from_bf16_bits(bits)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("shape,batch,fast", [(SMALL, 200, False), (SMALL, 300, False), (SMALL, 200, "first"),
                                              (SMALL, 300, True), (TILED, 200, False), (TILED, 300, "first"),
                                              (TILED, 420, True), (TILED, 129, False)],
                         ids=["B200_two_term", "B300_two_term", "B200_two_term_layer0_only", "B300_fast",
                              "tiled_B200_two_term", "tiled_B300_two_term_layer0_only", "tiled_B420_fast",
                              "tiled_B129_two_term"])
def test_every_row_of_a_large_ragged_batch(shape, batch, fast):
    """More sequences than one weight-streaming launch takes (128 rows), than one tile of the split-K decode GEMM
    (256 rows: 300 = 256 + a remainder on the weight-streaming kernel, 420 = 256 + 164) and than one 128-row group of
    the last prefill layer: every row of the prefill and of three decode steps is compared with the oracle."""
    g = np.random.default_rng(5 + batch)
    lens = g.integers(0, 13, size=batch)
    nps = g.integers(1, 25, size=batch)
    wl = W.Workload("Tb", 41, shape, batch=batch, n_patches=24, instr_len=(0, 12), n_tokens=4,
                    sampling="gumbel", temperature=1.0)
    obs = ragged_obs(wl, list(nps), list(lens), seed=93)
    stats, gpu, ora = run_both(wl, obs=obs, gumbel=W.make_gumbel(wl), fast=fast)
    assert stats["compared"] + stats["excused"] + stats["skipped"] == batch * wl.n_tokens
    assert stats["compared"] > 0.9 * batch * wl.n_tokens


def test_weights_outside_the_exact_range_are_refused():
    """A weight above 255 in magnitude or not finite cannot be re-encoded: the load reports it."""
    from paper_2603_18464_amd import VlaError
    wl = W.Workload("Tr", 43, SMALL, batch=2, n_patches=8, instr_len=(2, 2), n_tokens=2)
    good = W.make_weights(wl.shape, wl.seed)
    obs = W.make_observations(wl)
    for value in (300.0, -float("inf"), float("nan")):
        bad = dict(good)
        m = as_f32(good["layers.1.w_up"]).copy()
        m[17, 33] = value
        bad["layers.1.w_up"] = bf16(m)
        pol = make_policy(wl, good)
        with pytest.raises(VlaError) as e:
            pol.load_weights(bad)
        assert e.value.code == -6, value
        dev = P.device_inputs(pol, obs)
        with pytest.raises(VlaError) as e:                       # and nothing computes on them
            pol.prefill(dev["patch_emb"], obs["cu_patch"], dev["instr_ids"], obs["cu_instr"])
        assert e.value.code == -6
        pol.load_weights(good)                                   # a whole good set clears the finding
        pol.prefill(dev["patch_emb"], obs["cu_patch"], dev["instr_ids"], obs["cu_instr"])
        pol.close()
    # the edges themselves are exact, and values below 2^-25 are accepted (absolute error below 2^-33)
    edge = dict(good)
    m = as_f32(good["layers.0.wq"]).copy()
    m[0, 0], m[1, 1], m[2, 2], m[3, 3] = 255.0, -(2.0 ** -25), 0.0, 2.0 ** -40
    edge["layers.0.wq"] = bf16(m)
    run_both(wl, obs=obs, weights=edge)


def test_patch_embeddings_a_thousand_times_larger():
    """Inputs far above the half-precision range of a single rounded value stay in the float32 residual
    stream; the normalised rows that reach the matrix cores are of order one."""
    wl = W.Workload("Te", 45, SMALL, batch=5, n_patches=40, instr_len=(0, 9), n_tokens=4)
    obs = ragged_obs(wl, [40, 3, 40, 17, 40], [0, 9, 4, 1, 6], seed=95)
    obs["patch_emb"] = bf16(as_f32(obs["patch_emb"]) * 1000.0)
    assert np.abs(as_f32(obs["patch_emb"])).max() > 3000
    run_both(wl, obs=obs)


@pytest.mark.parametrize("fast", [False, True], ids=["two_term", "fast"])
def test_sharp_attention(fast):
    """Query / key projections scaled so that the attention scores have a standard deviation above 5: the
    softmax is far from uniform, and mistakes in the scale, the mask or the rotary embedding would show."""
    from oracle import vla_oracle as O
    wl = W.Workload("Ta", 47, SMALL, batch=4, n_patches=60, instr_len=(3, 20), n_tokens=4)
    weights = W.make_weights(wl.shape, wl.seed)
    for l in range(wl.shape.n_layers):
        for leaf in ("wq", "wk"):
            weights[f"layers.{l}.{leaf}"] = bf16(as_f32(weights[f"layers.{l}.{leaf}"]) * 8.0)   # exact in bf16
    obs = ragged_obs(wl, [60, 60, 31, 60], [3, 20, 11, 7], seed=97)
    # the premise, measured with the oracle's own functions on layer 0
    pol = O.OraclePolicy(wl.shape, weights)
    x = pol.prefix_rows(obs["patch_emb"][:60], obs["instr_ids"][:3])
    h = O.rms_norm(x, pol.W("layers.0.attn_norm"), wl.shape.rms_eps)
    n, H, hd = x.shape[0], wl.shape.n_heads, wl.shape.head_dim
    q = O.rope((h @ pol.W("layers.0.wq").T).reshape(n, H, hd), np.arange(n), wl.shape.rope_theta)
    k = O.rope((h @ pol.W("layers.0.wk").T).reshape(n, H, hd), np.arange(n), wl.shape.rope_theta)
    assert (np.einsum("ihd,jhd->hij", q, k) / np.sqrt(hd)).std() > 5
    run_both(wl, obs=obs, weights=weights, fast=fast)


def test_exact_ties_go_to_the_lowest_bin():
    """Duplicated head rows give bit-equal logits: the lower bin of each pair is chosen, as in the oracle."""
    import torch
    wl = W.Workload("Tt", 49, SMALL, batch=6, n_patches=20, instr_len=(0, 6), n_tokens=5)
    weights = W.make_weights(wl.shape, wl.seed)
    A, V = wl.shape.n_action_bins, wl.shape.vocab
    head = weights["lm_head"].copy()
    head[V - A // 2:] = head[V - A:V - A // 2]                    # bin j + 128 repeats bin j
    weights["lm_head"] = head
    obs = ragged_obs(wl, [20, 20, 5, 20, 1, 20], [0, 6, 2, 3, 0, 1], seed=99)
    stats, gpu, ora = run_both(wl, obs=obs, weights=weights)
    assert (gpu["tokens"] < A // 2).all() and (ora["tokens"] < A // 2).all()
    assert np.array_equal(gpu["logits"][..., :A // 2], gpu["logits"][..., A // 2:])
    # every bin equal: token 0 with log-prob -ln A
    head[V - A:] = head[V - A]
    weights["lm_head"] = head
    pol = make_policy(wl, weights)
    dev = P.device_inputs(pol, obs)
    out = P.to_numpy(pol.policy_step(dev["patch_emb"], obs["cu_patch"], dev["instr_ids"], obs["cu_instr"], wl.n_tokens))
    torch.cuda.synchronize()
    assert (out["tokens"] == 0).all()
    assert np.abs(out["logp"] + np.log(A)).max() < 1e-5
    assert np.allclose(out["actions"], -1.0 + 1.0 / A)
    pol.close()


def test_non_finite_logits_select_bin_zero_and_leave_other_sequences_alone():
    import torch
    wl = W.Workload("Tn", 51, SMALL, batch=4, n_patches=12, instr_len=(1, 5), n_tokens=3)
    weights = W.make_weights(wl.shape, wl.seed)
    obs = ragged_obs(wl, [12, 12, 12, 12], [1, 5, 2, 3], seed=101)
    pol = make_policy(wl, weights)
    dev = P.device_inputs(pol, obs)
    args = (obs["cu_patch"], dev["instr_ids"], obs["cu_instr"], wl.n_tokens)
    clean = P.to_numpy(pol.policy_step(dev["patch_emb"], *args, want_logits=True))
    pe = as_f32(obs["patch_emb"]).copy()
    pe[obs["cu_patch"][2] + 4, 7] = np.nan                      # one element of sequence 2
    dirty = P.to_numpy(pol.policy_step(pol.to_device(bf16(pe)), *args, want_logits=True))
    torch.cuda.synchronize()
    assert np.isnan(dirty["logits"][2]).all() and np.isnan(dirty["logp"][2]).all()
    assert (dirty["tokens"][2] == 0).all()
    for b in (0, 1, 3):
        for k in ("tokens", "logp", "logits", "actions"):
            assert np.array_equal(clean[k][b], dirty[k][b]), (b, k)
    pol.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_fewer_action_bins_than_lanes(dtype):
    shape = replace(SMALL, n_action_bins=40, dtype=dtype)
    wl = W.Workload("Tf", 53, shape, batch=5, n_patches=16, instr_len=(0, 8), n_tokens=4,
                    sampling="gumbel", temperature=0.8)
    obs = ragged_obs(wl, [16, 16, 2, 16, 9], [0, 8, 3, 5, 1], seed=103)
    stats, gpu, ora = run_both(wl, obs=obs, gumbel=W.make_gumbel(wl))
    assert (gpu["tokens"] < 40).all()
