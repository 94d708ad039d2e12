"""Pins for the fp64 oracle: closed forms, invariants, a hand-worked model and brute force.

None of these re-types the oracle's formulas: each compares it with something fixed by the
mathematics (a closed form, an identity, a special case) or with an independent evaluator.
"""
import math
import os
from types import SimpleNamespace

import numpy as np
import pytest

from oracle import vla_oracle as O
from tests import bruteforce_policy as BF

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def shape(L=2, d=16, H=2, hd=8, f=24, V=40, A=8, theta=1.0e4, eps=1.0e-5):
    return SimpleNamespace(n_layers=L, d_model=d, n_heads=H, head_dim=hd, d_ffn=f, vocab=V,
                           n_action_bins=A, rope_theta=theta, rms_eps=eps)


def rand_weights(s, seed=0, std=0.3):
    g = np.random.default_rng(seed)
    d, f, V = s.d_model, s.d_ffn, s.vocab
    w = {"embed": g.normal(0, 1.0, (V, d)), "lm_head": g.normal(0, std, (V, d)),
         "final_norm": 1 + g.normal(0, 0.1, d)}
    for l in range(s.n_layers):
        p = f"layers.{l}."
        w[p + "attn_norm"] = 1 + g.normal(0, 0.1, d)
        w[p + "ffn_norm"] = 1 + g.normal(0, 0.1, d)
        for n in ("wq", "wk", "wv", "wo"):
            w[p + n] = g.normal(0, std, (d, d))
        w[p + "w_gate"] = g.normal(0, std, (f, d))
        w[p + "w_up"] = g.normal(0, std, (f, d))
        w[p + "w_down"] = g.normal(0, std, (d, f))
    return w


def rand_obs(s, B, Np, lens, seed=1):
    g = np.random.default_rng(seed)
    pes = [g.normal(0, 1, (Np, s.d_model)) for _ in range(B)]
    ids = [g.integers(0, s.vocab - s.n_action_bins, size=n) for n in lens]
    return pes, ids


def read_golden(name):
    vals = {}
    for line in open(os.path.join(GOLDEN, name)):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        vals[k] = float(v)
    return vals


# ---- hand-worked one-layer model -----------------------------------------------------------

def handworked_model():
    s = shape(L=1, d=2, H=1, hd=2, f=2, V=4, A=2, theta=1.0e4, eps=0.0)
    I = np.eye(2)
    w = {"embed": np.zeros((4, 2)), "lm_head": np.vstack([np.zeros((2, 2)), I]),
         "final_norm": np.ones(2), "layers.0.attn_norm": np.ones(2), "layers.0.ffn_norm": np.ones(2)}
    for n in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
        w["layers.0." + n] = I.copy()
    return s, w


def test_handworked_values_match_fixture():
    gold = read_golden("handworked_1layer.txt")
    s, w = handworked_model()
    pol = O.OraclePolicy(s, w)
    x = np.array([[1.0, 1.0], [1.0, -1.0]])
    st = O.SeqState(1)
    out = pol.run_layers([x], [st])[0]
    # intermediates kept by the oracle: rotated key/query of position 1
    assert st.k[0][1, 0, 0] == pytest.approx(gold["q1_0"], abs=1e-11)
    assert st.k[0][1, 0, 1] == pytest.approx(gold["q1_1"], abs=1e-11)
    assert out[1, 0] == pytest.approx(gold["xout_0"], abs=1e-11)
    assert out[1, 1] == pytest.approx(gold["xout_1"], abs=1e-11)
    z = pol.action_logits(out[1])
    assert z[0] == pytest.approx(gold["z_0"], abs=1e-11)
    assert z[1] == pytest.approx(gold["z_1"], abs=1e-11)
    r = pol.policy_step([x], [np.zeros(0, dtype=np.int64)], 1, temperature=0.0)
    assert r["logp"][0, 0] == pytest.approx(gold["logp_0"], abs=1e-11)
    assert r["tokens"][0, 0] == int(gold["token"])
    assert r["actions"][0, 0] == gold["action"]
    # the other bin's log-prob
    assert O.log_softmax(z)[1] == pytest.approx(gold["logp_1"], abs=1e-11)


def test_handworked_closed_forms():
    """The same model through closed forms worked out by hand (trigonometric identities)."""
    s, w = handworked_model()
    pol = O.OraclePolicy(s, w)
    x = np.array([[1.0, 1.0], [1.0, -1.0]])
    st = O.SeqState(1)
    out = pol.run_layers([x], [st])[0]
    # position 0: z = (1,1), tie -> bin 0, logp = -ln 2, x'' = 2 + silu(1)
    silu1 = 1.0 / (1.0 + math.exp(-1.0))
    assert out[0] == pytest.approx([2 + silu1, 2 + silu1], abs=1e-14)
    r0 = pol.policy_step([x[:1]], [np.zeros(0, dtype=np.int64)], 1)
    assert r0["tokens"][0, 0] == 0 and r0["logp"][0, 0] == pytest.approx(-math.log(2), abs=1e-14)
    # position 1: attention weight on itself is a logistic of sqrt2 (1 - sin 1)
    a11 = 1.0 / (1.0 + math.exp(-math.sqrt(2) * (1 - math.sin(1))))
    x_mid1 = -1 + (1 - a11) - a11
    rms = math.sqrt((4 + x_mid1 ** 2) / 2)
    h = (2 / rms, x_mid1 / rms)
    f = [t * t / (1 + math.exp(-t)) for t in h]
    assert out[1] == pytest.approx([2 + f[0], x_mid1 + f[1]], abs=1e-13)


# ---- invariants and special cases ----------------------------------------------------------

def test_softmax_rows_and_logp_bounds():
    g = np.random.default_rng(3)
    s = g.normal(0, 5, (7, 33))
    assert np.allclose(O.softmax(s).sum(-1), 1.0, atol=1e-12)
    z = g.normal(0, 3, (5, 256))
    ell = O.log_softmax(z, 0.7)
    assert np.allclose(np.exp(ell).sum(-1), 1.0, atol=1e-12)
    assert (ell <= 0).all()
    # the greedy token is the mode: its probability is at least 1/A
    assert (ell.max(-1) >= -math.log(256) - 1e-12).all()
    # huge logits do not overflow
    assert np.isfinite(O.log_softmax(np.array([1e4, -1e4, 0.0]))).all()


def test_single_position_attention_returns_v():
    g = np.random.default_rng(4)
    q, k, v = g.normal(size=(1, 3, 8)), g.normal(size=(1, 3, 8)), g.normal(size=(1, 3, 8))
    out = O.causal_attention(q, k, v, np.array([0]))
    assert np.array_equal(out, v)


def test_attention_matches_scalar_loops():
    g = np.random.default_rng(5)
    n, H, hd = 5, 2, 4
    q, k, v = g.normal(size=(n, H, hd)), g.normal(size=(n, H, hd)), g.normal(size=(n, H, hd))
    out = O.causal_attention(q, k, v, np.arange(n))
    for p in range(n):
        for h in range(H):
            sc = [sum(q[p, h, j] * k[t, h, j] for j in range(hd)) / math.sqrt(hd) for t in range(p + 1)]
            e = [math.exp(c - max(sc)) for c in sc]
            for j in range(hd):
                ref = sum(e[t] * v[t, h, j] for t in range(p + 1)) / sum(e)
                assert out[p, h, j] == pytest.approx(ref, abs=1e-13)


def test_cached_equals_recompute():
    s = shape()
    pol = O.OraclePolicy(s, rand_weights(s))
    pes, ids = rand_obs(s, 3, 4, [3, 5, 2])
    a = pol.policy_step(pes, ids, 5, mode="recompute")
    b = pol.policy_step(pes, ids, 5, mode="cached")
    assert np.array_equal(a["tokens"], b["tokens"])
    assert np.abs(a["logits"] - b["logits"]).max() < 1e-12
    assert np.abs(a["logp"] - b["logp"]).max() < 1e-12
    # and under sampling with forced history
    gum = np.random.default_rng(9).gumbel(size=(3, 5, s.n_action_bins))
    forced = np.random.default_rng(10).integers(0, s.n_action_bins, size=(3, 5))
    a = pol.policy_step(pes, ids, 5, temperature=1.3, gumbel=gum, forced_tokens=forced, mode="recompute")
    b = pol.policy_step(pes, ids, 5, temperature=1.3, gumbel=gum, forced_tokens=forced, mode="cached")
    assert np.array_equal(a["tokens"], b["tokens"])
    assert np.abs(a["logits"] - b["logits"]).max() < 1e-12


def test_zero_output_projections_reduce_to_head():
    s = shape(L=3)
    w = rand_weights(s)
    for l in range(s.n_layers):
        w[f"layers.{l}.wo"][:] = 0
        w[f"layers.{l}.w_down"][:] = 0
    pol = O.OraclePolicy(s, w)
    pes, ids = rand_obs(s, 1, 3, [2])
    r = pol.policy_step(pes, ids, 1)
    x_last = w["embed"][ids[0][-1]]
    h = x_last / math.sqrt(float(np.mean(x_last ** 2)) + s.rms_eps) * w["final_norm"]
    z = w["lm_head"][s.vocab - s.n_action_bins:] @ h
    assert np.abs(r["logits"][0, 0] - z).max() < 1e-12


def test_zero_queries_give_running_mean_of_v():
    s = shape(L=1)
    w = rand_weights(s)
    w["layers.0.wq"][:] = 0
    pol = O.OraclePolicy(s, w)
    g = np.random.default_rng(6)
    x = g.normal(size=(6, s.d_model))
    st = O.SeqState(1)
    # make the rest of the layer transparent so the attention output is observable
    w["layers.0.wo"] = np.eye(s.d_model)
    w["layers.0.w_down"][:] = 0
    out = pol.run_layers([x], [st])[0]
    v = st.v[0].reshape(6, -1)
    run_mean = np.cumsum(v, axis=0) / np.arange(1, 7)[:, None]
    assert np.abs((out - x) - run_mean).max() < 1e-12


def test_rope_norm_and_shift_invariance():
    g = np.random.default_rng(7)
    u = g.normal(size=(5, 2, 8))
    pos = np.array([0, 1, 2, 10, 300])
    r = O.rope(u, pos, 1.0e4)
    assert np.allclose(np.linalg.norm(r, axis=-1), np.linalg.norm(u, axis=-1), atol=1e-12)
    assert np.array_equal(O.rope(u[:1], np.array([0]), 1.0e4), u[:1])
    # first pair of each head turns by exactly pos radians (frequency theta^0 = 1)
    assert r[3, 0, 0] == pytest.approx(u[3, 0, 0] * math.cos(10) - u[3, 0, 4] * math.sin(10), abs=1e-13)
    assert r[3, 0, 4] == pytest.approx(u[3, 0, 4] * math.cos(10) + u[3, 0, 0] * math.sin(10), abs=1e-13)
    # last pair turns by pos * theta^(-(hd-2)/hd)
    ang = 300 * 1.0e4 ** (-6 / 8)
    assert r[4, 1, 3] == pytest.approx(u[4, 1, 3] * math.cos(ang) - u[4, 1, 7] * math.sin(ang), abs=1e-12)
    # q.k depends on the position difference only
    q, k = g.normal(size=(1, 1, 8)), g.normal(size=(1, 1, 8))
    d0 = np.sum(O.rope(q, np.array([7]), 1e4) * O.rope(k, np.array([3]), 1e4))
    d1 = np.sum(O.rope(q, np.array([107]), 1e4) * O.rope(k, np.array([103]), 1e4))
    assert d0 == pytest.approx(d1, abs=1e-11)


def test_attention_invariant_to_global_position_shift():
    """Rotating queries and keys at positions p + c instead of p leaves attention unchanged."""
    g = np.random.default_rng(8)
    n, H, hd = 6, 2, 8
    q, k, v = g.normal(size=(n, H, hd)), g.normal(size=(n, H, hd)), g.normal(size=(n, H, hd))
    pos = np.arange(n)
    a = O.causal_attention(O.rope(q, pos, 1e4), O.rope(k, pos, 1e4), v, pos)
    b = O.causal_attention(O.rope(q, pos + 13, 1e4), O.rope(k, pos + 13, 1e4), v, pos)
    assert np.abs(a - b).max() < 1e-12
    # a non-uniform change of positions does change it (so positions are really used)
    c = O.causal_attention(O.rope(q, pos * 2, 1e4), O.rope(k, pos * 2, 1e4), v, pos)
    assert np.abs(a - c).max() > 1e-3


def test_causality():
    s = shape()
    pol = O.OraclePolicy(s, rand_weights(s))
    x = np.random.default_rng(11).normal(size=(6, s.d_model))
    y = x.copy()
    y[4] += 1.0
    sa, sb = O.SeqState(s.n_layers), O.SeqState(s.n_layers)
    a = pol.run_layers([x], [sa])[0]
    b = pol.run_layers([y], [sb])[0]
    assert np.array_equal(a[:4], b[:4])
    assert not np.allclose(a[4:], b[4:])
    for l in range(s.n_layers):
        assert np.array_equal(sa.k[l][:4], sb.k[l][:4]) and np.array_equal(sa.v[l][:4], sb.v[l][:4])


def test_batch_independence_and_permutation():
    s = shape()
    pol = O.OraclePolicy(s, rand_weights(s))
    pes, ids = rand_obs(s, 3, 4, [2, 6, 4])
    full = pol.policy_step(pes, ids, 4, mode="cached")
    for b in range(3):
        alone = pol.policy_step([pes[b]], [ids[b]], 4, mode="cached")
        assert np.array_equal(alone["tokens"][0], full["tokens"][b])
        assert np.abs(alone["logits"][0] - full["logits"][b]).max() < 1e-12
    perm = [2, 0, 1]
    pr = pol.policy_step([pes[i] for i in perm], [ids[i] for i in perm], 4, mode="cached")
    assert np.array_equal(pr["tokens"], full["tokens"][perm])


def test_slimming_equals_masked_full_vocab():
    """Cropping the head to the action rows == full-vocabulary logits with the rest at -inf."""
    s = shape()
    pol = O.OraclePolicy(s, rand_weights(s))
    x = np.random.default_rng(12).normal(size=(s.d_model,))
    z = pol.action_logits(x)
    full = pol.full_vocab_logits(x)
    masked = np.full(s.vocab, -np.inf)
    masked[s.vocab - s.n_action_bins:] = full[s.vocab - s.n_action_bins:]
    m = masked.max()
    lse = m + math.log(sum(math.exp(t - m) for t in masked if t > -np.inf))
    assert np.abs(O.log_softmax(z) - (masked - lse)[s.vocab - s.n_action_bins:]).max() < 1e-12
    # a pre-slimmed head gives the same logits
    w2 = dict(pol.w)
    w2["lm_head"] = pol.w["lm_head"][s.vocab - s.n_action_bins:]
    assert np.array_equal(O.OraclePolicy(s, w2).action_logits(x), z)


def test_chunk_logprob_is_sum_of_token_logprobs():
    """sum_k logp_k = log prod_k pi(a_k | o, a_<k), each factor evaluated separately."""
    s = shape()
    pol = O.OraclePolicy(s, rand_weights(s))
    pes, ids = rand_obs(s, 1, 3, [3])
    r = pol.policy_step(pes, ids, 4)
    prob = 1.0
    rows = pol.prefix_rows(pes[0], ids[0])
    for k in range(4):
        out = pol.run_layers([rows], [O.SeqState(s.n_layers)])[0]
        p = O.softmax(pol.action_logits(out[-1]))
        prob *= p[r["tokens"][0, k]]
        rows = np.concatenate([rows, pol.token_rows([s.vocab - s.n_action_bins + r["tokens"][0, k]])])
    assert r["logp"].shape == (1, 4)
    assert r["logp"][0].sum() == pytest.approx(math.log(prob), abs=1e-12)


def test_gumbel_zero_is_greedy_and_frequencies_match_softmax():
    g = np.random.default_rng(13)
    z = g.normal(0, 1.3, 16)
    t0, _ = O.select_token(z, 1.0, np.zeros(16))
    assert t0 == int(np.argmax(z)) == O.select_token(z, 0.0, None)[0]
    # exact ties -> lowest index
    assert O.select_token(np.array([1.0, 3.0, 3.0, 2.0]), 0.0, None)[0] == 1
    n = 200_000
    tau = 0.8
    noise = g.gumbel(size=(n, 16))
    counts = np.bincount(np.argmax(z / tau + noise, axis=1), minlength=16)
    # the oracle's selection on single draws agrees with the vectorised argmax
    for i in range(50):
        assert O.select_token(z, tau, noise[i])[0] == int(np.argmax(z / tau + noise[i]))
    p = np.exp(O.log_softmax(z, tau))
    chi2 = float(((counts - n * p) ** 2 / (n * p)).sum())
    assert chi2 < 50.0            # 15 d.o.f.: P(chi2 > 50) ~ 1e-5


def test_temperature_logprob_is_of_the_sampled_distribution():
    z = np.array([0.3, -1.2, 2.0, 0.1])
    ell = O.log_softmax(z, 2.0)
    p = np.exp(z / 2.0) / np.exp(z / 2.0).sum()
    assert np.allclose(np.exp(ell), p, atol=1e-15)


def test_detokeniser_closed_form():
    A = 256
    c = O.bin_centre(np.arange(A), A)
    assert c[0] == -1 + 1 / A == -0.99609375 and c[-1] == 1 - 1 / A
    assert np.array_equal(np.diff(c), np.full(A - 1, 2 / A))
    assert np.array_equal(c, -c[::-1])
    toks = np.array([[0, 255, 128, 127, 5, 6, 7, 0, 1]])
    sc, off = np.arange(1.0, 8.0), np.arange(7.0) * 0.5
    a = O.detokenise(toks, A, 7, sc, off)
    assert a[0, 1] == c[255] * 2.0 + 0.5 and a[0, 7] == c[0] * 1.0 + 0.0 and a[0, 8] == c[1] * 2.0 + 0.5


# ---- brute force -----------------------------------------------------------------------------

@pytest.mark.parametrize("seed", [0, 1])
def test_against_pure_python_loops(seed):
    s = shape(L=2, d=8, H=2, hd=4, f=6, V=12, A=4)
    w = rand_weights(s, seed=seed, std=0.5)
    cfg = dict(L=2, d=8, H=2, hd=4, f=6, V=12, A=4, theta=s.rope_theta, eps=s.rms_eps)
    Wt = {k: v.tolist() for k, v in w.items()}
    pes, ids = rand_obs(s, 1, 2, [2], seed=seed + 20)
    rows = [r.tolist() for r in pes[0]] + [Wt["embed"][i] for i in ids[0]]
    toks, lps = BF.greedy_rollout(cfg, Wt, rows, 3)
    z0 = BF.forward_logits(cfg, Wt, rows)
    pol = O.OraclePolicy(s, w)
    for mode in ("recompute", "cached"):
        r = pol.policy_step(pes, ids, 3, mode=mode)
        assert r["tokens"][0].tolist() == toks
        assert np.abs(r["logp"][0] - np.array(lps)).max() < 1e-12
        assert np.abs(r["logits"][0, 0] - np.array(z0)).max() < 1e-12


def test_widen_bf16_and_f32_exact():
    bits = np.array([0x3F80, 0xBF80, 0x3F81, 0x0000, 0x4049], dtype=np.uint16)
    assert O.widen(bits).tolist() == [1.0, -1.0, 1.0078125, 0.0, 3.140625]
    x = np.array([0.1], dtype=np.float32)
    assert O.widen(x)[0] == float(x[0])


# ---- value head (attention pooling over the action positions + step embedding + GELU MLP) --------------

def value_weights(d, n_steps=5, seed=0):
    g = np.random.default_rng(seed)
    return {"attn_w": g.normal(0, 0.5, d), "attn_b": np.array(0.3), "step_emb": g.normal(0, 0.5, (n_steps, d)),
            "w1": g.normal(0, 0.4, (d, d)), "b1": g.normal(0, 0.1, d), "w2": g.normal(0, 0.4, d), "b2": np.array(-0.2)}


def test_gelu_constants():
    # Phi(1) = 0.841344746068543, Phi(-1) = 0.158655253931457 (standard normal table)
    assert O.gelu(np.array([0.0]))[0] == 0.0
    assert O.gelu(np.array([1.0]))[0] == pytest.approx(0.841344746068543, abs=1e-14)
    assert O.gelu(np.array([-1.0]))[0] == pytest.approx(-0.158655253931457, abs=1e-14)
    assert O.gelu(np.array([10.0]))[0] == pytest.approx(10.0, abs=1e-12)


def test_value_head_special_cases():
    d, K = 6, 4
    g = np.random.default_rng(31)
    h = g.normal(size=(K, d))
    vw = value_weights(d)
    # zero attention projection -> uniform pooling -> the mean of the hidden states
    vw0 = dict(vw, attn_w=np.zeros(d), w1=np.eye(d), b1=np.zeros(d), w2=np.ones(d), b2=np.array(0.0),
               step_emb=np.zeros((5, d)))
    z = h.mean(0)
    assert O.value_head(h, 2, vw0) == pytest.approx(float(sum(t * 0.5 * (1 + math.erf(t / math.sqrt(2))) for t in z)), abs=1e-13)
    # one token: the pooled vector is that token whatever the scores
    v1 = O.value_head(h[:1], 1, vw)
    u = h[0] + vw["step_emb"][1]
    hid = [sum(vw["w1"][j, i] * u[i] for i in range(d)) + vw["b1"][j] for j in range(d)]
    ref = sum(vw["w2"][j] * hid[j] * 0.5 * (1 + math.erf(hid[j] / math.sqrt(2))) for j in range(d)) + float(vw["b2"])
    assert v1 == pytest.approx(ref, abs=1e-13)
    # the attention bias shifts every score equally: no effect; token order does not matter
    assert O.value_head(h, 3, dict(vw, attn_b=np.array(5.0))) == pytest.approx(O.value_head(h, 3, vw), abs=1e-12)
    assert O.value_head(h[::-1], 3, vw) == pytest.approx(O.value_head(h, 3, vw), abs=1e-12)
    # the step embedding matters
    assert abs(O.value_head(h, 0, vw) - O.value_head(h, 4, vw)) > 1e-3


def test_value_head_against_scalar_loops():
    d, K = 5, 3
    g = np.random.default_rng(32)
    h = g.normal(size=(K, d))
    vw = value_weights(d, seed=3)
    e = [sum(h[k, i] * vw["attn_w"][i] for i in range(d)) + float(vw["attn_b"]) for k in range(K)]
    m = max(e)
    a = [math.exp(t - m) for t in e]
    a = [t / sum(a) for t in a]
    z = [sum(a[k] * h[k, i] for k in range(K)) + vw["step_emb"][2, i] for i in range(d)]
    hid = [sum(vw["w1"][j, i] * z[i] for i in range(d)) + vw["b1"][j] for j in range(d)]
    v = sum(vw["w2"][j] * hid[j] * 0.5 * (1 + math.erf(hid[j] / math.sqrt(2))) for j in range(d)) + float(vw["b2"])
    assert O.value_head(h, 2, vw) == pytest.approx(v, abs=1e-13)


def test_policy_step_returns_the_hidden_rows_that_feed_the_head():
    s = shape()
    w = rand_weights(s)
    pol = O.OraclePolicy(s, w)
    pes, ids = rand_obs(s, 2, 3, [2, 4])
    r = pol.policy_step(pes, ids, 3, mode="cached")
    head = w["lm_head"][s.vocab - s.n_action_bins:]
    assert r["hidden"].shape == (2, 3, s.d_model)
    assert np.abs(r["hidden"] @ head.T - r["logits"]).max() < 1e-12


# ---- all K action rows in one pass: parallel decoding, stored-token evaluation, GIPO coefficients --------

def test_gipo_weight_closed_forms():
    """omega(rho; sigma) = exp(-(log rho / sigma)^2 / 2) (Section 3.3); rho from the two log-probabilities."""
    assert O.importance_ratio(-1.25, -1.25) == 1.0
    assert O.importance_ratio(math.log(0.3), math.log(0.6)) == pytest.approx(0.5, abs=1e-15)
    assert O.gipo_trust_weight(1.0, 0.7) == 1.0                                   # on-policy: no damping
    for sigma in (0.25, 1.0, 3.0):
        assert O.gipo_trust_weight(math.exp(sigma), sigma) == pytest.approx(math.exp(-0.5), abs=1e-15)
        assert O.gipo_trust_weight(math.exp(-2 * sigma), sigma) == pytest.approx(math.exp(-2.0), abs=1e-15)
    # a number worked by hand: sigma = 0.5, rho = 2: (ln 2 / 0.5)^2 / 2 = 0.960906 -> 0.382546
    assert O.gipo_trust_weight(2.0, 0.5) == pytest.approx(0.382546, abs=2e-6)
    rho = np.array([0.1, 0.5, 0.9, 1.1, 2.0, 10.0])
    w = O.gipo_trust_weight(rho, 0.8)
    assert np.allclose(w, O.gipo_trust_weight(1.0 / rho, 0.8), rtol=0, atol=1e-15)      # symmetric in log rho
    assert np.all(w < 1.0) and np.all(np.diff(w[:3]) > 0) and np.all(np.diff(w[3:]) < 0)  # peak at rho = 1
    assert O.gipo_trust_weight(1e6, 0.5) < 1e-100                                         # extreme ratios vanish smoothly


def test_chunk_rows_against_pure_python_prefixes():
    """Causality pins the chunk pass: row k of one pass over [prefix ; fed] equals the last-position logits of
    the sequence cut after S + k rows, computed by the pure-Python loops."""
    s = shape(L=2, d=8, H=2, hd=4, f=6, V=12, A=4)
    w = rand_weights(s, seed=5, std=0.5)
    cfg = dict(L=2, d=8, H=2, hd=4, f=6, V=12, A=4, theta=s.rope_theta, eps=s.rms_eps)
    Wt = {k: v.tolist() for k, v in w.items()}
    pes, ids = rand_obs(s, 1, 2, [3], seed=31)
    fed = np.array([[9, 2, 11]])                       # any vocabulary ids, K = 4
    rows = [r.tolist() for r in pes[0]] + [Wt["embed"][i] for i in ids[0]] + [Wt["embed"][i] for i in fed[0]]
    S = len(rows) - 3
    got = O.OraclePolicy(s, w).chunk_logits(pes, ids, fed)
    assert got.shape == (1, 4, 4)
    for k in range(4):
        want = np.array(BF.forward_logits(cfg, Wt, rows[:S + k]))
        assert np.abs(got[0, k] - want).max() < 1e-12, k


def test_parallel_decoding_reductions():
    s = shape()
    w = rand_weights(s, seed=2)
    pol = O.OraclePolicy(s, w)
    pes, ids = rand_obs(s, 3, 4, [0, 2, 5], seed=8)
    A, K = s.n_action_bins, 5
    ph_bin = 3
    ph = s.vocab - A + ph_bin
    par = pol.policy_step_parallel(pes, ids, K, ph)
    # (a) it is the autoregressive path with the placeholder fed back instead of the selected token
    for mode in ("recompute", "cached"):
        ar = pol.policy_step(pes, ids, K, mode=mode, forced_tokens=np.full((3, K), ph_bin))
        assert np.abs(par["logits"] - ar["logits"]).max() < 1e-11
        assert np.array_equal(par["tokens"], ar["tokens"]) and np.abs(par["logp"] - ar["logp"]).max() < 1e-11
    # (b) the first token does not depend on the placeholder at all, and K = 1 is the ordinary step
    other = pol.policy_step_parallel(pes, ids, K, 1)
    assert np.abs(other["logits"][:, 0] - par["logits"][:, 0]).max() < 1e-12
    assert np.abs(other["logits"][:, 1:] - par["logits"][:, 1:]).max() > 1e-3
    one = pol.policy_step_parallel(pes, ids, 1, ph)
    assert np.abs(one["logits"] - pol.policy_step(pes, ids, 1)["logits"]).max() < 1e-12
    # (c) conditional independence: noise at one position moves only that position's token
    g = np.random.default_rng(4).gumbel(size=(3, K, A))
    base = pol.policy_step_parallel(pes, ids, K, ph, temperature=0.9, gumbel=g)
    g2 = g.copy()
    g2[:, 2] = np.random.default_rng(5).gumbel(size=(3, A)) * 5
    moved = pol.policy_step_parallel(pes, ids, K, ph, temperature=0.9, gumbel=g2)
    keep = [0, 1, 3, 4]
    assert np.array_equal(base["tokens"][:, keep], moved["tokens"][:, keep])
    assert np.array_equal(base["logits"], moved["logits"])
    assert not np.array_equal(base["tokens"][:, 2], moved["tokens"][:, 2])
    assert np.all(base["actions"] == O.bin_centre(base["tokens"], A))
    # log-probs are a normalised distribution at temperature tau over the bins
    ell = O.log_softmax(base["logits"], 0.9)
    assert np.abs(np.exp(ell).sum(-1) - 1).max() < 1e-12
    assert np.abs(np.take_along_axis(ell, base["tokens"][..., None], -1)[..., 0] - base["logp"]).max() < 1e-12


def test_score_tokens_reproduces_behaviour_logp_and_gipo():
    s = shape()
    w = rand_weights(s, seed=6)
    pol = O.OraclePolicy(s, w)
    pes, ids = rand_obs(s, 2, 3, [1, 4], seed=9)
    A, K = s.n_action_bins, 4
    g = np.random.default_rng(7).gumbel(size=(2, K, A))
    beh = pol.policy_step(pes, ids, K, temperature=1.3, gumbel=g, mode="cached")
    sc = pol.score_tokens(pes, ids, beh["tokens"], temperature=1.3, mu_logp=beh["logp"], sigma=0.4)
    assert np.abs(sc["logp"] - beh["logp"]).max() < 1e-11          # same weights: learner == behaviour
    assert np.abs(sc["ratio"] - 1).max() < 1e-10 and np.abs(sc["weight"] - 1).max() < 1e-10
    assert np.abs(sc["logits"] - beh["logits"]).max() < 1e-11
    # other weights: rho = exp(logp' - mu), coefficient = omega * rho, token by token
    pol2 = O.OraclePolicy(s, rand_weights(s, seed=66))
    sc2 = pol2.score_tokens(pes, ids, beh["tokens"], temperature=1.3, mu_logp=beh["logp"], sigma=0.4)
    for b in range(2):
        for k in range(K):
            rho = math.exp(sc2["logp"][b, k] - beh["logp"][b, k])
            assert sc2["ratio"][b, k] == pytest.approx(rho, rel=1e-12)
            assert sc2["weight"][b, k] == pytest.approx(rho * math.exp(-0.5 * (math.log(rho) / 0.4) ** 2), rel=1e-10)
    assert np.abs(sc2["ratio"] - 1).max() > 0.05
    # placeholder conditioning scores the tokens of the parallel policy
    ph = s.vocab - A + 2
    par = pol.policy_step_parallel(pes, ids, K, ph, temperature=1.3, gumbel=g)
    scp = pol.score_tokens(pes, ids, par["tokens"], temperature=1.3, placeholder_id=ph)
    assert np.abs(scp["logp"] - par["logp"]).max() < 1e-11
