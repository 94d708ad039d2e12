"""fp64 CPU oracle for batched Vision-Language-Action policy inference.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what the
HIP library must compute.  Only the tests, the smoke check and the
`cpu_baseline` leg of the benchmark may import it; the product path never does,
and this file imports nothing from the product.

What is computed (one observation = one sequence; sequences never interact):

  * the rollout policy is a decoder-only transformer over the prefix
    [visual patch embeddings ; instruction tokens] that emits K discretised
    action tokens autoregressively (Appendix "Experiment Setup": OpenVLA-OFT on a
    Llama-2-7B backbone, discretised action tokens, action chunking);
  * the output head is the language-model head cut down to the rows of the
    action bins, so the distribution lives on the 256 bins only
    (Appendix "Vocabulary Slimming");
  * the behaviour probability of every chosen token is recorded for off-policy
    correction (Section 3.2, Eq. 2: mu_t in the trajectory tuple), one value per
    token, never summed over the chunk (Appendix "Token-level Policy
    Optimization"); it is returned as a log-probability.

The paper does not spell out the backbone.  The readings taken here are those of
a public Llama-family decoder: pre-norm RMSNorm (eps inside the square root,
gain applied after normalisation), rotary embedding on half-split pairs
(i, i + hd/2) with positions counted from the first patch, causal softmax
attention scaled by 1/sqrt(hd), SwiGLU feed-forward, no biases, final RMSNorm
before the head.  Action bin j is vocabulary id V - A + j and de-tokenises to the
centre of the j-th of A equal bins on [-1, 1].

Everything is float64.  Weights and patch embeddings arrive in their storage
dtype (float32, or bfloat16 bit patterns) and are widened exactly.  There is no
intermediate rounding, no tiling and no fusion.  Library matmul (numpy) is used
as a primitive step.

Two evaluation modes exist:
  "recompute": for every emitted token the whole sequence so far is pushed
               through all layers from scratch (the definition);
  "cached":    keys/values of earlier positions are kept and only the new
               position is pushed through (proved equal to "recompute" by the
               tests; used where recompute would take hours).

Pins (tests/test_oracle_*.py): softmax rows sum to one, one-position attention
returns v, cached == recompute, a hand-worked one-layer model, zeroed output
projections, zeroed queries (running mean of v), rotary shift invariance,
causality, batch independence, slimming == masking the full vocabulary, chunk
log-probability, Gumbel-max statistics, a separate pure-Python loop evaluator,
the de-tokeniser's closed form, and for the value head: uniform pooling, single
token, GELU constants, bias and permutation invariance, scalar loops.  Agreement with the paper's *trained*
policy is parity unpinned: its weights and datasets are not available.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Optional, Sequence

import numpy as np

_POOL = ThreadPoolExecutor(max_workers=8)


def widen(a: np.ndarray) -> np.ndarray:
    """Storage dtype -> float64, exactly.  uint16 arrays are bfloat16 bit patterns."""
    if a.dtype == np.float64:
        return a
    if a.dtype == np.float32:
        return a.astype(np.float64)
    if a.dtype != np.uint16:
        raise TypeError(a.dtype)

    out = np.empty(a.shape, dtype=np.float64)

    def one(rows):
        chunk = a[rows]
        out[rows] = (chunk.astype(np.uint32) << np.uint32(16)).view(np.float32)

    if a.size < (1 << 22) or a.ndim < 2:
        one(slice(None))
        return out
    step = -(-a.shape[0] // 16)
    list(_POOL.map(one, [slice(i, i + step) for i in range(0, a.shape[0], step)]))
    return out


# ----------------------------------------------------------------------------
# elementary operations
# ----------------------------------------------------------------------------

def rms_norm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """x * gain / sqrt(mean(x^2) + eps) over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope(u: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding.  u: [n, H, hd]; pos: [n] integer positions.

    Pair (i, i + hd/2) is rotated by the angle pos * theta^(-2i/hd).
    """
    hd = u.shape[-1]
    half = hd // 2
    i = np.arange(half, dtype=np.float64)
    inv_freq = theta ** (-2.0 * i / hd)
    phi = pos.astype(np.float64)[:, None] * inv_freq[None, :]       # [n, half]
    c, s = np.cos(phi)[:, None, :], np.sin(phi)[:, None, :]
    a, b = u[..., :half], u[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def softmax(s: np.ndarray) -> np.ndarray:
    e = np.exp(s - np.max(s, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


def causal_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, q_pos: np.ndarray) -> np.ndarray:
    """q: [n, H, hd] at absolute positions q_pos; k, v: [ctx, H, hd] at positions 0..ctx-1.

    Query at position p attends to keys p' <= p.  Returns [n, H, hd].
    """
    n, H, hd = q.shape
    ctx = k.shape[0]
    out = np.empty_like(q)
    allowed = np.arange(ctx)[None, :] <= q_pos[:, None]              # [n, ctx]
    for h in range(H):
        s = q[:, h, :] @ k[:, h, :].T / np.sqrt(hd)                  # [n, ctx]
        s = np.where(allowed, s, -np.inf)
        out[:, h, :] = softmax(s) @ v[:, h, :]
    return out


def silu(t: np.ndarray) -> np.ndarray:
    return t / (1.0 + np.exp(-t))


def log_softmax(z: np.ndarray, temperature: float = 1.0) -> np.ndarray:
    """log softmax(z / temperature) over the last axis."""
    y = z / temperature
    m = np.max(y, axis=-1, keepdims=True)
    return y - (m + np.log(np.sum(np.exp(y - m), axis=-1, keepdims=True)))


def select_token(z: np.ndarray, temperature: float, gumbel: Optional[np.ndarray]):
    """Selection scores z/temperature (+ Gumbel noise); lowest index among exact maxima.

    temperature == 0 means greedy with the log-prob taken at temperature 1.
    Returns (bin index, scores).
    """
    tau = 1.0 if temperature == 0 else temperature
    scores = z / tau
    if gumbel is not None and temperature != 0:
        scores = scores + gumbel.astype(np.float64)
    return int(np.argmax(scores)), scores


def bin_centre(t, n_bins: int):
    """Centre of the t-th of n_bins equal-width bins on [-1, 1]."""
    return -1.0 + (2.0 * np.asarray(t, dtype=np.float64) + 1.0) / n_bins


def detokenise(tokens: np.ndarray, n_bins: int, action_dim: int = 1,
               scale: Optional[np.ndarray] = None, offset: Optional[np.ndarray] = None) -> np.ndarray:
    """tokens [..., K] -> continuous actions; token k belongs to action dimension k mod action_dim
    (timestep-major chunk), and gets that dimension's optional affine map."""
    a = bin_centre(tokens, n_bins)
    dim = np.arange(a.shape[-1]) % action_dim
    if scale is not None:
        a = a * np.asarray(scale, dtype=np.float64)[dim]
    if offset is not None:
        a = a + np.asarray(offset, dtype=np.float64)[dim]
    return a


def gelu(t: np.ndarray) -> np.ndarray:
    """Exact GELU: t * Phi(t), Phi the standard normal CDF."""
    from math import erf, sqrt
    return t * 0.5 * (1.0 + np.vectorize(erf)(t / sqrt(2.0)))


def value_head(hidden: np.ndarray, step_t: int, vw: dict) -> float:
    """State value from the hidden states of the K action-related positions (Appendix "Value Head
    Design"): scores e_k = w_attn . h_k + b_attn, weights alpha = softmax_k(e), pooled z = sum_k alpha_k h_k,
    plus the embedding of the episode step, then Linear(d,d) -> GELU -> Linear(d,1).

    hidden: [K, d] float64 (the last hidden layer's output at the positions that emit the K action
    tokens; the policy's hidden states are inputs only, nothing flows back).
    vw: "attn_w" [d], "attn_b" scalar, "step_emb" [n_steps, d], "w1" [d, d] (nn.Linear layout), "b1" [d],
    "w2" [d], "b2" scalar, in storage dtype or float64."""
    h = np.asarray(hidden, dtype=np.float64)
    e = h @ widen(np.asarray(vw["attn_w"])).reshape(-1) + float(widen(np.asarray(vw["attn_b"]).reshape(1))[0])
    alpha = softmax(e)
    z = alpha @ h
    u = z + widen(np.asarray(vw["step_emb"]))[int(step_t)]
    hid = gelu(widen(np.asarray(vw["w1"])) @ u + widen(np.asarray(vw["b1"])).reshape(-1))
    return float(widen(np.asarray(vw["w2"])).reshape(-1) @ hid + float(widen(np.asarray(vw["b2"]).reshape(1))[0]))


def importance_ratio(logp: np.ndarray, mu_logp: np.ndarray) -> np.ndarray:
    """Token-level importance ratio rho = pi_theta(a_k | .) / mu(a_k | .) (Appendix "Token-level Policy
    Optimization"), from the two log-probabilities."""
    return np.exp(np.asarray(logp, dtype=np.float64) - np.asarray(mu_logp, dtype=np.float64))


def gipo_trust_weight(rho: np.ndarray, sigma: float) -> np.ndarray:
    """Gaussian trust weight omega(rho; sigma) = exp(-(log rho / sigma)^2 / 2) (Section 3.3, GIPO)."""
    return np.exp(-0.5 * (np.log(np.asarray(rho, dtype=np.float64)) / sigma) ** 2)


# ----------------------------------------------------------------------------
# the model
# ----------------------------------------------------------------------------

class SeqState:
    """Keys and values of one sequence, per layer, for positions 0..len-1."""

    def __init__(self, n_layers: int):
        self.k: List[Optional[np.ndarray]] = [None] * n_layers
        self.v: List[Optional[np.ndarray]] = [None] * n_layers
        self.len = 0


class OraclePolicy:
    def __init__(self, shape, weights: Dict[str, np.ndarray]):
        """shape: any object with n_layers, d_model, n_heads, head_dim, d_ffn, vocab,
        n_action_bins, rope_theta, rms_eps.  weights: name -> array in storage dtype,
        nn.Linear layout [out, in]."""
        self.s = shape
        self.w = weights
        assert shape.n_heads * shape.head_dim == shape.d_model

    def W(self, name: str) -> np.ndarray:
        return widen(self.w[name])

    # -- prefix ---------------------------------------------------------------
    def prefix_rows(self, patch_emb: np.ndarray, instr_ids: np.ndarray) -> np.ndarray:
        """[patches ; embed[instruction ids]] as float64 rows."""
        rows = [widen(patch_emb)]
        if len(instr_ids):
            rows.append(widen(self.w["embed"][np.asarray(instr_ids, dtype=np.int64)]))
        return np.concatenate(rows, axis=0)

    def token_rows(self, ids: Sequence[int]) -> np.ndarray:
        return widen(self.w["embed"][np.asarray(ids, dtype=np.int64)])

    # -- layers ---------------------------------------------------------------
    def run_layers(self, xs: List[np.ndarray], states: List[SeqState],
                   n_layers: Optional[int] = None) -> List[np.ndarray]:
        """Push new rows of several independent sequences through the layers.

        xs[b]: [n_b, d] input rows of sequence b at positions states[b].len ...;
        states[b] holds keys/values of its earlier positions and is extended.
        Returns the residual stream after the last layer for the new rows.
        """
        s = self.s
        H, hd = s.n_heads, s.head_dim
        L = s.n_layers if n_layers is None else n_layers
        counts = [x.shape[0] for x in xs]
        cuts = np.cumsum([0] + counts)
        x = np.concatenate(xs, axis=0)                                # rows of all sequences
        pos = [np.arange(st.len, st.len + n) for st, n in zip(states, counts)]
        for l in range(L):
            p = f"layers.{l}."
            h = rms_norm(x, self.W(p + "attn_norm"), s.rms_eps)
            q = h @ self.W(p + "wq").T
            k = h @ self.W(p + "wk").T
            v = h @ self.W(p + "wv").T
            att = np.empty_like(x)
            for b, st in enumerate(states):
                r0, r1 = cuts[b], cuts[b + 1]
                qb = rope(q[r0:r1].reshape(-1, H, hd), pos[b], s.rope_theta)
                kb = rope(k[r0:r1].reshape(-1, H, hd), pos[b], s.rope_theta)
                vb = v[r0:r1].reshape(-1, H, hd)
                st.k[l] = kb if st.k[l] is None else np.concatenate([st.k[l], kb], axis=0)
                st.v[l] = vb if st.v[l] is None else np.concatenate([st.v[l], vb], axis=0)
                att[r0:r1] = causal_attention(qb, st.k[l], st.v[l], pos[b]).reshape(-1, H * hd)
            x = x + att @ self.W(p + "wo").T
            h = rms_norm(x, self.W(p + "ffn_norm"), s.rms_eps)
            g = h @ self.W(p + "w_gate").T
            u = h @ self.W(p + "w_up").T
            x = x + (silu(g) * u) @ self.W(p + "w_down").T
        for st, n in zip(states, counts):
            st.len += n
        return [x[cuts[b]:cuts[b + 1]] for b in range(len(xs))]

    # -- head -----------------------------------------------------------------
    def action_logits(self, x_last: np.ndarray) -> np.ndarray:
        """Final RMSNorm, then the action-bin rows of the LM head.  x_last: [..., d] -> [..., A]."""
        s = self.s
        h = rms_norm(x_last, self.W("final_norm"), s.rms_eps)
        head = self.w["lm_head"]
        if head.shape[0] == s.vocab:            # full head: slim it to the action rows
            head = head[s.vocab - s.n_action_bins:]
        return h @ widen(head).T

    def final_hidden(self, x_last: np.ndarray) -> np.ndarray:
        """The last hidden layer's output for a row: the residual stream after the final RMSNorm."""
        return rms_norm(x_last, self.W("final_norm"), self.s.rms_eps)

    def full_vocab_logits(self, x_last: np.ndarray) -> np.ndarray:
        h = rms_norm(x_last, self.W("final_norm"), self.s.rms_eps)
        return h @ self.W("lm_head").T

    # -- policy step ----------------------------------------------------------
    def policy_step(self, patch_embs: List[np.ndarray], instr_ids: List[np.ndarray], n_tokens: int,
                    temperature: float = 0.0, gumbel: Optional[np.ndarray] = None,
                    mode: str = "recompute", forced_tokens: Optional[np.ndarray] = None,
                    n_layers: Optional[int] = None) -> dict:
        """K autoregressive action tokens for each of several sequences.

        gumbel: [B, K, A] or None.  forced_tokens: [B, K] bin indices fed back instead
        of the selected ones (teacher forcing); selection is still reported.
        Returns tokens [B,K] (bin index), logp [B,K], actions [B,K], logits [B,K,A],
        scores [B,K,A] (what the argmax ran over).
        """
        s = self.s
        B, A = len(patch_embs), s.n_action_bins
        tau = 1.0 if temperature == 0 else temperature
        tokens = np.zeros((B, n_tokens), dtype=np.int64)
        logp = np.zeros((B, n_tokens))
        logits = np.zeros((B, n_tokens, A))
        scores = np.zeros((B, n_tokens, A))
        hidden = np.zeros((B, n_tokens, s.d_model))
        seqs = [self.prefix_rows(pe, ids) for pe, ids in zip(patch_embs, instr_ids)]
        states = [SeqState(s.n_layers) for _ in range(B)]
        new_rows = seqs
        for k in range(n_tokens):
            if mode == "recompute":
                states = [SeqState(s.n_layers) for _ in range(B)]
                outs = self.run_layers(seqs, states, n_layers)
            elif mode == "cached":
                outs = self.run_layers(new_rows, states, n_layers)
            else:
                raise ValueError(mode)
            z = np.stack([self.action_logits(o[-1]) for o in outs])   # [B, A]
            hidden[:, k] = np.stack([self.final_hidden(o[-1]) for o in outs])
            logits[:, k] = z
            ell = log_softmax(z, tau)
            fed = []
            for b in range(B):
                gb = None if gumbel is None else gumbel[b, k]
                t, sc = select_token(z[b], temperature, gb)
                tokens[b, k], scores[b, k], logp[b, k] = t, sc, ell[b, t]
                fed.append(int(forced_tokens[b, k]) if forced_tokens is not None else t)
            new_rows = [self.token_rows([s.vocab - A + t]) for t in fed]
            seqs = [np.concatenate([sq, r], axis=0) for sq, r in zip(seqs, new_rows)]
        return {"tokens": tokens, "logp": logp, "actions": bin_centre(tokens, A),
                "logits": logits, "scores": scores, "hidden": hidden}

    # -- all K action rows in one forward pass ---------------------------------------
    def chunk_logits(self, patch_embs: List[np.ndarray], instr_ids: List[np.ndarray], fed_ids: np.ndarray,
                     n_layers: Optional[int] = None) -> np.ndarray:
        """One causal forward pass over [prefix ; fed_ids[b]] per sequence (fed_ids: [B, K-1] absolute vocabulary
        ids); returns the action-bin logits [B, K, A] of the last K positions: row k is the position that emits
        action token k (the last prefix position, then the K-1 fed positions)."""
        fed_ids = np.asarray(fed_ids).reshape(len(patch_embs), -1)
        K = fed_ids.shape[1] + 1
        seqs = [np.concatenate([self.prefix_rows(pe, ids), self.token_rows(list(f))], axis=0) if K > 1
                else self.prefix_rows(pe, ids) for pe, ids, f in zip(patch_embs, instr_ids, fed_ids)]
        states = [SeqState(self.s.n_layers) for _ in seqs]
        outs = self.run_layers(seqs, states, n_layers)
        return np.stack([np.stack([self.action_logits(o[len(o) - K + k]) for k in range(K)]) for o in outs])

    def policy_step_parallel(self, patch_embs, instr_ids, n_tokens: int, placeholder_id: int,
                             temperature: float = 0.0, gumbel: Optional[np.ndarray] = None) -> dict:
        """Parallel decoding: the K action tokens are conditionally independent given the observation (the
        token-level ratio of Appendix "Token-level Policy Optimization" conditions every token on o_t alone).
        The K-1 positions after the prefix hold a fixed placeholder token instead of sampled ones, so all K
        distributions come from one forward pass; each token is then selected on its own."""
        B, A = len(patch_embs), self.s.n_action_bins
        fed = np.full((B, n_tokens - 1), placeholder_id, dtype=np.int64)
        logits = self.chunk_logits(patch_embs, instr_ids, fed)
        tau = 1.0 if temperature == 0 else temperature
        tokens = np.zeros((B, n_tokens), dtype=np.int64)
        logp = np.zeros((B, n_tokens))
        scores = np.zeros((B, n_tokens, A))
        for b in range(B):
            ell = log_softmax(logits[b], tau)
            for k in range(n_tokens):
                t, sc = select_token(logits[b, k], temperature, None if gumbel is None else gumbel[b, k])
                tokens[b, k], scores[b, k], logp[b, k] = t, sc, ell[k, t]
        return {"tokens": tokens, "logp": logp, "actions": bin_centre(tokens, A), "logits": logits, "scores": scores}

    def score_tokens(self, patch_embs, instr_ids, tokens: np.ndarray, temperature: float = 0.0,
                     placeholder_id: Optional[int] = None, mu_logp: Optional[np.ndarray] = None,
                     sigma: float = 1.0) -> dict:
        """Learner-side evaluation of stored action tokens (bin indices [B, K]) under the current weights:
        logp[b,k] = log pi(a_k | o, a_<k) when placeholder_id is None (the stored tokens are fed back), or
        log pi(a_k | o) with the placeholder conditioning of policy_step_parallel.  With the behaviour
        log-probabilities mu_logp it also gives rho and the GIPO coefficient omega(rho; sigma) * rho that
        multiplies the advantage (Section 3.3)."""
        tokens = np.asarray(tokens)
        B, K = tokens.shape
        A = self.s.n_action_bins
        if placeholder_id is None:
            fed = self.s.vocab - A + tokens[:, :K - 1]
        else:
            fed = np.full((B, K - 1), placeholder_id, dtype=np.int64)
        logits = self.chunk_logits(patch_embs, instr_ids, fed)
        tau = 1.0 if temperature == 0 else temperature
        logp = np.zeros((B, K))
        for b in range(B):
            ell = log_softmax(logits[b], tau)
            logp[b] = ell[np.arange(K), tokens[b]]
        out = {"logp": logp, "logits": logits}
        if mu_logp is not None:
            rho = importance_ratio(logp, mu_logp)
            out["ratio"] = rho
            out["weight"] = gipo_trust_weight(rho, sigma) * rho
        return out
