"""What 16-bit matrix-core operands cost in accuracy, measured with the oracle's own arithmetic.

TEST INFRASTRUCTURE ONLY (same rules as vla_oracle.py).  The forward pass below is the oracle's
(it calls its functions), except that the tensors a 16-bit pipeline must round before feeding a
matrix core -- the normalised activations, rotated q and k, v, the attention output and the SwiGLU
output -- are rounded to a chosen 16-bit format and widened again.  Everything else stays float64,
so the difference to the exact oracle is a lower bound on the logit error of ANY implementation
that uses that operand format, whatever its kernels look like.  It is used to justify the
operand format (half precision instead of bfloat16) and the tolerances of the 7B-shaped tests.
"""
from __future__ import annotations

import numpy as np

from . import vla_oracle as O


def round_bf16(x: np.ndarray) -> np.ndarray:
    b = x.astype(np.float32).view(np.uint32)
    r = ((b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)
    return O.widen(r).reshape(x.shape)


def round_f16(x: np.ndarray) -> np.ndarray:
    return x.astype(np.float16).astype(np.float64)


POINTS = ("hn_a", "hn_f", "q", "k", "v", "att", "act")
# A split of the rounding points used to show that their contributions add in variance and that none of them can
# be left single-term for free: the normalised rows that feed the gate / up projections against the other six.
# (An operand carried as hi + lo terms has its rounding error cut by 2^-11 or, with 8-bit low terms, by a factor of
# about 2^-3 more than one term: out of the picture either way.)
TWO_TERM_POINTS = ("hn_a", "q", "k", "v", "att", "act")
SINGLE_TERM_LEFT = ("hn_f",)


def prefix_logits(pol: O.OraclePolicy, x: np.ndarray, rnd=None, points=POINTS, n_layers=None, first_layer=0):
    """Action logits at the last of the prefix rows x [S, d]; rnd (None = exact) is applied at `points`:
    hn_a / hn_f = the normalised rows that feed the QKV / the gate-up projections, q, k (after the rotary
    embedding), v, att = attention output, act = SwiGLU output; and only in layers >= first_layer (the layers
    before it stand for layers whose operands are carried as two terms)."""
    s = pol.s
    H, hd = s.n_heads, s.head_dim
    n = x.shape[0]
    pos = np.arange(n)
    for l in range(s.n_layers if n_layers is None else n_layers):
        p = f"layers.{l}."
        R = (lambda key, v: rnd(v) if (rnd is not None and key in points and l >= first_layer) else v)
        h = R("hn_a", O.rms_norm(x, pol.W(p + "attn_norm"), s.rms_eps))
        q = R("q", O.rope((h @ pol.W(p + "wq").T).reshape(n, H, hd), pos, s.rope_theta))
        k = R("k", O.rope((h @ pol.W(p + "wk").T).reshape(n, H, hd), pos, s.rope_theta))
        v = R("v", (h @ pol.W(p + "wv").T).reshape(n, H, hd))
        att = R("att", O.causal_attention(q, k, v, pos).reshape(n, -1))
        x = x + att @ pol.W(p + "wo").T
        h = R("hn_f", O.rms_norm(x, pol.W(p + "ffn_norm"), s.rms_eps))
        act = R("act", O.silu(h @ pol.W(p + "w_gate").T) * (h @ pol.W(p + "w_up").T))
        x = x + act @ pol.W(p + "w_down").T
    return pol.action_logits(x[-1])
