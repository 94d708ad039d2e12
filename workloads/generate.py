"""Counter-based, name-keyed generators for weights and observations.

Every tensor is drawn from its own Philox stream whose key is a hash of
(seed, tensor name), so any single tensor can be regenerated alone and the
result does not depend on generation order or threading.
"""
from __future__ import annotations

import hashlib
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, Iterable, List, Tuple

import numpy as np

from .configs import PolicyShape, Workload

WEIGHT_STD = 0.02


def tensor_rng(seed: int, name: str) -> np.random.Generator:
    digest = hashlib.blake2b(f"{seed}:{name}".encode(), digest_size=16).digest()
    key = np.frombuffer(digest, dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def bf16_bits_from_f32(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns the uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def f32_from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _store(x32: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return x32
    if dtype == "bf16":
        return bf16_bits_from_f32(x32)
    raise ValueError(dtype)


def weight_shape(shape: PolicyShape, name: str) -> Tuple[int, ...]:
    d, f, v = shape.d_model, shape.d_ffn, shape.vocab
    leaf = name.rsplit(".", 1)[-1]
    return {
        "embed": (v, d), "lm_head": (v, d), "final_norm": (d,),
        "attn_norm": (d,), "ffn_norm": (d,),
        "wq": (d, d), "wk": (d, d), "wv": (d, d), "wo": (d, d),
        "w_gate": (f, d), "w_up": (f, d), "w_down": (d, f),
    }[leaf]


def weight_names(shape: PolicyShape) -> List[str]:
    names = ["embed"]
    for l in range(shape.n_layers):
        names += [f"layers.{l}.{leaf}" for leaf in
                  ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")]
    names += ["final_norm", "lm_head"]
    return names


def make_weight(shape: PolicyShape, seed: int, name: str) -> np.ndarray:
    """One tensor in nn.Linear layout [out, in]; matrices N(0, 0.02^2), norm gains 1 + N(0, 0.02^2)."""
    shp = weight_shape(shape, name)
    g = tensor_rng(seed, name)
    x = g.standard_normal(shp, dtype=np.float32)
    x *= np.float32(WEIGHT_STD)
    if name.endswith("norm"):
        x += np.float32(1.0)
    return _store(x, shape.dtype)


def make_weights(shape: PolicyShape, seed: int, names: Iterable[str] | None = None,
                 threads: int = 8) -> Dict[str, np.ndarray]:
    names = list(names) if names is not None else weight_names(shape)
    with ThreadPoolExecutor(max_workers=threads) as ex:
        arrs = list(ex.map(lambda n: make_weight(shape, seed, n), names))
    return dict(zip(names, arrs))


def make_observations(wl: Workload) -> dict:
    """Patch embeddings ~N(0,1), instruction ids uniform over the non-action vocabulary.

    Returns packed, ragged-ready arrays:
      patch_emb  [B*Np, d]   storage dtype
      cu_patch   [B+1] int32 cumulative patch counts
      instr_ids  [sum Li] int32
      cu_instr   [B+1] int32 cumulative instruction lengths
    """
    s = wl.shape
    B, Np = wl.batch, wl.n_patches
    patch = tensor_rng(wl.seed, "patch").standard_normal((B * Np, s.d_model), dtype=np.float32)
    lo, hi = wl.instr_len
    if lo == hi:
        lens = np.full(B, lo, dtype=np.int64)
    else:
        lens = tensor_rng(wl.seed, "len").integers(lo, hi + 1, size=B)
    cu_instr = np.zeros(B + 1, dtype=np.int32)
    cu_instr[1:] = np.cumsum(lens)
    ids = tensor_rng(wl.seed, "instr").integers(0, s.action_id0, size=int(cu_instr[-1]))
    return {
        "patch_emb": _store(patch, s.dtype),
        "cu_patch": (np.arange(B + 1, dtype=np.int64) * Np).astype(np.int32),
        "instr_ids": ids.astype(np.int32),
        "cu_instr": cu_instr,
    }


def make_gumbel(wl: Workload) -> np.ndarray:
    """Standard Gumbel noise [B, K, A] float32: -log(-log u), u clamped to [2^-24, 1-2^-24]."""
    A = wl.shape.n_action_bins
    u = tensor_rng(wl.seed, "gumbel").random((wl.batch, wl.n_tokens, A), dtype=np.float32)
    u = np.clip(u.astype(np.float64), 2.0 ** -24, 1.0 - 2.0 ** -24)
    return (-np.log(-np.log(u))).astype(np.float32)


def make_value_weights(shape: PolicyShape, seed: int, n_steps: int) -> Dict[str, np.ndarray]:
    """Synthetic value-head weights in the storage dtype: every tensor N(0, 0.02^2)."""
    d = shape.d_model
    shapes = {"value.attn_w": (d,), "value.attn_b": (1,), "value.step_emb": (n_steps, d), "value.w1": (d, d),
              "value.b1": (d,), "value.w2": (d,), "value.b2": (1,)}
    out = {}
    for name, shp in shapes.items():
        x = tensor_rng(seed, name).standard_normal(shp, dtype=np.float32) * np.float32(WEIGHT_STD)
        out[name] = _store(x, shape.dtype)
    return out
