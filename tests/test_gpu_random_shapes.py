"""Seeded sweep over small model shapes, ragged batches and precision modes against the fp64 oracle: every
combination the configuration checks allow is fair game (head sizes, widths that are not multiples of the large
tiles, few bins, batches around the 128- and 256-row chunk sizes of the decode GEMMs, one to six layers)."""
import numpy as np
import pytest

import workloads as W
from tests.test_gpu_parity import ragged_obs, run_both

pytestmark = pytest.mark.gpu


def _case(rng, it):
    dtype = "bf16" if rng.random() < 0.8 else "f32"
    hd = int(rng.choice([64, 128])) if dtype == "bf16" else int(rng.choice([32, 64, 128]))
    heads = int(rng.choice([1, 2, 3, 4, 6]))
    if dtype == "bf16" and (hd * heads) % 128:
        heads += 1                                   # the 16-bit path wants d_model in multiples of 128
    shape = W.PolicyShape(int(rng.integers(1, 7)), hd * heads, heads, hd,
                          int(rng.choice([64, 128, 192, 320, 704, 1024, 1408])),
                          0, n_action_bins=int(rng.choice([256, 64, 40, 17])), dtype=dtype)
    shape = W.PolicyShape(shape.n_layers, shape.d_model, heads, hd, shape.d_ffn,
                          shape.n_action_bins + int(rng.integers(8, 600)), n_action_bins=shape.n_action_bins, dtype=dtype)
    B = int(rng.choice([1, 2, 3, 5, 17, 40, 131, 150, 260]))
    npmax, lmax = int(rng.choice([1, 8, 24, 70])), int(rng.choice([0, 3, 12, 40]))
    wl = W.Workload("Rs", 1000 + it, shape, batch=B, n_patches=npmax, instr_len=(0, lmax), n_tokens=int(rng.integers(1, 6)),
                    sampling="gumbel" if rng.random() < 0.5 else "greedy", temperature=float(rng.choice([1.0, 0.7])))
    nps, lens = rng.integers(1, npmax + 1, size=B), rng.integers(0, lmax + 1, size=B)
    mode = False if dtype == "f32" else [False, "first", True, "all"][int(rng.integers(0, 4))]
    rows = None
    if B > 40:      # the oracle runs a sample of the rows: the ends, the chunk boundary, and 24 at random
        rows = sorted(set(int(r) for r in rng.choice(B, size=24, replace=False)) | {0, B - 1, 127, 128})
    return wl, list(nps), list(lens), mode, rows


@pytest.mark.timeout(600)
@pytest.mark.parametrize("seed", [1, 2])
def test_random_shapes_batches_and_modes(seed):
    rng = np.random.default_rng(seed)
    for it in range(30):
        wl, nps, lens, mode, rows = _case(rng, it)
        s = wl.shape
        print(f"\ncase {seed}.{it}: {s.dtype} L{s.n_layers} d{s.d_model} H{s.n_heads} hd{s.head_dim} f{s.d_ffn} V{s.vocab} "
              f"A{s.n_action_bins} B{wl.batch} K{wl.n_tokens} mode {mode} {wl.sampling}", flush=True)
        obs = ragged_obs(wl, nps, lens, seed=7 + it)
        gum = W.make_gumbel(wl) if wl.sampling == "gumbel" else None
        run_both(wl, obs=obs, gumbel=gum, rows=rows, fast=mode)
