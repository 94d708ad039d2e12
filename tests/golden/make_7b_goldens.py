"""Writes the oracle's outputs for a few sequences of the 7B-shaped workloads (C3, C4, C5).

The full-size parity tests compare the HIP library with these stored values instead of running
the fp64 oracle on the GPU machine (one 7B sequence costs the oracle about 4 TFLOP of fp64).  This
script calls only `oracle/` and the seeded input generators; nothing in the files it writes comes
from the HIP path.  Usage:  python tests/golden/make_7b_goldens.py [C3 C4 C5] [--parallel]
With --parallel it writes <name>_parallel_oracle.npz instead: the one-pass (placeholder-fed) decoding of
the same rows, placeholder = the first action id.

For each workload it stores, for the chosen sequence indices `rows` of the seeded batch:
tokens [n,K], logp [n,K], logits [n,K,A], scores [n,K,A] from the oracle in "cached" mode
(proved equal to full recompute by tests/test_oracle_pins.py), free-running on its own tokens.
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import workloads as W                      # noqa: E402
from oracle import vla_oracle as O         # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))


def pick_rows(wl, obs, n=8):
    """n sequences of the batch: the first and last, the shortest and longest prefix, both sides of every
    128-row boundary (decode and last-layer kernels work on groups of 128 rows), then evenly spaced ones."""
    lens = np.diff(obs["cu_instr"])
    B = wl.batch
    rows = [0, B - 1, int(np.argmin(lens)), int(np.argmax(lens))]
    for edge in range(128, B, 128):
        rows += [edge - 1, edge]
    for r in np.linspace(0, B - 1, n + 2).astype(int)[1:-1]:
        if len(set(rows)) < n:
            rows.append(int(r))
    return sorted(set(rows))


def main(names, parallel=False):
    for name in names:
        wl = W.get_workload(name)
        t0 = time.time()
        weights = W.make_weights(wl.shape, wl.seed)
        obs = W.make_observations(wl)
        gum = W.make_gumbel(wl) if wl.sampling == "gumbel" else None
        rows = pick_rows(wl, obs)
        print(name, "inputs ready", round(time.time() - t0, 1), "s; rows", rows, flush=True)
        pol = O.OraclePolicy(wl.shape, weights)
        pes = [obs["patch_emb"][obs["cu_patch"][b]:obs["cu_patch"][b + 1]] for b in rows]
        ids = [obs["instr_ids"][obs["cu_instr"][b]:obs["cu_instr"][b + 1]] for b in rows]
        temp = wl.temperature if wl.sampling == "gumbel" else 0.0
        if parallel:
            ph = wl.shape.vocab - wl.shape.n_action_bins
            r = pol.policy_step_parallel(pes, ids, wl.n_tokens, ph, temperature=temp,
                                         gumbel=None if gum is None else gum[rows])
            np.savez(os.path.join(HERE, f"{name.lower()}_parallel_oracle.npz"), rows=np.array(rows),
                     tokens=r["tokens"], logp=r["logp"], logits=r["logits"], scores=r["scores"],
                     actions=r["actions"], seed=np.array(wl.seed), placeholder=np.array(ph))
            print(name, "parallel done", round(time.time() - t0, 1), "s", flush=True)
            del weights, pol
            continue
        r = pol.policy_step(pes, ids, wl.n_tokens, temperature=temp,
                            gumbel=None if gum is None else gum[rows], mode="cached")
        np.savez(os.path.join(HERE, f"{name.lower()}_oracle.npz"), rows=np.array(rows), tokens=r["tokens"],
                 logp=r["logp"], logits=r["logits"], scores=r["scores"], actions=r["actions"],
                 seed=np.array(wl.seed))
        print(name, "done", round(time.time() - t0, 1), "s", flush=True)
        del weights, pol


if __name__ == "__main__":
    args = [a for a in sys.argv[1:] if not a.startswith("--")]
    main(args or ["C3", "C4", "C5"], parallel="--parallel" in sys.argv)
