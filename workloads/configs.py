"""Shapes of the five synthetic policy workloads (C1..C5).

The paper fixes only the outline of the rollout policy: a Llama-2-7B based
OpenVLA-OFT backbone, 256 discretised action bins, one or two camera images per
observation, bf16, action chunking (Appendix "Experiment Setup"; Appendix
"Vocabulary Slimming"; hyper-parameter tables).  Everything else here is the
shape of a public Llama-family decoder (RMSNorm, RoPE, SwiGLU, MHA).
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Tuple

BASE_SEED = 260318464


@dataclass(frozen=True)
class PolicyShape:
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    n_action_bins: int = 256
    rope_theta: float = 1.0e4
    rms_eps: float = 1.0e-5
    dtype: str = "bf16"          # storage dtype of weights / patch embeddings: "f32" | "bf16"

    @property
    def action_id0(self) -> int:
        """First vocabulary id of the action bins (bins are the last ids)."""
        return self.vocab - self.n_action_bins

    @property
    def n_matrix_params(self) -> int:
        return self.n_layers * (4 * self.d_model * self.d_model + 3 * self.d_model * self.d_ffn)


@dataclass(frozen=True)
class Workload:
    name: str
    index: int                   # position in the list of configurations (seeds derive from it)
    shape: PolicyShape
    batch: int
    n_patches: int
    instr_len: Tuple[int, int]   # inclusive range of instruction lengths (equal => fixed)
    n_tokens: int                # K action tokens per policy step
    action_dim: int = 7
    sampling: str = "greedy"     # "greedy" | "gumbel"
    temperature: float = 1.0

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    @property
    def max_seq(self) -> int:
        return self.n_patches + self.instr_len[1] + self.n_tokens

    def scaled(self, **kw) -> "Workload":
        """Same workload with some fields replaced (e.g. a smaller batch)."""
        return replace(self, **kw)


_TINY = PolicyShape(2, 256, 4, 64, 704, 1024, dtype="f32")
_SMALL = PolicyShape(12, 768, 12, 64, 2048, 32000)
_7B = PolicyShape(32, 4096, 32, 128, 11008, 32000)

WORKLOADS = {
    "C1": Workload("C1", 0, _TINY, batch=4, n_patches=16, instr_len=(16, 16), n_tokens=7),
    "C2": Workload("C2", 1, _SMALL, batch=32, n_patches=256, instr_len=(32, 32), n_tokens=7),
    "C3": Workload("C3", 2, _7B, batch=64, n_patches=256, instr_len=(34, 34), n_tokens=7),
    "C4": Workload("C4", 3, _7B, batch=256, n_patches=256, instr_len=(20, 60), n_tokens=7,
                   sampling="gumbel", temperature=1.0),
    "C5": Workload("C5", 4, _7B, batch=128, n_patches=512, instr_len=(40, 40), n_tokens=56),
}


def get_workload(name: str) -> Workload:
    return WORKLOADS[name]
