"""Inference Worker loop of the rollout path (Section 3.2): requests are queued, the dynamic-window rule
(Eq. 1, evaluated by the native queue) releases ragged batches, each batch is one call of the policy step.

Argument marshalling only: the queue and its trigger are native host code, every step of the policy runs in
the HIP library.  torch is used to hold the requests' device buffers and to pack them into one batch."""
from __future__ import annotations

from typing import Dict, List, Optional

import numpy as np

from .binding import Batcher, VlaPolicy, VLA_ACCEPTING


class InferenceWorker:
    def __init__(self, policy: VlaPolicy, target_batch: int, t_max: float, n_tokens: int, action_dim: int = 7,
                 temperature: float = 0.0, with_value: bool = False):
        if target_batch > policy.cfg.max_batch:
            raise ValueError("target_batch exceeds the policy's max_batch")
        self.policy = policy
        self.queue = Batcher(target_batch, t_max, int(policy.cfg.max_prefill_tokens))
        self.n_tokens, self.action_dim, self.temperature = n_tokens, action_dim, temperature
        self.with_value = with_value
        self._pending: Dict[int, tuple] = {}

    def close(self):
        self.queue.close()

    def submit(self, request_id: int, patch_emb, instr_ids, t_arrival: float, gumbel=None, step_t: int = 0) -> None:
        """patch_emb: device tensor [n_patches, d] in storage dtype; instr_ids: device int32 [n_instr];
        gumbel: device float32 [n_tokens, n_action_bins] or None (needed iff temperature > 0)."""
        if request_id in self._pending:
            raise ValueError(f"request {request_id} is already queued")
        if patch_emb.shape[0] + instr_ids.shape[0] + self.n_tokens > self.policy.cfg.max_seq:
            raise ValueError("request does not fit max_seq")
        self.queue.push(request_id, int(patch_emb.shape[0]), int(instr_ids.shape[0]), t_arrival)
        self._pending[request_id] = (patch_emb, instr_ids, gumbel, step_t)

    def deadline(self) -> float:
        return self.queue.deadline()

    def poll(self, t_now: float) -> Optional[dict]:
        """Runs one batch if Eq. 1 fires and the policy accepts new batches.  Returns None, or
        {"ids": [...], "version": weights version used, "tokens"/"logp"/"actions": device tensors [n, K]
        (+ "values" [n])}; row i belongs to ids[i].  Nothing is synchronised."""
        pol = self.policy
        state, version = pol.state()
        if state != VLA_ACCEPTING:        # draining or updating: leave the queue alone
            return None
        batch = self.queue.poll(t_now)
        if not batch:
            return None
        torch = pol.torch
        ids = [r[0] for r in batch]
        items = [self._pending.pop(i) for i in ids]
        cu_p = np.zeros(len(ids) + 1, dtype=np.int32)
        cu_i = np.zeros(len(ids) + 1, dtype=np.int32)
        cu_p[1:] = np.cumsum([r[1] for r in batch])
        cu_i[1:] = np.cumsum([r[2] for r in batch])
        pe = torch.cat([it[0] for it in items], dim=0)
        ii = torch.cat([it[1] for it in items], dim=0)
        gum = None
        if self.temperature > 0:
            gum = torch.stack([it[2] for it in items], dim=0)
        step_t = None
        if self.with_value:
            step_t = torch.tensor([it[3] for it in items], dtype=torch.int32, device=pol.device)
        out = pol.policy_step(pe, cu_p, ii, cu_i, self.n_tokens, temperature=self.temperature, gumbel=gum,
                              action_dim=self.action_dim, step_t=step_t)
        out.pop("logits", None)
        out["ids"] = ids
        out["version"] = version
        return out


class ContinuousWorker:
    """Continuous batching on top of the same queue: requests are admitted into free cache slots whenever Eq. 1
    fires (cut to the number of free slots), and every call of step() runs ONE decode step shared by all the
    admitted batches that still have action tokens to emit, then prefills the newly admitted batch.  Each
    admitted batch keeps its own token index k, so selection is one call per batch on its rows of the shared
    logits.  Results are identical to running each admitted batch through vla_policy_step on its own."""

    def __init__(self, policy: VlaPolicy, target_batch: int, t_max: float, n_tokens: int, action_dim: int = 7,
                 temperature: float = 0.0):
        self.policy = policy
        self.queue = Batcher(min(target_batch, int(policy.cfg.max_batch)), t_max, int(policy.cfg.max_prefill_tokens))
        self.n_tokens, self.action_dim, self.temperature = n_tokens, action_dim, temperature
        self.free: List[int] = list(range(int(policy.cfg.max_batch)))
        self.running: List[dict] = []
        self._pending: Dict[int, tuple] = {}

    def close(self):
        self.queue.close()

    def submit(self, request_id: int, patch_emb, instr_ids, t_arrival: float, gumbel=None) -> None:
        if request_id in self._pending:
            raise ValueError(f"request {request_id} is already queued")
        if patch_emb.shape[0] + instr_ids.shape[0] + self.n_tokens > self.policy.cfg.max_seq:
            raise ValueError("request does not fit max_seq")
        self.queue.push(request_id, int(patch_emb.shape[0]), int(instr_ids.shape[0]), t_arrival)
        self._pending[request_id] = (patch_emb, instr_ids, gumbel)

    def _select(self, cohort: dict, logits) -> None:
        from .binding import vla_select
        pol = self.policy
        vla_select(pol.ctx, len(cohort["ids"]), logits, float(self.temperature), cohort["gumbel"], cohort["k"],
                   self.n_tokens, None, None, self.action_dim, cohort["tokens"], cohort["logp"], cohort["actions"],
                   self.n_tokens, cohort["next_ids"], pol._stream())
        cohort["k"] += 1

    def step(self, t_now: float) -> List[dict]:
        """One engine iteration.  Returns the batches that emitted their last token in this iteration:
        {"ids", "version", "tokens"/"logp"/"actions" device tensors [n, K]} (nothing is synchronised)."""
        pol = self.policy
        torch = pol.torch
        state, version = pol.state()
        done: List[dict] = []
        if self.running:                      # one decode step for everything in flight (allowed while draining)
            slots = np.concatenate([c["slots"] for c in self.running])
            toks = torch.cat([c["next_ids"] for c in self.running])
            logits = pol.decode_slots(slots, toks)
            off = 0
            for c in self.running:
                n = len(c["ids"])
                self._select(c, logits[off:off + n])
                off += n
        if state == VLA_ACCEPTING and self.free:
            batch = self.queue.poll(t_now, cap=len(self.free))
            if batch:
                ids = [r[0] for r in batch]
                items = [self._pending.pop(i) for i in ids]
                n = len(ids)
                slots = np.array([self.free.pop(0) for _ in range(n)], dtype=np.int32)
                cu_p = np.zeros(n + 1, dtype=np.int32)
                cu_i = np.zeros(n + 1, dtype=np.int32)
                cu_p[1:] = np.cumsum([r[1] for r in batch])
                cu_i[1:] = np.cumsum([r[2] for r in batch])
                pe = torch.cat([it[0] for it in items], dim=0)
                ii = torch.cat([it[1] for it in items], dim=0)
                K = self.n_tokens
                cohort = {"ids": ids, "slots": slots, "k": 0, "version": version,
                          "gumbel": torch.stack([it[2] for it in items], dim=0) if self.temperature > 0 else None,
                          "tokens": torch.empty((n, K), dtype=torch.int32, device=pol.device),
                          "logp": torch.empty((n, K), dtype=torch.float32, device=pol.device),
                          "actions": torch.empty((n, K), dtype=torch.float32, device=pol.device),
                          "next_ids": torch.empty((n,), dtype=torch.int32, device=pol.device)}
                self._select(cohort, pol.prefill_slots(slots, pe, cu_p, ii, cu_i))
                self.running.append(cohort)
        still = []
        for c in self.running:
            if c["k"] >= self.n_tokens:
                pol.release_slots(c["slots"])
                self.free.extend(int(s) for s in c["slots"])
                done.append({k: c[k] for k in ("ids", "version", "tokens", "logp", "actions")})
            else:
                still.append(c)
        self.running = still
        return done
