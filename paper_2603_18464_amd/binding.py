"""ctypes binding of include/vla.h.  Argument marshalling only: every step of the policy path
runs in the library's HIP kernels.  PyTorch provides device memory and the stream."""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import numpy as np

VLA_F32, VLA_BF16 = 0, 1
VLA_PREC_HIGH, VLA_PREC_FAST = 0, 1
STATUS = {0: "VLA_OK", -1: "VLA_E_NULL", -2: "VLA_E_CONFIG", -3: "VLA_E_SHAPE", -4: "VLA_E_CAPACITY",
          -5: "VLA_E_STATE", -6: "VLA_E_WEIGHTS", -7: "VLA_E_HIP", -8: "VLA_E_DRAINING"}
VLA_E_STATE, VLA_E_DRAINING = -5, -8
VLA_ACCEPTING, VLA_DRAINING, VLA_UPDATING = 0, 1, 2
EXPORTS = ["vla_create", "vla_destroy", "vla_last_error", "vla_query_sizes", "vla_bind_buffers",
           "vla_load_weights", "vla_check_weights", "vla_prefill", "vla_decode_step", "vla_decode_step_static", "vla_policy_step", "vla_select",
           "vla_load_value_head", "vla_policy_step_value",
           "vla_policy_step_parallel", "vla_score_tokens",
           "vla_prefill_slots", "vla_decode_slots", "vla_release_slots",
           "vla_probe",
           "vla_batcher_create", "vla_batcher_destroy", "vla_batcher_push", "vla_batcher_size",
           "vla_batcher_deadline", "vla_batcher_poll",
           "vla_get_state", "vla_drain_begin", "vla_update_begin", "vla_update_tensors", "vla_update_commit",
           "vla_prof_enable", "vla_prof_count", "vla_prof_read"]


class vla_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32),
                ("n_action_bins", C.c_int32), ("rope_theta", C.c_float), ("rms_eps", C.c_float),
                ("dtype", C.c_int32), ("max_batch", C.c_int32), ("max_seq", C.c_int32),
                ("max_prefill_tokens", C.c_int64), ("value_max_steps", C.c_int32), ("precision", C.c_int32),
                ("two_term_layers", C.c_int32)]


class vla_tensor(C.Structure):
    _fields_ = [("name", C.c_char_p), ("dev_ptr", C.c_void_p), ("dtype", C.c_int32),
                ("ndim", C.c_int32), ("shape", C.c_int64 * 4)]


class vla_request(C.Structure):
    _fields_ = [("id", C.c_uint64), ("n_patches", C.c_int32), ("n_instr", C.c_int32), ("t_arrival", C.c_double)]


class VlaError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{STATUS.get(code, code)}: {msg}")
        self.code = code


def library_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libvla.so")


_LIB = None


def lib() -> C.CDLL:
    """Loads libvla.so (built by `python -m paper_2603_18464_amd.build`).  Raises if it is missing."""
    global _LIB
    if _LIB is None:
        path = library_path()
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is not built; run __graft_entry__.build() "
                               "(there is no fallback path)")
        L = C.CDLL(path)
        vp, i32, f32 = C.c_void_p, C.c_int32, C.c_float
        L.vla_create.argtypes = [C.POINTER(vla_config), C.POINTER(vp)]
        L.vla_destroy.argtypes = [vp]
        L.vla_last_error.argtypes = [vp]
        L.vla_last_error.restype = C.c_char_p
        L.vla_query_sizes.argtypes = [C.POINTER(vla_config)] + [C.POINTER(C.c_size_t)] * 3
        L.vla_bind_buffers.argtypes = [vp, vp, vp, vp]
        L.vla_load_weights.argtypes = [vp, C.POINTER(vla_tensor), i32, vp]
        L.vla_check_weights.argtypes = [vp]
        L.vla_prefill.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp]
        L.vla_decode_step.argtypes = [vp, i32, vp, vp, vp]
        L.vla_decode_step_static.argtypes = [vp, i32, vp, vp, vp]
        L.vla_policy_step.argtypes = [vp, i32, vp, vp, vp, vp, i32, f32, vp, vp, vp, i32, vp, vp, vp, vp, vp]
        L.vla_load_value_head.argtypes = [vp, C.POINTER(vla_tensor), i32, vp]
        L.vla_policy_step_value.argtypes = [vp, i32, vp, vp, vp, vp, i32, f32, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp]
        L.vla_get_state.argtypes = [vp, C.POINTER(C.c_int32), C.POINTER(C.c_int64)]
        L.vla_drain_begin.argtypes = [vp]
        L.vla_update_begin.argtypes = [vp, vp]
        L.vla_update_tensors.argtypes = [vp, C.POINTER(vla_tensor), i32, vp]
        L.vla_update_commit.argtypes = [vp, vp, C.POINTER(C.c_int64)]
        L.vla_policy_step_parallel.argtypes = [vp, i32, vp, vp, vp, vp, i32, i32, f32, vp, vp, vp, i32, vp, vp, vp, vp, vp]
        L.vla_score_tokens.argtypes = [vp, i32, vp, vp, vp, vp, i32, vp, i32, f32, vp, f32, vp, vp, vp, vp, vp]
        L.vla_prefill_slots.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, vp]
        L.vla_decode_slots.argtypes = [vp, i32, vp, vp, vp, vp]
        L.vla_release_slots.argtypes = [vp, i32, vp]
        L.vla_probe.argtypes = [vp, i32, C.POINTER(C.c_double), vp]
        L.vla_batcher_create.argtypes = [i32, C.c_double, C.c_int64, C.POINTER(vp)]
        L.vla_batcher_destroy.argtypes = [vp]
        L.vla_batcher_push.argtypes = [vp, C.POINTER(vla_request)]
        L.vla_batcher_size.argtypes = [vp, C.POINTER(C.c_int32)]
        L.vla_batcher_deadline.argtypes = [vp, C.POINTER(C.c_double)]
        L.vla_batcher_poll.argtypes = [vp, C.c_double, C.POINTER(vla_request), i32, C.POINTER(C.c_int32)]
        L.vla_select.argtypes = [vp, i32, vp, f32, vp, i32, i32, vp, vp, i32, vp, vp, vp, i32, vp, vp]
        L.vla_prof_enable.argtypes = [vp, i32]
        L.vla_prof_count.argtypes = []
        L.vla_prof_read.argtypes = [vp, i32, C.POINTER(C.c_char_p), C.POINTER(C.c_int64), C.POINTER(C.c_double)]
        _LIB = L
    return _LIB


def _check(ctx, rc: int):
    if rc != 0:
        msg = lib().vla_last_error(ctx).decode() if ctx else ""
        raise VlaError(rc, msg)


def _ptr(t) -> Optional[int]:
    """Device (or host numpy) pointer of a tensor, None for None."""
    if t is None:
        return None
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


# ---- functions named as in include/vla.h -------------------------------------------------------------

def vla_create(cfg: vla_config) -> C.c_void_p:
    h = C.c_void_p()
    _check(None, lib().vla_create(C.byref(cfg), C.byref(h)))
    return h


def vla_destroy(ctx) -> None:
    _check(None, lib().vla_destroy(ctx))


def vla_last_error(ctx) -> str:
    return lib().vla_last_error(ctx).decode()


def vla_query_sizes(cfg: vla_config):
    a, k, w = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(None, lib().vla_query_sizes(C.byref(cfg), C.byref(a), C.byref(k), C.byref(w)))
    return a.value, k.value, w.value


def vla_bind_buffers(ctx, arena, kv, work) -> None:
    _check(ctx, lib().vla_bind_buffers(ctx, _ptr(arena), _ptr(kv), _ptr(work)))


def vla_load_weights(ctx, tensors: Dict[str, "object"], dtype: int, stream: int = 0) -> None:
    arr = (vla_tensor * len(tensors))()
    for i, (name, t) in enumerate(tensors.items()):
        arr[i].name = name.encode()
        arr[i].dev_ptr = t.data_ptr()
        arr[i].dtype = dtype
        arr[i].ndim = t.dim()
        for j, s in enumerate(t.shape):
            arr[i].shape[j] = s
    _check(ctx, lib().vla_load_weights(ctx, arr, len(tensors), stream))


def vla_check_weights(ctx) -> None:
    _check(ctx, lib().vla_check_weights(ctx))


def _tensor_array(tensors: Dict[str, "object"], dtype: int):
    arr = (vla_tensor * max(len(tensors), 1))()
    for i, (name, t) in enumerate(tensors.items()):
        arr[i].name = name.encode()
        arr[i].dev_ptr = t.data_ptr()
        arr[i].dtype = dtype
        arr[i].ndim = t.dim()
        for j, s in enumerate(t.shape):
            arr[i].shape[j] = s
    return arr


def vla_load_value_head(ctx, tensors: Dict[str, "object"], dtype: int, stream: int = 0) -> None:
    _check(ctx, lib().vla_load_value_head(ctx, _tensor_array(tensors, dtype), len(tensors), stream))


def vla_get_state(ctx):
    st, ver = C.c_int32(), C.c_int64()
    _check(ctx, lib().vla_get_state(ctx, C.byref(st), C.byref(ver)))
    return st.value, ver.value


def vla_drain_begin(ctx) -> None:
    _check(ctx, lib().vla_drain_begin(ctx))


def vla_update_begin(ctx, stream: int = 0) -> None:
    _check(ctx, lib().vla_update_begin(ctx, stream))


def vla_update_tensors(ctx, tensors: Dict[str, "object"], dtype: int, stream: int = 0) -> None:
    _check(ctx, lib().vla_update_tensors(ctx, _tensor_array(tensors, dtype), len(tensors), stream))


def vla_update_commit(ctx, stream: int = 0) -> int:
    ver = C.c_int64()
    _check(ctx, lib().vla_update_commit(ctx, stream, C.byref(ver)))
    return ver.value


def vla_policy_step_value(ctx, B, patch_emb, cu_patch, instr_ids, cu_instr, n_tokens, temperature, gumbel,
                          act_scale, act_offset, action_dim, step_t, tokens_out, logp_out, actions_out, logits_out,
                          values_out, stream: int = 0) -> None:
    _check(ctx, lib().vla_policy_step_value(ctx, B, _ptr(patch_emb), _ptr(cu_patch), _ptr(instr_ids),
                                            _ptr(cu_instr), n_tokens, temperature, _ptr(gumbel), _ptr(act_scale),
                                            _ptr(act_offset), action_dim, _ptr(step_t), _ptr(tokens_out),
                                            _ptr(logp_out), _ptr(actions_out), _ptr(logits_out), _ptr(values_out),
                                            stream))


def vla_policy_step_parallel(ctx, B, patch_emb, cu_patch, instr_ids, cu_instr, n_tokens, placeholder_id, temperature,
                             gumbel, act_scale, act_offset, action_dim, tokens_out, logp_out, actions_out,
                             logits_out, stream: int = 0) -> None:
    _check(ctx, lib().vla_policy_step_parallel(ctx, B, _ptr(patch_emb), _ptr(cu_patch), _ptr(instr_ids),
                                               _ptr(cu_instr), n_tokens, placeholder_id, temperature, _ptr(gumbel),
                                               _ptr(act_scale), _ptr(act_offset), action_dim, _ptr(tokens_out),
                                               _ptr(logp_out), _ptr(actions_out), _ptr(logits_out), stream))


def vla_score_tokens(ctx, B, patch_emb, cu_patch, instr_ids, cu_instr, n_tokens, tokens, placeholder_id, temperature,
                     mu_logp, sigma, logp_out, ratio_out, weight_out, logits_out, stream: int = 0) -> None:
    _check(ctx, lib().vla_score_tokens(ctx, B, _ptr(patch_emb), _ptr(cu_patch), _ptr(instr_ids), _ptr(cu_instr),
                                       n_tokens, _ptr(tokens), placeholder_id, temperature, _ptr(mu_logp), sigma,
                                       _ptr(logp_out), _ptr(ratio_out), _ptr(weight_out), _ptr(logits_out), stream))


def vla_prefill_slots(ctx, slot_ids, patch_emb, cu_patch, instr_ids, cu_instr, logits_out, stream: int = 0) -> None:
    slot_ids = np.ascontiguousarray(slot_ids, dtype=np.int32)
    _check(ctx, lib().vla_prefill_slots(ctx, len(slot_ids), _ptr(slot_ids), _ptr(patch_emb), _ptr(cu_patch),
                                        _ptr(instr_ids), _ptr(cu_instr), _ptr(logits_out), stream))


def vla_decode_slots(ctx, slot_ids, token_ids, logits_out, stream: int = 0) -> None:
    slot_ids = np.ascontiguousarray(slot_ids, dtype=np.int32)
    _check(ctx, lib().vla_decode_slots(ctx, len(slot_ids), _ptr(slot_ids), _ptr(token_ids), _ptr(logits_out), stream))


def vla_release_slots(ctx, slot_ids) -> None:
    slot_ids = np.ascontiguousarray(slot_ids, dtype=np.int32)
    _check(ctx, lib().vla_release_slots(ctx, len(slot_ids), _ptr(slot_ids)))


def vla_prefill(ctx, B, patch_emb, cu_patch: np.ndarray, instr_ids, cu_instr: np.ndarray, logits_out,
                stream: int = 0) -> None:
    _check(ctx, lib().vla_prefill(ctx, B, _ptr(patch_emb), _ptr(cu_patch), _ptr(instr_ids), _ptr(cu_instr),
                                  _ptr(logits_out), stream))


def vla_decode_step(ctx, B, token_ids, logits_out, stream: int = 0) -> None:
    _check(ctx, lib().vla_decode_step(ctx, B, _ptr(token_ids), _ptr(logits_out), stream))


def vla_decode_step_static(ctx, B, token_ids, logits_out, stream: int = 0) -> None:
    _check(ctx, lib().vla_decode_step_static(ctx, B, _ptr(token_ids), _ptr(logits_out), stream))


def vla_policy_step(ctx, B, patch_emb, cu_patch, instr_ids, cu_instr, n_tokens, temperature, gumbel,
                    act_scale, act_offset, action_dim, tokens_out, logp_out, actions_out, logits_out,
                    stream: int = 0) -> None:
    _check(ctx, lib().vla_policy_step(ctx, B, _ptr(patch_emb), _ptr(cu_patch), _ptr(instr_ids), _ptr(cu_instr),
                                      n_tokens, temperature, _ptr(gumbel), _ptr(act_scale), _ptr(act_offset),
                                      action_dim, _ptr(tokens_out), _ptr(logp_out), _ptr(actions_out),
                                      _ptr(logits_out), stream))


def vla_select(ctx, B, logits, temperature, gumbel, k, n_tokens, act_scale, act_offset, action_dim,
               tokens_out, logp_out, actions_out, out_stride, next_ids_out, stream: int = 0) -> None:
    _check(ctx, lib().vla_select(ctx, B, _ptr(logits), temperature, _ptr(gumbel), k, n_tokens, _ptr(act_scale),
                                 _ptr(act_offset), action_dim, _ptr(tokens_out), _ptr(logp_out),
                                 _ptr(actions_out), out_stride, _ptr(next_ids_out), stream))


def vla_probe(ctx, kind: int, stream: int = 0) -> float:
    v = C.c_double()
    _check(ctx, lib().vla_probe(ctx, kind, C.byref(v), stream))
    return v.value


def vla_prof_enable(ctx, mask: int) -> None:
    _check(ctx, lib().vla_prof_enable(ctx, mask))


def vla_prof_count() -> int:
    return lib().vla_prof_count()


def vla_prof_read(ctx, i: int):
    name, n, ms = C.c_char_p(), C.c_int64(), C.c_double()
    _check(ctx, lib().vla_prof_read(ctx, i, C.byref(name), C.byref(n), C.byref(ms)))
    return name.value.decode(), n.value, ms.value


# ---- convenience wrapper: owns the torch buffers ------------------------------------------------------

class Batcher:
    """Thin wrapper of the native request queue with the dynamic-window trigger (Section 3.2, Eq. 1)."""

    def __init__(self, target_batch: int, t_max: float, max_tokens: int = 0):
        self.h = C.c_void_p()
        rc = lib().vla_batcher_create(target_batch, t_max, max_tokens, C.byref(self.h))
        if rc:
            raise VlaError(rc, "vla_batcher_create")
        self.target = target_batch
        self._buf = (vla_request * target_batch)()

    def close(self):
        if self.h:
            lib().vla_batcher_destroy(self.h)
            self.h = None

    __del__ = close

    def push(self, rid: int, n_patches: int, n_instr: int, t_arrival: float) -> None:
        r = vla_request(rid, n_patches, n_instr, t_arrival)
        rc = lib().vla_batcher_push(self.h, C.byref(r))
        if rc:
            raise VlaError(rc, "vla_batcher_push")

    def __len__(self) -> int:
        n = C.c_int32()
        lib().vla_batcher_size(self.h, C.byref(n))
        return n.value

    def deadline(self) -> float:
        t = C.c_double()
        lib().vla_batcher_deadline(self.h, C.byref(t))
        return t.value

    def poll(self, t_now: float, cap: Optional[int] = None):
        """[(id, n_patches, n_instr, t_arrival)] of the released batch (at most min(target, cap) requests), [] if
        the rule did not fire."""
        n = C.c_int32()
        rc = lib().vla_batcher_poll(self.h, t_now, self._buf, self.target if cap is None else min(cap, self.target),
                                    C.byref(n))
        if rc:
            raise VlaError(rc, "vla_batcher_poll")
        return [(r.id, r.n_patches, r.n_instr, r.t_arrival) for r in self._buf[:n.value]]


def make_config(shape, max_batch: int, max_seq: int, max_prefill_tokens: int, value_max_steps: int = 0,
                precision: int = VLA_PREC_HIGH, two_term_layers: int = 0) -> vla_config:
    return vla_config(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn, shape.vocab,
                      shape.n_action_bins, shape.rope_theta, shape.rms_eps,
                      VLA_BF16 if shape.dtype == "bf16" else VLA_F32, max_batch, max_seq, max_prefill_tokens,
                      value_max_steps, precision, two_term_layers)


class VlaPolicy:
    """Holds a context plus the torch-allocated arena / KV cache / workspace it is bound to."""

    def __init__(self, shape, max_batch: int, max_seq: int, max_prefill_tokens: int, device="cuda:0",
                 value_max_steps: int = 0, precision: int = VLA_PREC_HIGH, two_term_layers: int = 0):
        import torch
        self.torch = torch
        self.shape = shape
        self.device = torch.device(device)
        self.dtype_code = VLA_BF16 if shape.dtype == "bf16" else VLA_F32
        self.cfg = make_config(shape, max_batch, max_seq, max_prefill_tokens, value_max_steps, precision,
                               two_term_layers)
        self.ctx = vla_create(self.cfg)
        a, k, w = vla_query_sizes(self.cfg)
        self.sizes = (a, k, w)
        self.arena = torch.empty(a, dtype=torch.uint8, device=self.device)
        self.kv = torch.empty(k, dtype=torch.uint8, device=self.device)
        self.work = torch.empty(w, dtype=torch.uint8, device=self.device)
        vla_bind_buffers(self.ctx, self.arena, self.kv, self.work)

    def close(self):
        if self.ctx is not None:
            self.torch.cuda.synchronize(self.device)
            vla_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _stream(self) -> int:
        return self.torch.cuda.current_stream(self.device).cuda_stream

    def to_device(self, arr: np.ndarray):
        """numpy array in storage dtype (float32, or uint16 holding bfloat16 bits) -> device tensor."""
        torch = self.torch
        if arr.dtype == np.uint16:
            return torch.from_numpy(arr.view(np.int16)).to(self.device).view(torch.bfloat16)
        return torch.from_numpy(arr).to(self.device)

    def load_weights(self, weights: Dict[str, "object"]):
        """weights: name -> device tensor (or numpy array in storage dtype, uploaded one at a time)."""
        dev = {}
        for n, t in weights.items():
            dev[n] = self.to_device(t) if isinstance(t, np.ndarray) else t
        vla_load_weights(self.ctx, dev, self.dtype_code, self._stream())
        self.torch.cuda.current_stream(self.device).synchronize()   # sources may now be freed
        vla_check_weights(self.ctx)                                 # raises VLA_E_WEIGHTS for unrepresentable values

    def load_value_head(self, weights: Dict[str, "object"]):
        dev = {n: (self.to_device(t) if isinstance(t, np.ndarray) else t) for n, t in weights.items()}
        vla_load_value_head(self.ctx, dev, self.dtype_code, self._stream())
        self.torch.cuda.current_stream(self.device).synchronize()

    # In-place weight update: drain, then overwrite on `stream` (a torch stream, default: the current one).
    def state(self):
        return vla_get_state(self.ctx)

    def drain_begin(self):
        vla_drain_begin(self.ctx)

    def update_begin(self, stream=None):
        vla_update_begin(self.ctx, stream.cuda_stream if stream is not None else self._stream())

    def update_tensors(self, tensors: Dict[str, "object"], stream=None):
        """tensors: name -> device tensor in storage dtype (they must stay alive until the stream has passed them)."""
        vla_update_tensors(self.ctx, tensors, self.dtype_code, stream.cuda_stream if stream is not None else self._stream())

    def update_commit(self, stream=None) -> int:
        return vla_update_commit(self.ctx, stream.cuda_stream if stream is not None else self._stream())

    def prefill(self, patch_emb, cu_patch, instr_ids, cu_instr, want_logits=True):
        torch = self.torch
        B = len(cu_patch) - 1
        out = torch.empty((B, self.shape.n_action_bins), dtype=torch.float32, device=self.device) if want_logits else None
        vla_prefill(self.ctx, B, patch_emb, np.ascontiguousarray(cu_patch, dtype=np.int32), instr_ids,
                    np.ascontiguousarray(cu_instr, dtype=np.int32), out, self._stream())
        return out

    def prefill_slots(self, slot_ids, patch_emb, cu_patch, instr_ids, cu_instr):
        torch = self.torch
        out = torch.empty((len(slot_ids), self.shape.n_action_bins), dtype=torch.float32, device=self.device)
        vla_prefill_slots(self.ctx, slot_ids, patch_emb, np.ascontiguousarray(cu_patch, dtype=np.int32), instr_ids,
                          np.ascontiguousarray(cu_instr, dtype=np.int32), out, self._stream())
        return out

    def decode_slots(self, slot_ids, token_ids):
        torch = self.torch
        out = torch.empty((len(slot_ids), self.shape.n_action_bins), dtype=torch.float32, device=self.device)
        vla_decode_slots(self.ctx, slot_ids, token_ids, out, self._stream())
        return out

    def release_slots(self, slot_ids):
        vla_release_slots(self.ctx, slot_ids)

    def decode_step(self, token_ids, want_logits=True, static=False, out=None):
        """static=True: vla_decode_step_static (staging in the library's own device array, nothing allocated)."""
        torch = self.torch
        B = token_ids.shape[0]
        if out is None and want_logits:
            out = torch.empty((B, self.shape.n_action_bins), dtype=torch.float32, device=self.device)
        (vla_decode_step_static if static else vla_decode_step)(self.ctx, B, token_ids, out, self._stream())
        return out

    def policy_step_parallel(self, patch_emb, cu_patch, instr_ids, cu_instr, n_tokens, placeholder_id,
                             temperature=0.0, gumbel=None, act_scale=None, act_offset=None, action_dim=7,
                             want_logits=False, out=None):
        """All K action tokens from one forward pass (placeholder-fed positions)."""
        torch = self.torch
        B = len(cu_patch) - 1
        A = self.shape.n_action_bins
        if out is None:
            out = {
                "tokens": torch.empty((B, n_tokens), dtype=torch.int32, device=self.device),
                "logp": torch.empty((B, n_tokens), dtype=torch.float32, device=self.device),
                "actions": torch.empty((B, n_tokens), dtype=torch.float32, device=self.device),
                "logits": torch.empty((B, n_tokens, A), dtype=torch.float32, device=self.device) if want_logits else None,
            }
        vla_policy_step_parallel(self.ctx, B, patch_emb, np.ascontiguousarray(cu_patch, dtype=np.int32), instr_ids,
                                 np.ascontiguousarray(cu_instr, dtype=np.int32), n_tokens, int(placeholder_id),
                                 float(temperature), gumbel, act_scale, act_offset, action_dim, out["tokens"],
                                 out["logp"], out["actions"], out.get("logits"), self._stream())
        return out

    def score_tokens(self, patch_emb, cu_patch, instr_ids, cu_instr, tokens, placeholder_id=-1, temperature=0.0,
                     mu_logp=None, sigma=1.0, want_logits=False):
        """Log-probabilities of stored tokens [B, K] under the current weights (+ ratio and GIPO coefficient)."""
        torch = self.torch
        B, K = tokens.shape
        A = self.shape.n_action_bins
        mk = lambda *s: torch.empty(s, dtype=torch.float32, device=self.device)   # noqa: E731
        out = {"logp": mk(B, K), "ratio": mk(B, K) if mu_logp is not None else None,
               "weight": mk(B, K) if mu_logp is not None else None, "logits": mk(B, K, A) if want_logits else None}
        vla_score_tokens(self.ctx, B, patch_emb, np.ascontiguousarray(cu_patch, dtype=np.int32), instr_ids,
                         np.ascontiguousarray(cu_instr, dtype=np.int32), K, tokens, int(placeholder_id),
                         float(temperature), mu_logp, float(sigma), out["logp"], out["ratio"], out["weight"],
                         out["logits"], self._stream())
        return out

    def policy_step(self, patch_emb, cu_patch, instr_ids, cu_instr, n_tokens, temperature=0.0, gumbel=None,
                    act_scale=None, act_offset=None, action_dim=7, want_logits=False, out=None, step_t=None):
        """step_t (device int32 [B]) switches the value head on: out["values"] [B] is filled as well."""
        torch = self.torch
        B = len(cu_patch) - 1
        A = self.shape.n_action_bins
        if out is None:
            out = {
                "tokens": torch.empty((B, n_tokens), dtype=torch.int32, device=self.device),
                "logp": torch.empty((B, n_tokens), dtype=torch.float32, device=self.device),
                "actions": torch.empty((B, n_tokens), dtype=torch.float32, device=self.device),
                "logits": torch.empty((B, n_tokens, A), dtype=torch.float32, device=self.device) if want_logits else None,
            }
        if step_t is not None:
            if out.get("values") is None:
                out["values"] = torch.empty((B,), dtype=torch.float32, device=self.device)
            vla_policy_step_value(self.ctx, B, patch_emb, np.ascontiguousarray(cu_patch, dtype=np.int32), instr_ids,
                                  np.ascontiguousarray(cu_instr, dtype=np.int32), n_tokens, float(temperature),
                                  gumbel, act_scale, act_offset, action_dim, step_t, out["tokens"], out["logp"],
                                  out["actions"], out.get("logits"), out["values"], self._stream())
            return out
        vla_policy_step(self.ctx, B, patch_emb, np.ascontiguousarray(cu_patch, dtype=np.int32), instr_ids,
                        np.ascontiguousarray(cu_instr, dtype=np.int32), n_tokens, float(temperature), gumbel,
                        act_scale, act_offset, action_dim, out["tokens"], out["logp"], out["actions"],
                        out.get("logits"), self._stream())
        return out
