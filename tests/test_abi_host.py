"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the header
declares, and validates configurations."""
import ctypes as C
import os
import re

import pytest

import workloads as W
from paper_2603_18464_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(vla_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = declared_symbols()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert hasattr(L, n), n


def test_config_validation_and_sizes():
    wl = W.get_workload("C3")
    cfg = B.make_config(wl.shape, wl.batch, wl.max_seq, wl.batch * 290, precision=B.VLA_PREC_FAST)
    arena, kv, work = B.vla_query_sizes(cfg)
    s = wl.shape
    assert kv == 2 * s.n_layers * wl.batch * s.n_heads * (wl.max_seq | 1) * s.head_dim * 2     # odd position pitch
    # two-term layers keep a second set of planes with the low terms of their cached keys and values, one byte each,
    # and an 8-bit copy of their matrices for the 8-bit low terms of the operands
    hi = B.make_config(wl.shape, wl.batch, wl.max_seq, wl.batch * 290)
    assert hi.precision == B.VLA_PREC_HIGH and hi.two_term_layers == 0          # 0 = the default of 4 layers
    per_layer_kv = kv // s.n_layers
    per_layer_w8 = 4 * s.d_model ** 2 + 3 * s.d_model * s.d_ffn
    arena_hi, kv_hi, work_hi = B.vla_query_sizes(hi)
    assert kv_hi == kv + 4 * per_layer_kv // 2 and work_hi > work
    assert 4 * per_layer_w8 <= arena_hi - arena < 4 * per_layer_w8 + (1 << 20)
    for n, n_eff in [(1, 1), (7, 7), (32, 32), (1000, 32)]:
        cn = B.make_config(wl.shape, wl.batch, wl.max_seq, wl.batch * 290, two_term_layers=n)
        arena_n, kv_n, work_n = B.vla_query_sizes(cn)
        assert kv_n == kv + n_eff * per_layer_kv // 2 and work_n == work_hi
        assert n_eff * per_layer_w8 <= arena_n - arena < n_eff * per_layer_w8 + (1 << 20)
    assert arena >= 2 * (s.n_matrix_params + (s.vocab + 256) * s.d_model)
    assert arena < 2 * (s.n_matrix_params + (s.vocab + 256) * s.d_model) + (4 << 20)   # head is slimmed: no second [V,d] matrix
    ctx = B.vla_create(cfg)
    B.vla_destroy(ctx)
    for field, value in [("n_heads", 31), ("dtype", 5), ("n_action_bins", 0), ("n_action_bins", 40000),
                         ("max_seq", 0), ("head_dim", 100), ("rope_theta", 0.0), ("precision", 2),
                         ("two_term_layers", -1)]:
        bad = B.make_config(wl.shape, wl.batch, wl.max_seq, wl.batch * 290)
        setattr(bad, field, value)
        with pytest.raises(B.VlaError) as e:
            B.vla_create(bad)
        assert e.value.code == -2, field
        with pytest.raises(B.VlaError):
            B.vla_query_sizes(bad)


def test_null_arguments_and_unbound_state():
    L = B.lib()
    assert L.vla_create(None, None) == -1
    assert L.vla_destroy(None) == -1
    assert L.vla_prefill(None, 1, None, None, None, None, None, None) == -1
    wl = W.get_workload("C1")
    ctx = B.vla_create(B.make_config(wl.shape, 4, 64, 256))
    with pytest.raises(B.VlaError) as e:
        B.vla_bind_buffers(ctx, None, None, None)
    assert e.value.code == -1
    # nothing bound yet: every compute entry point refuses
    cu = (C.c_int32 * 2)(0, 1)
    assert L.vla_prefill(ctx, 1, None, cu, None, cu, None, None) == -5
    assert L.vla_decode_step(ctx, 1, None, None, None) == -5
    assert L.vla_load_weights(ctx, None, 0, None) == -1
    assert "bound" in B.vla_last_error(ctx) or "NULL" in B.vla_last_error(ctx)
    assert B.vla_prof_count() == 18
    B.vla_destroy(ctx)


def test_serving_state_transitions_on_the_host():
    """Drain / update state machine (Appendix "High-Performance NCCL-based Weight Synchronization"): the
    transitions that touch no device state."""
    L = B.lib()
    wl = W.get_workload("C1")
    ctx = B.vla_create(B.make_config(wl.shape, 4, 64, 256, value_max_steps=3))
    assert B.vla_get_state(ctx) == (B.VLA_ACCEPTING, 0)
    B.vla_drain_begin(ctx)
    B.vla_drain_begin(ctx)                                   # repeating the signal is harmless
    assert B.vla_get_state(ctx) == (B.VLA_DRAINING, 0)
    # no update is open: tensors and commit are refused, and the state does not move
    dummy = (B.vla_tensor * 1)()
    assert L.vla_update_tensors(ctx, dummy, 0, None) == B.VLA_E_STATE
    assert L.vla_update_commit(ctx, None, None) == B.VLA_E_STATE
    # an update cannot open on a context without bound buffers / loaded weights
    assert L.vla_update_begin(ctx, None) == B.VLA_E_STATE
    assert B.vla_get_state(ctx) == (B.VLA_DRAINING, 0)
    assert L.vla_get_state(None, None, None) == -1
    assert L.vla_drain_begin(None) == -1
    B.vla_destroy(ctx)


def test_later_entry_points_refuse_null_and_unbound_contexts():
    """Every compute entry point added after the first path checks the context before anything else."""
    L = B.lib()
    wl = W.get_workload("C1")
    ctx = B.vla_create(B.make_config(wl.shape, 4, 64, 256, value_max_steps=2))
    cu = (C.c_int32 * 2)(0, 1)
    one = (C.c_int32 * 1)(0)
    assert L.vla_policy_step_parallel(None, 1, None, cu, None, cu, 1, 0, 0.0, None, None, None, 7, None, None, None, None, None) == -1
    assert L.vla_score_tokens(None, 1, None, cu, None, cu, 1, None, -1, 0.0, None, 1.0, None, None, None, None, None) == -1
    assert L.vla_prefill_slots(None, 1, one, None, cu, None, cu, None, None) == -1
    assert L.vla_decode_slots(None, 1, one, None, None, None) == -1
    assert L.vla_release_slots(None, 1, one) == -1
    assert L.vla_load_value_head(None, None, 0, None) == -1
    assert L.vla_policy_step_value(None, 1, None, cu, None, cu, 1, 0.0, None, None, None, 7, None, None, None, None, None, None, None) == -1
    # unbound context: state error, nothing touched
    assert L.vla_policy_step_parallel(ctx, 1, None, cu, None, cu, 1, 0, 0.0, None, None, None, 7, None, None, None, None, None) == -5
    assert L.vla_score_tokens(ctx, 1, None, cu, None, cu, 1, None, -1, 0.0, None, 1.0, None, None, None, None, None) == -5
    assert L.vla_prefill_slots(ctx, 1, one, None, cu, None, cu, None, None) == -5
    assert L.vla_decode_slots(ctx, 1, one, None, None, None) == -5
    assert L.vla_policy_step_value(ctx, 1, None, cu, None, cu, 1, 0.0, None, None, None, 7, None, None, None, None, None, None, None) == -5
    # slot lists are validated on the host
    bad = (C.c_int32 * 2)(1, 1)
    assert L.vla_release_slots(ctx, 2, bad) == -3
    assert L.vla_release_slots(ctx, 1, (C.c_int32 * 1)(4)) == -3
    assert L.vla_release_slots(ctx, 0, one) == -3
    assert L.vla_release_slots(ctx, 1, one) == 0
    B.vla_destroy(ctx)
