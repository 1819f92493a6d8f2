"""CPU-side checks of the library: it loads, exports every symbol the headers
declare, its schedule generator agrees with the oracle's, and the slot allocator /
validator return the documented error codes (dry-run stages: no kernel runs)."""
import os
import re

import pytest

from oracle import stage_oracle as O
from paper_2007_01045_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(header):
    txt = open(os.path.join(ROOT, "include", header)).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return set(re.findall(r"\b((?:stage|dapple|pipeline)_[a-z0-9_]+)\s*\(", txt))


def test_library_exports_every_declared_symbol():
    lib = B.load()
    names = _declared("dapple_stage.h") | _declared("dapple_kernels.h") | _declared("dapple_pipeline.h")
    assert len(names) >= 20
    for n in names:
        assert hasattr(lib, n), n
    assert names == set(B.SYMBOLS), names ^ set(B.SYMBOLS)


@pytest.mark.parametrize("order", [O.GPIPE, O.EARLY_BACKWARD])
def test_schedule_matches_oracle(order):
    for M in range(1, 12):
        for K in range(1, 12):
            assert B.stage_schedule_ops(M, K, order) == O.schedule_ops(M, K, order)


def test_schedule_bad_arguments():
    for args in [(0, 1, 1), (3, 0, 1), (3, 2, 5)]:
        with pytest.raises(B.StageError) as e:
            B.stage_schedule_ops(*args)
        assert e.value.code == B.STAGE_E_BAD_ORDER


def dry(max_slots=2, **kw):
    base = dict(n_layers=2, hidden=64, n_heads=4, ffn=256, seq=16, micro_batch=2, max_slots=max_slots,
                dtype=B.DTYPE_F32, flags=B.FLAG_DRY_RUN)
    base.update(kw)
    return B.make_config(**base)


def test_config_errors():
    for kw in [dict(n_heads=5), dict(hidden=0), dict(max_slots=0), dict(dtype=7), dict(hidden=66, n_heads=6),
               dict(ln_eps=-1.0), dict(hidden=8192, n_heads=8)]:
        with pytest.raises(B.StageError) as e:
            B.stage_query_sizes(dry(**kw))
        assert e.value.code == B.STAGE_E_CONFIG, kw
    # not a dry run and no device memory given
    cfg = dry(); cfg.flags = 0
    with pytest.raises(B.StageError) as e:
        B.stage_init(cfg, None, None, 0)
    assert e.value.code == B.STAGE_E_NULL
    with pytest.raises(B.StageError) as e:          # arena too small (pointer never dereferenced)
        B.stage_init(cfg, 4096, 4096, 1024)
    assert e.value.code == B.STAGE_E_ARENA_SMALL


def test_recompute_keeps_only_the_boundary_per_slot():
    # section VI-E: with re-computation a resident micro-batch keeps its input only; the activation
    # buffers (one for the forward tasks, one per backward lane) do not scale with the slots
    full = B.stage_query_sizes(dry(2))
    rc2 = B.stage_query_sizes(dry(2, flags=B.FLAG_DRY_RUN | B.FLAG_RECOMPUTE))
    rc8 = B.stage_query_sizes(dry(8, flags=B.FLAG_DRY_RUN | B.FLAG_RECOMPUTE))
    T, H = 2 * 16, 64
    assert rc2.slot_bytes == T * H * 4 < full.slot_bytes
    assert rc8.arena_bytes - rc2.arena_bytes == 6 * rc2.slot_bytes
    assert rc2.workspace_bytes >= full.workspace_bytes + full.slot_bytes          # a backward lane's buffer
    grads_and_slots = lambda q, k: q.grad_bytes + k * q.slot_bytes
    assert rc2.arena_bytes - grads_and_slots(rc2, 2) >= 2 * rc2.workspace_bytes + full.slot_bytes   # + the forward tasks' buffer
    one = B.stage_query_sizes(dry(2, flags=B.FLAG_DRY_RUN | B.FLAG_RECOMPUTE | B.FLAG_ONE_STREAM))
    assert one.arena_bytes - grads_and_slots(one, 2) < rc2.arena_bytes - grads_and_slots(rc2, 2) - full.slot_bytes
    # first stage: token ids; last stage: input and targets
    emb = B.stage_query_sizes(dry(2, flags=B.FLAG_DRY_RUN | B.FLAG_RECOMPUTE, has_embedding=1, vocab=100, max_pos=16))
    assert emb.slot_bytes == 256          # T int32 ids, rounded up to the 256-byte granule
    head = B.stage_query_sizes(dry(2, flags=B.FLAG_DRY_RUN | B.FLAG_RECOMPUTE, has_mlm_head=1, vocab=100))
    assert head.slot_bytes == T * H * 4 + 256


def test_sizes_scale_with_slots_only():
    a, b = B.stage_query_sizes(dry(2)), B.stage_query_sizes(dry(4))
    assert a.slot_bytes == b.slot_bytes and a.grad_bytes == b.grad_bytes
    assert b.arena_bytes - a.arena_bytes == 2 * a.slot_bytes
    H, F = 64, 256
    assert a.n_params == 2 * (4 * (H * H + H) + 2 * H * F + F + H + 4 * H)


def test_slot_allocator_error_paths():
    h = B.stage_init(dry(2), None, None, 0)
    try:
        B.stage_fwd(h, 0, None, None)
        with pytest.raises(B.StageError) as e:
            B.stage_fwd(h, 0, None, None)
        assert e.value.code == B.STAGE_E_DUP_MB
        B.stage_fwd(h, 1, None, None)
        with pytest.raises(B.StageError) as e:      # K+1-th forward without a backward
            B.stage_fwd(h, 2, None, None)
        assert e.value.code == B.STAGE_E_NO_SLOT
        with pytest.raises(B.StageError) as e:
            B.stage_bwd(h, 5, None, None)
        assert e.value.code == B.STAGE_E_NOT_RESIDENT
        st = B.stage_stats(h)
        assert st.live_slots == 2 and st.peak_live_slots == 2 and st.fwd_tasks == 2
        B.stage_bwd(h, 0, None, None)
        B.stage_fwd(h, 2, None, None)               # reuses the slot B_0 released
        with pytest.raises(B.StageError) as e:
            B.stage_bwd(h, 0, None, None)
        assert e.value.code == B.STAGE_E_NOT_RESIDENT
        B.stage_bwd(h, 1, None, None)
        B.stage_bwd(h, 2, None, None)
        st = B.stage_stats(h)
        assert st.live_slots == 0 and st.peak_live_slots == 2 and st.bwd_tasks == 3
        assert st.peak_activation_bytes == 2 * st.slot_bytes
    finally:
        B.stage_destroy(h)


@pytest.mark.parametrize("M,K", [(1, 1), (4, 2), (8, 4), (16, 4), (5, 7)])
def test_peak_is_K_for_early_backward_and_M_for_gpipe(M, K):
    slots = max(M, K)
    h = B.stage_init(dry(slots), None, None, 0)
    try:
        B.stage_run_schedule(h, M, K, B.ORDER_EARLY_BACKWARD)
        st = B.stage_stats(h)
        assert st.peak_live_slots == min(K, M) and st.live_slots == 0
        assert st.fwd_tasks == M and st.bwd_tasks == M
        B.stage_reset_stats(h)
        B.stage_run_schedule(h, M, K, B.ORDER_GPIPE)
        assert B.stage_stats(h).peak_live_slots == M
    finally:
        B.stage_destroy(h)


def test_run_schedule_rejects_bad_orders_before_running_anything():
    h = B.stage_init(dry(2), None, None, 0)
    try:
        bad = [
            (4, 2, B.ORDER_GPIPE, None),                                   # needs 4 slots, stage has 2
            (4, 3, B.ORDER_EARLY_BACKWARD, None),                          # K > max_slots
            (2, 2, B.ORDER_EXPLICIT, [("B", 0), ("F", 0), ("F", 1), ("B", 1)]),   # B before F
            (2, 2, B.ORDER_EXPLICIT, [("F", 0), ("F", 0), ("B", 0), ("B", 0)]),   # twice
            (3, 2, B.ORDER_EXPLICIT, [("F", 0), ("F", 1), ("F", 2), ("B", 0), ("B", 1), ("B", 2)]),  # 3 resident
            (2, 2, B.ORDER_EXPLICIT, [("F", 0), ("B", 0)]),                # incomplete
            (0, 1, B.ORDER_GPIPE, None),
        ]
        for M, K, order, ops in bad:
            with pytest.raises(B.StageError) as e:
                B.stage_run_schedule(h, M, K, order, explicit_ops=ops)
            assert e.value.code == B.STAGE_E_BAD_ORDER, (M, K, order, ops)
            assert B.stage_stats(h).fwd_tasks == 0
        # a steady phase that ran the forward first would need K+1 slots
        fb = [("F", 0), ("F", 1), ("F", 2), ("B", 0), ("B", 1), ("F", 3), ("B", 2), ("B", 3)]
        with pytest.raises(B.StageError):
            B.stage_run_schedule(h, 4, 2, B.ORDER_EXPLICIT, explicit_ops=fb)
        # descending backwards are a valid explicit order
        ok = [("F", 0), ("F", 1), ("B", 1), ("B", 0)]
        B.stage_run_schedule(h, 2, 2, B.ORDER_EXPLICIT, explicit_ops=ok)
        assert B.stage_stats(h).bwd_tasks == 2
        # leftovers from single calls block a schedule run
        B.stage_fwd(h, 9, None, None)
        with pytest.raises(B.StageError) as e:
            B.stage_run_schedule(h, 2, 2, B.ORDER_GPIPE)
        assert e.value.code == B.STAGE_E_BAD_ORDER
    finally:
        B.stage_destroy(h)


def test_null_handle_and_error_text():
    with pytest.raises(B.StageError) as e:
        B.stage_fwd(None, 0, None, None)
    assert e.value.code == B.STAGE_E_NULL and "NULL" in str(e.value)


def test_pipeline_host_functions_follow_the_oracle():
    import random
    from oracle import pipeline_oracle as PO
    rng = random.Random(7)
    for _ in range(300):
        S, M = rng.randint(1, 6), rng.randint(1, 12)
        F = [rng.uniform(0.2, 3.0) for _ in range(S)]
        Bt = [rng.uniform(0.2, 6.0) for _ in range(S)]
        if rng.random() < 0.3:
            F[0] *= 4; Bt[0] *= 4
        assert B.pipeline_pivot_stage(M, F, Bt) == PO.pivot_stage(F, Bt, M)
        assert B.pipeline_latency_model(M, F, Bt) == pytest.approx(PO.latency_model(F, Bt, M), rel=1e-13)
        Q = rng.randrange(S)
        assert B.pipeline_latency_model(M, F, Bt, Q) == pytest.approx(PO.latency_model(F, Bt, M, Q), rel=1e-13)
        for pol, name in ((B.POLICY_A, "A"), (B.POLICY_B, "B")):
            D = rng.choice([0, 1, 2, 5, 100])
            assert B.pipeline_warmup_depths(S, M, pol, D) == PO.warmup_depths(S, M, name, None if D == 0 else D)
    with pytest.raises(B.StageError):
        B.pipeline_latency_model(3, [1.0, 1.0], [1.0, 1.0], Q=2)
    assert B.pipeline_boundary_bytes(3, 4, 1000) == 2 * 2 * 4 * 1024
