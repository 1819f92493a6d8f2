"""S stages on one GPU run as a pipeline through the C-ABI of dapple_pipeline.h: results against the
float64 oracle of the unsplit model and against the single-stage HIP path, residency per stage,
and the measured timeline against the dependences of the schedule."""
import numpy as np
import pytest

from oracle import pipeline_oracle as PO
from paper_2007_01045_amd import binding as B
from paper_2007_01045_amd import inputs as I
from tests.stage_util import c_config, compare, make_inputs, run_gpu, run_oracle, to_np

pytestmark = pytest.mark.gpu

SEED = 20200701
TOL_F32, TOL_BF16 = 1e-4, 2e-2


class Pipe:
    """S equal stages cut from one L-layer configuration, each on a stream of its own (a partition of the
    compute units when parts > 1, an ordinary stream when parts == 0), with the boundary buffer between them."""

    def __init__(self, cfg, S, slots, theta, max_M, parts=1, flags=0):
        import torch
        assert cfg.n_layers % S == 0
        self.torch, self.S, self.cfg = torch, S, cfg
        part = I.StageConfig(cfg.n_layers // S, cfg.hidden, cfg.n_heads, cfg.ffn, cfg.seq, cfg.micro_batch,
                             cfg.M, cfg.K, cfg.dtype, ln_eps=cfg.ln_eps)
        n = I.n_params(part)
        assert n * S == theta.size
        self.pr = B.PipelineRunner([c_config(part, slots[i], flags=flags) for i in range(S)],
                                   [theta[i * n:(i + 1) * n] for i in range(S)], max_M, parts)
        self.runners = self.pr.runners

    def run(self, M, K, order, mbs):
        torch, r0, cfg = self.torch, self.runners[0], self.cfg
        T, H = cfg.tokens, cfg.hidden
        xs = [r0.to_dev(mb["x"].reshape(T, H)) for mb in mbs]
        dys = [r0.to_dev(mb["dy"].reshape(T, H)) for mb in mbs]
        ys = [r0.empty_act() for _ in range(M)]
        dxs = [r0.empty_act() for _ in range(M)]
        for r in self.runners:
            B.stage_zero_grads(r.h)
            B.stage_reset_stats(r.h)
        torch.cuda.synchronize()
        self.pr.run(M, K, order, xs, dys, None, ys, dxs)
        torch.cuda.synchronize()
        return dict(ys=[to_np(y) for y in ys], dxs=[to_np(d) for d in dxs],
                    grads=np.concatenate([r.grads.cpu().numpy() for r in self.runners]),
                    peak=[B.stage_stats(r.h).peak_live_slots for r in self.runners],
                    timeline=self.pr.timeline(M))

    def close(self):
        self.pr.close()


def check_timeline(tl, S, M, lists):
    """Every dependence of the schedule shows in the measured times: a stage's tasks in list order, a forward after
    the forward of the stage before, a backward after the backward of the stage behind."""
    eps = 1e-3   # ms: an event pair on one stream can read equal
    for i in range(S):
        prev = None
        for kind, m in lists[i]:
            t0, t1 = tl[(kind, i, m)]
            assert t1 >= t0 >= 0
            if prev is not None:
                assert t0 >= prev - eps, (kind, i, m)
            prev = t1
            if kind == "F" and i > 0:
                assert t0 >= tl[("F", i - 1, m)][1] - eps
            if kind == "B":
                dep = ("F", i, m) if i == S - 1 else ("B", i + 1, m)
                assert t0 >= tl[dep][1] - eps


@pytest.mark.parametrize("parts", [0, 1, 3])
def test_three_stages_fp32_equal_the_single_stage_bitwise(parts):
    cfg = I.StageConfig(6, 64, 4, 128, 16, 2, 5, 3, "f32", ln_eps=1e-5)
    S, M = 3, 5
    theta, mbs = make_inputs(cfg, SEED, M)
    K = B.pipeline_warmup_depths(S, M, B.POLICY_A)
    assert K == [3, 2, 1] == PO.warmup_depths(S, M, "A")
    one = run_gpu(cfg, theta, mbs, M, 3, B.ORDER_EARLY_BACKWARD)
    pipe = Pipe(cfg, S, K, theta, M, parts)
    try:
        got = pipe.run(M, K, B.ORDER_EARLY_BACKWARD, mbs)
        again = pipe.run(M, K, B.ORDER_EARLY_BACKWARD, mbs)
    finally:
        pipe.close()
    assert got["peak"] == K                      # stage i never holds more than K_i = S - i micro-batches
    assert np.array_equal(got["grads"], one["grads"]) and np.array_equal(again["grads"], one["grads"])
    for m in range(M):
        assert np.array_equal(got["ys"][m], one["ys"][m]) and np.array_equal(got["dxs"][m], one["dxs"][m])
    st, ref = run_oracle(cfg, theta, mbs, M, 3)
    compare(cfg, st, ref, got, TOL_F32, M)
    check_timeline(got["timeline"], S, M, PO.stage_lists(S, M, K))


def test_gpipe_order_and_policy_b_give_the_same_bits_with_more_residents():
    cfg = I.StageConfig(4, 64, 4, 128, 16, 2, 6, 3, "f32", ln_eps=1e-5)
    S, M = 2, 6
    theta, mbs = make_inputs(cfg, SEED, M)
    KA, KB = B.pipeline_warmup_depths(S, M, B.POLICY_A), B.pipeline_warmup_depths(S, M, B.POLICY_B)
    assert KA == [2, 1] and KB == [3, 1] == PO.warmup_depths(S, M, "B")
    pipe = Pipe(cfg, S, [M, M], theta, M)
    try:
        a = pipe.run(M, KA, B.ORDER_EARLY_BACKWARD, mbs)
        b = pipe.run(M, KB, B.ORDER_EARLY_BACKWARD, mbs)
        g = pipe.run(M, None, B.ORDER_GPIPE, mbs)
        check_timeline(g["timeline"], S, M, PO.stage_lists(S, M, None, PO.GPIPE))
        assert a["peak"] == KA and b["peak"] == KB and g["peak"] == [M, M]
        assert np.array_equal(a["grads"], b["grads"]) and np.array_equal(a["grads"], g["grads"])
        # depths that grow along the pipeline deadlock: refused before anything is enqueued
        with pytest.raises(B.StageError) as e:
            pipe.run(M, [1, 2], B.ORDER_EARLY_BACKWARD, mbs)
        assert e.value.code == B.STAGE_E_BAD_ORDER
        with pytest.raises(B.StageError):
            pipe.run(M + 1, KA, B.ORDER_EARLY_BACKWARD, mbs + mbs[:1])     # more than max_M
        c = pipe.run(M, KA, B.ORDER_EARLY_BACKWARD, mbs)                   # still usable afterwards
        assert np.array_equal(a["grads"], c["grads"])
    finally:
        pipe.close()


@pytest.mark.parametrize("flags", [0, B.FLAG_ONE_STREAM])
def test_four_bf16_stages_on_four_partitions_follow_the_oracle(flags):
    cfg = I.StageConfig(4, 256, 4, 512, 128, 2, 6, 4, "bf16")
    S, M = 4, 6
    theta, mbs = make_inputs(cfg, SEED, M)
    K = B.pipeline_warmup_depths(S, M, B.POLICY_A)
    pipe = Pipe(cfg, S, K, theta, M, parts=4, flags=flags)
    try:
        got = pipe.run(M, K, B.ORDER_EARLY_BACKWARD, mbs)
    finally:
        pipe.close()
    assert got["peak"] == [4, 3, 2, 1]
    st, ref = run_oracle(cfg, theta, mbs, M, 4)
    compare(cfg, st, ref, got, TOL_BF16, M)
    tl = got["timeline"]
    check_timeline(tl, S, M, PO.stage_lists(S, M, K))
    # the stages really ran beside each other: the iteration is shorter than its tasks laid end to end,
    # and no shorter than the busiest stage
    span = max(v[1] for v in tl.values())
    busy = [sum(tl[(k, i, m)][1] - tl[(k, i, m)][0] for k in "FB" for m in range(M)) for i in range(S)]
    assert max(busy) <= span * 1.001 and span < sum(busy)


def test_pipeline_create_error_paths():
    cfg = I.StageConfig(2, 64, 4, 128, 16, 2, 2, 2, "f32", ln_eps=1e-5)
    theta, _ = make_inputs(cfg, SEED, 2)
    r = B.StageRunner(c_config(cfg, 2), theta)          # on torch's default (NULL) stream
    try:
        import torch
        buf = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
        with pytest.raises(B.StageError) as e:
            B.pipeline_create([r.h], buf.data_ptr(), buf.numel(), cfg.tokens * cfg.hidden * 4, 2)
        assert e.value.code == B.STAGE_E_CONFIG            # no stream of its own
    finally:
        r.close()
    with pytest.raises(B.StageError):
        B.pipeline_partition_stream_create(3, 3)
    with pytest.raises(B.StageError):
        B.pipeline_warmup_depths(0, 4)


@pytest.mark.parametrize("dtype,tol", [("f32", TOL_F32), ("bf16", TOL_BF16)])
def test_whole_model_as_three_stages_follows_the_oracle(dtype, tol):
    """Embedding block on the first stage, MLM head on the last: token ids in, losses out, every gradient of the
    unsplit model against the float64 oracle of the unsplit model."""
    import torch
    if dtype == "f32":
        full = I.StageConfig(3, 64, 4, 128, 16, 2, 4, 3, "f32", has_embedding=True, has_mlm_head=True, vocab=200,
                             max_pos=16, ln_eps=1e-5)
    else:
        full = I.StageConfig(3, 128, 2, 256, 64, 2, 4, 3, "bf16", has_embedding=True, has_mlm_head=True, vocab=520,
                             max_pos=64)
    S, M = 3, 4
    theta, mbs = make_inputs(full, SEED, M)
    kw = dict(vocab=full.vocab, max_pos=full.max_pos, ln_eps=full.ln_eps)
    parts = [I.StageConfig(1, full.hidden, full.n_heads, full.ffn, full.seq, full.micro_batch, M, 3, dtype,
                           has_embedding=(i == 0), has_mlm_head=(i == S - 1), **kw) for i in range(S)]
    sizes = [I.n_params(p) for p in parts]
    assert sum(sizes) == theta.size
    cuts = np.cumsum([0] + sizes)
    K = B.pipeline_warmup_depths(S, M, B.POLICY_A)
    pr = B.PipelineRunner([c_config(parts[i], K[i]) for i in range(S)], [theta[cuts[i]:cuts[i + 1]] for i in range(S)], M,
                          parts=0)
    try:
        T = full.tokens
        r0 = pr.runners[0]
        xs = [r0.to_dev(mb["ids"].reshape(T).astype(np.int32)) for mb in mbs]
        auxs = [r0.to_dev(mb["targets"].reshape(T).astype(np.int32)) for mb in mbs]
        ys = [torch.zeros(1, dtype=torch.float32, device="cuda") for _ in range(M)]
        for r in pr.runners:
            B.stage_zero_grads(r.h)
        torch.cuda.synchronize()
        pr.run(M, K, B.ORDER_EARLY_BACKWARD, xs, None, auxs, ys, None)
        torch.cuda.synchronize()
        got = dict(ys=[to_np(y) for y in ys], dxs=None,
                   grads=np.concatenate([r.grads.cpu().numpy() for r in pr.runners]))
        assert [B.stage_stats(r.h).peak_live_slots for r in pr.runners] == K
    finally:
        pr.close()
    st, ref = run_oracle(full, theta, mbs, M, 3)
    compare(full, st, ref, got, tol, M)


@pytest.mark.parametrize("S,M", [(1, 3), (2, 1), (3, 2)])
def test_degenerate_pipelines(S, M):
    # one stage (no boundary at all), one micro-batch, fewer micro-batches than stages: K_i is capped at M
    cfg = I.StageConfig(6, 64, 4, 128, 16, 2, M, 3, "f32", ln_eps=1e-5)
    theta, mbs = make_inputs(cfg, SEED, M)
    K = B.pipeline_warmup_depths(S, M, B.POLICY_A)
    assert K == PO.warmup_depths(S, M, "A") and max(K) <= M
    one = run_gpu(cfg, theta, mbs, M, max(K), B.ORDER_EARLY_BACKWARD)
    pipe = Pipe(cfg, S, K, theta, M, parts=0)
    try:
        got = pipe.run(M, K, B.ORDER_EARLY_BACKWARD, mbs)
    finally:
        pipe.close()
    assert got["peak"] == K
    assert np.array_equal(got["grads"], one["grads"])
    for m in range(M):
        assert np.array_equal(got["ys"][m], one["ys"][m]) and np.array_equal(got["dxs"][m], one["dxs"][m])
    check_timeline(got["timeline"], S, M, PO.stage_lists(S, M, K))


def test_recomputing_stages_in_a_pipeline_give_the_same_bits():
    cfg = I.StageConfig(4, 64, 4, 128, 16, 2, 5, 2, "f32", ln_eps=1e-5)
    S, M = 2, 5
    theta, mbs = make_inputs(cfg, SEED, M)
    K = B.pipeline_warmup_depths(S, M, B.POLICY_A)
    out = []
    for flags in (0, B.FLAG_RECOMPUTE, B.FLAG_RECOMPUTE | B.FLAG_ONE_STREAM):
        pipe = Pipe(cfg, S, K, theta, M, parts=0, flags=flags)
        try:
            out.append(pipe.run(M, K, B.ORDER_EARLY_BACKWARD, mbs))
        finally:
            pipe.close()
    for o in out[1:]:
        assert o["peak"] == K and np.array_equal(o["grads"], out[0]["grads"])
        for m in range(M):
            assert np.array_equal(o["dxs"][m], out[0]["dxs"][m]) and np.array_equal(o["ys"][m], out[0]["ys"][m])
