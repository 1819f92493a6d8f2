"""The Apply step (Adam) on the GPU against the oracle.  Gradients are written into the stage's
accumulators from the seeded generator, so both sides update from identical values; a second
test runs whole iterations (forward, backward, update) on both sides."""
import numpy as np
import pytest
import torch

from oracle import stage_oracle as O
from paper_2007_01045_amd import binding as B
from paper_2007_01045_amd import inputs as I
from tests.stage_util import c_config, make_inputs, rel_l2, run_oracle

pytestmark = pytest.mark.gpu
SEED = I.DEFAULT_SEED


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_adam_three_steps_from_given_gradients(dtype):
    cfg = I.StageConfig(1, 64, 4, 136, 16, 2, 2, 2, dtype)      # n_params is not a multiple of 4
    theta = I.make_params(cfg, SEED)
    n = theta.size
    r = B.StageRunner(c_config(cfg, 2), theta)
    try:
        r.init_adam()
        th = r.master.cpu().numpy().astype(np.float64)        # the weights as the stage holds them
        m, v = np.zeros(n), np.zeros(n)
        lr, b1, b2, eps, scale = 1e-2, 0.9, 0.98, 1e-6, 1.0 / 8
        for step in range(1, 4):
            # gradients of very different magnitudes, some exactly zero
            G = I.normal(SEED, f"adam.G{step}", n).astype(np.float32) * np.float32(10.0 ** (step - 2))
            G[::7] = 0.0
            r.grads.copy_(torch.from_numpy(G))
            r.apply_adam(lr, b1, b2, eps, scale, zero_grads=(step == 2))
            torch.cuda.synchronize()
            th, m, v = O.adam_apply(th, m, v, G.astype(np.float64), step, lr, b1, b2, eps, scale)
            got = r.master.cpu().numpy().astype(np.float64)
            assert np.abs(got - th).max() <= 2e-6 * lr + 1e-6 * np.abs(th).max()
            assert rel_l2(r.m.cpu().numpy(), m) < 1e-6 and rel_l2(r.v.cpu().numpy(), v) < 1e-6
            # the stage's weights are the fp32 master rounded to the stage's dtype, nothing else
            assert torch.equal(r.weights, r.master.to(r.weights.dtype))
            left = r.grads.cpu().numpy()
            assert (np.count_nonzero(left) == 0) if step == 2 else np.array_equal(left, G)
    finally:
        r.close()


def test_adam_error_paths():
    cfg = I.StageConfig(1, 64, 4, 128, 16, 2, 2, 2, "f32")
    theta = I.make_params(cfg, SEED)
    r = B.StageRunner(c_config(cfg, 2), theta)
    try:
        r.init_adam()
        args = (r.h, r.weights.data_ptr(), r.master.data_ptr(), r.m.data_ptr(), r.v.data_ptr())
        for bad, code in [((0, 1e-3), B.STAGE_E_CONFIG), ((1, 1e-3, 1.0), B.STAGE_E_CONFIG),
                          ((1, 1e-3, 0.9, 0.999, 0.0), B.STAGE_E_CONFIG)]:
            with pytest.raises(B.StageError) as e:
                B.stage_apply_adam(*args, *bad)
            assert e.value.code == code
        with pytest.raises(B.StageError) as e:      # not the buffer the stage reads its weights from
            B.stage_apply_adam(r.h, r.master.data_ptr(), r.master.data_ptr(), r.m.data_ptr(), r.v.data_ptr(), 1, 1e-3)
        assert e.value.code == B.STAGE_E_CONFIG
        x = r.to_dev(np.zeros((cfg.tokens, cfg.hidden), np.float32))
        y = r.empty_act()
        B.stage_fwd(r.h, 0, x.data_ptr(), y.data_ptr())
        with pytest.raises(B.StageError) as e:      # a micro-batch is still resident
            B.stage_apply_adam(*args, 1, 1e-3)
        assert e.value.code == B.STAGE_E_BAD_ORDER
        B.stage_bwd(r.h, 0, y.data_ptr(), x.data_ptr())
        torch.cuda.synchronize()
    finally:
        r.close()


@pytest.mark.parametrize("dtype,tol", [("f32", 1e-4), ("bf16", 3e-2)])
def test_two_training_iterations_follow_the_oracle(dtype, tol):
    # forward, backward, update, twice: the second iteration runs on the updated weights
    cfg = I.StageConfig(2, 128, 4, 256, 32, 2, 3, 2, dtype)
    theta, mbs = make_inputs(cfg, SEED, 3)
    lr, scale = 1e-3, 1.0 / (3 * cfg.micro_batch)
    r = B.StageRunner(c_config(cfg, 2), theta)
    try:
        r.init_adam()
        T, H = cfg.tokens, cfg.hidden
        xs = [r.to_dev(mb["x"].reshape(T, H)) for mb in mbs]
        dys = [r.to_dev(mb["dy"].reshape(T, H)) for mb in mbs]
        th0 = r.master.cpu().numpy().astype(np.float64)
        th, m, v = th0.copy(), np.zeros_like(th0), np.zeros_like(th0)
        # the key-bias gradient is analytically zero: both sides hold rounding noise there, and Adam
        # turns the sign of noise into a step of lr -- those entries are not compared
        keep = np.ones(th0.size, bool)
        for name, (off, shape) in I.param_offsets(cfg).items():
            if name.endswith(".bk"):
                keep[off:off + int(np.prod(shape))] = False
        eps = None
        for it in range(2):
            # the oracle's iteration from the oracle's own weights
            _, ref = run_oracle(cfg, th.astype(np.float32) if dtype == "f32" else I.round_to_bf16(th.astype(np.float32)),
                                mbs, 3, 2)
            if eps is None:
                # eps of the size of a typical gradient: with the usual 1e-8 the first Adam step is
                # lr * sign(g), and the sign of a small gradient is not something bf16 arithmetic fixes
                eps = float(np.sqrt(np.mean((ref["grads"] * scale) ** 2)))
            r.run(3, 2, B.ORDER_EARLY_BACKWARD, xs, dys)
            r.apply_adam(lr, eps=eps, grad_scale=scale, zero_grads=True)
            torch.cuda.synchronize()
            prev = th
            th, m, v = O.adam_apply(th, m, v, ref["grads"], it + 1, lr, eps=eps, grad_scale=scale)
            got = r.master.cpu().numpy().astype(np.float64)
            # compare the motion of the weights, not the weights (the update is 1e-3 of them)
            assert rel_l2((got - th0)[keep], (th - th0)[keep]) < tol, (it, rel_l2((got - th0)[keep], (th - th0)[keep]))
            assert rel_l2(r.m.cpu().numpy()[keep], m[keep]) < tol and rel_l2(r.v.cpu().numpy()[keep], v[keep]) < 2 * tol
            assert np.abs(th - prev).max() > 0
    finally:
        r.close()
