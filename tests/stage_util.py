"""Helpers shared by the GPU parity tests: build the oracle and the HIP stage
from the same seeded inputs and compare tensor by tensor."""
import numpy as np

from oracle import stage_oracle as O
from paper_2007_01045_amd import binding as B
from paper_2007_01045_amd import inputs as I


def rel_l2(a, ref):
    a, ref = np.asarray(a, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm(a - ref) / max(np.linalg.norm(ref), 1e-300))


def to_np(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def c_config(cfg: I.StageConfig, max_slots, loss_scale=1.0, flags=0):
    return B.config_for(cfg, max_slots, loss_scale, flags)


def oracle_stage(cfg, theta, loss_scale=1.0):
    return O.Stage(I.param_layout(cfg), theta.astype(np.float64), cfg.n_layers, cfg.n_heads, cfg.ln_eps,
                   cfg.has_embedding, cfg.has_mlm_head, loss_scale)


def make_inputs(cfg, seed, M=None):
    M = cfg.M if M is None else M
    theta = I.make_params(cfg, seed)
    mbs = [I.make_microbatch(cfg, seed, m) for m in range(M)]
    return theta, mbs


def run_gpu(cfg, theta, mbs, M, K, order, max_slots=None, loss_scale=1.0, explicit_ops=None, flags=0):
    """Run one iteration on the GPU; returns dict(ys, dxs, grads, stats) as numpy float64."""
    import torch
    slots = max_slots if max_slots is not None else (M if order == B.ORDER_GPIPE else min(K, M))
    r = B.StageRunner(c_config(cfg, slots, loss_scale, flags), theta)
    try:
        T, H = cfg.tokens, cfg.hidden
        if cfg.has_embedding:
            xs = [r.to_dev(mb["ids"].reshape(T).astype(np.int32)) for mb in mbs]
        else:
            xs = [r.to_dev(mb["x"].reshape(T, H)) for mb in mbs]
        dys = None if cfg.has_mlm_head else [r.to_dev(mb["dy"].reshape(T, H)) for mb in mbs]
        auxs = [r.to_dev(mb["targets"].reshape(T).astype(np.int32)) for mb in mbs] if cfg.has_mlm_head else None
        ys, dxs = r.run(M, K, order, xs, dys, auxs, explicit_ops)
        B.stage_sync(r.h)
        torch.cuda.synchronize()
        st = B.stage_stats(r.h)
        out = dict(ys=[to_np(y) for y in ys], dxs=None if dxs is None else [to_np(d) for d in dxs],
                   grads=r.grads.detach().cpu().numpy().copy(),
                   stats=dict(peak_live=st.peak_live_slots, peak_bytes=st.peak_activation_bytes,
                              slot_bytes=st.slot_bytes, launches=st.kernel_launches))
        return out
    finally:
        r.close()


def run_oracle(cfg, theta, mbs, M, K, order=O.EARLY_BACKWARD, loss_scale=1.0):
    st = oracle_stage(cfg, theta, loss_scale)
    xs = [mb["ids"] if cfg.has_embedding else mb["x"].astype(np.float64) for mb in mbs]
    dys = None if cfg.has_mlm_head else [mb["dy"].astype(np.float64) for mb in mbs]
    tg = [mb["targets"] for mb in mbs] if cfg.has_mlm_head else None
    return st, O.run_schedule(st, M, K, order, xs, dys, tg)


def compare(cfg, st, ref, got, tol, M):
    """Per-tensor relative L2 of every y_m, dx_m and every parameter-gradient tensor,
    and of the whole flat gradient.  Returns the worst (name, value)."""
    T, H = cfg.tokens, cfg.hidden
    worst = ("", 0.0)

    def upd(name, v):
        nonlocal worst
        assert v <= tol, (name, v, tol)
        if v > worst[1]:
            worst = (name, v)

    for m in range(M):
        if cfg.has_mlm_head:
            upd(f"loss{m}", abs(float(got["ys"][m].reshape(-1)[0]) - ref["ys"][m]) / abs(ref["ys"][m]))
        else:
            upd(f"y{m}", rel_l2(got["ys"][m], ref["ys"][m].reshape(T, H)))
        if not cfg.has_embedding:
            upd(f"dx{m}", rel_l2(got["dxs"][m], ref["dxs"][m].reshape(T, H)))
    G, Gr = got["grads"].astype(np.float64), ref["grads"]
    upd("grads(all)", rel_l2(G, Gr))
    gscale = np.sqrt(np.mean(Gr ** 2))
    for name, (off, shape) in st.offsets.items():
        n = int(np.prod(shape))
        a, b = G[off:off + n], Gr[off:off + n]
        if name.endswith(".bk"):
            # analytically zero (softmax ignores a common shift of the keys): the
            # oracle holds rounding noise, so compare on the scale of the query bias
            qoff, _ = st.offsets[name[:-2] + "bq"]
            scale = np.linalg.norm(Gr[qoff:qoff + n])
            upd(name, float(np.linalg.norm(a - b) / scale))
        else:
            upd(name, rel_l2(a, b))
    return worst
