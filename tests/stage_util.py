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


# Element-wise bound beside the norm: |a - ref| <= ELEM_C * tol * rms(ref) for every element of every compared
# tensor.  Rounding errors of a tensor that passes the relative-L2 tolerance are spread over its elements:
# with n elements of error scale tol * rms(ref) the largest of them sits near sqrt(2 ln n) ~ 5.5 scales for
# n = 2e6..1e8, and gradient elements with heavier tails reach a few times that; 25 scales leaves room for
# that and still rejects any element that is plainly wrong (an element of typical size that is missing,
# doubled or misplaced is off by rms(ref) = 50 scales at the bf16 tolerance, 1e4 scales at the fp32 one).
ELEM_C = 25.0
# Per-row bound for the two vocabulary-sized gradient tables (token embedding, output projection): every row
# with a contribution must itself meet ROW_C * tol in relative L2 (a row has H elements, so its own relative
# error scatters around the tensor's by a factor 1 +- a few / sqrt(H); a wrong row is off by about 1), and a
# row of the token-embedding gradient that no token id names must be exactly zero.
ROW_C = 3.0


def elem_excess(a, ref):
    """max |a - ref| / rms(ref)"""
    a, ref = np.asarray(a, dtype=np.float64).reshape(-1), np.asarray(ref, dtype=np.float64).reshape(-1)
    rms = float(np.sqrt(np.mean(ref * ref)))
    return float(np.max(np.abs(a - ref)) / max(rms, 1e-300))


def row_check(name, a, ref, tol, touched=None):
    """Per-row relative L2 of a [V, H] gradient table; rows outside `touched` (if given) must be exactly 0.
    Returns the worst row's relative L2."""
    d = np.linalg.norm(a - ref, axis=1)
    n = np.linalg.norm(ref, axis=1)
    if touched is not None:
        mask = np.zeros(a.shape[0], dtype=bool)
        mask[touched] = True
        assert not a[~mask].any(), (name, "a row that no token id names is not exactly zero")
        assert not ref[~mask].any()
    else:
        mask = n > 0
    r = d[mask] / n[mask]
    w = float(r.max())
    assert w <= ROW_C * tol, (name, "row", int(np.flatnonzero(mask)[int(r.argmax())]), w, ROW_C * tol)
    # element-wise, on the scale of the element's own row (the rows of these tables differ in size by orders of
    # magnitude: a row that a target or a token id names against one that only the softmax tail reaches)
    e = np.max(np.abs(a - ref), axis=1)[mask] / (n[mask] / np.sqrt(a.shape[1]))
    assert float(e.max()) <= ELEM_C * tol, (name, "row element", int(np.flatnonzero(mask)[int(e.argmax())]), float(e.max()))
    return w


def compare(cfg, st, ref, got, tol, M, mbs=None, report=None):
    """Per-tensor relative L2 of every y_m, dx_m and every parameter-gradient tensor,
    and of the whole flat gradient, each with the element-wise bound; per-row checks of the
    vocabulary-sized tables (the token ids come from `mbs`).  Returns the worst (name, value);
    `report` (a dict) receives the worst element-wise and per-row figures."""
    T, H = cfg.tokens, cfg.hidden
    worst = ("", 0.0)
    worst_elem = ("", 0.0)

    def upd(name, v, a=None, b=None):
        nonlocal worst, worst_elem
        assert v <= tol, (name, v, tol)
        if v > worst[1]:
            worst = (name, v)
        if a is not None:
            e = elem_excess(a, b)
            assert e <= ELEM_C * tol, (name, "element-wise", e, ELEM_C * tol)
            if e > worst_elem[1]:
                worst_elem = (name, e)

    for m in range(M):
        if cfg.has_mlm_head:
            upd(f"loss{m}", abs(float(got["ys"][m].reshape(-1)[0]) - ref["ys"][m]) / abs(ref["ys"][m]))
        else:
            upd(f"y{m}", rel_l2(got["ys"][m], ref["ys"][m].reshape(T, H)), got["ys"][m], ref["ys"][m])
        if not cfg.has_embedding:
            upd(f"dx{m}", rel_l2(got["dxs"][m], ref["dxs"][m].reshape(T, H)), got["dxs"][m], ref["dxs"][m])
    G, Gr = got["grads"], ref["grads"]
    upd("grads(all)", rel_l2(G, Gr))
    rows = {}
    for name, (off, shape) in st.offsets.items():
        n = int(np.prod(shape))
        a, b = G[off:off + n].astype(np.float64), Gr[off:off + n]
        if name.endswith(".bk"):
            # analytically zero (softmax ignores a common shift of the keys): the
            # oracle holds rounding noise, so compare on the scale of the query bias
            qoff, _ = st.offsets[name[:-2] + "bq"]
            scale = np.linalg.norm(Gr[qoff:qoff + n])
            upd(name, float(np.linalg.norm(a - b) / scale))
        elif name in ("emb.E_w", "head.E_out"):
            upd(name, rel_l2(a, b))          # element-wise: per row, below
        else:
            upd(name, rel_l2(a, b), a, b)
        if name == "emb.E_w":
            touched = None if mbs is None else np.unique(np.concatenate([mb["ids"].reshape(-1) for mb in mbs[:M]]))
            rows[name] = row_check(name, a.reshape(shape), b.reshape(shape), tol, touched)
        elif name == "head.E_out":
            rows[name] = row_check(name, a.reshape(shape), b.reshape(shape), tol)
    if report is not None:
        report.update(worst=worst, worst_elem=worst_elem, rows=rows)
    return worst
