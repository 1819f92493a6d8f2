"""Pins for the oracle's layer math: an independent library implementation
(torch's TransformerEncoderLayer, float64, autograd), central finite
differences, and closed forms for the elementary pieces."""
import math

import numpy as np
import pytest
import torch

from oracle import stage_oracle as O
from paper_2007_01045_amd import inputs as I


def rel(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


def make_stage(cfg, seed=3, loss_scale=1.0):
    theta = I.make_params(cfg, seed).astype(np.float64)
    return O.Stage(I.param_layout(cfg), theta, cfg.n_layers, cfg.n_heads, cfg.ln_eps,
                   cfg.has_embedding, cfg.has_mlm_head, loss_scale)


SMALL = I.StageConfig(2, 32, 4, 64, 8, 2, 3, 2, "f32", ln_eps=1e-5)


def _torch_layer(st, l, H, A, F, eps):
    p = st.group(f"l{l}.")
    m = torch.nn.TransformerEncoderLayer(H, A, F, dropout=0.0, activation="gelu",
                                         layer_norm_eps=eps, batch_first=True,
                                         norm_first=False).double()
    t = lambda a: torch.tensor(np.ascontiguousarray(a))
    with torch.no_grad():
        m.self_attn.in_proj_weight.copy_(t(np.concatenate([p["Wq"].T, p["Wk"].T, p["Wv"].T])))
        m.self_attn.in_proj_bias.copy_(t(np.concatenate([p["bq"], p["bk"], p["bv"]])))
        m.self_attn.out_proj.weight.copy_(t(p["Wo"].T)); m.self_attn.out_proj.bias.copy_(t(p["bo"]))
        m.linear1.weight.copy_(t(p["W1"].T)); m.linear1.bias.copy_(t(p["b1"]))
        m.linear2.weight.copy_(t(p["W2"].T)); m.linear2.bias.copy_(t(p["b2"]))
        m.norm1.weight.copy_(t(p["ln1_g"])); m.norm1.bias.copy_(t(p["ln1_b"]))
        m.norm2.weight.copy_(t(p["ln2_g"])); m.norm2.bias.copy_(t(p["ln2_b"]))
    m.train()      # keeps torch on its plain (non-fused) path; dropout is 0
    return m


def test_stage_matches_torch_encoder_forward_and_backward():
    cfg = SMALL
    st = make_stage(cfg)
    mb = I.make_microbatch(cfg, 5, 0)
    x, dy = mb["x"].astype(np.float64), mb["dy"].astype(np.float64)
    y, cache = st.forward(x)
    dx, G = st.backward(dy, cache)

    layers = [_torch_layer(st, l, cfg.hidden, cfg.n_heads, cfg.ffn, cfg.ln_eps)
              for l in range(cfg.n_layers)]
    xt = torch.tensor(x, requires_grad=True)
    h = xt
    for m in layers:
        h = m(h)
    (h * torch.tensor(dy)).sum().backward()
    assert rel(y, h.detach().numpy()) < 1e-13
    assert rel(dx, xt.grad.numpy()) < 1e-12
    H = cfg.hidden
    for l, m in enumerate(layers):
        gw = m.self_attn.in_proj_weight.grad.numpy()
        gb = m.self_attn.in_proj_bias.grad.numpy()
        want = {"Wq": gw[:H].T, "Wk": gw[H:2 * H].T, "Wv": gw[2 * H:].T,
                "bq": gb[:H], "bk": gb[H:2 * H], "bv": gb[2 * H:],
                "Wo": m.self_attn.out_proj.weight.grad.numpy().T,
                "bo": m.self_attn.out_proj.bias.grad.numpy(),
                "W1": m.linear1.weight.grad.numpy().T, "b1": m.linear1.bias.grad.numpy(),
                "W2": m.linear2.weight.grad.numpy().T, "b2": m.linear2.bias.grad.numpy(),
                "ln1_g": m.norm1.weight.grad.numpy(), "ln1_b": m.norm1.bias.grad.numpy(),
                "ln2_g": m.norm2.weight.grad.numpy(), "ln2_b": m.norm2.bias.grad.numpy()}
        for name, w in want.items():
            off, shape = st.offsets[f"l{l}.{name}"]
            got = G[off:off + w.size].reshape(shape)
            if name == "bk":
                # a shift of every key moves all logits of a row alike, which softmax
                # ignores: this gradient is zero up to rounding
                assert np.abs(got).max() < 1e-15 and np.abs(w).max() < 1e-15
                continue
            assert rel(got, w) < 1e-11, (l, name)


def _objective(cfg, theta, mb, loss_scale=1.0):
    st = O.Stage(I.param_layout(cfg), theta, cfg.n_layers, cfg.n_heads, cfg.ln_eps,
                 cfg.has_embedding, cfg.has_mlm_head, loss_scale)
    x = mb["ids"] if cfg.has_embedding else mb["x"].astype(np.float64)
    out, _ = st.forward(x, mb.get("targets"))
    return out if cfg.has_mlm_head else float((out * mb["dy"]).sum())


@pytest.mark.parametrize("kind", ["plain", "embedding", "head"])
def test_finite_differences_every_parameter_tensor(kind):
    base = dict(n_layers=2, hidden=16, n_heads=2, ffn=32, seq=6, micro_batch=2, M=2, K=1,
                dtype="f32", vocab=23, max_pos=8, ln_eps=1e-5)
    cfg = I.StageConfig(**base, has_embedding=(kind == "embedding"), has_mlm_head=(kind == "head"))
    seed, ls = 11, 0.37
    theta = I.make_params(cfg, seed).astype(np.float64)
    # larger weights than the workload's N(0,0.02) so that no path is nearly linear
    theta = theta + 0.3 * I.normal(seed, "fd.bump", theta.size)
    mb = I.make_microbatch(cfg, seed, 0)
    if kind == "head":      # ceil(0.15*12) = 2 rows; fine
        assert (mb["targets"] >= 0).sum() == 2
    st = O.Stage(I.param_layout(cfg), theta, cfg.n_layers, cfg.n_heads, cfg.ln_eps,
                 cfg.has_embedding, cfg.has_mlm_head, ls)
    x = mb["ids"] if cfg.has_embedding else mb["x"].astype(np.float64)
    _, cache = st.forward(x, mb.get("targets"))
    dx, G = st.backward(None if kind == "head" else mb["dy"].astype(np.float64), cache)
    h = 1e-5
    f = lambda th: _objective(cfg, th, mb, ls)
    rng = np.random.default_rng(0)
    for name, (off, shape) in st.offsets.items():
        n = int(np.prod(shape))
        # a random direction inside this tensor
        v = np.zeros_like(theta); v[off:off + n] = rng.standard_normal(n)
        num = (f(theta + h * v) - f(theta - h * v)) / (2 * h)
        ana = float(G @ v)
        assert abs(num - ana) <= 2e-6 * max(abs(ana), abs(num), 1e-3), (name, num, ana)
        # and a few single coordinates
        for j in rng.choice(n, size=min(3, n), replace=False):
            e = np.zeros_like(theta); e[off + j] = 1.0
            num = (f(theta + h * e) - f(theta - h * e)) / (2 * h)
            assert abs(num - G[off + j]) <= 2e-6 * max(abs(num), 1e-3) + 1e-9, (name, j)
    if kind == "plain":      # input gradient
        for _ in range(3):
            v = rng.standard_normal(mb["x"].shape)
            mp, mm = dict(mb), dict(mb)
            mp["x"] = mb["x"].astype(np.float64) + h * v
            mm["x"] = mb["x"].astype(np.float64) - h * v
            num = (_objective(cfg, theta, mp) - _objective(cfg, theta, mm)) / (2 * h)
            assert abs(num - float((dx * v).sum())) <= 2e-6 * max(abs(num), 1e-3)


def test_layernorm_closed_forms():
    rng = np.random.default_rng(1)
    z = rng.standard_normal((5, 7, 48)) * 3 + 2
    H, eps = 48, 1e-12
    y, cache = O.layernorm_fwd(z, np.ones(H), np.zeros(H), eps)
    assert np.abs(y.mean(-1)).max() < 1e-14
    assert np.abs((y ** 2).mean(-1) - 1).max() < 1e-10
    # affine map of the input leaves the output unchanged (shift) / flips sign
    y2, _ = O.layernorm_fwd(-2.5 * z + 9, np.ones(H), np.zeros(H), eps)
    assert np.abs(y2 + y).max() < 1e-12
    g = rng.standard_normal(H); dy = rng.standard_normal(z.shape)
    dz, dg, db = O.layernorm_bwd(dy, cache, g)
    assert np.abs(dz.sum(-1)).max() < 1e-12                 # orthogonal to constants
    assert np.abs((dz * cache[0]).sum(-1)).max() < 1e-10    # and to x-hat (up to eps/var)
    assert np.allclose(db, dy.reshape(-1, H).sum(0))
    # eps enters inside the square root: a constant row maps to exactly beta
    y3, _ = O.layernorm_fwd(np.full((1, H), 4.0), g, g + 1, 1e-5)
    assert np.allclose(y3, g + 1)
    # known value: row (0, 2): mean 1, biased var 1
    y4, _ = O.layernorm_fwd(np.array([[0.0, 2.0]]), np.array([2.0, 3.0]), np.array([0.5, -0.5]), 0.0)
    assert np.allclose(y4, [[-1.5, 2.5]])


def test_gelu_closed_forms():
    assert O.gelu(np.array([0.0]))[0] == 0.0
    assert abs(O.gelu_grad(np.array([0.0]))[0] - 0.5) < 1e-16
    u = np.linspace(-4, 4, 33)
    assert np.allclose(O.gelu(u) - O.gelu(-u), u)                  # u Phi(u) - (-u) Phi(-u) = u
    assert np.allclose(O.gelu_grad(u) + O.gelu_grad(-u), 1.0)
    # against the normal CDF written with erfc, and a printed value
    want = np.array([v * 0.5 * math.erfc(-v / math.sqrt(2)) for v in u])
    assert np.allclose(O.gelu(u), want, atol=1e-15)
    assert abs(O.gelu(np.array([1.0]))[0] - 0.8413447460685429) < 1e-15
    h = 1e-6
    assert np.allclose((O.gelu(u + h) - O.gelu(u - h)) / (2 * h), O.gelu_grad(u), atol=1e-9)


def test_attention_closed_forms():
    cfg = I.StageConfig(1, 16, 2, 32, 5, 1, 1, 1, "f32")
    st = make_stage(cfg)
    p = dict(st.group("l0."))
    rng = np.random.default_rng(2)
    # all keys equal => P is uniform and ctx is the column mean of V
    p["Wk"] = np.zeros_like(p["Wk"])
    x = rng.standard_normal((1, 5, 16))
    _, c = O.layer_fwd(x, p, 2, 1e-12)
    assert np.allclose(c["P"], 1.0 / 5)
    v = x @ p["Wv"] + p["bv"]
    assert np.allclose(c["ctx"], np.broadcast_to(v.mean(1, keepdims=True), v.shape))
    # rows of P sum to one in general
    _, c = O.layer_fwd(x, st.group("l0."), 2, 1e-12)
    assert np.allclose(c["P"].sum(-1), 1.0)
    # scale: logits are q.k/sqrt(d): doubling q's weights and bias doubles log-odds
    S = np.log(c["P"])
    p2 = dict(st.group("l0.")); p2["Wq"] = 2 * p2["Wq"]; p2["bq"] = 2 * p2["bq"]
    _, c2 = O.layer_fwd(x, p2, 2, 1e-12)
    S2 = np.log(c2["P"])
    assert np.allclose((S2 - S2[..., :1]), 2 * (S - S[..., :1]))
    d = 8
    q, k = c["q"], c["k"]
    logit = (q[0, 1, 2] * k[0, 1, 4]).sum() / math.sqrt(d) - (q[0, 1, 2] * k[0, 1, 0]).sum() / math.sqrt(d)
    assert abs((S[0, 1, 2, 4] - S[0, 1, 2, 0]) - logit) < 1e-12


def test_brute_force_tiny_layer_forward():
    """Pure-Python loops on a tiny layer, written from the definitions."""
    cfg = I.StageConfig(1, 4, 2, 6, 3, 1, 1, 1, "f32", ln_eps=1e-3)
    st = make_stage(cfg, seed=9)
    p = {k: v.tolist() for k, v in st.group("l0.").items()}
    x = (I.normal(1, "bf.x", 12).reshape(3, 4)).tolist()
    H, A, F, s, d = 4, 2, 6, 3, 2

    def lin(rows, W, b):
        return [[sum(r[i] * W[i][j] for i in range(len(r))) + b[j] for j in range(len(b))] for r in rows]

    def ln(rows, g, b):
        out = []
        for r in rows:
            mu = sum(r) / len(r)
            var = sum((t - mu) ** 2 for t in r) / len(r)
            out.append([(t - mu) / math.sqrt(var + 1e-3) * g[j] + b[j] for j, t in enumerate(r)])
        return out

    q, k, v = lin(x, p["Wq"], p["bq"]), lin(x, p["Wk"], p["bk"]), lin(x, p["Wv"], p["bv"])
    ctx = [[0.0] * H for _ in range(s)]
    for a in range(A):
        for i in range(s):
            sc = [sum(q[i][a * d + t] * k[j][a * d + t] for t in range(d)) / math.sqrt(d) for j in range(s)]
            mx = max(sc); e = [math.exp(t - mx) for t in sc]; Z = sum(e)
            for t in range(d):
                ctx[i][a * d + t] = sum(e[j] / Z * v[j][a * d + t] for j in range(s))
    att = lin(ctx, p["Wo"], p["bo"])
    y1 = ln([[x[i][j] + att[i][j] for j in range(H)] for i in range(s)], p["ln1_g"], p["ln1_b"])
    u = lin(y1, p["W1"], p["b1"])
    g = [[t * 0.5 * (1 + math.erf(t / math.sqrt(2))) for t in r] for r in u]
    f = lin(g, p["W2"], p["b2"])
    y = ln([[y1[i][j] + f[i][j] for j in range(H)] for i in range(s)], p["ln2_g"], p["ln2_b"])
    got, _ = O.layer_fwd(np.array(x)[None], st.group("l0."), A, 1e-3)
    assert np.allclose(got[0], np.array(y), rtol=1e-12, atol=1e-14)
