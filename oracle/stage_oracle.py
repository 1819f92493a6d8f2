"""CPU oracle for one pipeline stage of synchronous pipelined training.

THIS IS TEST INFRASTRUCTURE, not a product path: only the tests, the smoke
check and the benchmark's cpu_baseline leg may call it.  It shares no code with
the HIP library and imports nothing from it.  Everything is plain numpy in
float64; matmul, exp, erf, sqrt are used as library primitives, there is no
blocking, fusion or reordering beyond what the definitions state.

What the stage computes (synchronous training, weights theta frozen for the
whole iteration; early-backward scheduling section III-B and micro-batch unit
scheduling section V-C of the DAPPLE paper; synchronous weights update section
V-B-3 for the accumulation):

    y_m  = stage(x_m; theta)
    dx_m = d<dy_m, stage(x_m; theta)>/dx_m
    G    = sum_{m=0}^{M-1} d<dy_m, stage(x_m; theta)>/dtheta     (summed, not averaged:
                                                                 averaging belongs to Apply)

The schedule only reorders the forward (F_m) and backward (B_m) tasks; the paper
states (section VI-A, section VI-D) that all its orders give equivalent
gradients, so the definition above is the result for every order.  The oracle
evaluates it by walking the task list of the chosen order with an activation
store that refuses to hold more than K micro-batches.

The paper does not define the math inside a layer (it names BERT-48 and
BERT-Large as workloads).  The layer is the standard post-LayerNorm transformer
encoder layer; the readings taken where nothing is stated:
  * GELU is the exact one, u * Phi(u), with Phi the normal CDF (erf form).
  * no attention mask, no dropout.
  * LayerNorm over the H features of one token, biased variance, eps inside the
    square root; eps is a config field.
  * softmax subtracts the row maximum.
  * embedding stage: x = LN(E_w[id] + E_p[pos]), pos = 0..s-1, no segment table.
  * MLM head: masked rows r -> t = LN(GELU(r Wt + bt)) -> z = t E_out^T + b_out ->
    loss = loss_scale * sum_rows (logsumexp(z) - z[target]).

Pins (tests/test_oracle_*.py): central finite differences in float64; an
independent library implementation of the same layer (torch's
TransformerEncoderLayer with autograd, float64); the paper's worked two-stage
schedule example and its control-edge rules; closed forms for LayerNorm,
softmax, GELU and cross-entropy; the invariants sum-of-micro-batch-gradients =
full-batch gradient and GPipe order = early-backward order.
bf16 end-to-end values are "parity unpinned" by the paper (it trains in fp32
only); they are pinned by this float64 oracle within the bf16 tolerance.
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erf

GPIPE = 0
EARLY_BACKWARD = 1


# --------------------------------------------------------------------------
# schedule (sections III-B and V-C)
# --------------------------------------------------------------------------

def schedule_ops(M: int, K: int, order: int):
    """Task list of one stage for one iteration: [('F'|'B', m), ...].

    GPipe order (section III-A): every forward, then every backward; the
    activations of all M micro-batches are alive at the turn.
    Early-backward order (section III-B): inject K' = min(K, M) micro-batches,
    then alternate strictly one backward, one forward -- B_j releases its
    activations and F_{j+K'} reuses them (control edge B_m -> F_{m+K'} of section
    V-C) -- then drain the remaining backwards.  Backwards run in ascending
    micro-batch order in both orders.
    """
    if M < 1 or K < 1:
        raise ValueError("M and K must be positive")
    if order == GPIPE:
        return [("F", m) for m in range(M)] + [("B", m) for m in range(M)]
    if order != EARLY_BACKWARD:
        raise ValueError("unknown order")
    Kp = min(K, M)
    ops = [("F", m) for m in range(Kp)]
    for j in range(M - Kp):
        ops.append(("B", j))
        ops.append(("F", j + Kp))
    ops += [("B", m) for m in range(M - Kp, M)]
    return ops


def warmup_depth(policy: str, S: int, i: int, D: int) -> int:
    """Number of micro-batches stage i of S injects before its first backward
    (section V-C): policy A  K_i = min(S - i, D); policy B  K_i = min(2(S-i)-1, D);
    D = how many micro-batches fit in device memory."""
    if policy == "A":
        return min(S - i, D)
    if policy == "B":
        return min(2 * (S - i) - 1, D)
    raise ValueError("policy must be 'A' or 'B'")


def live_trace(ops):
    """Number of micro-batches whose activations are alive after each task."""
    live, out = set(), []
    for kind, m in ops:
        if kind == "F":
            live.add(m)
        else:
            live.remove(m)
        out.append(len(live))
    return out


# --------------------------------------------------------------------------
# elementary pieces
# --------------------------------------------------------------------------

def gelu(u):
    return u * 0.5 * (1.0 + erf(u / math.sqrt(2.0)))


def gelu_grad(u):
    # d/du [u Phi(u)] = Phi(u) + u phi(u)
    Phi = 0.5 * (1.0 + erf(u / math.sqrt(2.0)))
    phi = np.exp(-0.5 * u * u) / math.sqrt(2.0 * math.pi)
    return Phi + u * phi


def layernorm_fwd(z, g, beta, eps):
    mean = z.mean(axis=-1, keepdims=True)
    var = ((z - mean) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (z - mean) * rstd
    return xhat * g + beta, (xhat, rstd)


def layernorm_bwd(dy, cache, g):
    xhat, rstd = cache
    lead = tuple(range(dy.ndim - 1))
    dg = (dy * xhat).sum(axis=lead)
    dbeta = dy.sum(axis=lead)
    dxhat = dy * g
    dz = rstd * (dxhat - dxhat.mean(axis=-1, keepdims=True)
                 - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    return dz, dg, dbeta


def softmax_rows(S):
    e = np.exp(S - S.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def _split_heads(t, A):
    b, s, H = t.shape
    return t.reshape(b, s, A, H // A).transpose(0, 2, 1, 3)      # [b,A,s,d]


def _merge_heads(t):
    b, A, s, d = t.shape
    return t.transpose(0, 2, 1, 3).reshape(b, s, A * d)


def attention_fwd(q, k, v):
    """q, k, v [b,A,s,d] -> ctx [b,A,s,d] and P = softmax_rows(q k^T / sqrt(d)) [b,A,s,s]."""
    d = q.shape[-1]
    P = softmax_rows(q @ k.transpose(0, 1, 3, 2) / math.sqrt(d))
    return P @ v, P


def attention_bwd(dctx, q, k, v, P):
    """Exact derivative of attention_fwd: dq, dk, dv [b,A,s,d]."""
    d = q.shape[-1]
    dv = P.transpose(0, 1, 3, 2) @ dctx
    dP = dctx @ v.transpose(0, 1, 3, 2)
    dS = P * (dP - (dP * P).sum(axis=-1, keepdims=True))
    dq = dS @ k / math.sqrt(d)
    dk = dS.transpose(0, 1, 3, 2) @ q / math.sqrt(d)
    return dq, dk, dv


# --------------------------------------------------------------------------
# one encoder layer
# --------------------------------------------------------------------------

def layer_fwd(x, p, A, eps):
    """x [b,s,H] -> y [b,s,H]; p maps the layer's parameter names to arrays."""
    q = _split_heads(x @ p["Wq"] + p["bq"], A)
    k = _split_heads(x @ p["Wk"] + p["bk"], A)
    v = _split_heads(x @ p["Wv"] + p["bv"], A)
    ctx_h, P = attention_fwd(q, k, v)
    ctx = _merge_heads(ctx_h)
    a = ctx @ p["Wo"] + p["bo"]
    y1, ln1 = layernorm_fwd(x + a, p["ln1_g"], p["ln1_b"], eps)
    u = y1 @ p["W1"] + p["b1"]
    gl = gelu(u)
    f = gl @ p["W2"] + p["b2"]
    y, ln2 = layernorm_fwd(y1 + f, p["ln2_g"], p["ln2_b"], eps)
    cache = dict(x=x, q=q, k=k, v=v, P=P, ctx=ctx, ln1=ln1, y1=y1, u=u, gl=gl, ln2=ln2)
    return y, cache


def layer_bwd(dy, c, p, A):
    """Exact derivative of layer_fwd: returns dx and this layer's parameter gradients."""
    g = {}
    flat = lambda t: t.reshape(-1, t.shape[-1])
    dz2, g["ln2_g"], g["ln2_b"] = layernorm_bwd(dy, c["ln2"], p["ln2_g"])
    # f = gl W2 + b2
    g["W2"] = flat(c["gl"]).T @ flat(dz2)
    g["b2"] = flat(dz2).sum(axis=0)
    du = (dz2 @ p["W2"].T) * gelu_grad(c["u"])
    g["W1"] = flat(c["y1"]).T @ flat(du)
    g["b1"] = flat(du).sum(axis=0)
    dy1 = dz2 + du @ p["W1"].T
    dz1, g["ln1_g"], g["ln1_b"] = layernorm_bwd(dy1, c["ln1"], p["ln1_g"])
    g["Wo"] = flat(c["ctx"]).T @ flat(dz1)
    g["bo"] = flat(dz1).sum(axis=0)
    dctx = _split_heads(dz1 @ p["Wo"].T, A)                      # [b,A,s,d]
    dq, dk, dv = attention_bwd(dctx, c["q"], c["k"], c["v"], c["P"])
    dq, dk, dv = _merge_heads(dq), _merge_heads(dk), _merge_heads(dv)
    x = c["x"]
    dx = dz1.copy()
    for n, dt in (("q", dq), ("k", dk), ("v", dv)):
        g["W" + n] = flat(x).T @ flat(dt)
        g["b" + n] = flat(dt).sum(axis=0)
        dx = dx + dt @ p["W" + n].T
    return dx, g


# --------------------------------------------------------------------------
# embedding block (first stage) and MLM head (last stage)
# --------------------------------------------------------------------------

def embedding_fwd(ids, p, eps):
    """ids [b,s] -> x [b,s,H] = LN(E_w[id] + E_p[pos]), pos = 0..s-1."""
    s = ids.shape[1]
    e = p["E_w"][ids] + p["E_p"][np.arange(s)][None, :, :]
    x, ln = layernorm_fwd(e, p["ln_g"], p["ln_b"], eps)
    return x, dict(ids=ids, ln=ln)


def embedding_bwd(dx, c, p):
    de, dg, dbeta = layernorm_bwd(dx, c["ln"], p["ln_g"])
    g = {"ln_g": dg, "ln_b": dbeta}
    dEw = np.zeros_like(p["E_w"])
    np.add.at(dEw, c["ids"].reshape(-1), de.reshape(-1, de.shape[-1]))   # repeated ids add
    dEp = np.zeros_like(p["E_p"])
    dEp[: de.shape[1]] = de.sum(axis=0)
    g["E_w"], g["E_p"] = dEw, dEp
    return g


def mlm_head_fwd(y, targets, p, eps, loss_scale):
    """y [b,s,H]; targets [b,s] with -1 on positions that are not predicted.
    Returns loss = loss_scale * sum over predicted positions of
    (logsumexp(z) - z[target])."""
    H = y.shape[-1]
    rows = np.flatnonzero(targets.reshape(-1) >= 0)
    tgt = targets.reshape(-1)[rows]
    r = y.reshape(-1, H)[rows]
    h = r @ p["Wt"] + p["bt"]
    gl = gelu(h)
    t, ln = layernorm_fwd(gl, p["ln_g"], p["ln_b"], eps)
    z = t @ p["E_out"].T + p["b_out"]
    zmax = z.max(axis=-1, keepdims=True)
    lse = zmax[:, 0] + np.log(np.exp(z - zmax).sum(axis=-1))
    loss = loss_scale * (lse - z[np.arange(len(rows)), tgt]).sum()
    return loss, dict(rows=rows, tgt=tgt, r=r, h=h, gl=gl, ln=ln, t=t, z=z, lse=lse,
                      shape=y.shape, loss_scale=loss_scale)


def mlm_head_bwd(c, p):
    """Gradient of the loss w.r.t. the head's parameters and w.r.t. y."""
    n = len(c["rows"])
    dz = np.exp(c["z"] - c["lse"][:, None])
    dz[np.arange(n), c["tgt"]] -= 1.0
    dz *= c["loss_scale"]
    g = {"E_out": dz.T @ c["t"], "b_out": dz.sum(axis=0)}
    dt = dz @ p["E_out"]
    dgl, g["ln_g"], g["ln_b"] = layernorm_bwd(dt, c["ln"], p["ln_g"])
    dh = dgl * gelu_grad(c["h"])
    g["Wt"] = c["r"].T @ dh
    g["bt"] = dh.sum(axis=0)
    dy = np.zeros(c["shape"], dtype=np.float64).reshape(-1, c["shape"][-1])
    dy[c["rows"]] = dh @ p["Wt"].T
    return dy.reshape(c["shape"]), g


# --------------------------------------------------------------------------
# the stage: parameter views, F task, B task, schedule walk
# --------------------------------------------------------------------------

class Stage:
    """A stage with frozen parameters theta (flat vector, order given by `layout`:
    a list of (name, shape); names 'emb.*', 'l<i>.*', 'head.*')."""

    def __init__(self, layout, theta, n_layers, n_heads, ln_eps,
                 has_embedding=False, has_mlm_head=False, loss_scale=1.0):
        self.layout = list(layout)
        self.n_layers, self.A, self.eps = n_layers, n_heads, ln_eps
        self.has_embedding, self.has_mlm_head = has_embedding, has_mlm_head
        self.loss_scale = loss_scale
        theta = np.asarray(theta, dtype=np.float64)
        self.offsets, off = {}, 0
        for name, shape in self.layout:
            n = int(np.prod(shape))
            self.offsets[name] = (off, shape)
            off += n
        if off != theta.size:
            raise ValueError("theta has the wrong length")
        self.theta = theta
        self.n_params = off

    def group(self, prefix):
        out = {}
        for name, (off, shape) in self.offsets.items():
            if name.startswith(prefix):
                out[name[len(prefix):]] = self.theta[off:off + int(np.prod(shape))].reshape(shape)
        return out

    # F_m: forward task of one micro-batch; returns the boundary output and the
    # activations its backward will need
    def forward(self, x, targets=None):
        cache = {}
        if self.has_embedding:
            h, cache["emb"] = embedding_fwd(np.asarray(x), self.group("emb."), self.eps)
        else:
            h = np.asarray(x, dtype=np.float64)
        cache["layers"] = []
        for l in range(self.n_layers):
            h, c = layer_fwd(h, self.group(f"l{l}."), self.A, self.eps)
            cache["layers"].append(c)
        if self.has_mlm_head:
            loss, cache["head"] = mlm_head_fwd(h, np.asarray(targets), self.group("head."),
                                               self.eps, self.loss_scale)
            return loss, cache
        return h, cache

    # B_m: backward task; returns dx (None for an embedding stage) and this
    # micro-batch's parameter gradient as a flat vector
    def backward(self, dy, cache):
        G = np.zeros(self.n_params, dtype=np.float64)

        def put(prefix, g):
            for k, v in g.items():
                off, shape = self.offsets[prefix + k]
                G[off:off + v.size] += np.asarray(v).reshape(-1)

        if self.has_mlm_head:
            dh, g = mlm_head_bwd(cache["head"], self.group("head."))
            put("head.", g)
        else:
            dh = np.asarray(dy, dtype=np.float64)
        for l in reversed(range(self.n_layers)):
            dh, g = layer_bwd(dh, cache["layers"][l], self.group(f"l{l}."), self.A)
            put(f"l{l}.", g)
        if self.has_embedding:
            put("emb.", embedding_bwd(dh, cache["emb"], self.group("emb.")))
            dh = None
        return dh, G


def run_schedule(stage: Stage, M, K, order, xs, dys=None, targets=None):
    """Walk the task list of `order`; gradients accumulate over micro-batches in
    the order their backwards run (section V-B-3).  The activation store raises
    if it would hold more than K (early-backward) or M (GPipe) micro-batches.
    Returns dict(ys, dxs, grads, peak_live, ops)."""
    limit = min(K, M) if order == EARLY_BACKWARD else M
    store, ys, dxs = {}, [None] * M, [None] * M
    G = np.zeros(stage.n_params, dtype=np.float64)
    peak = 0
    ops = schedule_ops(M, K, order)
    for kind, m in ops:
        if kind == "F":
            if m in store:
                raise RuntimeError("micro-batch already resident")
            if len(store) >= limit:
                raise RuntimeError("activation store is full")
            ys[m], store[m] = stage.forward(xs[m], None if targets is None else targets[m])
            peak = max(peak, len(store))
        else:
            cache = store.pop(m)                         # released after its backward
            dxs[m], g = stage.backward(None if dys is None else dys[m], cache)
            G += g
    if store:
        raise RuntimeError("activations left resident")
    return dict(ys=ys, dxs=dxs, grads=G, peak_live=peak, ops=ops)


def full_batch(stage: Stage, xs, dys=None, targets=None):
    """The same iteration as one task over the concatenation of all micro-batches
    along the batch axis (the plain definition of the accumulated gradient)."""
    X = np.concatenate([np.asarray(x) for x in xs], axis=0)
    Tg = None if targets is None else np.concatenate([np.asarray(t) for t in targets], axis=0)
    Y, cache = stage.forward(X, Tg)
    DY = None if dys is None else np.concatenate([np.asarray(d) for d in dys], axis=0)
    dX, G = stage.backward(DY, cache)
    return dict(y=Y, dx=dX, grads=G)


# ---------------------------------------------------------------- synchronous weights update
def adam_apply(theta, m, v, G, step, lr, beta1=0.9, beta2=0.999, eps=1e-8, grad_scale=1.0):
    """The Apply of section V-B-3 for the optimizer the paper trains BERT-48 with (Adam, section
    VI-A): one update of the weights theta from the gradients G accumulated over the iteration's
    micro-batches, averaged by grad_scale (1 / number of samples or micro-batches, the caller's
    choice).  Adam as its authors state it (Kingma & Ba, Algorithm 1), step counted from 1:

        g = grad_scale * G
        m <- beta1 m + (1 - beta1) g          v <- beta2 v + (1 - beta2) g^2
        theta <- theta - lr * (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps)

    Returns the new (theta, m, v) as float64 arrays; the inputs are not modified.
    Pins (tests/test_oracle_adam.py): torch.optim.Adam in float64 over several steps; the closed
    form of the first step (|update| = lr |g| / (|g| + eps)); a zero gradient leaves theta alone."""
    theta, m, v, G = (np.asarray(a, dtype=np.float64) for a in (theta, m, v, G))
    g = grad_scale * G
    m1 = beta1 * m + (1.0 - beta1) * g
    v1 = beta2 * v + (1.0 - beta2) * g * g
    mhat = m1 / (1.0 - beta1 ** step)
    vhat = v1 / (1.0 - beta2 ** step)
    return theta - lr * mhat / (np.sqrt(vhat) + eps), m1, v1
