"""Seeded synthetic inputs for one pipeline stage.

This module draws numbers and lays them out; it contains none of the stage's
arithmetic (no layer math, no schedule).  Both the CPU oracle's tests and the
HIP path's tests/bench take their inputs from here, so that the two sides see
identical, reproducible values.

Generator: a counter-based splitmix64 stream (state_i = seed + (i+1)*gamma,
then the splitmix64 finaliser), turned into uniforms in (0,1) and into normals
by the Box-Muller transform.  Every tensor gets its own sub-stream keyed by
(seed, tensor tag), so the value of one tensor does not depend on whether the
others were drawn.

Workload recipe (it stands in for the BERT-48 / BERT-Large fine-tuning
workloads of the paper's evaluation, section VI; only shapes matter for
throughput and memory): stage input x_m ~ N(0,1) [b,s,H]; output gradient
dy_m ~ N(0,1) [b,s,H]; every weight matrix and bias ~ N(0,0.02); LayerNorm gain
1 + N(0,0.02), shift N(0,0.02); token ids uniform in [0,V); MLM targets on
exactly ceil(0.15*T) distinct positions per micro-batch, uniform in [0,V).
For bf16 configs all floating-point tensors are rounded once to bf16
(round-to-nearest-even), so that the oracle and the GPU consume identical
bf16-representable values.
"""
from __future__ import annotations

import dataclasses
import math
import zlib

import numpy as np

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


@dataclasses.dataclass(frozen=True)
class StageConfig:
    """Shape of one stage.  Names follow the usual transformer notation:
    L layers, H hidden, A heads, F ffn width, s sequence length, b samples per
    micro-batch; M micro-batches per iteration, K resident limit."""
    n_layers: int
    hidden: int
    n_heads: int
    ffn: int
    seq: int
    micro_batch: int
    M: int
    K: int
    dtype: str = "bf16"          # "f32" or "bf16"
    has_embedding: bool = False
    has_mlm_head: bool = False
    vocab: int = 30522
    max_pos: int = 512
    ln_eps: float = 1e-12
    name: str = ""

    @property
    def tokens(self) -> int:
        return self.micro_batch * self.seq

    @property
    def head_dim(self) -> int:
        return self.hidden // self.n_heads


CONFIGS = {
    "tiny": StageConfig(2, 64, 4, 256, 16, 2, 4, 2, "f32", name="tiny"),
    "bert_large": StageConfig(6, 1024, 16, 4096, 512, 4, 8, 4, "bf16", name="bert_large"),
    "bert48_quarter": StageConfig(12, 1024, 16, 4096, 512, 2, 16, 4, "bf16", name="bert48_quarter"),
    "first_stage": StageConfig(12, 1024, 16, 4096, 512, 2, 16, 4, "bf16", has_embedding=True,
                               name="first_stage"),
    "last_stage": StageConfig(12, 1024, 16, 4096, 512, 2, 32, 4, "bf16", has_mlm_head=True,
                              name="last_stage"),
}


def param_layout(cfg: StageConfig):
    """Flat parameter order: [(name, shape)].  Linear weights are stored
    [in, out] row-major so that y = x @ W + b.  Embedding block first, encoder
    layers next, MLM-head block last."""
    H, F = cfg.hidden, cfg.ffn
    out = []
    if cfg.has_embedding:
        out += [("emb.E_w", (cfg.vocab, H)), ("emb.E_p", (cfg.max_pos, H)),
                ("emb.ln_g", (H,)), ("emb.ln_b", (H,))]
    for l in range(cfg.n_layers):
        p = f"l{l}."
        out += [(p + "Wq", (H, H)), (p + "bq", (H,)), (p + "Wk", (H, H)), (p + "bk", (H,)),
                (p + "Wv", (H, H)), (p + "bv", (H,)), (p + "Wo", (H, H)), (p + "bo", (H,)),
                (p + "ln1_g", (H,)), (p + "ln1_b", (H,)),
                (p + "W1", (H, F)), (p + "b1", (F,)), (p + "W2", (F, H)), (p + "b2", (H,)),
                (p + "ln2_g", (H,)), (p + "ln2_b", (H,))]
    if cfg.has_mlm_head:
        out += [("head.Wt", (H, H)), ("head.bt", (H,)), ("head.ln_g", (H,)), ("head.ln_b", (H,)),
                ("head.E_out", (cfg.vocab, H)), ("head.b_out", (cfg.vocab,))]
    return out


def n_params(cfg: StageConfig) -> int:
    return sum(int(np.prod(s)) for _, s in param_layout(cfg))


def param_offsets(cfg: StageConfig):
    """name -> (offset, shape) into the flat parameter / gradient vector."""
    off, d = 0, {}
    for name, shape in param_layout(cfg):
        d[name] = (off, shape)
        off += int(np.prod(shape))
    return d


def _mix(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _stream_key(seed: int, tag: str) -> np.uint64:
    k = np.array([(seed & 0xFFFFFFFFFFFFFFFF)], dtype=np.uint64)
    t = np.array([zlib.crc32(tag.encode()) | (len(tag) << 32)], dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _mix(_mix(k + _GAMMA) ^ (t * _GAMMA))[0]


def raw_u64(seed: int, tag: str, n: int) -> np.ndarray:
    """n 64-bit words of the (seed, tag) stream."""
    key = _stream_key(seed, tag)
    with np.errstate(over="ignore"):
        ctr = (np.arange(1, n + 1, dtype=np.uint64)) * _GAMMA + key
        return _mix(ctr)


def uniform01(seed: int, tag: str, n: int) -> np.ndarray:
    """n float64 uniforms strictly inside (0,1) (53-bit mantissa, offset half an ulp)."""
    return ((raw_u64(seed, tag, n) >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / (1 << 53))


def normal(seed: int, tag: str, n: int) -> np.ndarray:
    """n float64 standard normals by Box-Muller (two uniforms -> two normals)."""
    m = (n + 1) // 2
    u = uniform01(seed, tag, 2 * m)
    r = np.sqrt(-2.0 * np.log(u[:m]))
    th = (2.0 * math.pi) * u[m:]
    return np.concatenate([r * np.cos(th), r * np.sin(th)])[:n]


def randint(seed: int, tag: str, n: int, hi: int) -> np.ndarray:
    """n integers uniform in [0, hi) (multiply-shift on the top 32 bits)."""
    w = raw_u64(seed, tag, n) >> np.uint64(32)
    return ((w * np.uint64(hi)) >> np.uint64(32)).astype(np.int64)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float values to the nearest bf16 (ties to even); returns float32
    holding exactly bf16-representable values."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))) & np.uint64(0xFFFF0000)
    return u.astype(np.uint32).view(np.float32).reshape(f.shape)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of values that are already bf16-representable."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    return (f.view(np.uint32) >> np.uint32(16)).astype(np.uint16).reshape(f.shape)


def bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """float32 values of uint16 bf16 bit patterns."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _maybe_round(cfg: StageConfig, a: np.ndarray) -> np.ndarray:
    return round_to_bf16(a) if cfg.dtype == "bf16" else a.astype(np.float32)


def make_params(cfg: StageConfig, seed: int) -> np.ndarray:
    """Flat float32 parameter vector in `param_layout` order."""
    theta = np.empty(n_params(cfg), dtype=np.float32)
    off = 0
    for name, shape in param_layout(cfg):
        n = int(np.prod(shape))
        v = 0.02 * normal(seed, "theta." + name, n)
        if name.endswith("_g"):          # LayerNorm gains sit around one
            v = 1.0 + v
        theta[off:off + n] = _maybe_round(cfg, v)
        off += n
    return theta


def make_microbatch(cfg: StageConfig, seed: int, m: int):
    """Inputs of micro-batch m: dict with
    x   [b,s,H] float32 (or ids [b,s] int32 for a stage with embeddings),
    dy  [b,s,H] float32 (absent for a stage with the MLM head),
    targets [b,s] int32, -1 = not predicted (MLM head only)."""
    b, s, H = cfg.micro_batch, cfg.seq, cfg.hidden
    T = b * s
    out = {}
    if cfg.has_embedding:
        out["ids"] = randint(seed, f"ids.{m}", T, cfg.vocab).astype(np.int32).reshape(b, s)
    else:
        out["x"] = _maybe_round(cfg, normal(seed, f"x.{m}", T * H)).reshape(b, s, H)
    if cfg.has_mlm_head:
        n_mask = math.ceil(0.15 * T)
        # the n_mask positions with the smallest keys: a seeded partial shuffle
        keys = raw_u64(seed, f"maskpos.{m}", T)
        pos = np.sort(np.argsort(keys, kind="stable")[:n_mask])
        tgt = np.full(T, -1, dtype=np.int32)
        tgt[pos] = randint(seed, f"target.{m}", n_mask, cfg.vocab).astype(np.int32)
        out["targets"] = tgt.reshape(b, s)
    else:
        out["dy"] = _maybe_round(cfg, normal(seed, f"dy.{m}", T * H)).reshape(b, s, H)
    return out


DEFAULT_SEED = 20200701
