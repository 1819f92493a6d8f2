"""ctypes binding of libdapple_stage.so: the same names as the C ABI
(include/dapple_stage.h, include/dapple_kernels.h), argument marshalling only.
Every step of a task runs in the library's kernels; there is no Python or CPU
fallback -- if the library is missing, loading raises.

PyTorch appears only in `StageRunner`, a convenience that allocates device
buffers with torch and hands raw pointers to the library.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdapple_stage.so")

STAGE_OK = 0
STAGE_E_CONFIG, STAGE_E_NULL, STAGE_E_ARENA_SMALL, STAGE_E_NO_SLOT = -1, -2, -3, -4
STAGE_E_NOT_RESIDENT, STAGE_E_DUP_MB, STAGE_E_BAD_ORDER, STAGE_E_DEVICE = -5, -6, -7, -8
ORDER_GPIPE, ORDER_EARLY_BACKWARD, ORDER_EXPLICIT = 0, 1, 2
DTYPE_F32, DTYPE_BF16 = 0, 1
FLAG_DRY_RUN = 1
FLAG_RECOMPUTE = 2
FLAG_ONE_STREAM = 4
EPI_BIAS, EPI_ADD, EPI_MUL, EPI_GELU, EPI_ACC32, EPI_BSUM = 1, 2, 4, 8, 16, 128
EPI_OUT32, EPI_AUX32, EPI_ROWDOT = 32, 64, 256


class stage_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "hidden", "n_heads", "ffn", "seq", "micro_batch", "max_slots", "dtype",
                 "has_embedding", "has_mlm_head", "vocab", "max_pos", "flags")] + \
               [("ln_eps", C.c_float), ("loss_scale", C.c_float), ("mlm_max_rows", C.c_int32)]


class stage_sizes(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in
                ("n_params", "weight_bytes", "grad_bytes", "slot_bytes", "workspace_bytes", "arena_bytes")]


class stage_stats_t(C.Structure):
    _fields_ = [("slot_bytes", C.c_uint64), ("peak_activation_bytes", C.c_uint64),
                ("live_slots", C.c_int32), ("peak_live_slots", C.c_int32),
                ("fwd_tasks", C.c_uint64), ("bwd_tasks", C.c_uint64), ("kernel_launches", C.c_uint64)]


class dapple_gemm_desc(C.Structure):
    _fields_ = [("A", C.c_void_p), ("B", C.c_void_p), ("C", C.c_void_p), ("C2", C.c_void_p),
                ("bias", C.c_void_p), ("aux", C.c_void_p), ("bsum", C.c_void_p), ("rowdot", C.c_void_p),
                ("M", C.c_int32), ("N", C.c_int32), ("K", C.c_int32),
                ("lda", C.c_int32), ("ldb", C.c_int32), ("ldc", C.c_int32), ("ldaux", C.c_int32),
                ("a_kstrided", C.c_int32), ("b_kstrided", C.c_int32), ("kseg_len", C.c_int32),
                ("segA", C.c_int64), ("segB", C.c_int64), ("batch", C.c_int32),
                ("sA", C.c_int64), ("sB", C.c_int64), ("sC", C.c_int64), ("sBias", C.c_int64),
                ("k_valid", C.c_int32), ("epi", C.c_int32), ("tile", C.c_int32)]


# every symbol the two headers declare: name -> (restype, argtypes)
_vp, _i, _f = C.c_void_p, C.c_int, C.c_float
_pp = C.POINTER(C.c_void_p)
SYMBOLS = {
    "stage_query_sizes": (_i, [C.POINTER(stage_config), C.POINTER(stage_sizes)]),
    "stage_init": (_i, [C.POINTER(_vp), C.POINTER(stage_config), _vp, _vp, C.c_size_t, _vp]),
    "stage_fwd": (_i, [_vp, _i, _vp, _vp, _vp]),
    "stage_bwd": (_i, [_vp, _i, _vp, _vp]),
    "stage_schedule_ops": (_i, [_i, _i, _i, C.POINTER(C.c_int32), _i]),
    "stage_run_schedule": (_i, [_vp, _i, _i, _i, _pp, _pp, _pp, _pp, _pp, C.POINTER(C.c_int32), _i]),
    "stage_graph_capture": (_i, [_vp, _i, _i, _i, _pp, _pp, _pp, _pp, _pp, C.POINTER(C.c_int32), _i, _i]),
    "stage_graph_launch": (_i, [_vp]),
    "stage_stream": (_i, [_vp, C.POINTER(_vp)]),
    "stage_get_config": (_i, [_vp, C.POINTER(stage_config)]),
    "stage_grads": (_i, [_vp, C.POINTER(_vp), C.POINTER(C.c_uint64)]),
    "stage_zero_grads": (_i, [_vp]),
    "stage_apply_adam": (_i, [_vp, _vp, _vp, _vp, _vp, _i, _f, _f, _f, _f, _f, _i]),
    "stage_stats": (_i, [_vp, C.POINTER(stage_stats_t)]),
    "stage_reset_stats": (_i, [_vp]),
    "stage_profile_enable": (_i, [_vp, _i]),
    "stage_profile_read": (_i, [_vp, _i, C.POINTER(C.c_uint64), C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "stage_profile_launches": (_i, [_vp, _vp, _i]),
    "stage_profile_class_name": (C.c_char_p, [_i]),
    "stage_sync": (_i, [_vp]),
    "stage_destroy": (_i, [_vp]),
    "stage_last_error": (C.c_char_p, []),
    "pipeline_warmup_depths": (_i, [_i, _i, _i, _i, C.POINTER(C.c_int32)]),
    "pipeline_pivot_stage": (_i, [_i, _i, C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "pipeline_latency_model": (_i, [_i, _i, C.POINTER(C.c_double), C.POINTER(C.c_double), _i, C.POINTER(C.c_double)]),
    "pipeline_partition_stream_create": (_i, [_i, _i, C.POINTER(_vp)]),
    "pipeline_partition_stream_destroy": (_i, [_vp]),
    "pipeline_boundary_bytes": (C.c_size_t, [_i, _i, C.c_size_t]),
    "pipeline_create": (_i, [C.POINTER(_vp), _i, C.POINTER(_vp), _vp, C.c_size_t, C.c_size_t, _i]),
    "pipeline_destroy": (_i, [_vp]),
    "pipeline_run": (_i, [_vp, _i, C.POINTER(C.c_int32), _i, _pp, _pp, _pp, _pp, _pp]),
    "pipeline_sync": (_i, [_vp]),
    "pipeline_timeline": (_i, [_vp, C.POINTER(C.c_double), C.POINTER(C.c_double), _i]),
    "dapple_gemm": (_i, [_i, C.POINTER(dapple_gemm_desc), _vp]),
    "dapple_attention_fwd": (_i, [_i, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _vp]),
    "dapple_attention_bwd": (_i, [_i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _vp]),
    "dapple_layernorm_fwd": (_i, [_i, _vp, _vp, _vp, _vp, _vp, _i, _i, _f, _vp]),
    "dapple_layernorm_bwd": (_i, [_i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _vp]),
    "dapple_colsum": (_i, [_i, _vp, _i, _i, _i, _vp, _vp, _vp]),
    "dapple_colsum_static": (_i, [_i, _vp, _i, _i, _i, _vp, _vp]),
}

_lib = None


def load():
    """Load the shared library (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2007_01045_amd.build` "
                               "(there is no fallback path)")
        # PyTorch brings its own copy of the HIP runtime.  The library shares streams and device memory
        # with it, so both must sit on the same copy: with torch loaded first, the dynamic linker gives
        # ours the runtime that is already there; loaded the other way round the process would hold two
        # runtimes, and the second one finds no device.
        import torch  # noqa: F401
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in SYMBOLS.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


class StageError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"stage error {code}: {msg}")
        self.code = code


def last_error() -> str:
    return (load().stage_last_error() or b"").decode()


def _check(rc):
    if rc < 0:
        raise StageError(rc, last_error())
    return rc


def make_config(n_layers, hidden, n_heads, ffn, seq, micro_batch, max_slots, dtype, has_embedding=0,
                has_mlm_head=0, vocab=0, max_pos=0, flags=0, ln_eps=1e-12, loss_scale=1.0,
                mlm_max_rows=0) -> stage_config:
    return stage_config(n_layers, hidden, n_heads, ffn, seq, micro_batch, max_slots, dtype,
                        int(has_embedding), int(has_mlm_head), vocab, max_pos, flags, ln_eps, loss_scale,
                        mlm_max_rows)


# ---- thin wrappers, one per C entry point ---------------------------------
def config_for(cfg, max_slots, loss_scale=1.0, flags=0) -> stage_config:
    """The C configuration of a stage described by inputs.StageConfig (the seeded-input module's shape record);
    a stage with the MLM head gets room for the 15% of positions the input recipe predicts."""
    import math
    tokens = cfg.micro_batch * cfg.seq
    return make_config(cfg.n_layers, cfg.hidden, cfg.n_heads, cfg.ffn, cfg.seq, cfg.micro_batch, max_slots,
                       DTYPE_BF16 if cfg.dtype == "bf16" else DTYPE_F32, cfg.has_embedding, cfg.has_mlm_head,
                       cfg.vocab if (cfg.has_embedding or cfg.has_mlm_head) else 0,
                       cfg.max_pos if cfg.has_embedding else 0, flags, cfg.ln_eps, loss_scale,
                       math.ceil(0.15 * tokens) if cfg.has_mlm_head else 0)


def stage_query_sizes(cfg: stage_config) -> stage_sizes:
    out = stage_sizes()
    _check(load().stage_query_sizes(C.byref(cfg), C.byref(out)))
    return out


def stage_init(cfg: stage_config, weights_ptr, arena_ptr, arena_bytes, stream_ptr=None):
    h = C.c_void_p()
    _check(load().stage_init(C.byref(h), C.byref(cfg), weights_ptr, arena_ptr, arena_bytes, stream_ptr))
    return h


def stage_fwd(h, mb, x_ptr, y_ptr, aux_ptr=None):
    _check(load().stage_fwd(h, mb, x_ptr, y_ptr, aux_ptr))


def stage_bwd(h, mb, dy_ptr, dx_ptr):
    _check(load().stage_bwd(h, mb, dy_ptr, dx_ptr))


def stage_schedule_ops(M, K, order):
    cap = max(2 * M, 1)
    buf = (C.c_int32 * cap)()
    n = _check(load().stage_schedule_ops(M, K, order, buf, cap))
    return [("F", v - 1) if v > 0 else ("B", -v - 1) for v in buf[:n]]


def _ptr_array(ptrs, M):
    if ptrs is None:
        return None
    return (C.c_void_p * M)(*[p for p in ptrs])


def stage_run_schedule(h, M, K, order, xs=None, dys=None, ys=None, dxs=None, auxs=None, explicit_ops=None):
    ops, n = None, 0
    if explicit_ops is not None:
        enc = [(m + 1) if k == "F" else -(m + 1) for k, m in explicit_ops]
        ops, n = (C.c_int32 * max(len(enc), 1))(*enc), len(enc)
    _check(load().stage_run_schedule(h, M, K, order, _ptr_array(xs, M), _ptr_array(dys, M), _ptr_array(ys, M),
                                     _ptr_array(dxs, M), _ptr_array(auxs, M), ops, n))


def stage_graph_capture(h, M, K, order, xs=None, dys=None, ys=None, dxs=None, auxs=None, explicit_ops=None,
                        zero_grads_first=True):
    ops, n = None, 0
    if explicit_ops is not None:
        enc = [(m + 1) if k == "F" else -(m + 1) for k, m in explicit_ops]
        ops, n = (C.c_int32 * max(len(enc), 1))(*enc), len(enc)
    _check(load().stage_graph_capture(h, M, K, order, _ptr_array(xs, M), _ptr_array(dys, M), _ptr_array(ys, M),
                                      _ptr_array(dxs, M), _ptr_array(auxs, M), ops, n, int(zero_grads_first)))


def stage_graph_launch(h):
    _check(load().stage_graph_launch(h))


def stage_stream(h):
    p = C.c_void_p()
    _check(load().stage_stream(h, C.byref(p)))
    return p.value


def stage_get_config(h) -> stage_config:
    c = stage_config()
    _check(load().stage_get_config(h, C.byref(c)))
    return c


POLICY_A, POLICY_B = 0, 1


def pipeline_warmup_depths(S, M, policy=POLICY_A, D=0):
    buf = (C.c_int32 * max(S, 1))()
    _check(load().pipeline_warmup_depths(S, M, policy, D, buf))
    return list(buf[:S])


def pipeline_pivot_stage(M, F, B):
    S = len(F)
    return _check(load().pipeline_pivot_stage(S, M, (C.c_double * S)(*F), (C.c_double * S)(*B)))


def pipeline_latency_model(M, F, B, Q=-1):
    S = len(F)
    out = C.c_double()
    _check(load().pipeline_latency_model(S, M, (C.c_double * S)(*F), (C.c_double * S)(*B), Q, C.byref(out)))
    return out.value


def pipeline_partition_stream_create(part, nparts):
    p = C.c_void_p()
    _check(load().pipeline_partition_stream_create(part, nparts, C.byref(p)))
    return p.value


def pipeline_partition_stream_destroy(stream):
    _check(load().pipeline_partition_stream_destroy(stream))


def pipeline_boundary_bytes(S, max_M, act_bytes):
    return load().pipeline_boundary_bytes(S, max_M, act_bytes)


def pipeline_create(stage_handles, boundary_ptr, boundary_bytes, act_bytes, max_M):
    S = len(stage_handles)
    arr = (C.c_void_p * S)(*[h.value if isinstance(h, C.c_void_p) else h for h in stage_handles])
    out = C.c_void_p()
    _check(load().pipeline_create(C.byref(out), S, arr, boundary_ptr, boundary_bytes, act_bytes, max_M))
    return out


def pipeline_destroy(p):
    _check(load().pipeline_destroy(p))


def pipeline_run(p, M, K, order, xs, dys=None, auxs=None, ys=None, dxs=None):
    Ka = None if K is None else (C.c_int32 * len(K))(*K)
    _check(load().pipeline_run(p, M, Ka, order, _ptr_array(xs, M), _ptr_array(dys, M), _ptr_array(auxs, M),
                               _ptr_array(ys, M), _ptr_array(dxs, M)))


def pipeline_sync(p):
    _check(load().pipeline_sync(p))


def pipeline_timeline(p, S, M):
    """{(kind, stage, m): (start_ms, end_ms)} of the last run, kind 'F' or 'B'."""
    n = 2 * S * M
    a, b = (C.c_double * n)(), (C.c_double * n)()
    _check(load().pipeline_timeline(p, a, b, n))
    return {(("F", "B")[k], i, m): (a[(k * S + i) * M + m], b[(k * S + i) * M + m])
            for k in range(2) for i in range(S) for m in range(M)}


def stage_grads(h):
    p, n = C.c_void_p(), C.c_uint64()
    _check(load().stage_grads(h, C.byref(p), C.byref(n)))
    return p.value, n.value


def stage_zero_grads(h):
    _check(load().stage_zero_grads(h))


def stage_apply_adam(h, weights_ptr, master_ptr, m_ptr, v_ptr, step, lr, beta1=0.9, beta2=0.999, eps=1e-8,
                     grad_scale=1.0, zero_grads=False):
    _check(load().stage_apply_adam(h, weights_ptr, master_ptr, m_ptr, v_ptr, step, lr, beta1, beta2, eps,
                                   grad_scale, int(zero_grads)))


def stage_stats(h) -> stage_stats_t:
    out = stage_stats_t()
    _check(load().stage_stats(h, C.byref(out)))
    return out


def stage_reset_stats(h):
    _check(load().stage_reset_stats(h))


def stage_profile_enable(h, on):
    _check(load().stage_profile_enable(h, int(on)))


def stage_profile_read(h):
    names = []
    while True:
        s = load().stage_profile_class_name(len(names))
        if s is None:
            break
        names.append(s.decode())
    n = len(names)
    launches, ms, flops = (C.c_uint64 * n)(), (C.c_double * n)(), (C.c_double * n)()
    _check(load().stage_profile_read(h, n, launches, ms, flops))
    return {names[i]: dict(launches=launches[i], ms=ms[i], flops=flops[i]) for i in range(n)}


class stage_launch_record(C.Structure):
    _fields_ = [("cls", C.c_int32), ("lane", C.c_int32), ("M", C.c_int32), ("N", C.c_int32), ("K", C.c_int32),
                ("batch", C.c_int32), ("ms", C.c_double), ("flops", C.c_double)]


def stage_profile_launches(h, capacity=1 << 16):
    """The launches timed since profiling was enabled (call before stage_profile_read): a list of dicts."""
    buf = (stage_launch_record * capacity)()
    n = _check(load().stage_profile_launches(h, buf, capacity))
    lib = load()
    return [dict(cls=(lib.stage_profile_class_name(r.cls) or b"?").decode(), lane=r.lane, M=r.M, N=r.N, K=r.K,
                 batch=r.batch, ms=r.ms, flops=r.flops) for r in buf[:n]]


def stage_sync(h):
    _check(load().stage_sync(h))


def stage_destroy(h):
    _check(load().stage_destroy(h))


def dapple_gemm(dtype, desc: dapple_gemm_desc, stream_ptr=None) -> int:
    rc = load().dapple_gemm(dtype, C.byref(desc), stream_ptr)
    if rc < 0:
        raise StageError(rc, "dapple_gemm rejected its arguments")
    return rc


def _kcheck(rc, name):
    if rc < 0:
        raise StageError(rc, name + " rejected its arguments")


def dapple_attention_fwd(dtype, q, k, v, ctx, lse, b, s, A, H, stream_ptr=None):
    _kcheck(load().dapple_attention_fwd(dtype, q, k, v, ctx, lse, b, s, A, H, stream_ptr), "dapple_attention_fwd")


def dapple_attention_bwd(dtype, q, k, v, ctx, lse, dctx, dq, dk, dv, delta, b, s, A, H, stream_ptr=None):
    _kcheck(load().dapple_attention_bwd(dtype, q, k, v, ctx, lse, dctx, dq, dk, dv, delta, b, s, A, H, stream_ptr),
            "dapple_attention_bwd")


def dapple_layernorm_fwd(dtype, z, gamma, beta, y, stats, rows, H, eps, stream_ptr=None):
    _kcheck(load().dapple_layernorm_fwd(dtype, z, gamma, beta, y, stats, rows, H, eps, stream_ptr),
            "dapple_layernorm_fwd")


def dapple_layernorm_bwd(dtype, dy, z, stats, gamma, dz, partial, dgamma, dbeta, dbias, rows, H, stream_ptr=None):
    _kcheck(load().dapple_layernorm_bwd(dtype, dy, z, stats, gamma, dz, partial, dgamma, dbeta, dbias, rows, H,
                                        stream_ptr), "dapple_layernorm_bwd")


def dapple_colsum(dtype, X, rows, cols, ld, partial, out, stream_ptr=None):
    _kcheck(load().dapple_colsum(dtype, X, rows, cols, ld, partial, out, stream_ptr), "dapple_colsum")


COLSUM_STATIC_MAX_FLOATS = 1 << 20


def dapple_colsum_static(dtype, X, rows, cols, ld, out, stream_ptr=None):
    rc = load().dapple_colsum_static(dtype, X, rows, cols, ld, out, stream_ptr)
    if rc < 0:
        raise StageError(rc, last_error())


# ---- convenience: device memory through torch ------------------------------
class StageRunner:
    """Owns the device buffers of one stage (weights, arena, per-micro-batch inputs
    and outputs) as torch tensors and passes their addresses to the library."""

    def __init__(self, cfg: stage_config, theta_f32, device="cuda:0", stream_ptr=None):
        import torch
        load()
        self.torch, self.cfg, self.device = torch, cfg, device
        self.tdtype = torch.bfloat16 if cfg.dtype == DTYPE_BF16 else torch.float32
        self.sizes = stage_query_sizes(cfg)
        th = torch.as_tensor(theta_f32, dtype=torch.float32)
        assert th.numel() == self.sizes.n_params
        self.weights = th.to(device).to(self.tdtype).contiguous()
        self.arena = torch.empty(self.sizes.arena_bytes + 256, dtype=torch.uint8, device=device)
        base = self.arena.data_ptr()
        self.arena_ptr = (base + 255) // 256 * 256
        # stream_ptr: a raw hipStream_t (a partition stream of the pipeline); else torch's current stream
        self.stream = torch.cuda.current_stream(device) if stream_ptr is None else torch.cuda.ExternalStream(stream_ptr)
        self.h = stage_init(cfg, self.weights.data_ptr(), self.arena_ptr, self.sizes.arena_bytes,
                            self.stream.cuda_stream)
        off = self.arena_ptr - base
        self.grads = self.arena[off:off + 4 * self.sizes.n_params].view(torch.float32)
        p, n = stage_grads(self.h)
        assert p == self.grads.data_ptr() and n == self.sizes.n_params
        self.T = cfg.micro_batch * cfg.seq

    def init_adam(self):
        """fp32 master copy of the weights and zeroed moments (the optimizer state is the caller's)."""
        torch = self.torch
        self.master = self.weights.to(torch.float32).clone().contiguous()
        self.m = torch.zeros_like(self.master)
        self.v = torch.zeros_like(self.master)
        self.step = 0

    def apply_adam(self, lr, beta1=0.9, beta2=0.999, eps=1e-8, grad_scale=1.0, zero_grads=False):
        self.step += 1
        stage_apply_adam(self.h, self.weights.data_ptr(), self.master.data_ptr(), self.m.data_ptr(),
                         self.v.data_ptr(), self.step, lr, beta1, beta2, eps, grad_scale, zero_grads)

    def to_dev(self, a, dtype=None):
        t = self.torch.as_tensor(a)
        if t.dtype.is_floating_point:
            t = t.to(dtype or self.tdtype)
        return t.to(self.device).contiguous()

    def empty_act(self):
        return self.torch.empty(self.T, self.cfg.hidden, dtype=self.tdtype, device=self.device)

    def run(self, M, K, order, xs, dys=None, auxs=None, explicit_ops=None):
        """xs/dys/auxs: lists of device tensors.  Returns (ys, dxs) device tensors."""
        torch = self.torch
        head, emb = self.cfg.has_mlm_head, self.cfg.has_embedding
        ys = [torch.zeros(1, dtype=torch.float32, device=self.device) if head else self.empty_act() for _ in range(M)]
        dxs = None if emb else [self.empty_act() for _ in range(M)]
        ptr = lambda ts: None if ts is None else [t.data_ptr() for t in ts]
        stage_run_schedule(self.h, M, K, order, ptr(xs), ptr(dys), ptr(ys), ptr(dxs), ptr(auxs), explicit_ops)
        return ys, dxs

    def close(self):
        if self.h is not None:
            stage_destroy(self.h)
            self.h = None


class PipelineRunner:
    """S stages on one GPU tied into a pipeline (dapple_pipeline.h): owns the stage runners, their streams
    (one partition of the compute units each when parts > 1, ordinary torch streams when parts == 0)
    and the boundary buffer."""

    def __init__(self, cfgs, thetas, max_M, parts=1, device="cuda:0"):
        import torch
        load()
        self.torch, self.S, self.max_M = torch, len(cfgs), max_M
        self.streams, self.tstreams, self.runners, self.p = [], [], [], None
        for i, (cfg, th) in enumerate(zip(cfgs, thetas)):
            if parts == 0:
                self.tstreams.append(torch.cuda.Stream(device))
                sp = self.tstreams[-1].cuda_stream
            else:
                self.streams.append(pipeline_partition_stream_create(i if parts > 1 else 0, parts))
                sp = self.streams[-1]
            self.runners.append(StageRunner(cfg, th, device, stream_ptr=sp))
        c = cfgs[0]
        self.act_bytes = c.micro_batch * c.seq * c.hidden * (2 if c.dtype == DTYPE_BF16 else 4)
        nb = pipeline_boundary_bytes(self.S, max_M, self.act_bytes)
        self.boundary = torch.zeros(nb + 256, dtype=torch.uint8, device=device)
        torch.cuda.synchronize()
        self.p = pipeline_create([r.h for r in self.runners], (self.boundary.data_ptr() + 255) // 256 * 256, nb,
                                 self.act_bytes, max_M)

    def run(self, M, K, order, xs, dys=None, auxs=None, ys=None, dxs=None):
        """Enqueue one iteration (device tensors in, device tensors written) and wait for it."""
        ptr = lambda ts: None if ts is None else [t.data_ptr() for t in ts]
        pipeline_run(self.p, M, K, order, ptr(xs), ptr(dys), ptr(auxs), ptr(ys), ptr(dxs))
        pipeline_sync(self.p)

    def timeline(self, M):
        return pipeline_timeline(self.p, self.S, M)

    def close(self):
        if self.p is not None:
            pipeline_destroy(self.p)
            self.p = None
        for r in self.runners:
            r.close()
        for s in self.streams:
            pipeline_partition_stream_destroy(s)
        self.streams = []
