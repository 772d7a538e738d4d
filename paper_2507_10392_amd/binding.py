"""ctypes binding of libstage.so: argument marshalling only.

PyTorch is used for device memory (torch.empty on the GPU) and for the stream handle; no
computation of the stage step happens in Python or in torch.  The library must have been built
(python -m paper_2507_10392_amd.build, or __graft_entry__.build()); loading fails loudly if
it is missing - there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libstage.so")

STAGE_OK, STAGE_ERR_ARG, STAGE_ERR_STATE, STAGE_ERR_WORKSPACE, STAGE_ERR_BUDGET, STAGE_ERR_DEVICE = range(6)
_ERR_NAMES = {1: "STAGE_ERR_ARG", 2: "STAGE_ERR_STATE", 3: "STAGE_ERR_WORKSPACE", 4: "STAGE_ERR_BUDGET",
              5: "STAGE_ERR_DEVICE"}


class StageError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"{_ERR_NAMES.get(code, code)}: {msg}")
        self.code = code


class StageConfigC(C.Structure):
    _fields_ = [("arch", C.c_int32), ("dtype", C.c_int32), ("layers", C.c_int32), ("hidden", C.c_int32),
                ("heads", C.c_int32), ("ffn", C.c_int32), ("seq", C.c_int32), ("microbatch", C.c_int32),
                ("max_microbatches", C.c_int32), ("vocab", C.c_int32), ("has_embed", C.c_int32),
                ("has_head", C.c_int32), ("recompute", C.c_int32), ("pair_wgrad", C.c_int32),
                ("act_budget_bytes", C.c_int64), ("shard_begin", C.c_int64), ("shard_end", C.c_int64),
                ("norm_eps", C.c_float), ("rope_base", C.c_float), ("lr", C.c_float), ("beta1", C.c_float),
                ("beta2", C.c_float), ("adam_eps", C.c_float), ("weight_decay", C.c_float), ("offload_acts", C.c_int32)]


class StageMemoryC(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("params", "grads", "optim", "activations", "scratch", "workspace", "host_stash")]


class MinistagesConfigC(C.Structure):
    _fields_ = [("stage", StageConfigC), ("n_ministages", C.c_int32), ("reserved", C.c_int32)]


class MinistagesMemoryC(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("per_stage_host", "host_bytes", "off_params", "off_master", "off_m", "off_v",
                                         "off_stash", "param_slot", "state_slot", "grad", "workspace_each", "scratch",
                                         "device_bytes", "resident_bytes")]


class StageLinearFitC(C.Structure):
    _fields_ = [("intercept", C.c_double), ("slope", C.c_double), ("r2", C.c_double)]


class StageSegmentC(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("offset", C.c_int64), ("rows", C.c_int64), ("cols", C.c_int64)]


class StageKernelStatC(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("launches", C.c_int64), ("ms", C.c_double), ("flops", C.c_double),
                ("bytes", C.c_double)]


_lib = None


def lib():
    """The loaded library; raises if it was not built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2507_10392_amd.build` "
                               "(there is no fallback implementation)")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
        L.stage_query.argtypes = [C.POINTER(StageConfigC), C.POINTER(i64), C.POINTER(StageMemoryC), C.POINTER(i32)]
        L.stage_layout.argtypes = [C.POINTER(StageConfigC), C.POINTER(StageSegmentC), i32]
        L.stage_init.argtypes = [C.POINTER(StageConfigC), vp, vp, vp, vp, vp, vp, vp, i64, C.POINTER(vp)]
        L.stage_init_split.argtypes = [C.POINTER(StageConfigC), vp, vp, vp, vp, vp, vp, vp, i64, vp, i64, C.POINTER(vp)]
        L.stage_attach_host_stash.argtypes = [vp, vp, i64]
        L.stage_forward.argtypes = [vp, i32, vp, vp, vp, vp]
        L.stage_backward.argtypes = [vp, i32, vp, vp, f32]
        L.stage_accumulate.argtypes = [vp, i32]
        L.stage_optimizer_step.argtypes = [vp, i64, f32]
        L.stage_graph_replayed.argtypes = [vp, i32]
        L.stage_profile.argtypes = [vp, i32]
        L.stage_profile_read.argtypes = [vp, C.POINTER(StageKernelStatC), i32]
        L.stage_set_overflow_flag.argtypes = [vp, vp]
        L.stage_loss_scale_update.argtypes = [C.POINTER(f32), C.POINTER(i32), i32, f32, f32, i32]
        L.stage_time_layers.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.stage_fit_linear.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_double), i32, C.POINTER(StageLinearFitC)]
        L.stage_last_error.argtypes = [vp]
        L.stage_last_error.restype = C.c_char_p
        L.stage_destroy.argtypes = [vp]
        L.stage_destroy.restype = None
        L.ministages_query.argtypes = [C.POINTER(MinistagesConfigC), C.POINTER(MinistagesMemoryC)]
        L.ministages_init.argtypes = [C.POINTER(MinistagesConfigC), vp, vp, i64, vp, i64, C.POINTER(vp)]
        L.ministages_forward.argtypes = [vp, i32, i32, vp, vp, vp, vp]
        L.ministages_backward.argtypes = [vp, i32, i32, vp, vp, f32]
        L.ministages_accumulate.argtypes = [vp, i32, i32]
        L.ministages_optimizer_step.argtypes = [vp, i32, i64, f32]
        L.ministages_stage.argtypes = [vp, i32]
        L.ministages_stage.restype = vp
        L.ministages_traffic.argtypes = [vp, C.POINTER(i64), C.POINTER(i64)]
        L.ministages_last_error.argtypes = [vp]
        L.ministages_last_error.restype = C.c_char_p
        L.ministages_destroy.argtypes = [vp]
        L.ministages_destroy.restype = None
        L.stage_op_gemm.argtypes = [vp, i32, i32, i32, i32, i32, i32, vp, i64, vp, i64, vp, i64, i32, vp, vp, i64, i32,
                                    i64, i64, i64, i64, i32, i64, i32]
        L.stage_op_gemm_rope.argtypes = L.stage_op_gemm.argtypes + [vp, i32, i32, i32]
        L.stage_op_gemm_glu.argtypes = [vp, i32, i32, i32, i32, i32, vp, i64, vp, i64, i64, vp, vp, i32]
        L.stage_op_rope_table.argtypes = [vp, i32, i32, f32, vp]
        L.stage_op_wgrad_pair.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, i64, vp, vp, i64, vp, i64, i32, i64, i64, i64, i32]
        L.stage_op_wgrad_parts.argtypes = [vp, i32, i32, i32, i32, i32, i32, C.POINTER(vp), i64, C.POINTER(vp), i64, vp, i64, i32,
                                           i64, i64, i64, i32]
        L.stage_op_wgrad_parts_cut.argtypes = [vp, i32, i32, i32, i32, i32, i32, C.POINTER(vp), i64, C.POINTER(vp), i64, vp, i64, i32,
                                               i64, i64, i64, vp, i64]
        L.stage_op_wgrad_parts_scratch_bytes.argtypes = [i32, i32, i32, i32, i32, i32]
        L.stage_op_wgrad_parts_scratch_bytes.restype = i64
        L.stage_op_norm_fwd.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, f32, vp, vp, vp]
        L.stage_op_norm_bwd.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32]
        L.stage_op_rope.argtypes = [vp, i32, i32, i32, i32, i32, vp, i64, f32, f32, vp]
        L.stage_op_gelu.argtypes = [vp, i32, i64, vp, vp, vp, i32]
        L.stage_op_swiglu.argtypes = [vp, i32, i32, i32, vp, vp, vp, i32]
        L.stage_op_attention_fwd.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, vp, i64, vp, i64, vp, i32]
        L.stage_op_attention_bwd.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, vp, i64, vp, vp, i64, vp, vp, vp, vp,
                                             vp, i64, i32]
        L.stage_op_attention_bwd_rope.argtypes = L.stage_op_attention_bwd.argtypes + [vp]
        L.stage_op_attention_bwd_noalloc.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, vp, i64, vp, vp, i64, vp, vp, vp, vp,
                                                     i64, i32]
        L.stage_op_embed.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, i32]
        L.stage_op_cross_entropy.argtypes = [vp, i32, i32, i32, vp, i64, vp, vp, vp, vp, f32, i32]
        L.stage_op_adamw.argtypes = [vp, i32, i64, i64, vp, vp, vp, vp, vp, f32, f32, f32, f32, f32, i64, f32]
        L.stage_op_mfma_rate.argtypes = [vp, i32, i32, vp, vp]
        L.stage_op_lds_probe.argtypes = [vp, i32, C.POINTER(i32), vp, i32, vp]
        _lib = L
    return _lib


def make_config(cfg, shard=None, max_microbatches=None) -> StageConfigC:
    """Builds the C struct from any object with the attributes of workloads.StageConfig."""
    b, e = cfg.shard_range if shard is None else shard
    return StageConfigC(cfg.arch, cfg.dtype, cfg.layers, cfg.hidden, cfg.heads, cfg.ffn, cfg.seq, cfg.microbatch,
                        cfg.num_microbatches if max_microbatches is None else max_microbatches, cfg.vocab,
                        cfg.has_embed, cfg.has_head, cfg.recompute, int(getattr(cfg, "pair_wgrad", 0)), cfg.act_budget_bytes, b, e,
                        cfg.norm_eps,
                        cfg.rope_base, cfg.lr, cfg.beta1, cfg.beta2, cfg.adam_eps, cfg.weight_decay,
                        int(getattr(cfg, "offload_acts", 0)))


def _check(code, handle=None):
    if code != STAGE_OK:
        raise StageError(code, (lib().stage_last_error(handle) or b"").decode())


def query(cc: StageConfigC):
    """-> (n_params, dict of memory terms in bytes, n_segments); raises StageError on a bad config."""
    n, mem, ns = C.c_int64(), StageMemoryC(), C.c_int32()
    _check(lib().stage_query(C.byref(cc), C.byref(n), C.byref(mem), C.byref(ns)))
    return n.value, {k: getattr(mem, k) for k, _ in StageMemoryC._fields_}, ns.value


def fit_linear(x, y):
    """Least-squares line through (x, y) by the library (stage_fit_linear) -> (intercept, slope, r2)."""
    n = len(x)
    xa, ya, out = (C.c_double * n)(*x), (C.c_double * n)(*y), StageLinearFitC()
    _check(lib().stage_fit_linear(xa, ya, n, C.byref(out)))
    return out.intercept, out.slope, out.r2


def loss_scale_update(scale, good_steps, found_inf, backoff=0.5, growth=2.0, growth_interval=2000):
    """The library's dynamic loss-scaling rule (stage_loss_scale_update) -> (scale, good_steps)."""
    sc, gd = C.c_float(scale), C.c_int32(good_steps)
    _check(lib().stage_loss_scale_update(C.byref(sc), C.byref(gd), int(bool(found_inf)), backoff, growth, growth_interval))
    return sc.value, gd.value


def layout(cc: StageConfigC):
    _, _, ns = query(cc)
    segs = (StageSegmentC * ns)()
    _check(lib().stage_layout(C.byref(cc), segs, ns))
    return [(s.name.decode(), s.offset, s.rows, s.cols) for s in segs]


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


class Stage:
    """One stage bound to torch device tensors.  The tensors are kept alive by this object."""

    def __init__(self, cc: StageConfigC, params, master, grad_acc, adam_m, adam_v, workspace, stream=None):
        import torch
        self.cc = cc
        self._keep = (params, master, grad_acc, adam_m, adam_v, workspace)
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        h = C.c_void_p()
        _check(lib().stage_init(C.byref(cc), C.c_void_p(self.stream.cuda_stream), _ptr(params), _ptr(master),
                                _ptr(grad_acc), _ptr(adam_m), _ptr(adam_v), _ptr(workspace),
                                workspace.numel() * workspace.element_size(), C.byref(h)))
        self.h = h

    def attach_host_stash(self, host):
        """host: a pinned CPU tensor (torch.empty(..., pin_memory=True)) of at least mem['host_stash'] bytes."""
        self._keep = self._keep + (host,)
        _check(lib().stage_attach_host_stash(self.h, _ptr(host), host.numel() * host.element_size()), self.h)

    def forward(self, mb, x_or_ids, y_out=None, targets=None, loss_out=None):
        _check(lib().stage_forward(self.h, mb, _ptr(x_or_ids), _ptr(y_out), _ptr(targets), _ptr(loss_out)), self.h)

    def backward(self, mb, dy=None, dx_out=None, loss_scale=1.0):
        _check(lib().stage_backward(self.h, mb, _ptr(dy), _ptr(dx_out), loss_scale), self.h)

    def accumulate(self, mb):
        _check(lib().stage_accumulate(self.h, mb), self.h)

    def graph_replayed(self, n_microbatches):
        _check(lib().stage_graph_replayed(self.h, n_microbatches), self.h)

    def optimizer_step(self, t, grad_scale=1.0):
        _check(lib().stage_optimizer_step(self.h, t, grad_scale), self.h)

    def profile(self, enable):
        _check(lib().stage_profile(self.h, 1 if enable else 0), self.h)

    def time_layers(self, x_or_ids, y_out, dy, dx_out, targets=None, loss_out=None, reps=3):
        """-> (forward ms, backward ms) of one microbatch through the whole stage (stage_time_layers)."""
        f, b = C.c_double(), C.c_double()
        _check(lib().stage_time_layers(self.h, _ptr(x_or_ids), _ptr(y_out), _ptr(dy), _ptr(dx_out), _ptr(targets),
                                       _ptr(loss_out), reps, C.byref(f), C.byref(b)), self.h)
        return f.value, b.value

    def profile_read(self):
        out = (StageKernelStatC * 64)()
        n = lib().stage_profile_read(self.h, out, 64)
        if n < 0:
            raise StageError(-n, "stage_profile_read failed")
        return {out[i].name.decode(): dict(launches=out[i].launches, ms=out[i].ms, flops=out[i].flops,
                                           bytes=out[i].bytes) for i in range(n)}

    def close(self):
        if self.h:
            lib().stage_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def ministages_query(cc: StageConfigC, n_ministages: int):
    """-> dict of the sizes and offsets of include/ministages.h's ministages_memory."""
    mc, mem = MinistagesConfigC(cc, n_ministages, 0), MinistagesMemoryC()
    code = lib().ministages_query(C.byref(mc), C.byref(mem))
    if code != STAGE_OK:
        raise StageError(code, (lib().ministages_last_error(None) or b"").decode())
    return {k: getattr(mem, k) for k, _ in MinistagesMemoryC._fields_}


class Ministages:
    """K ministages of one shape sharing two parameter slots on the device (include/ministages.h).
    host: pinned CPU uint8 tensor (the host block, filled by the caller); arena: device uint8 tensor."""

    def __init__(self, cc: StageConfigC, n_ministages, host, arena, stream=None):
        import torch
        self.mc = MinistagesConfigC(cc, n_ministages, 0)
        self._keep = (host, arena)
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        h = C.c_void_p()
        code = lib().ministages_init(C.byref(self.mc), C.c_void_p(self.stream.cuda_stream), _ptr(host), host.numel(),
                                     _ptr(arena), arena.numel(), C.byref(h))
        if code != STAGE_OK:
            raise StageError(code, (lib().ministages_last_error(None) or b"").decode())
        self.h = h

    def _check(self, code):
        if code != STAGE_OK:
            raise StageError(code, (lib().ministages_last_error(self.h) or b"").decode())

    def forward(self, k, mb, x_or_ids, y_out=None, targets=None, loss_out=None):
        self._check(lib().ministages_forward(self.h, k, mb, _ptr(x_or_ids), _ptr(y_out), _ptr(targets), _ptr(loss_out)))

    def backward(self, k, mb, dy=None, dx_out=None, loss_scale=1.0):
        self._check(lib().ministages_backward(self.h, k, mb, _ptr(dy), _ptr(dx_out), loss_scale))

    def accumulate(self, k, mb):
        self._check(lib().ministages_accumulate(self.h, k, mb))

    def optimizer_step(self, k, t, grad_scale=1.0):
        self._check(lib().ministages_optimizer_step(self.h, k, t, grad_scale))

    def traffic(self):
        a, b = C.c_int64(), C.c_int64()
        self._check(lib().ministages_traffic(self.h, C.byref(a), C.byref(b)))
        return a.value, b.value

    def stage_profile(self, k, enable):
        _check(lib().stage_profile(lib().ministages_stage(self.h, k), 1 if enable else 0))

    def stage_profile_read(self, k):
        out = (StageKernelStatC * 64)()
        n = lib().stage_profile_read(lib().ministages_stage(self.h, k), out, 64)
        if n < 0:
            raise StageError(-n, "stage_profile_read failed")
        return {out[i].name.decode(): dict(launches=out[i].launches, ms=out[i].ms, flops=out[i].flops,
                                           bytes=out[i].bytes) for i in range(n)}

    def close(self):
        if self.h:
            lib().ministages_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class _Ops:
    """Single-kernel entry points (stage_op_*), same names as in include/stage_ops.h."""

    def __getattr__(self, name):
        fn = getattr(lib(), "stage_op_" + name)

        def call(*args):
            conv = [(_ptr(a) if hasattr(a, "data_ptr") else a) for a in args]
            code = fn(*conv)
            if code != STAGE_OK:
                raise StageError(code, f"stage_op_{name}")
        return call


ops = _Ops()


def wgrad_parts_scratch_bytes(M, N, K_each, K_last, nparts, batch=1):
    """stage_op_wgrad_parts_scratch_bytes (host only)."""
    n = lib().stage_op_wgrad_parts_scratch_bytes(M, N, K_each, K_last, nparts, batch)
    if n < 0:
        raise StageError(-n, "stage_op_wgrad_parts_scratch_bytes")
    return n


def wgrad_parts_cut(stream, dtype, M, N, K_each, K_last, A_parts, lda, B_parts, ldb, Cbuf, ldc, batch=1, sA=0, sB=0, sC=0,
                    scratch=None, scratch_bytes=0):
    """stage_op_wgrad_parts_cut with lists of device tensors for the parts."""
    n = len(A_parts)
    pa = (C.c_void_p * n)(*[t.data_ptr() for t in A_parts])
    pb = (C.c_void_p * n)(*[t.data_ptr() for t in B_parts])
    code = lib().stage_op_wgrad_parts_cut(stream, dtype, M, N, K_each, K_last, n, pa, lda, pb, ldb, _ptr(Cbuf), ldc, batch, sA, sB, sC,
                                          _ptr(scratch), scratch_bytes)
    if code != STAGE_OK:
        raise StageError(code, "stage_op_wgrad_parts_cut")


def wgrad_parts(stream, dtype, M, N, K_each, K_last, A_parts, lda, B_parts, ldb, Cbuf, ldc, batch=1, sA=0, sB=0, sC=0, impl=0):
    """stage_op_wgrad_parts with lists of device tensors for the parts."""
    n = len(A_parts)
    pa = (C.c_void_p * n)(*[t.data_ptr() for t in A_parts])
    pb = (C.c_void_p * n)(*[t.data_ptr() for t in B_parts])
    code = lib().stage_op_wgrad_parts(stream, dtype, M, N, K_each, K_last, n, pa, lda, pb, ldb, _ptr(Cbuf), ldc, batch, sA, sB, sC, impl)
    if code != STAGE_OK:
        raise StageError(code, "stage_op_wgrad_parts")
