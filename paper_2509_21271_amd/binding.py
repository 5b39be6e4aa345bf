"""ctypes binding of libso_adam.so: same names as include/so_adam.h, marshalling only."""
from __future__ import annotations

import ctypes as C
import os

from .build import LIB

# PyTorch-ROCm ships its own copy of the HIP runtime.  Callers hand this library torch's
# device pointers and streams, so both must live in ONE runtime: load torch's first, and the
# dynamic loader resolves libso_adam.so's dependency on libamdhip64 to the copy already there.
try:
    import torch  # noqa: F401
except ImportError:      # pure C-ABI use without torch: the system HIP runtime is used
    pass

if not os.path.exists(LIB):
    raise ImportError(
        f"{LIB} is missing: build it first (python -m paper_2509_21271_amd.build, or "
        "__graft_entry__.build()).  There is no fallback path.")

_lib = C.CDLL(LIB)

SO_OK = 0
SO_ERR_INVALID_ARG, SO_ERR_ALIGNMENT, SO_ERR_STATE, SO_ERR_OOM, SO_ERR_HIP, SO_ERR_UNSUPPORTED = \
    -1, -2, -3, -4, -5, -6
SO_GRAD_BF16, SO_GRAD_FP16 = 0, 1
SO_LP_BF16, SO_LP_FP16 = 0, 1
SO_SYNC, SO_SPEC_PINGPONG, SO_SPEC_SAVE = 0, 1, 2
SO_COMMIT, SO_ROLLBACK_SKIP, SO_ROLLBACK_REDO = 0, 1, 2


class so_bucket(C.Structure):
    _fields_ = [("grad", C.c_void_p), ("param", C.c_void_p), ("exp_avg", C.c_void_p),
                ("exp_avg_sq", C.c_void_p), ("param_lp", C.c_void_p),
                ("alt_param", C.c_void_p), ("alt_exp_avg", C.c_void_p),
                ("alt_exp_avg_sq", C.c_void_p), ("alt_param_lp", C.c_void_p),
                ("n", C.c_uint64), ("grad_dtype", C.c_int32), ("pending", C.c_int32),
                ("lp_dtype", C.c_int32), ("reserved", C.c_int32)]


class so_hparams(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("weight_decay", C.c_float), ("adamw", C.c_int32),
                ("bias_correction", C.c_int32)]


class so_stats(C.Structure):
    _fields_ = [("sumsq", C.c_double), ("norm", C.c_double), ("nonfinite", C.c_uint64),
                ("overflow", C.c_int32), ("reserved", C.c_int32)]


class so_decision(C.Structure):
    _fields_ = [("action", C.c_int32), ("reserved", C.c_int32), ("clip", C.c_double),
                ("grad_scale", C.c_float), ("next_loss_scale", C.c_float)]


class so_slice(C.Structure):
    _fields_ = [("tensor", C.c_uint64), ("tensor_offset", C.c_uint64), ("bucket", C.c_uint64),
                ("bucket_offset", C.c_uint64), ("len", C.c_uint64)]


class so_arena_alt(C.Structure):
    _fields_ = [("param", C.c_uint64), ("exp_avg", C.c_uint64), ("exp_avg_sq", C.c_uint64),
                ("param_lp", C.c_uint64)]


class so_arena_layout(C.Structure):
    _fields_ = [("bytes", C.c_uint64), ("param", C.c_uint64), ("grad", C.c_uint64), ("exp_avg", C.c_uint64),
                ("param_lp", C.c_uint64), ("exp_avg_sq", C.c_uint64)]


class so_stream_report(C.Structure):
    _fields_ = [("total_ms", C.c_double), ("h2d_gbps", C.c_double), ("d2h_gbps", C.c_double),
                ("kernel_ms", C.c_double), ("buckets", C.c_uint64)]


class so_stream_state(C.Structure):
    _fields_ = [("host_param", C.c_void_p), ("host_exp_avg", C.c_void_p),
                ("host_exp_avg_sq", C.c_void_p), ("grad", C.c_void_p), ("param_lp", C.c_void_p),
                ("n_total", C.c_uint64), ("bucket_elems", C.c_uint64),
                ("grad_dtype", C.c_int32), ("lp_dtype", C.c_int32),
                ("staging", C.c_void_p), ("staging_bytes", C.c_uint64)]


_P = C.POINTER
_ctx = C.c_void_p
_sig = {
    "so_version": (C.c_char_p, []),
    "so_create": (C.c_int, [_P(_ctx), C.c_int, C.c_void_p]),
    "so_destroy": (C.c_int, [_ctx]),
    "so_set_stream": (C.c_int, [_ctx, C.c_void_p]),
    "so_last_error": (C.c_char_p, [_ctx]),
    "so_set_limits": (C.c_int, [_ctx, C.c_uint64, C.c_uint32]),
    "so_set_profiling": (C.c_int, [_ctx, C.c_int]),
    "so_read_step_kernel_ms": (C.c_int, [_ctx, _P(C.c_double), C.c_size_t, _P(C.c_size_t)]),
    "so_layout_plan": (C.c_int, [_P(C.c_uint64), C.c_size_t, C.c_uint64, _P(so_slice), C.c_size_t,
                                 _P(C.c_size_t), _P(C.c_uint64)]),
    "so_arena_plan": (C.c_int, [C.c_uint64, _P(so_arena_layout)]),
    "so_arena_candidate": (C.c_int, [C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint32, _P(so_arena_layout),
                                     _P(so_arena_alt)]),
    "so_arena_tune": (C.c_int, [_ctx, C.c_void_p, C.c_uint64, C.c_uint64, C.c_int, C.c_uint32, C.c_uint64,
                                _P(so_arena_layout), _P(so_arena_alt), _P(C.c_double), _P(C.c_double)]),
    "so_flatten": (C.c_int, [_ctx, _P(so_slice), C.c_size_t, _P(C.c_void_p), _P(C.c_void_p),
                             C.c_int, C.c_int]),
    "so_flatten_grad_stats": (C.c_int, [_ctx, _P(so_slice), C.c_size_t, _P(C.c_void_p), _P(C.c_void_p),
                                        C.c_int, C.c_float, C.c_float]),
    "so_grad_stats": (C.c_int, [_ctx, _P(so_bucket), C.c_size_t, C.c_float, _P(so_stats)]),
    "so_grad_stats_static": (C.c_int, [_P(so_bucket), C.c_size_t, C.c_float, C.c_void_p, C.c_void_p]),
    "so_grad_stats_enqueue": (C.c_int, [_ctx, _P(so_bucket), C.c_size_t, C.c_float, C.c_float]),
    "so_grad_stats_fetch": (C.c_int, [_ctx, _P(so_stats), _P(so_decision)]),
    "so_validate": (C.c_int, [_P(so_stats), C.c_double, C.c_double, C.c_double, _P(so_decision)]),
    "so_train_reset": (C.c_int, [_ctx, _P(so_hparams), C.c_int64, C.c_float, C.c_float, C.c_float, C.c_uint32,
                                 C.c_float]),
    "so_train_iteration": (C.c_int, [_ctx, _P(so_bucket), C.c_size_t]),
    "so_train_capture": (C.c_int, [_ctx, _P(so_bucket), C.c_size_t]),
    "so_train_replay": (C.c_int, [_ctx]),
    "so_train_fetch": (C.c_int, [_ctx, _P(so_stats), _P(so_decision), _P(C.c_int64), _P(C.c_float)]),
    "so_loss_scale_next": (C.c_int, [C.c_float, C.c_int, _P(C.c_uint32), C.c_uint32, C.c_float, C.c_float,
                                     _P(C.c_float)]),
    "so_adam_step": (C.c_int, [_ctx, _P(so_bucket), _P(so_hparams), C.c_int64, C.c_float, C.c_int]),
    "so_adam_step_multi": (C.c_int, [_ctx, _P(so_bucket), C.c_size_t, _P(so_hparams), C.c_int64,
                                     C.c_float, C.c_int]),
    "so_adam_step_groups": (C.c_int, [_ctx, _P(so_bucket), C.c_size_t, _P(so_hparams), C.c_int64,
                                      C.c_float, C.c_int]),
    "so_adam_step_guarded": (C.c_int, [_ctx, _P(so_bucket), C.c_size_t, _P(so_hparams), C.c_int64]),
    "so_adam_step_stats": (C.c_int, [_ctx, _P(so_stats)]),
    "so_adam_commit": (C.c_int, [_ctx, _P(so_bucket)]),
    "so_adam_rollback": (C.c_int, [_ctx, _P(so_bucket)]),
    "so_plan_resident": (C.c_int, [C.c_double] * 5 + [C.c_uint64, C.c_uint64, _P(C.c_uint64)]),
    "so_pinned_alloc": (C.c_int, [C.c_size_t, _P(C.c_void_p)]),
    "so_pinned_free": (C.c_int, [C.c_void_p]),
    "so_stream_step": (C.c_int, [_ctx, _P(so_stream_state), _P(so_hparams), C.c_int64, C.c_float,
                                 _P(so_stream_report)]),
    "so_hybrid_step": (C.c_int, [_ctx, _P(so_stream_state), _P(so_bucket), C.c_size_t, _P(so_hparams),
                                 C.c_int64, C.c_float, _P(so_stream_report), _P(C.c_double)]),
    "so_cast_params": (C.c_int, [_ctx, C.c_void_p, C.c_void_p, C.c_uint64, C.c_int]),
    "so_stream_cast_params": (C.c_int, [_ctx, C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint64, C.c_int,
                                        _P(C.c_double)]),
}
for _name, (_res, _args) in _sig.items():
    _f = getattr(_lib, _name)
    _f.restype = _res
    _f.argtypes = _args

EXPORTS = tuple(_sig)


class SoError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"so_adam status {status}: {message}")
        self.status = status


def _check(ctx, rc):
    if rc != SO_OK:
        msg = _lib.so_last_error(ctx).decode() if ctx else ""
        raise SoError(rc, msg)


def _arr(buckets):
    """Accept one so_bucket, a ctypes array of them, or a Python list (copied in and out)."""
    if isinstance(buckets, so_bucket):
        return C.pointer(buckets), 1, None
    if isinstance(buckets, C.Array):
        return buckets, len(buckets), None
    arr = (so_bucket * len(buckets))(*buckets)
    return arr, len(buckets), buckets


def _writeback(arr, src):
    if src is not None:
        for i, b in enumerate(src):
            C.memmove(C.byref(b), C.byref(arr[i]), C.sizeof(so_bucket))


def so_version() -> str:
    return _lib.so_version().decode()


def so_create(device: int = 0, hip_stream: int | None = None):
    ctx = _ctx()
    rc = _lib.so_create(C.byref(ctx), device, C.c_void_p(hip_stream or 0))
    if rc != SO_OK:
        raise SoError(rc, "so_create failed")
    return ctx


def so_destroy(ctx):
    _check(None, _lib.so_destroy(ctx))


def so_set_stream(ctx, hip_stream):
    _check(ctx, _lib.so_set_stream(ctx, C.c_void_p(hip_stream or 0)))


def so_last_error(ctx) -> str:
    return _lib.so_last_error(ctx).decode()


def so_set_limits(ctx, max_grid_workgroups: int = 0, max_grid_rows: int = 0):
    _check(ctx, _lib.so_set_limits(ctx, max_grid_workgroups, max_grid_rows))


def so_set_profiling(ctx, enable: bool):
    _check(ctx, _lib.so_set_profiling(ctx, int(enable)))


def so_read_step_kernel_ms(ctx, cap: int = 8192):
    buf = (C.c_double * cap)()
    n = C.c_size_t()
    _check(ctx, _lib.so_read_step_kernel_ms(ctx, buf, cap, C.byref(n)))
    return [buf[i] for i in range(n.value)]


def so_layout_plan(tensor_numel, bucket_elems: int):
    """Returns (list of so_slice, number of buckets)."""
    nt = len(tensor_numel)
    numel = (C.c_uint64 * max(nt, 1))(*tensor_numel)
    ns, nb = C.c_size_t(), C.c_uint64()
    rc = _lib.so_layout_plan(numel, nt, bucket_elems, None, 0, C.byref(ns), C.byref(nb))
    if rc != SO_OK:
        raise SoError(rc, "so_layout_plan: invalid argument")
    out = (so_slice * max(ns.value, 1))()
    rc = _lib.so_layout_plan(numel, nt, bucket_elems, out, ns.value, C.byref(ns), C.byref(nb))
    if rc != SO_OK:
        raise SoError(rc, "so_layout_plan: invalid argument")
    return [out[i] for i in range(ns.value)], nb.value


def so_arena_plan(n_total: int) -> so_arena_layout:
    out = so_arena_layout()
    rc = _lib.so_arena_plan(n_total, C.byref(out))
    if rc != SO_OK:
        raise SoError(rc, "so_arena_plan: invalid argument")
    return out


def arena_views(n_total: int, grad_dtype, device="cuda", extra_16bit: int = 0):
    """Marshalling helper: ONE torch allocation carved as so_arena_plan says.  Returns
    (p, g, m, q, v, [extra 16-bit arrays of the gradients' type, after v], owner tensor); m, v
    and q are zeroed, p and g are not."""
    import torch
    lay = so_arena_plan(n_total)
    two_mib = 2 << 20
    a2 = (2 * n_total + two_mib - 1) // two_mib * two_mib
    owner = torch.empty(lay.bytes + extra_16bit * a2, dtype=torch.uint8, device=device)
    base = (owner.data_ptr() + two_mib - 1) // two_mib * two_mib - owner.data_ptr()

    def view(off, width, dt):
        return owner[base + off:base + off + width * n_total].view(dt)
    p, m, v = (view(o, 4, torch.float32) for o in (lay.param, lay.exp_avg, lay.exp_avg_sq))
    g, q = view(lay.grad, 2, grad_dtype), view(lay.param_lp, 2, torch.bfloat16)
    end = lay.bytes - two_mib
    extras = [view(end + k * a2, 2, grad_dtype) for k in range(extra_16bit)]
    m.zero_()
    v.zero_()
    q.zero_()
    return p, g, m, q, v, extras, owner


def so_arena_candidate(n_total: int, workspace_bytes: int, seed: int, index: int, second_set: bool = False):
    """Returns (so_arena_layout, so_arena_alt or None)."""
    out, alt = so_arena_layout(), so_arena_alt()
    rc = _lib.so_arena_candidate(n_total, workspace_bytes, seed, index, C.byref(out),
                                 C.byref(alt) if second_set else None)
    if rc != SO_OK:
        raise SoError(rc, "so_arena_candidate: invalid argument")
    return out, (alt if second_set else None)


def so_arena_tune(ctx, workspace: int, workspace_bytes: int, n_total: int, grad_dtype: int = SO_GRAD_BF16,
                  trials: int = 60, seed: int = 1, second_set: bool = False):
    """workspace: device address.  Returns (so_arena_layout, so_arena_alt or None, tight_ms, tuned_ms)."""
    out, alt = so_arena_layout(), so_arena_alt()
    t0, t1 = C.c_double(), C.c_double()
    _check(ctx, _lib.so_arena_tune(ctx, workspace, workspace_bytes, n_total, grad_dtype, trials, seed,
                                   C.byref(out), C.byref(alt) if second_set else None,
                                   C.byref(t0), C.byref(t1)))
    return out, (alt if second_set else None), t0.value, t1.value


def tuned_arena_views(ctx, n_total: int, grad_dtype, workspace_bytes: int, device="cuda", trials: int = 60,
                      seed: int = 1, second_set: bool = False):
    """Marshalling helper: ONE torch allocation of workspace_bytes with the arenas where
    so_arena_tune puts them.  Returns (p, g, m, q, v, [p', m', v', q'] or None, owner tensor,
    tight_ms, tuned_ms); everything is zero."""
    import torch
    owner = torch.empty(workspace_bytes, dtype=torch.uint8, device=device)
    code = SO_GRAD_FP16 if grad_dtype == torch.float16 else SO_GRAD_BF16
    lay, alt, t0, t1 = so_arena_tune(ctx, owner.data_ptr(), workspace_bytes, n_total, code, trials, seed, second_set)
    owner.zero_()

    def view(off, width, dt):
        return owner[off:off + width * n_total].view(dt)
    p, m, v = (view(o, 4, torch.float32) for o in (lay.param, lay.exp_avg, lay.exp_avg_sq))
    g, q = view(lay.grad, 2, grad_dtype), view(lay.param_lp, 2, torch.bfloat16)
    second = None
    if second_set:
        second = [view(o, 4, torch.float32) for o in (alt.param, alt.exp_avg, alt.exp_avg_sq)] + \
                 [view(alt.param_lp, 2, torch.bfloat16)]
    return p, g, m, q, v, second, owner, t0, t1


def so_flatten(ctx, slices, tensor_ptrs, bucket_ptrs, elem_size: int, direction: int = 0):
    sl = (so_slice * max(len(slices), 1))(*slices)
    tp = (C.c_void_p * max(len(tensor_ptrs), 1))(*tensor_ptrs)
    bp = (C.c_void_p * max(len(bucket_ptrs), 1))(*bucket_ptrs)
    _check(ctx, _lib.so_flatten(ctx, sl, len(slices), tp, bp, elem_size, direction))


def so_flatten_grad_stats(ctx, slices, tensor_ptrs, bucket_ptrs, grad_dtype: int, loss_scale: float = 1.0,
                          max_norm: float = 0.0):
    sl = (so_slice * max(len(slices), 1))(*slices)
    tp = (C.c_void_p * max(len(tensor_ptrs), 1))(*tensor_ptrs)
    bp = (C.c_void_p * max(len(bucket_ptrs), 1))(*bucket_ptrs)
    _check(ctx, _lib.so_flatten_grad_stats(ctx, sl, len(slices), tp, bp, grad_dtype, loss_scale, max_norm))


def so_grad_stats(ctx, buckets, inv_loss_scale: float = 1.0) -> so_stats:
    arr, nb, _ = _arr(buckets)
    out = so_stats()
    _check(ctx, _lib.so_grad_stats(ctx, arr, nb, inv_loss_scale, C.byref(out)))
    return out


def so_grad_stats_static(buckets, inv_loss_scale: float, hip_stream, out_device_ptr: int):
    """Context-free, allocation-free statistics; the so_stats lands in device memory at
    ``out_device_ptr`` when the stream gets there."""
    arr, nb, _ = _arr(buckets)
    rc = _lib.so_grad_stats_static(arr, nb, inv_loss_scale, C.c_void_p(hip_stream or 0), C.c_void_p(out_device_ptr))
    if rc != SO_OK:
        raise SoError(rc, _lib.so_last_error(None).decode())


def so_grad_stats_enqueue(ctx, buckets, loss_scale: float = 1.0, max_norm: float = 0.0):
    arr, nb, _ = _arr(buckets)
    _check(ctx, _lib.so_grad_stats_enqueue(ctx, arr, nb, loss_scale, max_norm))


def so_grad_stats_fetch(ctx):
    st, dec = so_stats(), so_decision()
    _check(ctx, _lib.so_grad_stats_fetch(ctx, C.byref(st), C.byref(dec)))
    return st, dec


def so_validate(stats: so_stats, max_norm: float, loss_scale: float = 1.0,
                min_loss_scale: float = 1.0) -> so_decision:
    dec = so_decision()
    rc = _lib.so_validate(C.byref(stats), max_norm, loss_scale, min_loss_scale, C.byref(dec))
    if rc != SO_OK:
        raise SoError(rc, "so_validate: invalid argument")
    return dec


def so_train_reset(ctx, hp: so_hparams, first_step: int = 1, loss_scale: float = 1.0,
                   min_loss_scale: float = 1.0, max_loss_scale: float = 2.0 ** 24, growth_interval: int = 0,
                   max_norm: float = 0.0):
    _check(ctx, _lib.so_train_reset(ctx, C.byref(hp), first_step, loss_scale, min_loss_scale, max_loss_scale,
                                    growth_interval, max_norm))


def so_train_iteration(ctx, buckets):
    arr, nb, src = _arr(buckets)
    rc = _lib.so_train_iteration(ctx, arr, nb)
    _writeback(arr, src)
    _check(ctx, rc)


def so_train_capture(ctx, buckets):
    arr, nb, src = _arr(buckets)
    rc = _lib.so_train_capture(ctx, arr, nb)
    _writeback(arr, src)
    _check(ctx, rc)


def so_train_replay(ctx):
    _check(ctx, _lib.so_train_replay(ctx))


def so_train_fetch(ctx):
    """Returns (so_stats, so_decision, applied steps, loss scale of the next iteration)."""
    st, dec = so_stats(), so_decision()
    applied, scale = C.c_int64(), C.c_float()
    _check(ctx, _lib.so_train_fetch(ctx, C.byref(st), C.byref(dec), C.byref(applied), C.byref(scale)))
    return st, dec, applied.value, scale.value


def so_loss_scale_next(loss_scale: float, overflow: bool, clean_iterations: int, growth_interval: int,
                       min_loss_scale: float = 1.0, max_loss_scale: float = 2.0 ** 24):
    """Returns (next loss scale, new count of clean iterations)."""
    clean = C.c_uint32(clean_iterations)
    nxt = C.c_float()
    rc = _lib.so_loss_scale_next(loss_scale, int(bool(overflow)), C.byref(clean), growth_interval,
                                 min_loss_scale, max_loss_scale, C.byref(nxt))
    if rc != SO_OK:
        raise SoError(rc, "so_loss_scale_next: invalid argument")
    return nxt.value, clean.value


def so_adam_step(ctx, bucket: so_bucket, hp: so_hparams, step: int, clip_coef: float = 1.0,
                 speculative: int = SO_SYNC):
    _check(ctx, _lib.so_adam_step(ctx, C.byref(bucket), C.byref(hp), step, clip_coef, speculative))


def so_adam_step_multi(ctx, buckets, hp: so_hparams, step: int, clip_coef: float = 1.0,
                       speculative: int = SO_SYNC):
    arr, nb, src = _arr(buckets)
    rc = _lib.so_adam_step_multi(ctx, arr, nb, C.byref(hp), step, clip_coef, speculative)
    _writeback(arr, src)
    _check(ctx, rc)


def so_adam_step_groups(ctx, buckets, hps, step: int, clip_coef: float = 1.0,
                        speculative: int = SO_SYNC):
    arr, nb, src = _arr(buckets)
    assert len(hps) == nb
    hp_arr = (so_hparams * max(nb, 1))(*hps)
    rc = _lib.so_adam_step_groups(ctx, arr, nb, hp_arr, step, clip_coef, speculative)
    _writeback(arr, src)
    _check(ctx, rc)


def so_adam_step_guarded(ctx, buckets, hp: so_hparams, step: int):
    arr, nb, src = _arr(buckets)
    rc = _lib.so_adam_step_guarded(ctx, arr, nb, C.byref(hp), step)
    _writeback(arr, src)
    _check(ctx, rc)


def so_adam_step_stats(ctx) -> so_stats:
    out = so_stats()
    _check(ctx, _lib.so_adam_step_stats(ctx, C.byref(out)))
    return out


def so_adam_commit(ctx, bucket: so_bucket):
    _check(ctx, _lib.so_adam_commit(ctx, C.byref(bucket)))


def so_adam_rollback(ctx, bucket: so_bucket):
    _check(ctx, _lib.so_adam_rollback(ctx, C.byref(bucket)))


def so_plan_resident(move_grad_ms, step_offloaded_ms, move_param_ms, bwd_ms_per_bucket,
                     step_resident_ms_per_bucket, n_buckets, max_resident) -> int:
    n = C.c_uint64()
    rc = _lib.so_plan_resident(move_grad_ms, step_offloaded_ms, move_param_ms, bwd_ms_per_bucket,
                               step_resident_ms_per_bucket, n_buckets, max_resident, C.byref(n))
    if rc != SO_OK:
        raise SoError(rc, "so_plan_resident: invalid argument")
    return n.value


def so_pinned_alloc(nbytes: int) -> int:
    ptr = C.c_void_p()
    rc = _lib.so_pinned_alloc(nbytes, C.byref(ptr))
    if rc != SO_OK:
        raise SoError(rc, f"cannot pin {nbytes} bytes of host memory")
    return ptr.value


def so_pinned_free(ptr: int):
    _check(None, _lib.so_pinned_free(C.c_void_p(ptr)))


class PinnedArray:
    """n fp32 values in page-locked host memory, viewed as a torch CPU tensor (``.t``)."""

    def __init__(self, n: int):
        import numpy as np
        import torch
        self.ptr = so_pinned_alloc(4 * n)
        buf = (C.c_float * n).from_address(self.ptr)
        self.t = torch.from_numpy(np.frombuffer(buf, dtype=np.float32, count=n))

    def free(self):
        if self.ptr:
            self.t = None
            so_pinned_free(self.ptr)
            self.ptr = 0


def so_stream_step(ctx, state: so_stream_state, hp: so_hparams, step: int,
                   clip_coef: float = 1.0) -> so_stream_report:
    rep = so_stream_report()
    _check(ctx, _lib.so_stream_step(ctx, C.byref(state), C.byref(hp), step, clip_coef, C.byref(rep)))
    return rep


def so_hybrid_step(ctx, state: so_stream_state, resident, hp: so_hparams, step: int,
                   clip_coef: float = 1.0):
    """Returns (so_stream_report of the streamed part, resident_ms)."""
    arr, nb, src = _arr(resident)
    rep = so_stream_report()
    ms = C.c_double()
    rc = _lib.so_hybrid_step(ctx, C.byref(state), arr, nb, C.byref(hp), step, clip_coef,
                             C.byref(rep), C.byref(ms))
    _writeback(arr, src)
    _check(ctx, rc)
    return rep, ms.value


def so_cast_params(ctx, param: int, param_lp: int, n: int, lp_dtype: int = SO_LP_BF16):
    """param, param_lp: device addresses."""
    _check(ctx, _lib.so_cast_params(ctx, param, param_lp, n, lp_dtype))


def so_stream_cast_params(ctx, host_param: int, param_lp: int, n: int, chunk_elems: int,
                          lp_dtype: int = SO_LP_BF16) -> float:
    """host_param: host address, param_lp: device address.  Returns the wall time of the pass in ms."""
    ms = C.c_double()
    _check(ctx, _lib.so_stream_cast_params(ctx, host_param, param_lp, n, chunk_elems, lp_dtype, C.byref(ms)))
    return ms.value


# ------------------------------------------------------------------ marshalling helpers
def hparams(lr, beta1, beta2, eps, wd, adamw=1, bias_correction=1) -> so_hparams:
    return so_hparams(lr, beta1, beta2, eps, wd, adamw, bias_correction)


def bucket_of(grad, param, exp_avg, exp_avg_sq, param_lp, alt=None) -> so_bucket:
    """Describe torch device tensors as one so_bucket (addresses only; the tensors stay owned
    by the caller and must outlive the bucket).  ``alt`` = (param, exp_avg, exp_avg_sq,
    param_lp-or-None) tensors of the second state set."""
    import torch
    n = grad.numel()
    assert grad.dtype in (torch.bfloat16, torch.float16)
    assert param_lp.dtype in (torch.bfloat16, torch.float16)
    for t in (param, exp_avg, exp_avg_sq):
        assert t.dtype == torch.float32 and t.numel() == n and t.is_contiguous()
    assert param_lp.numel() == n
    b = so_bucket()
    b.grad, b.param, b.exp_avg, b.exp_avg_sq, b.param_lp = (
        grad.data_ptr(), param.data_ptr(), exp_avg.data_ptr(), exp_avg_sq.data_ptr(),
        param_lp.data_ptr())
    if alt is not None:
        b.alt_param, b.alt_exp_avg, b.alt_exp_avg_sq = (alt[0].data_ptr(), alt[1].data_ptr(),
                                                        alt[2].data_ptr())
        b.alt_param_lp = alt[3].data_ptr() if alt[3] is not None else None
    b.n = n
    b.grad_dtype = SO_GRAD_FP16 if grad.dtype == torch.float16 else SO_GRAD_BF16
    b.lp_dtype = SO_LP_FP16 if param_lp.dtype == torch.float16 else SO_LP_BF16
    b.pending = 0
    return b
