"""CPU oracle for the Adam(W) bucket step -- TEST INFRASTRUCTURE ONLY.

Only tests, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline`` leg may import
this package.  It wraps the scalar C file ``adam_oracle.c`` (compiled with gcc into
``liboracle.so`` next to it) and adds the per-iteration validation protocol of the paper's
speculation-then-validation scheme (Sec. 4.4) in plain Python.  It shares nothing with the
GPU library and never imports it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "adam_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
# tests/test_sanitizers.py points this at an UndefinedBehaviorSanitizer build of the same file
_OVERRIDE = os.environ.get("ORACLE_LIB_OVERRIDE")

GRAD_BF16 = 0
GRAD_FP16 = 1


def build(force: bool = True) -> str:
    """Compile the C oracle with gcc.  No FMA contraction, no fast-math: the file's double
    arithmetic is evaluated exactly as written."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-ffp-contract=off",
               "-fno-fast-math", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if _OVERRIDE is None:
            build(force=False)
        L = ctypes.CDLL(_OVERRIDE or _LIB)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        f32p = ctypes.POINTER(ctypes.c_float)
        L.orc_decode16.restype = ctypes.c_double
        L.orc_decode16.argtypes = [ctypes.c_uint16, ctypes.c_int]
        L.orc_is_nonfinite16.restype = ctypes.c_int
        L.orc_is_nonfinite16.argtypes = [ctypes.c_uint16, ctypes.c_int]
        L.orc_f32_to_bf16.restype = ctypes.c_uint16
        L.orc_f32_to_bf16.argtypes = [ctypes.c_float]
        L.orc_grad_stats.restype = None
        L.orc_grad_stats.argtypes = [u16p, ctypes.c_uint64, ctypes.c_int, ctypes.c_float,
                                     ctypes.POINTER(ctypes.c_double),
                                     ctypes.POINTER(ctypes.c_uint64)]
        L.orc_adamw_step.restype = None
        L.orc_adamw_step.argtypes = [u16p, ctypes.c_int, f32p, f32p, f32p, u16p,
                                     ctypes.c_uint64] + [ctypes.c_float] * 5 + \
                                    [ctypes.c_int64, ctypes.c_float, ctypes.c_int, ctypes.c_int,
                                     ctypes.c_int]
        L.orc_f32_to_fp16.restype = ctypes.c_uint16
        L.orc_f32_to_fp16.argtypes = [ctypes.c_float]
        L.orc_cast_lp.restype = None
        L.orc_cast_lp.argtypes = [f32p, u16p, ctypes.c_uint64, ctypes.c_int]
        L.orc_clip_coef.restype = ctypes.c_double
        L.orc_clip_coef.argtypes = [ctypes.c_double, ctypes.c_double]
        _lib = L
    return _lib


def _u16(a: np.ndarray):
    assert a.dtype == np.uint16 and a.flags.c_contiguous
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def _f32(a: np.ndarray):
    assert a.dtype == np.float32 and a.flags.c_contiguous
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def decode16(bits: int, dtype: int) -> float:
    return lib().orc_decode16(int(bits), dtype)


def is_nonfinite16(bits: int, dtype: int) -> bool:
    return bool(lib().orc_is_nonfinite16(int(bits), dtype))


def f32_to_bf16(x) -> int:
    return int(lib().orc_f32_to_bf16(ctypes.c_float(x)))


def f32_to_fp16(x) -> int:
    return int(lib().orc_f32_to_fp16(ctypes.c_float(x)))


def cast_lp(p: np.ndarray, lp_fp16: int = 0) -> np.ndarray:
    """16-bit working copy (uint16 bit patterns) of a float32 array (Sec. 4.5)."""
    p = np.ascontiguousarray(p, dtype=np.float32)
    q = np.empty(p.shape, dtype=np.uint16)
    lib().orc_cast_lp(_f32(p), _u16(q), p.size, int(lp_fp16))
    return q


def grad_stats(g: np.ndarray, dtype: int, inv_scale=1.0):
    """(sumsq, nonfinite) of one bucket of 16-bit gradient bit patterns (uint16 array)."""
    s = ctypes.c_double()
    c = ctypes.c_uint64()
    lib().orc_grad_stats(_u16(g), g.size, dtype, ctypes.c_float(inv_scale),
                         ctypes.byref(s), ctypes.byref(c))
    return s.value, c.value


def count_nonfinite_blas(g16, chunk=1 << 28) -> int:
    """Number of NaN/Inf elements of a torch CPU bf16/fp16 tensor (library isfinite)."""
    import torch
    flat = g16.reshape(-1)
    bad = 0
    for c0 in range(0, flat.numel(), chunk):
        x = flat[c0:c0 + chunk]
        bad += int(x.numel() - int(torch.isfinite(x).sum()))
    return bad


def grad_stats_blas(g16, inv_scale=1.0, chunk=1 << 26):
    """The same two quantities by their plain definition with library primitives: view the
    16-bit patterns as a torch CPU tensor (bf16 or fp16), widen to double, mask the non-finite
    elements, multiply by inv_scale, square, sum -- chunk by chunk, in index order of the
    chunks.  Used for the global norm of multi-billion-element workloads, where the scalar C
    loop would take minutes; pinned against it in tests/test_oracle_pins.py."""
    import torch
    assert g16.dtype in (torch.bfloat16, torch.float16) and g16.device.type == "cpu"
    s = float(np.float32(inv_scale))
    total, bad = 0.0, 0
    flat = g16.reshape(-1)
    for c0 in range(0, flat.numel(), chunk):
        x = flat[c0:c0 + chunk].to(torch.float64)
        fin = torch.isfinite(x)
        bad += int(x.numel() - int(fin.sum()))
        y = torch.where(fin, x, torch.zeros((), dtype=torch.float64)) * s
        total += float((y * y).sum())
    return total, bad


def grad_stats_threaded(g: np.ndarray, dtype: int, inv_scale=1.0, threads=1, chunk=1 << 22):
    """(sumsq, nonfinite) of a long uint16 array of gradient bit patterns by the scalar C loop:
    the array is cut into chunks of `chunk` elements, each chunk is summed in index order by
    orc_grad_stats (one chunk per host thread at a time), and the chunk sums are added in chunk
    order.  The result does not depend on `threads`."""
    spans = [(c0, min(chunk, g.size - c0)) for c0 in range(0, g.size, chunk)]

    def one(span):
        c0, n = span
        return grad_stats(g[c0:c0 + n], dtype, inv_scale)

    if threads <= 1:
        parts = [one(sp) for sp in spans]
    else:
        with ThreadPoolExecutor(threads) as ex:
            parts = list(ex.map(one, spans))
    sumsq, bad = 0.0, 0
    for s_, c_ in parts:
        sumsq += s_
        bad += c_
    return sumsq, bad


def layout_plan(numel, bucket):
    """Bucket layout by its definition (Sec. 4.3, bucketisation): the tensors are laid back to
    back in one flat index space, and flat index i lives in bucket i // bucket at offset
    i % bucket.  Walks every element; maximal runs that stay inside one tensor and one bucket
    become one slice (tensor, tensor_offset, bucket, bucket_offset, len).  Returns (slices,
    number of buckets).  Pure Python: for small cases only."""
    out, flat = [], 0
    for t, n in enumerate(numel):
        for j in range(n):
            bk, bo = divmod(flat, bucket)
            if out and out[-1][0] == t and out[-1][2] == bk and out[-1][1] + out[-1][4] == j:
                out[-1][4] += 1
            else:
                out.append([t, j, bk, bo, 1])
            flat += 1
    return [tuple(x) for x in out], -(-flat // bucket)


def adamw_step(g, dtype, p, m, v, q, *, lr, beta1, beta2, eps, wd, t, s=1.0, adamw=1,
               bias_correction=1, lp_fp16=0):
    """In-place step of one bucket: p, m, v float32 arrays, q uint16 (bf16 or fp16 bits), g uint16."""
    n = g.size
    assert p.size == n and m.size == n and v.size == n and q.size == n
    lib().orc_adamw_step(_u16(g), dtype, _f32(p), _f32(m), _f32(v), _u16(q), n,
                         ctypes.c_float(lr), ctypes.c_float(beta1), ctypes.c_float(beta2),
                         ctypes.c_float(eps), ctypes.c_float(wd), int(t), ctypes.c_float(s),
                         int(adamw), int(bias_correction), int(lp_fp16))


def clip_coef(norm: float, max_norm: float) -> float:
    return lib().orc_clip_coef(float(norm), float(max_norm))


class Bucket:
    """State of one flat bucket on the host: fp32 p, m, v; bf16 working copy q."""

    def __init__(self, p: np.ndarray):
        self.p = np.ascontiguousarray(p, dtype=np.float32).copy()
        self.m = np.zeros_like(self.p)
        self.v = np.zeros_like(self.p)
        self.q = np.zeros(self.p.size, dtype=np.uint16)

    def snapshot(self):
        return (self.p.copy(), self.m.copy(), self.v.copy(), self.q.copy())

    def restore(self, snap):
        self.p[:], self.m[:], self.v[:], self.q[:] = snap


class Trainer:
    """The per-iteration protocol of Sec. 4.4, written synchronously.

    Each iteration first looks at all gradients: if any is NaN/Inf the iteration has no
    effect on the state (scenario 1: skipped) and the loss scale is halved; otherwise the
    global L2 norm of the unscaled gradients gives the clipping coefficient and every bucket
    takes one Adam(W) step with gradients multiplied by clip / loss_scale.  The step counter
    t advances only when a step is applied.  A speculative schedule that runs the step first
    and rolls it back must leave exactly this state (the scheme is exact)."""

    def __init__(self, buckets, *, lr, beta1, beta2, eps, wd, grad_dtype=GRAD_BF16,
                 max_norm=0.0, loss_scale=1.0, min_loss_scale=1.0, adamw=1,
                 bias_correction=1, threads=1, stats_fn=None, growth_interval=0,
                 max_loss_scale=2.0 ** 24):
        self.buckets = buckets
        self.hp = dict(lr=lr, beta1=beta1, beta2=beta2, eps=eps, wd=wd)
        self.grad_dtype = grad_dtype
        self.max_norm = max_norm
        self.loss_scale = float(loss_scale)
        self.min_loss_scale = float(min_loss_scale)
        # Growth of the loss scale (the paper gives no schedule; the usual one): after
        # `growth_interval` iterations in a row without NaN/Inf the scale doubles.  0 = never.
        self.growth_interval = int(growth_interval)
        self.max_loss_scale = float(max_loss_scale)
        self.clean = 0
        self.adamw = adamw
        self.bias_correction = bias_correction
        self.t = 1
        self.threads = threads
        self.stats_fn = stats_fn       # optional: (grads) -> (sumsq, nonfinite), e.g. grad_stats_blas
        self.log = []

    def _map(self, fn, items):
        if self.threads <= 1:
            return [fn(x) for x in items]
        with ThreadPoolExecutor(self.threads) as ex:
            return list(ex.map(fn, items))

    def stats(self, grads):
        """Global (sumsq, nonfinite, norm) over the per-bucket gradient arrays."""
        inv = np.float32(1.0 / self.loss_scale)
        if self.stats_fn is not None:
            sumsq, bad = self.stats_fn(grads, inv)
            return sumsq, bad, float(np.sqrt(sumsq))
        parts = self._map(lambda g: grad_stats(g, self.grad_dtype, inv), grads)
        sumsq = 0.0
        bad = 0
        for s, c in parts:              # bucket order
            sumsq += s
            bad += c
        return sumsq, bad, float(np.sqrt(sumsq))

    def scale_for(self, norm):
        """fp32 multiplier handed to the step: clip coefficient / loss scale."""
        clip = clip_coef(norm, self.max_norm)
        return np.float32(clip / self.loss_scale), clip

    def iteration(self, grads, only=None):
        """Run one iteration.  ``grads``: one uint16 array per bucket.  ``only``: optional
        set of bucket indices whose state is carried (the norm always uses all gradients)."""
        sumsq, bad, norm = self.stats(grads)
        if bad > 0:
            self.loss_scale = max(self.loss_scale * 0.5, self.min_loss_scale)
            self.clean = 0
            self.log.append(dict(applied=False, nonfinite=bad, norm=None, clip=None,
                                 loss_scale=self.loss_scale, t=self.t))
            return False
        s, clip = self.scale_for(norm)

        def one(i):
            b = self.buckets[i]
            if b is None:
                return
            adamw_step(grads[i], self.grad_dtype, b.p, b.m, b.v, b.q, t=self.t, s=s,
                       adamw=self.adamw, bias_correction=self.bias_correction, **self.hp)

        idx = [i for i in range(len(grads)) if only is None or i in only]
        self._map(one, idx)
        self.log.append(dict(applied=True, nonfinite=0, norm=norm, clip=clip, s=float(s),
                             loss_scale=self.loss_scale, t=self.t))
        self.t += 1
        self.clean += 1
        if self.growth_interval and self.clean >= self.growth_interval:
            self.loss_scale = min(self.loss_scale * 2.0, self.max_loss_scale)
            self.clean = 0
        return True
