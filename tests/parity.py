"""Shared helpers of the GPU parity tests: build device buckets and oracle buckets from the
same seeded inputs, run both, compare to the stated tolerances.

Tolerances (from the benchmark spec): fp32 p, m, v  |a-b| <= max(1e-6 |b|, 1e-9);
bf16 working copy within 1 ulp; gradient norm relative 1e-5; counts, flags and rollback
bit-exact."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import synth

REL, ABS = 1e-6, 1e-9
# The stated tolerance of the gradient norm is 1e-5 relative.  Both sides accumulate exact
# products in fp64 and differ only in summation order, which leaves ~1e-13; the tests hold the
# library to 1e-10, so that a float accumulator sneaking in would be noticed.
NORM_REL = 1e-10


def bits16(t: torch.Tensor) -> np.ndarray:
    """uint16 bit patterns of a bf16/fp16 tensor (copied to the host)."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16).copy()


def dtype_code(t: torch.Tensor) -> int:
    return oracle.GRAD_FP16 if t.dtype == torch.float16 else oracle.GRAD_BF16


class DevBucket:
    """Device arrays of one bucket + the so_bucket that describes them."""

    def __init__(self, B, p0: torch.Tensor, grad_dtype=torch.bfloat16, alt=False, m0=None, v0=None,
                 device="cuda", lp_dtype=torch.bfloat16):
        n = p0.numel()
        self.n = n
        self.p = p0.to(device).clone()
        self.m = torch.zeros(n, dtype=torch.float32, device=device) if m0 is None else m0.to(device).clone()
        self.v = torch.zeros(n, dtype=torch.float32, device=device) if v0 is None else v0.to(device).clone()
        self.q = torch.zeros(n, dtype=lp_dtype, device=device)
        self.g = torch.zeros(n, dtype=grad_dtype, device=device)
        self.alt = None
        if alt:
            self.alt = [torch.full((n,), float("nan"), dtype=torch.float32, device=device) for _ in range(3)]
            self.alt.append(torch.zeros(n, dtype=lp_dtype, device=device))
        self.B = B
        self.c = B.bucket_of(self.g, self.p, self.m, self.v, self.q, self.alt)
        self._by_ptr = {t.data_ptr(): t for t in [self.p, self.m, self.v, self.q] + (self.alt or [])}

    def current(self):
        """(p, m, v, q) tensors that the so_bucket currently names (they swap on commit)."""
        if self.n == 0:
            return self.p, self.m, self.v, self.q
        c = self.c
        return (self._by_ptr[c.param], self._by_ptr[c.exp_avg], self._by_ptr[c.exp_avg_sq],
                self._by_ptr[c.param_lp])

    def host_state(self):
        p, m, v, q = self.current()
        return (p.cpu().numpy(), m.cpu().numpy(), v.cpu().numpy(), bits16(q))


def ordered16(bits: np.ndarray) -> np.ndarray:
    """Map 16-bit float patterns to integers ordered like the values (for ulp distance)."""
    b = bits.astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7FFF), b)


def compare_state(dev_state, ob: "oracle.Bucket", what="", lp=torch.bfloat16, sharp=True):
    """Element-by-element comparison of a device bucket with an oracle bucket.

    Stated tolerance: |a - b| <= max(1e-6 |b|, 1e-9).  With gradients of the workloads' scale
    (1e-3) the moments are small -- m ~ 1e-4, v ~ 1e-9 -- and the absolute floor of 1e-9 alone
    would accept any v at all.  `sharp` therefore also holds m and v to
    |a - b| <= 1e-6 max(|b|, rms(b)): relative to the element, or, where an element of m nearly
    cancels, relative to the typical magnitude of the array."""
    p, m, v, q = dev_state
    worst = {}
    for name, a, b in (("p", p, ob.p), ("m", m, ob.m), ("v", v, ob.v)):
        assert a.shape == b.shape
        a64, b64 = a.astype(np.float64), b.astype(np.float64)
        assert np.all(np.isfinite(a64)), f"{what}{name}: non-finite on device"
        err = np.abs(a64 - b64)
        tol = np.maximum(REL * np.abs(b64), ABS)
        bad = err > tol
        if bad.any():
            i = int(np.argmax(err - tol))
            raise AssertionError(f"{what}{name}[{i}]: device {a[i]!r} oracle {b[i]!r} "
                                 f"err {err[i]:.3e} tol {tol[i]:.3e} ({int(bad.sum())} bad)")
        with np.errstate(divide="ignore", invalid="ignore"):
            rel = np.where(np.abs(b64) > 0, err / np.abs(b64), 0.0)
        worst[name] = float(rel[err > ABS].max()) if (err > ABS).any() else 0.0
        if name != "p" and b64.size:
            rms = float(np.sqrt(np.mean(b64 * b64)))
            scale = np.maximum(np.abs(b64), rms)
            if rms == 0.0:
                assert not err.any(), f"{what}{name}: oracle is all zero, device is not"
                worst[name + "_sharp"] = 0.0
                continue
            ratio = err / scale
            worst[name + "_sharp"] = float(ratio.max())
            if sharp and worst[name + "_sharp"] > REL:
                i = int(np.argmax(ratio))
                raise AssertionError(f"{what}{name}[{i}]: device {a[i]!r} oracle {b[i]!r} err {err[i]:.3e} "
                                     f"exceeds 1e-6 x max(|oracle|, rms {rms:.3e})")
    # the working copy is exactly the round-to-nearest-even 16-bit value of the device's own p
    q_from_p = bits16(torch.from_numpy(p).to(lp))
    assert np.array_equal(q, q_from_p), f"{what}q is not the 16-bit rounding of p"
    # ... and within 1 bf16 ulp of the oracle's; next to zero, where the fp32 comparison
    # itself falls back to its absolute floor, the same floor applies to the values
    dq = np.abs(ordered16(q) - ordered16(ob.q))
    if lp == torch.bfloat16:
        qv = (q.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        ov = (ob.q.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    else:
        qv = q.view(np.float16).astype(np.float64)
        ov = ob.q.view(np.float16).astype(np.float64)
    with np.errstate(invalid="ignore"):                 # inf - inf where both copies overflowed
        badq = (dq > 1) & (np.abs(qv - ov) > ABS * (1 + 2.0 ** -7))
    if badq.any():
        i = int(np.argmax(badq))
        raise AssertionError(f"{what}q[{i}]: device {q[i]:#06x} oracle {ob.q[i]:#06x} "
                             f"(p device {p[i]!r} oracle {ob.p[i]!r}); {int(badq.sum())} bad")
    # how many elements are more than 1 ulp apart and were accepted only because the two values
    # agree within the absolute floor (next to zero an ulp is far smaller than the floor)
    worst["q_beyond_1ulp_within_abs_floor"] = int((dq > 1).sum())
    worst["q_ulp"] = int(dq.max(initial=0))
    worst["q_mismatch_frac"] = float((dq > 0).mean()) if dq.size else 0.0
    return worst


def assert_bits_equal(a: torch.Tensor, b: torch.Tensor, what=""):
    """Bit-for-bit equality of two tensors of the same dtype (NaNs included)."""
    assert a.dtype == b.dtype and a.numel() == b.numel(), what
    ia = a.contiguous().view(torch.int32 if a.element_size() == 4 else torch.int16)
    ib = b.contiguous().view(torch.int32 if b.element_size() == 4 else torch.int16)
    assert torch.equal(ia, ib), f"{what}: bit patterns differ"


def gen_params(cfg, start, n, device):
    return synth.normal_f32(cfg["seed"], synth.STREAM_PARAM, 0, start, n, cfg["sigma_p"], device)


def gen_grads(cfg, step, start, n, device, loss_scale=1.0):
    dt = torch.float16 if cfg["grad_dtype"] == "fp16" else torch.bfloat16
    return synth.normal_16bit(cfg["seed"], synth.STREAM_GRAD, step, start, n,
                              cfg["sigma_g"] * loss_scale, dt, device)


def bucket_ranges(total, bucket):
    return [(s, min(bucket, total - s)) for s in range(0, total, bucket)]
