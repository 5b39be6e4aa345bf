"""The benchmark workloads at full size, in the launch configuration bench.py times, against
the CPU oracle: every element where the oracle finishes in seconds (workload 1), sampled
buckets plus size-independent properties where it does not (workloads 2 and 3)."""
import math

import numpy as np
import pytest
import torch

import oracle
import synth
from parity import (assert_bits_equal, bits16, bucket_ranges, compare_state, gen_grads, gen_params,
                    NORM_REL)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2509_21271_amd import binding
    return binding


@pytest.fixture()
def ctx(B):
    c = B.so_create(0, torch.cuda.current_stream().cuda_stream)
    yield c
    B.so_destroy(c)
    torch.cuda.empty_cache()


def make_say(capsys):
    """Progress lines that reach the terminal even when pytest captures output: the full-size
    tests run for minutes, and a harness that watches for silence must see them alive."""
    def say(*args, **_):
        with capsys.disabled():
            print(*args, flush=True)
    return say


class Arena:
    """Flat arenas, one per array kind, cut into buckets (the layout bench.py uses)."""

    def __init__(self, B, cfg, total, alt=False, one_allocation=False, tuned_ctx=None):
        self.B, self.cfg, self.total = B, cfg, total
        self.ranges = bucket_ranges(total, cfg["bucket"])
        dev = "cuda"
        gdt = torch.float16 if cfg["grad_dtype"] == "fp16" else torch.bfloat16
        second = None
        if tuned_ctx is not None:   # bench.py --config 2: both state sets where so_arena_tune puts them
            ws = int(B.so_arena_plan(total).bytes * 1.75 * 3.0) // (2 << 20) * (2 << 20)
            (self.p, self.g, self.m, self.q, self.v, second, self.big, self.tight_ms,
             self.tuned_ms) = B.tuned_arena_views(tuned_ctx, total, gdt, ws, dev, trials=60, second_set=alt)
        elif one_allocation:        # bench.py's default: one allocation laid out by so_arena_plan
            self.p, self.g, self.m, self.q, self.v, _, self.big = B.arena_views(total, gdt, dev)
        else:
            self.p = torch.empty(total, dtype=torch.float32, device=dev)
            self.m = torch.zeros(total, dtype=torch.float32, device=dev)
            self.v = torch.zeros(total, dtype=torch.float32, device=dev)
            self.q = torch.zeros(total, dtype=torch.bfloat16, device=dev)
            self.g = torch.empty(total, dtype=gdt, device=dev)
        for s, n in self.ranges:
            self.p[s:s + n] = gen_params(cfg, s, n, dev)
        self.alt = second
        if alt and second is None:
            self.alt = [torch.empty(total, dtype=torch.float32, device=dev) for _ in range(3)]
            self.alt.append(torch.zeros(total, dtype=torch.bfloat16, device=dev))
        self.buckets = []
        for s, n in self.ranges:
            a = [t[s:s + n] for t in self.alt] if alt else None
            self.buckets.append(B.bucket_of(self.g[s:s + n], self.p[s:s + n], self.m[s:s + n],
                                            self.v[s:s + n], self.q[s:s + n], a))
        self.arr = (B.so_bucket * len(self.buckets))(*self.buckets)
        self._by_ptr = {}
        for k, (s, n) in enumerate(self.ranges):
            sets = [(self.p, self.m, self.v, self.q)] + ([tuple(self.alt)] if alt else [])
            for st in sets:
                for t in st:
                    self._by_ptr[t[s:s + n].data_ptr()] = t[s:s + n]

    def fresh_grads(self, step, loss_scale=1.0):
        for s, n in self.ranges:
            self.g[s:s + n] = gen_grads(self.cfg, step, s, n, "cuda", loss_scale)

    def host_state(self, k):
        c = self.arr[k]
        t = [self._by_ptr[x] for x in (c.param, c.exp_avg, c.exp_avg_sq, c.param_lp)]
        return (t[0].cpu().numpy(), t[1].cpu().numpy(), t[2].cpu().numpy(), bits16(t[3]))

    def current(self, k):
        c = self.arr[k]
        return [self._by_ptr[x] for x in (c.param, c.exp_avg, c.exp_avg_sq, c.param_lp)]


CHUNK = 1 << 22


class Sampled:
    """Oracle state of a few sampled buckets, cut into 4 Mi-element chunks so that the scalar
    oracle can be spread over the host threads (each chunk is an independent oracle bucket)."""

    def __init__(self, arena, sample):
        self.arena, self.sample = arena, sample
        self.spans = []                      # (bucket k, global start, length)
        for k in sample:
            s, n = arena.ranges[k]
            for c0 in range(0, n, CHUNK):
                self.spans.append((k, s + c0, min(CHUNK, n - c0)))
        self.buckets = [oracle.Bucket(arena.p[s:s + n].cpu().numpy()) for _, s, n in self.spans]

    def grads(self):
        return [bits16(self.arena.g[s:s + n]) for _, s, n in self.spans]

    def joined(self, k):
        """One oracle.Bucket-like object for bucket k (concatenated chunks)."""
        parts = [b for (kk, _, _), b in zip(self.spans, self.buckets) if kk == k]
        out = oracle.Bucket(np.concatenate([b.p for b in parts]))
        out.m = np.concatenate([b.m for b in parts])
        out.v = np.concatenate([b.v for b in parts])
        out.q = np.concatenate([b.q for b in parts])
        return out


@pytest.mark.timeout(300)
def test_one_bucket_longer_than_2_32_elements(B, ctx, capsys):
    """ONE bucket of 2^32 + 2^20 + 77 elements (no workload has one; workload 3 reaches 8 x 10^9
    only as a merged range of 81 buckets): the statistics pass against a closed form with NaN and
    infinities planted on both sides of index 2^32, then two steps against the oracle on windows
    at the start, across index 2^32 and at the ragged end.  Speculative (save-mode) step too: its
    by-product statistics must give the same closed form, its rollback the old bits."""
    say = make_say(capsys)
    n = (1 << 32) + (1 << 20) + 77
    dev = "cuda"
    g = torch.full((n,), 2.0 ** -8, dtype=torch.bfloat16, device=dev)
    bad = {5: float("nan"), (1 << 32) + 123: float("inf"), n - 1: float("-inf")}
    for i, x in bad.items():
        g[i] = x
    p = torch.empty(n, dtype=torch.float32, device=dev)
    for s0 in range(0, n, 1 << 28):
        k = min(1 << 28, n - s0)
        p[s0:s0 + k] = synth.normal_f32(41, synth.STREAM_PARAM, 0, s0, k, 0.02, dev)
    m = torch.zeros(n, dtype=torch.float32, device=dev)
    v = torch.zeros(n, dtype=torch.float32, device=dev)
    q = torch.zeros(n, dtype=torch.bfloat16, device=dev)
    bk = B.bucket_of(g, p, m, v, q)
    st = B.so_grad_stats(ctx, [bk], 0.5)
    assert st.nonfinite == 3 and st.overflow == 1
    assert st.sumsq == (n - 3) * 2.0 ** -18, (st.sumsq, (n - 3) * 2.0 ** -18)      # exact: equal dyadic terms
    say(f"statistics over one bucket of {n} elements: exact")
    for i in bad:
        g[i] = 2.0 ** -8
    windows = [(0, 4096), ((1 << 32) - 2048, 4096), (n - 4096 - 77, 4096 + 77)]
    obs = []
    for w, (s0, k) in enumerate(windows):
        g[s0:s0 + k] = synth.normal_16bit(41, synth.STREAM_GRAD, w, s0, k, 1e-3, torch.bfloat16, dev)
        obs.append(oracle.Bucket(p[s0:s0 + k].cpu().numpy()))
    gw = [bits16(g[s0:s0 + k]) for s0, k in windows]
    hp = B.hparams(**{**dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, wd=0.01)})
    for t in (1, 2):
        B.so_adam_step(ctx, bk, hp, t, 0.37)
        for ob, gb in zip(obs, gw):
            oracle.adamw_step(gb, oracle.GRAD_BF16, ob.p, ob.m, ob.v, ob.q, t=t, s=np.float32(0.37),
                              lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, wd=0.01)
    torch.cuda.synchronize()
    for (s0, k), ob in zip(windows, obs):
        state = (p[s0:s0 + k].cpu().numpy(), m[s0:s0 + k].cpu().numpy(), v[s0:s0 + k].cpu().numpy(),
                 bits16(q[s0:s0 + k]))
        compare_state(state, ob, f"window at {s0}: ")
    say("two steps: windows at 0, across 2^32 and at the end match the oracle")
    # save-mode speculative step: statistics as a by-product, rollback restores the bits
    g.fill_(2.0 ** -8)
    g[(1 << 32) + 7] = float("nan")
    saves = [torch.empty(n, dtype=torch.float32, device=dev) for _ in range(3)]
    spec = B.bucket_of(g, p, m, v, q, saves + [None])
    before = [x[s0:s0 + k].clone() for x in (p, m, v, q) for s0, k in windows]
    B.so_adam_step(ctx, spec, hp, 3, 0.5, B.SO_SPEC_SAVE)
    st = B.so_adam_step_stats(ctx)
    assert st.nonfinite == 1 and st.sumsq == (n - 1) * 2.0 ** -18, (st.nonfinite, st.sumsq)
    B.so_adam_rollback(ctx, spec)
    torch.cuda.synchronize()
    after = [x[s0:s0 + k] for x in (p, m, v, q) for s0, k in windows]
    for x, y in zip(before, after):
        assert_bits_equal(x, y, "rollback beyond 2^32")
    say("save-mode step over the same bucket: by-product statistics exact, rollback bit-exact")


@pytest.mark.timeout(300)
@pytest.mark.parametrize("src_off", [0, 3])
def test_gather_of_one_slice_longer_than_2_32_elements(B, ctx, capsys, src_off):
    """One slice of 2^32 + 2^20 + 77 16-bit gradients gathered with fused statistics, from a
    source aligned with its destination and from one that is 6 bytes off: every element must
    arrive, and the statistics must equal their closed form with NaN / infinities planted on
    both sides of index 2^32."""
    say = make_say(capsys)
    n = (1 << 32) + (1 << 20) + 77
    src = torch.full((n + 8,), 2.0 ** -8, dtype=torch.bfloat16, device="cuda")
    mark = torch.arange(0, n, 1 << 16, device="cuda")                  # a different value every 65,536 elements
    src[mark + src_off] = (mark >> 16).to(torch.float32).mul_(2.0 ** -8).to(torch.bfloat16)
    bad = [9, (1 << 32) - 1, (1 << 32) + 4097, n - 1]
    for k, i in enumerate(bad):
        src[i + src_off] = float("nan") if k % 2 == 0 else float("inf")
    dst = torch.zeros(n + 8, dtype=torch.bfloat16, device="cuda")
    B.so_flatten_grad_stats(ctx, [B.so_slice(0, src_off, 0, 0, n)], [src.data_ptr()], [dst.data_ptr()],
                            B.SO_GRAD_BF16, 2.0, 0.0)
    st, dec = B.so_grad_stats_fetch(ctx)
    assert torch.equal(dst[:n].view(torch.int16), src[src_off:src_off + n].view(torch.int16))
    assert not dst[n:].any(), "wrote past the slice"
    assert st.nonfinite == len(bad) and dec.action == B.SO_ROLLBACK_SKIP
    assert all(i % (1 << 16) for i in bad)                           # no planted value sits on a marked element
    vals = src[mark + src_off].to(torch.float64)                       # the marked values as stored (8-bit mantissas)
    plain = n - mark.numel() - len(bad)
    # every square is a multiple of 2^-16 and the total is below 2^33: all sums are exact in fp64
    want = (plain * 2.0 ** -16 + float((vals * vals).sum())) * 0.25
    assert st.sumsq == want, (st.sumsq, want)
    say(f"gather of one slice of {n} elements, source offset {src_off}: copy bit-exact, statistics {st.sumsq} ~ {want}")


def hp_of(B, cfg):
    h = cfg["hp"]
    return B.hparams(h["lr"], h["beta1"], h["beta2"], h["eps"], h["wd"])


@pytest.mark.timeout(600)
def test_workload1_gpt2_small_every_element(B, ctx, capsys):
    """124,439,808 parameters, 5 buckets of 25 M (last 24,439,808), clipping at 1.0, 20 steps.
    Gradients arrive as per-tensor arrays and are flattened into the buckets (148 tensors that
    straddle bucket boundaries); odd steps run GPU-validated, even steps host-validated."""
    say = make_say(capsys)
    cfg = synth.config(1)
    total = synth.total_params(1)
    assert total == 124_439_808
    A = Arena(B, cfg, total)
    assert len(A.ranges) == 5 and A.ranges[-1][1] == 24_439_808
    numel = [n for _, n in synth.tensor_list(1)]
    slices, nb = B.so_layout_plan(numel, cfg["bucket"])
    assert nb == 5
    offs = np.cumsum([0] + numel)
    orcs = [oracle.Bucket(A.p[s:s + n].cpu().numpy()) for s, n in A.ranges]
    tr = oracle.Trainer(orcs, max_norm=cfg["max_norm"], threads=5, **cfg["hp"])
    hp = hp_of(B, cfg)
    flat = torch.empty(total, dtype=torch.bfloat16, device="cuda")
    norm_rel = 0.0
    for t in range(1, cfg["steps"] + 1):
        for s, n in A.ranges:
            flat[s:s + n] = gen_grads(cfg, t, s, n, "cuda")
        tensors = [flat[offs[i]:offs[i + 1]] for i in range(len(numel))]
        A.g.zero_()
        B.so_flatten(ctx, slices, [x.data_ptr() for x in tensors], [A.g[s:s + n].data_ptr() for s, n in A.ranges], 2, 0)
        if t == 1:
            assert_bits_equal(A.g, flat, "flattened gradients")
        if t % 2:
            B.so_grad_stats_enqueue(ctx, A.arr, 1.0, cfg["max_norm"])
            B.so_adam_step_guarded(ctx, A.arr, hp, t)
            st, dec = B.so_grad_stats_fetch(ctx)
        else:
            st = B.so_grad_stats(ctx, A.arr, 1.0)
            dec = B.so_validate(st, cfg["max_norm"], 1.0, 1.0)
            B.so_adam_step_multi(ctx, A.arr, hp, t, dec.grad_scale)
        assert tr.iteration([bits16(A.g[s:s + n]) for s, n in A.ranges])
        ref = tr.log[-1]
        assert st.overflow == 0 and abs(st.norm - ref["norm"]) <= NORM_REL * ref["norm"]
        assert abs(dec.clip - ref["clip"]) <= 1e-9 and abs(ref["clip"] - 0.0896) < 2e-3
        norm_rel = max(norm_rel, abs(st.norm - ref["norm"]) / ref["norm"])
        if t % 5 == 0:
            say("workload 1 step", t, "norm rel err so far", norm_rel)
    worst = {"norm_rel": norm_rel}
    for k in range(5):
        w = compare_state(A.host_state(k), orcs[k], f"workload 1 bucket {k}: ")
        for key, val in w.items():
            worst[key] = max(worst.get(key, 0), val)
    say("workload 1 worst:", worst)


@pytest.mark.timeout(900)
def test_workload2_speculative_rollback_sampled_buckets(B, ctx, capsys):
    """1,310,986,240 parameters, 27 buckets of 50 M, fp16 gradients x loss scale 2^16, ping-pong
    speculation per bucket; iterations 5, 10, ... are poisoned, rolled back bit for bit and the
    scale halved.  The oracle carries three buckets through all 25 iterations and computes the
    global norm and NaN/Inf count of ALL gradients on each; the count is checked exactly against
    the seeded plan on every poisoned iteration."""
    say = make_say(capsys)
    cfg = synth.config(2)
    total = synth.total_params(2)
    assert total == 1_310_986_240
    A = Arena(B, cfg, total, alt=True, tuned_ctx=ctx)
    say(f"placement tuned: ping-pong step {A.tight_ms:.3f} ms in the tight layout, {A.tuned_ms:.3f} ms where the arenas lie")
    nbk = len(A.ranges)
    assert nbk == 27
    sample = [0, 13, nbk - 1]
    S = Sampled(A, sample)
    tr = oracle.Trainer(S.buckets, grad_dtype=oracle.GRAD_FP16, loss_scale=cfg["loss_scale"], threads=16,
                        **cfg["hp"])
    hp = hp_of(B, cfg)
    scale, t = cfg["loss_scale"], 1
    norm_checked = 0
    for it in range(1, cfg["steps"] + 1):
        A.fresh_grads(it, scale)
        poisoned = cfg["poison_every"] and it % cfg["poison_every"] == 0
        if poisoned:
            plan = synth.poison_plan(cfg["seed"], it, total)
            hits = sum(synth.apply_poison(A.g[s:s + n], s, plan) for s, n in A.ranges)
            assert hits == len(plan) == 132
            distinct = len({pos for pos, _ in plan})
            before = {k: [x.clone() for x in A.current(k)] for k in sample}
        inv = float(np.float32(1.0 / scale))
        for k in range(nbk):                       # speculative step, bucket by bucket
            B.so_adam_step(ctx, A.arr[k], hp, t, inv, B.SO_SPEC_PINGPONG)
        st = B.so_adam_step_stats(ctx)
        dec = B.so_validate(st, cfg["max_norm"], scale, 1.0)
        # oracle side: NaN/Inf count (it decides the skip) and norm from ALL gradients, by the
        # scalar loop, on every iteration
        g_bits = bits16(A.g)
        want_norm = True
        tr.stats_fn = lambda grads, inv_, gb=g_bits: oracle.grad_stats_threaded(gb, oracle.GRAD_FP16, inv_, threads=16)
        applied = tr.iteration(S.grads())
        assert applied == (not poisoned)
        assert (dec.action == B.SO_COMMIT) == applied
        if poisoned:
            assert st.overflow == 1 and st.nonfinite == distinct == tr.log[-1]["nonfinite"]
            for k in range(nbk):
                B.so_adam_rollback(ctx, A.arr[k])
            torch.cuda.synchronize()
            for k in sample:
                for x, y in zip(A.current(k), before[k]):
                    assert_bits_equal(x, y, f"rollback it {it} bucket {k}")
            say("workload 2 iteration", it, "poisoned:", int(st.nonfinite), "NaN/Inf found, rolled back bit for bit")
        else:
            assert st.nonfinite == 0
            if want_norm:
                ref = tr.log[-1]["norm"]
                assert abs(st.norm - ref) <= NORM_REL * ref
                say("workload 2 iteration", it, "norm rel err", abs(st.norm - ref) / ref)
                assert abs(ref / (cfg["sigma_g"] * math.sqrt(total)) - 1) < 2e-3
                norm_checked += 1
            for k in range(nbk):
                B.so_adam_commit(ctx, A.arr[k])
            t += 1
        scale = dec.next_loss_scale
        assert scale == tr.loss_scale and t == tr.t
    assert t == 21 and scale == 2048.0 and norm_checked == 20
    for k in sample:
        w = compare_state(A.host_state(k), S.joined(k), f"workload 2 bucket {k}: ")
        say("workload 2 bucket", k, w)


def _seeded_interior(seed, nbk, count):
    """`count` distinct interior bucket indices (neither first nor last) drawn from the seed."""
    picked, k = [], 0
    while len(picked) < count:
        b = 1 + synth.mix32_int(seed ^ (0x9E3779B9 * (k + 1) & 0xFFFFFFFF)) % (nbk - 2)
        if b not in picked:
            picked.append(b)
        k += 1
    return sorted(picked)


@pytest.mark.timeout(1500)
def test_workload3_llama8b_sampled_buckets(B, ctx, capsys):
    """8,030,261,248 parameters resident in HBM, 81 buckets of 100 M (last 30,261,248), clipping
    at 1.0, the schedule bench.py times (statistics -> GPU-side validation -> guarded step in
    one launch).  All 10 steps at full size: on every step the oracle computes the global norm
    from ALL gradients with its scalar loop (which fixes the clip coefficient), and it carries
    ten buckets -- the first, the last (partial) one and eight seeded interior ones -- element
    by element through all ten steps; all other buckets are covered by properties that hold at
    any size."""
    say = make_say(capsys)
    import time
    cfg = synth.config(3)
    total = synth.total_params(3)
    assert total == 8_030_261_248 and cfg["steps"] == 10
    t_start = time.time()
    A = Arena(B, cfg, total, one_allocation=True)
    nbk = len(A.ranges)
    assert nbk == 81 and A.ranges[-1][1] == 30_261_248
    sample = sorted([0, nbk - 1] + _seeded_interior(cfg["seed"], nbk, 8))
    assert len(sample) == 10
    say("workload 3 sampled buckets:", sample)
    S = Sampled(A, sample)
    tr = oracle.Trainer(S.buckets, max_norm=cfg["max_norm"], threads=16, **cfg["hp"])
    hp = hp_of(B, cfg)
    p0_probe = A.p[5_000_000_000:5_000_001_000].clone()
    assert total % 2 == 0
    g_pin = B.PinnedArray(total // 2)         # exact size (torch's pinned pool rounds up and keeps it)
    g_host = g_pin.t.view(torch.bfloat16)
    g_bits = g_host.view(torch.int16).numpy().view(np.uint16)
    say(f"workload 3 set-up {time.time() - t_start:.0f} s")
    for t in range(1, cfg["steps"] + 1):
        t0 = time.time()
        A.fresh_grads(t)
        B.so_grad_stats_enqueue(ctx, A.arr, 1.0, cfg["max_norm"])
        B.so_adam_step_guarded(ctx, A.arr, hp, t)
        st, dec = B.so_grad_stats_fetch(ctx)
        g_host.copy_(A.g)
        tr.stats_fn = lambda grads, inv_: oracle.grad_stats_threaded(g_bits, oracle.GRAD_BF16, inv_, threads=16)
        assert tr.iteration(S.grads())
        ref = tr.log[-1]
        assert st.overflow == 0 and abs(st.norm - ref["norm"]) <= NORM_REL * ref["norm"]
        assert abs(ref["norm"] - 89.61) < 0.2 and abs(dec.clip - ref["clip"]) <= 1e-9
        assert dec.grad_scale == np.float32(ref["s"])
        say(f"workload 3 step {t}: norm rel err {abs(st.norm - ref['norm']) / ref['norm']:.2e}, "
              f"{time.time() - t0:.0f} s", flush=True)
        if t in (1, cfg["steps"]):
            # additivity: the global sum of squares is the sum over buckets (any size)
            parts = sum(B.so_grad_stats(ctx, A.arr[k], 1.0).sumsq for k in range(0, nbk, 9))
            rest = B.so_grad_stats(ctx, [A.arr[k] for k in range(nbk) if k % 9], 1.0).sumsq
            assert abs(parts + rest - st.sumsq) <= 1e-12 * st.sumsq
    worst = {}
    for k in sample:
        w = compare_state(A.host_state(k), S.joined(k), f"workload 3 bucket {k}: ")
        say("workload 3 bucket", k, w)
        for key, val in w.items():
            worst[key] = max(worst.get(key, 0), val)
    say("workload 3 worst over 10 buckets after 10 steps:", worst)
    # properties over ALL elements: finite, working copy is exactly the bf16 rounding of p,
    # every parameter moved by at most 10 steps of size ~lr, v is non-negative
    for s, n in A.ranges:
        p, v, q = A.p[s:s + n], A.v[s:s + n], A.q[s:s + n]
        assert bool(torch.isfinite(p).all()) and bool((v >= 0).all())
        assert torch.equal(p.to(torch.bfloat16).view(torch.int16), q.view(torch.int16))
    moved = (A.p[5_000_000_000:5_000_001_000] - p0_probe).abs()
    assert 0 < float(moved.max()) < 10 * 1e-4 * 4
    g_host = g_bits = None
    tr.stats_fn = None
    g_pin.free()
    say(f"workload 3 total {time.time() - t_start:.0f} s")


W4_LAYERS = 7      # what bench.py --config 4 runs: 57 GB of pinned state (the machines pin at most 64 GB)


@pytest.mark.timeout(900)
def test_workload4_streamed_state_scaled(B, ctx, capsys):
    """Workload 4's schedule -- fp32 state in pinned host memory streamed through device
    staging slots, gradients and working copy resident -- with its real bucket size (200 M
    elements) at the largest size the test machines can pin: 7 of the 48 layers
    (4,746,995,712 parameters, 57 GB pinned; the full set needs 280 GB).  Three steps; the
    oracle carries the first bucket, an interior one past the first reuse of a staging slot
    (bucket index >= 3) and the last (partial) one.  The staging slots are caller-provided and
    refilled with NaN before every pass, so a missed wait shows up as NaN or stale state."""
    say = make_say(capsys)
    import time
    t_start = time.time()
    cfg = synth.config(4)
    total = synth.total_params(4, layers=W4_LAYERS)
    bucket = cfg["bucket"]
    ranges = bucket_ranges(total, bucket)
    assert total == 4_746_995_712 and len(ranges) == 24
    pinned = [B.PinnedArray(total) for _ in range(3)]
    host = [a.t for a in pinned]
    host[1].zero_()
    host[2].zero_()
    for s, n in ranges:
        host[0][s:s + n].copy_(gen_params(cfg, s, n, "cuda"))
    g = torch.empty(total, dtype=torch.bfloat16, device="cuda")
    q = torch.zeros(total, dtype=torch.bfloat16, device="cuda")
    interior = 3 + synth.mix32_int(cfg["seed"]) % (len(ranges) - 4)
    sample = [0, interior, len(ranges) - 1]
    assert 3 <= interior < len(ranges) - 1
    say("workload 4 sampled buckets:", sample, f"set-up {time.time() - t_start:.0f} s")
    orcs = {}
    for k in sample:                      # oracle state in 4 Mi chunks, one host thread each
        s, n = ranges[k]
        orcs[k] = [(s + c0, min(CHUNK, n - c0), oracle.Bucket(host[0][s + c0:s + c0 + min(CHUNK, n - c0)].numpy()))
                   for c0 in range(0, n, CHUNK)]
    staging = torch.empty(9 * bucket, dtype=torch.float32, device="cuda")
    st = B.so_stream_state()
    st.host_param, st.host_exp_avg, st.host_exp_avg_sq = (h.data_ptr() for h in host)
    st.grad, st.param_lp = g.data_ptr(), q.data_ptr()
    st.n_total, st.bucket_elems, st.grad_dtype = total, bucket, B.SO_GRAD_BF16
    st.staging, st.staging_bytes = staging.data_ptr(), 36 * bucket
    hp = hp_of(B, cfg)
    from concurrent.futures import ThreadPoolExecutor
    for t in (1, 2, 3):
        for s, n in ranges:
            g[s:s + n] = gen_grads(cfg, t, s, n, "cuda")
        staging.fill_(float("nan"))
        rep = B.so_stream_step(ctx, st, hp, t, 1.0)
        assert rep.buckets == 24 and rep.h2d_gbps > 5 and rep.d2h_gbps > 5 and rep.kernel_ms > 0
        say(f"step {t}: {rep.total_ms:.0f} ms, H2D {rep.h2d_gbps:.1f} GB/s, D2H {rep.d2h_gbps:.1f} GB/s, "
              f"kernels {rep.kernel_ms:.1f} ms", flush=True)

        def one(item):
            s0, n0, ob = item
            oracle.adamw_step(bits16(g[s0:s0 + n0]), 0, ob.p, ob.m, ob.v, ob.q, t=t, s=1.0, **cfg["hp"])

        with ThreadPoolExecutor(16) as ex:
            list(ex.map(one, [it for k in sample for it in orcs[k]]))
    for k in sample:
        s, n = ranges[k]
        ob = oracle.Bucket(np.concatenate([o.p for _, _, o in orcs[k]]))
        ob.m = np.concatenate([o.m for _, _, o in orcs[k]])
        ob.v = np.concatenate([o.v for _, _, o in orcs[k]])
        ob.q = np.concatenate([o.q for _, _, o in orcs[k]])
        state = (host[0][s:s + n].numpy(), host[1][s:s + n].numpy(), host[2][s:s + n].numpy(), bits16(q[s:s + n]))
        say("workload 4 bucket", k, compare_state(state, ob, f"workload 4 bucket {k}: "))
    # every element: finite, and the device working copy is the bf16 rounding of the host p
    for s, n in ranges:
        p = host[0][s:s + n]
        assert bool(torch.isfinite(p).all())
        assert torch.equal(p.to(torch.bfloat16).view(torch.int16), q[s:s + n].cpu().view(torch.int16))
    host = p = None
    for a in pinned:
        a.free()
    say(f"workload 4 total {time.time() - t_start:.0f} s")
