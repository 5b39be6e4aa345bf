"""GPU parity of the fused Adam(W) step, the gradient statistics and the speculative
commit/rollback path against the CPU oracle, element by element, through the C ABI."""
import math

import numpy as np
import pytest
import torch

import oracle
import synth
from parity import (DevBucket, assert_bits_equal, bits16, compare_state, dtype_code, gen_grads,
                    gen_params, NORM_REL)

pytestmark = pytest.mark.gpu

HP = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, wd=0.01)
CFG0 = synth.config(0)


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


def hp_struct(B, hp=HP, **kw):
    return B.hparams(hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["wd"], **kw)


def rand_state(n, seed, device="cuda"):
    """A mid-training state: Adam keeps |m| <= sqrt(v) up to constants, so the synthetic second
    moment is built on top of m^2 (independent m and v would allow |m| >> sqrt(v), i.e. updates
    thousands of times larger than any real one, which cancel against p)."""
    p = synth.normal_f32(seed, synth.STREAM_PARAM, 0, 0, n, 0.02, device)
    m = synth.normal_f32(seed, synth.STREAM_PARAM, 1, 0, n, 1e-4, device)
    v = (m.abs() + synth.normal_f32(seed, synth.STREAM_PARAM, 2, 0, n, 1e-4, device).abs()) ** 2
    return p, m, v


def oracle_bucket(p, m=None, v=None):
    ob = oracle.Bucket(p.cpu().numpy())
    if m is not None:
        ob.m[:] = m.cpu().numpy()
        ob.v[:] = v.cpu().numpy()
    return ob


# --------------------------------------------------------------------------------- step
@pytest.mark.parametrize("gdt", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("n", [1, 3, 4, 7, 8, 255, 1024, 4095, 4096, 4097, 16383, 16384, 16385,
                               3 * 16384 + 123, (1 << 20) + 13, 300 * 16384 + 5])
def test_step_sizes_and_tails(B, ctx, n, gdt):
    p, m, v = rand_state(n, 100 + n)
    sig, s = (1e-3, 0.37) if gdt == torch.bfloat16 else (60.0, 1.0 / 65536.0)
    db = DevBucket(B, p, gdt, m0=m, v0=v)
    db.g.copy_(synth.normal_16bit(7, synth.STREAM_GRAD, n, 0, n, sig, gdt, "cuda"))
    ob = oracle_bucket(p, m, v)
    for t in (1, 2, 9):
        B.so_adam_step(ctx, db.c, hp_struct(B), t, s)
        oracle.adamw_step(bits16(db.g), dtype_code(db.g), ob.p, ob.m, ob.v, ob.q, t=t,
                          s=np.float32(s), **HP)
    torch.cuda.synchronize()
    compare_state(db.host_state(), ob, f"n={n}: ")


@pytest.mark.parametrize("kw", [dict(adamw=0), dict(bias_correction=0), dict(adamw=0, bias_correction=0)])
def test_step_variants(B, ctx, kw):
    n = 50_000
    p, m, v = rand_state(n, 5)
    db = DevBucket(B, p, m0=m, v0=v)
    db.g.copy_(synth.normal_16bit(8, synth.STREAM_GRAD, 0, 0, n, 1e-3, torch.bfloat16, "cuda"))
    ob = oracle_bucket(p, m, v)
    for t in (1, 2, 3):
        B.so_adam_step(ctx, db.c, hp_struct(B, **kw), t, 1.0)
        oracle.adamw_step(bits16(db.g), 0, ob.p, ob.m, ob.v, ob.q, t=t, s=1.0, **HP, **kw)
    compare_state(db.host_state(), ob)


def test_fp16_working_copy(B, ctx):
    """The 16-bit working copy as IEEE fp16 instead of bf16: sync step, and a save-mode
    speculative step rolled back (the restore pass re-derives the fp16 copy)."""
    n = 70_001
    p, m, v = rand_state(n, 31)
    p[:4] = torch.tensor([70000.0, -65519.0, 3e-8, 65504.0])       # overflow to inf, max finite, subnormal
    db = DevBucket(B, p, m0=m, v0=v, alt=True, lp_dtype=torch.float16)
    assert db.c.lp_dtype == B.SO_LP_FP16
    db.g.copy_(synth.normal_16bit(8, synth.STREAM_GRAD, 3, 0, n, 1e-3, torch.bfloat16, "cuda"))
    ob = oracle_bucket(p, m, v)
    for t in (1, 2):
        B.so_adam_step(ctx, db.c, hp_struct(B), t, 1.0)
        oracle.adamw_step(bits16(db.g), 0, ob.p, ob.m, ob.v, ob.q, t=t, s=1.0, lp_fp16=1, **HP)
    compare_state(db.host_state(), ob, "fp16 copy: ", lp=torch.float16)
    before = [x.clone() for x in db.current()]
    B.so_adam_step(ctx, db.c, hp_struct(B), 3, 1.0, B.SO_SPEC_SAVE)
    B.so_adam_step_stats(ctx)
    B.so_adam_rollback(ctx, db.c)
    torch.cuda.synchronize()
    for x, y in zip(db.current(), before):
        assert_bits_equal(x, y, "fp16 copy rollback")


def test_parameter_groups_in_one_launch(B, ctx):
    """One so_hparams per bucket (learning rate, betas, decay, decay mode differ) in a single
    launch, against the oracle stepping each bucket with its own hyper-parameters."""
    groups = [dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, wd=0.01),
              dict(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, wd=0.0),
              dict(lr=1e-5, beta1=0.8, beta2=0.99, eps=1e-6, wd=0.1),
              dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, wd=0.01)]
    kws = [dict(), dict(), dict(adamw=0), dict(bias_correction=0)]
    sizes = [20_000, 20_000, 20_000, 7_777]
    devs, orcs = [], []
    for i, n in enumerate(sizes):
        p, m, v = rand_state(n, 40 + i)
        d = DevBucket(B, p, m0=m, v0=v)
        d.g.copy_(synth.normal_16bit(9, synth.STREAM_GRAD, i, 0, n, 1e-3, torch.bfloat16, "cuda"))
        devs.append(d)
        orcs.append(oracle_bucket(p, m, v))
    hps = [hp_struct(B, g, **kw) for g, kw in zip(groups, kws)]
    for t in (1, 2, 3):
        B.so_adam_step_groups(ctx, [d.c for d in devs], hps, t, 0.9)
        for d, ob, g, kw in zip(devs, orcs, groups, kws):
            oracle.adamw_step(bits16(d.g), 0, ob.p, ob.m, ob.v, ob.q, t=t, s=np.float32(0.9), **g, **kw)
    for i, (d, ob) in enumerate(zip(devs, orcs)):
        compare_state(d.host_state(), ob, f"group {i}: ")
    # contiguous buckets with different groups must not be merged into one entry
    n = 8192
    P, M, V = rand_state(2 * n, 50)
    G = synth.normal_16bit(9, synth.STREAM_GRAD, 9, 0, 2 * n, 1e-3, torch.bfloat16, "cuda")
    Q = torch.zeros(2 * n, dtype=torch.bfloat16, device="cuda")
    o1, o2 = oracle_bucket(P[:n], M[:n], V[:n]), oracle_bucket(P[n:], M[n:], V[n:])
    bks = [B.bucket_of(G[:n], P[:n], M[:n], V[:n], Q[:n]), B.bucket_of(G[n:], P[n:], M[n:], V[n:], Q[n:])]
    B.so_adam_step_groups(ctx, bks, hps[:2], 1, 1.0)
    oracle.adamw_step(bits16(G[:n]), 0, o1.p, o1.m, o1.v, o1.q, t=1, s=1.0, **groups[0])
    oracle.adamw_step(bits16(G[n:]), 0, o2.p, o2.m, o2.v, o2.q, t=1, s=1.0, **groups[1])
    compare_state((P[:n].cpu().numpy(), M[:n].cpu().numpy(), V[:n].cpu().numpy(), bits16(Q[:n])), o1, "adjacent group 0: ")
    compare_state((P[n:].cpu().numpy(), M[n:].cpu().numpy(), V[n:].cpu().numpy(), bits16(Q[n:])), o2, "adjacent group 1: ")


def test_step_edge_values(B, ctx):
    """Zero, subnormal, huge-but-finite gradients and zero state."""
    pats = np.array([0x0000, 0x8000, 0x0001, 0x8001, 0x007F, 0x0080, 0x3F80, 0xBF80, 0x7F7F, 0xFF7F,
                     0x4000, 0x1234, 0x0F00], dtype=np.uint16)
    n = pats.size
    p = torch.linspace(-1, 1, n)
    db = DevBucket(B, p)
    db.g.copy_(torch.from_numpy(pats.view(np.int16)).view(torch.bfloat16))
    ob = oracle_bucket(p)
    B.so_adam_step(ctx, db.c, hp_struct(B), 1, 1.0)
    oracle.adamw_step(pats, 0, ob.p, ob.m, ob.v, ob.q, t=1, s=1.0, **HP)
    pd, md, vd, qd = db.host_state()
    fin = np.isfinite(ob.v)                 # max-finite g squares to inf in fp32 on both sides
    assert np.array_equal(np.isinf(vd), np.isinf(ob.v))
    # where g*g leaves the fp32 range the fp32 kernel sees v = inf (update 0) while the
    # oracle's double intermediate does not: such elements are outside the method's range
    for a, b in ((pd[fin], ob.p[fin]), (md, ob.m), (vd[fin], ob.v[fin])):
        assert np.allclose(a, b, rtol=1e-6, atol=1e-9)
    assert np.all(np.isfinite(pd))


def test_config0_flat_bucket_10_steps(B, ctx):
    cfg = CFG0
    n = 1 << 24
    p0 = gen_params(cfg, 0, n, "cuda")
    db = DevBucket(B, p0)
    ob = oracle_bucket(p0)
    hp = hp_struct(B, cfg["hp"])
    for t in range(1, cfg["steps"] + 1):
        db.g.copy_(gen_grads(cfg, t, 0, n, "cuda"))
        st = B.so_grad_stats(ctx, db.c, 1.0)
        assert st.overflow == 0 and st.nonfinite == 0
        B.so_adam_step(ctx, db.c, hp, t, 1.0)
        gb = bits16(db.g)
        s, c = oracle.grad_stats(gb, 0, 1.0)
        assert c == 0 and abs(st.sumsq - s) <= NORM_REL * s and abs(st.norm - math.sqrt(s)) <= NORM_REL * math.sqrt(s)
        oracle.adamw_step(gb, 0, ob.p, ob.m, ob.v, ob.q, t=t, s=1.0, **cfg["hp"])
    w = compare_state(db.host_state(), ob, "config 0: ")
    print("config0 worst rel err", w)


# --------------------------------------------------------------------------------- stats
def _mk_grad_buckets(B, sizes, gdt, seed):
    out = []
    for i, n in enumerate(sizes):
        db = DevBucket(B, torch.zeros(n), gdt)
        if n:
            sig = 1e-3 if gdt == torch.bfloat16 else 40.0
            db.g.copy_(synth.normal_16bit(seed, synth.STREAM_GRAD, i, 0, n, sig, gdt, "cuda"))
        out.append(db)
    return out


@pytest.mark.parametrize("gdt", [torch.bfloat16, torch.float16])
def test_grad_stats_multi_bucket_ragged(B, ctx, gdt):
    sizes = [0, 1, 8191, 8192, 8193, 0, 100_003, (1 << 21) + 5, 7]
    dbs = _mk_grad_buckets(B, sizes, gdt, 21)
    inf, nan = (0x7F80, 0x7FC0) if gdt == torch.bfloat16 else (0x7C00, 0x7E00)
    inv = 1.0 if gdt == torch.bfloat16 else 1.0 / 64.0
    for poison in (False, True):
        if poison:
            dbs[2].g.view(torch.int16)[8190] = inf
            dbs[6].g.view(torch.int16)[100_002] = nan
            dbs[7].g.view(torch.int16)[0] = (inf | 0x8000) - 0x10000          # -inf
            dbs[8].g.view(torch.int16)[6] = nan
        st = B.so_grad_stats(ctx, [d.c for d in dbs], inv)
        tot, bad = 0.0, 0
        for d in dbs:
            s, c = oracle.grad_stats(bits16(d.g), dtype_code(d.g), np.float32(inv))
            tot += s
            bad += c
        assert st.nonfinite == bad and st.overflow == (1 if bad else 0)
        assert bad == (4 if poison else 0)
        assert abs(st.sumsq - tot) <= NORM_REL * tot
        assert abs(st.norm - math.sqrt(tot)) <= NORM_REL * math.sqrt(tot)
        assert abs(st.sumsq - tot) <= 1e-12 * tot           # in fact fp64-accurate
        st2 = B.so_grad_stats(ctx, [d.c for d in dbs], inv)   # deterministic
        assert (st2.sumsq, st2.nonfinite) == (st.sumsq, st.nonfinite)


def test_grad_stats_empty_and_extremes(B, ctx):
    st = B.so_grad_stats(ctx, [], 1.0)
    assert (st.sumsq, st.norm, st.nonfinite, st.overflow) == (0.0, 0.0, 0, 0)
    db = DevBucket(B, torch.zeros(1000))
    db.g.view(torch.int16).fill_(0x7F7F)              # largest finite bf16: squares overflow fp32
    st = B.so_grad_stats(ctx, db.c, 1.0)
    s, c = oracle.grad_stats(bits16(db.g), 0, 1.0)
    assert st.nonfinite == 0 and math.isfinite(st.sumsq) and abs(st.sumsq - s) <= 1e-12 * s
    db.g.view(torch.int16).fill_(0x0001)              # smallest subnormal: squares underflow fp32
    st = B.so_grad_stats(ctx, db.c, 1.0)
    s, c = oracle.grad_stats(bits16(db.g), 0, 1.0)
    assert s > 0 and abs(st.sumsq - s) <= 1e-12 * s
    # every bf16 and fp16 bit pattern once
    for gdt, code in ((torch.bfloat16, 0), (torch.float16, 1)):
        allb = DevBucket(B, torch.zeros(65536), gdt)
        allb.g.view(torch.int16).copy_(torch.arange(65536, dtype=torch.int32).to(torch.int16))
        st = B.so_grad_stats(ctx, allb.c, 1.0)
        s, c = oracle.grad_stats(bits16(allb.g), code, 1.0)
        assert st.nonfinite == c and abs(st.sumsq - s) <= 1e-12 * s


# --------------------------------------------------------------------------------- multi launch
def test_multi_bucket_launch_equals_per_bucket(B, ctx):
    sizes = [5000, 0, 16384, 1, 270_001, 49_152, 3, 16384 * 40 + 77]
    hp = hp_struct(B)
    a, b = [], []
    for i, n in enumerate(sizes):
        p, m, v = rand_state(n, 300 + i) if n else (torch.zeros(0),) * 3
        for lst in (a, b):
            db = DevBucket(B, p, m0=m, v0=v)
            if n:
                db.g.copy_(synth.normal_16bit(9, synth.STREAM_GRAD, i, 0, n, 1e-3, torch.bfloat16, "cuda"))
            lst.append(db)
    for t in (1, 2):
        B.so_adam_step_multi(ctx, [d.c for d in a], hp, t, 0.5)
        for d in b:
            B.so_adam_step(ctx, d.c, hp, t, 0.5)
    for da, dbb in zip(a, b):
        for x, y in zip(da.current(), dbb.current()):
            assert_bits_equal(x, y, "multi vs single")



@pytest.mark.parametrize("sizes", [[33_000] * 4 + [20_001], [512 * 7] * 3, [70_000, 70_000]])
def test_multi_bucket_equal_sizes_all_modes(B, ctx, sizes):
    """Equal-size buckets in separate allocations (the two-dimensional launch form), in the
    synchronous, ping-pong and save-old-state modes, against per-bucket calls."""
    hp = hp_struct(B)
    for mode in (B.SO_SYNC, B.SO_SPEC_PINGPONG, B.SO_SPEC_SAVE):
        a, b = [], []
        for i, n in enumerate(sizes):
            p, m, v = rand_state(n, 700 + i)
            for lst in (a, b):
                db = DevBucket(B, p, m0=m, v0=v, alt=True)
                db.g.copy_(synth.normal_16bit(15, synth.STREAM_GRAD, i, 0, n, 1e-3, torch.bfloat16, "cuda"))
                lst.append(db)
        arr = (B.so_bucket * len(a))(*[d.c for d in a])
        B.so_adam_step_multi(ctx, arr, hp, 3, 0.5, mode)
        for i, d in enumerate(a):
            d.c = arr[i]
        st_multi = B.so_adam_step_stats(ctx) if mode != B.SO_SYNC else None
        for d in b:
            B.so_adam_step(ctx, d.c, hp, 3, 0.5, mode)
        if mode != B.SO_SYNC:
            st_single = B.so_adam_step_stats(ctx)
            assert st_multi.nonfinite == st_single.nonfinite == 0
            assert abs(st_multi.sumsq - st_single.sumsq) <= 1e-12 * st_single.sumsq
            tot = sum(oracle.grad_stats(bits16(d.g), 0, np.float32(0.5))[0] for d in a)
            assert abs(st_multi.sumsq - tot) <= 1e-12 * tot
            for d in a + b:
                B.so_adam_commit(ctx, d.c)
        for da, dbb in zip(a, b):
            for x, y in zip(da.current(), dbb.current()):
                assert_bits_equal(x, y, f"mode {mode}")


@pytest.mark.parametrize("limits", [(7, 0), (0, 2), (5, 1), (1, 1)])
@pytest.mark.parametrize("sizes", [[33_000] * 5, [5000, 0, 16384, 1, 70_001], [300_003]])
def test_step_cut_into_several_launches(B, ctx, sizes, limits):
    """A step that exceeds the size of one launch is cut into several (by tiles per grid row,
    by rows of the two-dimensional grid, and by the room for partial sums).  The hardware's
    limits are out of reach of a test, so they are lowered; state and statistics must not
    change."""
    hp = hp_struct(B)
    for mode in (B.SO_SYNC, B.SO_SPEC_PINGPONG, B.SO_SPEC_SAVE):
        a, b = [], []
        for i, n in enumerate(sizes):
            p, m, v = rand_state(n, 740 + i) if n else (torch.zeros(0),) * 3
            for lst in (a, b):
                db = DevBucket(B, p, m0=m, v0=v, alt=True)
                if n:
                    db.g.copy_(synth.normal_16bit(17, synth.STREAM_GRAD, i, 0, n, 1e-3, torch.bfloat16, "cuda"))
                lst.append(db)
        stats = []
        for lst, lim in ((a, limits), (b, (0, 0))):
            B.so_set_limits(ctx, *lim)
            arr = (B.so_bucket * len(lst))(*[d.c for d in lst])
            B.so_adam_step_multi(ctx, arr, hp, 2, 0.5, mode)
            for i, d in enumerate(lst):
                d.c = arr[i]
            if mode != B.SO_SYNC:
                stats.append(B.so_adam_step_stats(ctx))
                for d in lst:
                    B.so_adam_commit(ctx, d.c)
        B.so_set_limits(ctx, 0, 0)
        if stats:
            assert stats[0].nonfinite == stats[1].nonfinite == 0
            assert abs(stats[0].sumsq - stats[1].sumsq) <= 1e-12 * stats[1].sumsq
        for da, dbb in zip(a, b):
            for x, y in zip(da.current(), dbb.current()):
                assert_bits_equal(x, y, f"mode {mode} limits {limits}")
    with pytest.raises(B.SoError):
        B.so_set_limits(ctx, 1 << 40, 0)


@pytest.mark.parametrize("seed", range(12))
def test_random_bucket_lists_equal_per_bucket_steps(B, ctx, seed):
    """Seeded random bucket lists -- sizes from 0 to a few hundred tiles, some buckets adjacent
    in one arena (so the runtime merges them), some in allocations of their own, random
    per-launch limits, every mode -- stepped in one call, against one call per bucket."""
    rng = np.random.default_rng(1000 + seed)
    nb = int(rng.integers(1, 9))
    sizes = [int(rng.choice([0, 1, 8, 256, 1000, 4096, 8 * int(rng.integers(1, 9000))])) for _ in range(nb)]
    sizes = [n - n % 8 if n > 8 else n for n in sizes]          # arena slices must stay 16-byte aligned
    mode = [B.SO_SYNC, B.SO_SPEC_PINGPONG, B.SO_SPEC_SAVE][seed % 3]
    gdt = torch.float16 if seed % 2 else torch.bfloat16
    hp = hp_struct(B)
    total = sum(sizes) + 8
    arena = {k: torch.zeros(total, dtype=torch.float32, device="cuda") for k in "pmv"}
    arena["g"] = torch.zeros(total, dtype=gdt, device="cuda")
    arena["q"] = torch.zeros(total, dtype=torch.bfloat16, device="cuda")
    alt = {k: torch.zeros(total, dtype=torch.float32, device="cuda") for k in "pmv"}
    alt["q"] = torch.zeros(total, dtype=torch.bfloat16, device="cuda")
    multi, single, off = [], [], 0
    for i, n in enumerate(sizes):
        p, m, v = rand_state(n, 5000 + 17 * seed + i) if n else (torch.zeros(0, device="cuda"),) * 3
        g = synth.normal_16bit(50 + seed, synth.STREAM_GRAD, i, 0, n, 1e-3 if gdt == torch.bfloat16 else 0.5, gdt, "cuda")
        ref = DevBucket(B, p, gdt, alt=True, m0=m, v0=v)
        ref.g.copy_(g)
        single.append(ref)
        if n >= 8 and rng.random() < 0.6:       # a slice of the arena, right behind the previous slice
            sl = slice(off, off + n)
            off += n
            for k, src in (("p", p), ("m", m), ("v", v), ("g", g)):
                arena[k][sl].copy_(src)
            bk = B.bucket_of(arena["g"][sl], arena["p"][sl], arena["m"][sl], arena["v"][sl], arena["q"][sl],
                             [alt["p"][sl], alt["m"][sl], alt["v"][sl], alt["q"][sl]])
            views = {"cur": (arena["p"][sl], arena["m"][sl], arena["v"][sl], arena["q"][sl]),
                     "alt": (alt["p"][sl], alt["m"][sl], alt["v"][sl], alt["q"][sl])}
            multi.append((bk, views))
        else:
            d = DevBucket(B, p, gdt, alt=True, m0=m, v0=v)
            d.g.copy_(g)
            multi.append((d.c, d))
    B.so_set_limits(ctx, int(rng.choice([0, 3, 50])), int(rng.choice([0, 1, 2])))
    arr = (B.so_bucket * nb)(*[bk for bk, _ in multi])
    B.so_adam_step_multi(ctx, arr, hp, 3, 0.25, mode)
    B.so_set_limits(ctx, 0, 0)
    st_multi = B.so_adam_step_stats(ctx) if mode != B.SO_SYNC else None
    for d in single:
        B.so_adam_step(ctx, d.c, hp, 3, 0.25, mode)
    if mode != B.SO_SYNC:
        st_single = B.so_adam_step_stats(ctx)
        assert st_multi.nonfinite == st_single.nonfinite == 0
        assert abs(st_multi.sumsq - st_single.sumsq) <= 1e-12 * max(st_single.sumsq, 1e-300)
    torch.cuda.synchronize()
    for i, ((bk, holder), ref) in enumerate(zip(multi, single)):
        if sizes[i] == 0:
            continue
        assert arr[i].pending == ref.c.pending == (mode if mode != B.SO_SYNC else 0)
        want = ref.alt if mode == B.SO_SPEC_PINGPONG else [ref.p, ref.m, ref.v, ref.q]
        if isinstance(holder, dict):
            got = holder["alt"] if mode == B.SO_SPEC_PINGPONG else holder["cur"]
        else:
            got = holder.alt if mode == B.SO_SPEC_PINGPONG else [holder.p, holder.m, holder.v, holder.q]
        for x, y, name in zip(got, want, "pmvq"):
            assert_bits_equal(x, y, f"seed {seed} bucket {i} (n={sizes[i]}) {name}")


def test_contiguous_buckets_are_stepped_as_one(B, ctx):
    """Buckets that are consecutive slices of flat arenas (the benchmark's layout), with bucket
    sizes that are not multiples of the tile, against the same data in separate allocations."""
    sizes = [10_001, 4_099, 512, 30_000]
    total = sum(sizes)
    hp = hp_struct(B)
    p, m, v = rand_state(total, 808)
    g = synth.normal_16bit(16, synth.STREAM_GRAD, 0, 0, total, 1e-3, torch.bfloat16, "cuda")
    P, M, V = p.clone(), m.clone(), v.clone()
    Q = torch.zeros(total, dtype=torch.bfloat16, device="cuda")
    offs = np.cumsum([0] + sizes)
    # element offsets of the slices are not multiples of 8: the 16-bit arrays of the later
    # buckets are then not 16-byte aligned, so pad the arena so that they are
    flat, sep = [], []
    ok = all(o % 8 == 0 for o in offs[:-1])
    for i, n in enumerate(sizes):
        s = int(offs[i])
        d = DevBucket(B, p[s:s + n], m0=m[s:s + n], v0=v[s:s + n])
        d.g.copy_(g[s:s + n])
        sep.append(d)
    if not ok:
        sizes = [10_000, 4_096 + 8, 512, 30_000]
        total = sum(sizes)
        offs = np.cumsum([0] + sizes)
        sep = []
        for i, n in enumerate(sizes):
            s = int(offs[i])
            d = DevBucket(B, p[s:s + n], m0=m[s:s + n], v0=v[s:s + n])
            d.g.copy_(g[s:s + n])
            sep.append(d)
    for i, n in enumerate(sizes):
        s = int(offs[i])
        flat.append(B.bucket_of(g[s:s + n], P[s:s + n], M[s:s + n], V[s:s + n], Q[s:s + n]))
    for t in (1, 2):
        B.so_adam_step_multi(ctx, flat, hp, t, 0.7)
        for d in sep:
            B.so_adam_step(ctx, d.c, hp, t, 0.7)
    for i, d in enumerate(sep):
        s, n = int(offs[i]), sizes[i]
        for x, y in zip((P[s:s + n], M[s:s + n], V[s:s + n], Q[s:s + n]), d.current()):
            assert_bits_equal(x.contiguous(), y, "contiguous buckets")


# --------------------------------------------------------------------------------- speculation
@pytest.mark.parametrize("mode_name", ["pingpong", "save"])
def test_speculative_rollback_redo_equals_synchronous(B, ctx, mode_name):
    """Speculative step -> validation says clip -> rollback -> clipped redo must leave exactly
    the state of the synchronous schedule (stats first, then one clipped step)."""
    mode = B.SO_SPEC_PINGPONG if mode_name == "pingpong" else B.SO_SPEC_SAVE
    sizes = [140_000, 16384 * 3, 9_999]
    hp = hp_struct(B)
    spec, sync, orc = [], [], []
    for i, n in enumerate(sizes):
        p, m, v = rand_state(n, 400 + i)
        g = synth.normal_16bit(10, synth.STREAM_GRAD, i, 0, n, 0.05, torch.bfloat16, "cuda")
        for lst, alt in ((spec, True), (sync, False)):
            db = DevBucket(B, p, m0=m, v0=v, alt=alt)
            db.g.copy_(g)
            db.q.copy_(p.to(torch.bfloat16))
            lst.append(db)
        orc.append(oracle_bucket(p, m, v))
    before = [[t.clone() for t in d.current()] for d in spec]
    # speculative schedule
    for d in spec:
        B.so_adam_step(ctx, d.c, hp, 1, 1.0, mode)
        assert d.c.pending == mode
    st = B.so_adam_step_stats(ctx)
    dec = B.so_validate(st, 1.0, 1.0, 1.0)
    assert dec.action == B.SO_ROLLBACK_REDO and dec.clip < 1.0
    for d in spec:
        B.so_adam_rollback(ctx, d.c)
        assert d.c.pending == 0
    torch.cuda.synchronize()
    for d, bef in zip(spec, before):
        for x, y in zip(d.current(), bef):
            assert_bits_equal(x, y, "rollback")
    for d in spec:
        B.so_adam_step(ctx, d.c, hp, 1, dec.grad_scale, B.SO_SYNC)
    # synchronous schedule
    st2 = B.so_grad_stats(ctx, [d.c for d in sync], 1.0)
    dec2 = B.so_validate(st2, 1.0, 1.0, 1.0)
    assert st2.nonfinite == st.nonfinite == 0
    assert abs(st2.sumsq - st.sumsq) <= 1e-12 * st.sumsq
    B.so_adam_step_multi(ctx, [d.c for d in sync], hp, 1, dec.grad_scale)
    for a, b in zip(spec, sync):
        for x, y in zip(a.current(), b.current()):
            assert_bits_equal(x, y, "speculative+redo vs synchronous")
    # and both agree with the oracle's synchronous iteration
    tr = oracle.Trainer(orc, max_norm=1.0, **HP)
    tr.iteration([bits16(d.g) for d in sync])
    assert abs(st.norm - tr.log[-1]["norm"]) <= NORM_REL * st.norm
    assert abs(dec.clip - tr.log[-1]["clip"]) <= 1e-12
    assert abs(dec2.grad_scale - tr.log[-1]["s"]) <= 1.2e-7 * tr.log[-1]["s"]
    for d, ob in zip(spec, orc):
        compare_state(d.host_state(), ob, mode_name + ": ")


@pytest.mark.parametrize("mode_name", ["pingpong", "save"])
def test_speculative_overflow_is_rolled_back_bit_exact(B, ctx, mode_name):
    mode = B.SO_SPEC_PINGPONG if mode_name == "pingpong" else B.SO_SPEC_SAVE
    n = 123_457
    p, m, v = rand_state(n, 77)
    d = DevBucket(B, p, torch.float16, m0=m, v0=v, alt=True)
    d.q.copy_(p.to(torch.bfloat16))
    d.g.copy_(synth.normal_16bit(12, synth.STREAM_GRAD, 0, 0, n, 60.0, torch.float16, "cuda"))
    d.g.view(torch.int16)[[5, 70_000, n - 1]] = torch.tensor([0x7C00, 0x7E00, -1024], dtype=torch.int16,
                                                              device="cuda")   # +inf, NaN, -inf
    before = [t.clone() for t in d.current()]
    B.so_adam_step(ctx, d.c, hp_struct(B), 4, 1.0 / 65536.0, mode)
    st = B.so_adam_step_stats(ctx)
    _, bad = oracle.grad_stats(bits16(d.g), 1, np.float32(1.0 / 65536.0))
    assert st.nonfinite == bad == 3 and st.overflow == 1
    dec = B.so_validate(st, 0.0, 65536.0, 1.0)
    assert dec.action == B.SO_ROLLBACK_SKIP and dec.next_loss_scale == 32768.0
    with pytest.raises(B.SoError) as ei:            # cannot step again while pending
        B.so_adam_step(ctx, d.c, hp_struct(B), 4, 1.0, mode)
    assert ei.value.status == B.SO_ERR_STATE
    B.so_adam_rollback(ctx, d.c)
    torch.cuda.synchronize()
    for x, y in zip(d.current(), before):
        assert_bits_equal(x, y, "overflow rollback")
    with pytest.raises(B.SoError) as ei:
        B.so_adam_rollback(ctx, d.c)
    assert ei.value.status == B.SO_ERR_STATE


@pytest.mark.parametrize("mode_name", ["pingpong", "save"])
@pytest.mark.parametrize("density", ["every element", "every 97th", "one wavefront's worth", "one per bucket tail"])
def test_overflow_patterns_dense_and_sparse(B, ctx, mode_name, density):
    """Rollbacks are frequent early in a run and rare later (Sec. 5.7): the NaN/Inf count is exact
    and the rollback bit-exact whether every gradient is bad, many are, or a single one in the
    ragged tail of a bucket -- through the speculative step's by-product statistics, the
    standalone pass and the gather with statistics alike."""
    mode = B.SO_SPEC_PINGPONG if mode_name == "pingpong" else B.SO_SPEC_SAVE
    sizes = [70_001, 256 * 40, 33]
    hp = hp_struct(B)
    dbs = []
    for i, n in enumerate(sizes):
        p, m, v = rand_state(n, 400 + i)
        d = DevBucket(B, p, m0=m, v0=v, alt=True)
        d.q.copy_(p.to(torch.bfloat16))
        d.g.copy_(synth.normal_16bit(44, synth.STREAM_GRAD, i, 0, n, 1e-3, torch.bfloat16, "cuda"))
        raw = d.g.view(torch.int16)
        if density == "every element":
            raw[0::2] = 0x7F80
            raw[1::2] = 0x7FC0
        elif density == "every 97th":
            raw[5::97] = 0x7FC1
        elif density == "one wavefront's worth" and i == 0:
            raw[256 * 7:256 * 8] = -128                  # -inf over exactly one tile
        elif density == "one per bucket tail":
            raw[n - 1] = 0x7F80
        dbs.append(d)
    want = sum(oracle.grad_stats(bits16(d.g), 0, 1.0)[1] for d in dbs)
    assert want > 0
    before = [[t.clone() for t in d.current()] for d in dbs]
    B.so_adam_step_multi(ctx, [d.c for d in dbs], hp, 7, 1.0, mode)
    st = B.so_adam_step_stats(ctx)
    assert st.nonfinite == want and st.overflow == 1
    assert B.so_grad_stats(ctx, [d.c for d in dbs], 1.0).nonfinite == want
    flat = torch.cat([d.g for d in dbs])
    dst = torch.zeros_like(flat)
    B.so_flatten_grad_stats(ctx, [B.so_slice(0, 0, 0, 0, flat.numel())], [flat.data_ptr()], [dst.data_ptr()],
                            B.SO_GRAD_BF16, 1.0, 1.0)
    st2, dec = B.so_grad_stats_fetch(ctx)
    assert st2.nonfinite == want and dec.action == B.SO_ROLLBACK_SKIP
    assert_bits_equal(dst, flat, "gather of poisoned gradients")
    for d in dbs:
        B.so_adam_rollback(ctx, d.c)
    torch.cuda.synchronize()
    for d, bef in zip(dbs, before):
        for x, y in zip(d.current(), bef):
            assert_bits_equal(x, y, f"rollback, {density}")


def test_speculative_commit_matches_oracle_over_iterations(B, ctx):
    """Ping-pong speculation over several iterations with an overflow in the middle."""
    n, nb = 30_011, 3
    hp = hp_struct(B)
    devs, orcs = [], []
    for i in range(nb):
        p = synth.normal_f32(55, synth.STREAM_PARAM, 0, i * n, n, 0.02, "cuda")
        devs.append(DevBucket(B, p, torch.float16, alt=True))
        orcs.append(oracle_bucket(p))
    tr = oracle.Trainer(orcs, grad_dtype=oracle.GRAD_FP16, loss_scale=65536.0, **HP)
    scale, t = 65536.0, 1
    for it in range(1, 8):
        for i, d in enumerate(devs):
            d.g.copy_(synth.normal_16bit(56, synth.STREAM_GRAD, it, i * n, n, 1e-3 * scale, torch.float16, "cuda"))
        if it in (3, 6):
            devs[it % nb].g.view(torch.int16)[it * 100] = 0x7C00 if it == 3 else 0x7FFF
        inv = float(np.float32(1.0 / scale))
        for d in devs:
            B.so_adam_step(ctx, d.c, hp, t, inv, B.SO_SPEC_PINGPONG)
        st = B.so_adam_step_stats(ctx)
        dec = B.so_validate(st, 0.0, scale, 1.0)
        applied = tr.iteration([bits16(d.g) for d in devs])
        assert (dec.action == B.SO_COMMIT) == applied
        for d in devs:
            (B.so_adam_commit if applied else B.so_adam_rollback)(ctx, d.c)
        if applied:
            assert abs(st.norm - tr.log[-1]["norm"]) <= NORM_REL * st.norm
            t += 1
        scale = dec.next_loss_scale
        assert scale == tr.loss_scale and t == tr.t
    assert t == 6 and scale == 16384.0
    for d, ob in zip(devs, orcs):
        compare_state(d.host_state(), ob, "spec iterations: ")


# --------------------------------------------------------------------------------- guarded step
def test_guarded_step_equals_host_validated_step(B, ctx):
    sizes = [33_000, 8_191, 50_000]
    hp = hp_struct(B)
    a, b = [], []
    for i, n in enumerate(sizes):
        p, m, v = rand_state(n, 600 + i)
        g = synth.normal_16bit(13, synth.STREAM_GRAD, i, 0, n, 0.02, torch.bfloat16, "cuda")
        for lst in (a, b):
            d = DevBucket(B, p, m0=m, v0=v)
            d.g.copy_(g)
            lst.append(d)
    # host-validated
    st = B.so_grad_stats(ctx, [d.c for d in a], 1.0)
    dec = B.so_validate(st, 1.0, 1.0, 1.0)
    assert dec.clip < 1.0
    B.so_adam_step_multi(ctx, [d.c for d in a], hp, 2, dec.grad_scale)
    # device-validated, no host round trip
    B.so_grad_stats_enqueue(ctx, [d.c for d in b], 1.0, 1.0)
    B.so_adam_step_guarded(ctx, [d.c for d in b], hp, 2)
    st2, dec2 = B.so_grad_stats_fetch(ctx)
    assert (st2.sumsq, st2.nonfinite) == (st.sumsq, st.nonfinite)
    assert (dec2.clip, dec2.grad_scale, dec2.action) == (dec.clip, dec.grad_scale, B.SO_ROLLBACK_REDO)
    for x, y in zip(a, b):
        for u, w in zip(x.current(), y.current()):
            assert_bits_equal(u, w, "guarded")
    # overflow: the guarded step must leave everything untouched
    b[1].g.view(torch.int16)[17] = 0x7F80
    before = [[t.clone() for t in d.current()] for d in b]
    B.so_grad_stats_enqueue(ctx, [d.c for d in b], 1.0, 1.0)
    B.so_adam_step_guarded(ctx, [d.c for d in b], hp, 3)
    st3, dec3 = B.so_grad_stats_fetch(ctx)
    assert st3.overflow == 1 and dec3.action == B.SO_ROLLBACK_SKIP
    for d, bef in zip(b, before):
        for u, w in zip(d.current(), bef):
            assert_bits_equal(u, w, "guarded skip")


# --------------------------------------------------------------------------------- layout
@pytest.mark.parametrize("gdt,scale0", [(torch.float16, 1024.0), (torch.bfloat16, 1.0)])
def test_autonomous_iterations_match_the_oracle_protocol(B, ctx, gdt, scale0):
    """Twelve iterations enqueued back to back without a single host round trip: step count,
    bias corrections, loss scale (halving and growth) and clipping all live on the GPU.  Some
    iterations carry Inf/NaN.  The oracle's Trainer runs the same protocol on the host."""
    sizes = [70_001, 16_384, 0, 33_333]
    hp = hp_struct(B)
    code = dtype_code(torch.empty(0, dtype=gdt))
    devs, obs = [], []
    for i, n in enumerate(sizes):
        p, m, v = rand_state(n, 960 + i) if n else (torch.zeros(0),) * 3
        devs.append(DevBucket(B, p, gdt, m0=m, v0=v))
        obs.append(oracle_bucket(p, m, v) if n else oracle.Bucket(np.zeros(0, dtype=np.float32)))
    growth = 2 if scale0 > 1 else 0
    tr = oracle.Trainer(obs, grad_dtype=code, max_norm=0.25, loss_scale=scale0, min_loss_scale=1.0,
                        growth_interval=growth, max_loss_scale=4096.0, **HP)
    tr.t = 5                                            # resume in the middle of a run
    B.so_train_reset(ctx, hp, 5, scale0, 1.0, 4096.0, growth, 0.25)   # exact in fp32
    poisoned = {3, 4, 8}
    grads = {}
    for it in range(1, 13):
        # gradients follow the loss scale the ORACLE holds (a real backward pass would scale its loss)
        for i, d in enumerate(devs):
            if d.n:
                g = synth.normal_16bit(41, synth.STREAM_GRAD, it, i << 20, d.n, 1e-3 * tr.loss_scale, gdt, "cuda")
                if it in poisoned and i == (it % 2) * 3:
                    g.view(torch.int16)[d.n // 2] = 0x7C00 if gdt == torch.float16 else 0x7F80
                    g.view(torch.int16)[7] = 0x7E01 if gdt == torch.float16 else 0x7FC1
                d.g.copy_(g)
        B.so_train_iteration(ctx, [d.c for d in devs])
        applied = tr.iteration([bits16(d.g) for d in devs])
        assert applied == (it not in poisoned)
    st, dec, applied_steps, next_scale = B.so_train_fetch(ctx)
    assert applied_steps == tr.t - 1 == 4 + 9
    assert next_scale == tr.loss_scale
    last = tr.log[-1]
    assert st.overflow == 0 and abs(st.norm - last["norm"]) <= NORM_REL * last["norm"]
    assert abs(dec.clip - last["clip"]) <= 1e-12 and dec.clip < 1.0
    for d, ob in zip(devs, obs):
        if d.n:
            compare_state(d.host_state(), ob, "autonomous: ")
    # a context without train state refuses, and a bad bucket is rejected before anything runs
    fresh = B.so_create(0, torch.cuda.current_stream().cuda_stream)
    with pytest.raises(B.SoError) as ei:
        B.so_train_iteration(fresh, [devs[0].c])
    assert ei.value.status == B.SO_ERR_STATE
    B.so_destroy(fresh)


def test_recorded_iteration_replays_like_the_eager_one(B):
    """so_train_capture / so_train_replay: one recorded iteration replayed eight times, with
    fresh gradients, other GPU work and synchronisations in between; after EVERY replay the
    state must equal, bit for bit, a twin that ran the eager so_train_iteration, and at the end
    both must match the oracle's protocol (two iterations carry Inf/NaN and are skipped)."""
    sizes = [70_001, 16_384, 33_333]
    hp = hp_struct(B)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    ctxs = [B.so_create(0, st.cuda_stream) for st in streams]
    twins, obs = [[], []], []
    for i, n in enumerate(sizes):
        p, m, v = rand_state(n, 970 + i)
        for tw in twins:
            tw.append(DevBucket(B, p, torch.float16, m0=m, v0=v))
        obs.append(oracle_bucket(p, m, v))
    tr = oracle.Trainer(obs, grad_dtype=oracle.GRAD_FP16, max_norm=0.25, loss_scale=256.0, min_loss_scale=1.0,
                        growth_interval=3, max_loss_scale=4096.0, **HP)
    for c in ctxs:
        B.so_train_reset(c, hp, 1, 256.0, 1.0, 4096.0, 3, 0.25)
    with pytest.raises(B.SoError) as ei:
        B.so_train_replay(ctxs[0])                      # nothing recorded yet
    assert ei.value.status == B.SO_ERR_STATE
    poisoned = {3, 6}
    scratch = torch.zeros(1 << 20, device="cuda")
    for it in range(1, 9):
        for i, n in enumerate(sizes):
            g = synth.normal_16bit(43, synth.STREAM_GRAD, it, i << 20, n, 1e-3 * tr.loss_scale, torch.float16, "cuda")
            if it in poisoned and i == 1:
                g.view(torch.int16)[n // 3] = 0x7C00
            for tw in twins:
                tw[i].g.copy_(g)
        scratch.add_(1.0)                               # unrelated eager work between replays
        torch.cuda.synchronize()
        if it == 1:
            B.so_train_capture(ctxs[0], [d.c for d in twins[0]])
            torch.cuda.synchronize()
            for d, e in zip(*twins):                    # recording runs nothing
                assert_bits_equal(d.p, e.p, "state after recording")
        B.so_train_replay(ctxs[0])
        B.so_train_iteration(ctxs[1], [d.c for d in twins[1]])
        assert tr.iteration([bits16(d.g) for d in twins[1]]) == (it not in poisoned)
        torch.cuda.synchronize()
        for d, e in zip(*twins):
            for name in ("p", "m", "v", "q"):
                assert_bits_equal(getattr(d, name), getattr(e, name), f"replay {it}: {name}")
    for c in ctxs:
        st, dec, applied, scale = B.so_train_fetch(c)
        assert applied == 6 == tr.t - 1 and scale == tr.loss_scale and st.overflow == 0
    for d, ob in zip(twins[0], obs):
        compare_state(d.host_state(), ob, "recorded iteration: ")
    assert float(scratch[0]) == 8.0
    for c in ctxs:
        B.so_destroy(c)


def test_flatten_roundtrip_matches_slicing(B, ctx):
    numel = [5, 4096, 1, 10_007, 0, 8192, 333]
    bucket = 6000
    total = sum(numel)
    slices, nb = B.so_layout_plan(numel, bucket)
    assert nb == -(-total // bucket)
    for elem, dt in ((2, torch.bfloat16), (4, torch.float32)):
        flat = synth.normal_f32(3, 1, 0, 0, total, 1.0, "cuda").to(dt)
        offs = np.cumsum([0] + numel)
        tensors = [flat[offs[i]:offs[i + 1]].clone() for i in range(len(numel))]
        buckets = [torch.zeros(bucket, dtype=dt, device="cuda") for _ in range(nb)]
        B.so_flatten(ctx, slices, [t.data_ptr() if t.numel() else 0 for t in tensors],
                     [b.data_ptr() for b in buckets], elem, 0)
        got = torch.cat(buckets)[:total]
        assert_bits_equal(got, flat, "flatten")
        back = [torch.zeros_like(t) for t in tensors]
        B.so_flatten(ctx, slices, [t.data_ptr() if t.numel() else 0 for t in back],
                     [b.data_ptr() for b in buckets], elem, 1)
        for x, y in zip(back, tensors):
            if x.numel():
                assert_bits_equal(x, y, "unflatten")


@pytest.mark.parametrize("elem,dt", [(2, torch.bfloat16), (4, torch.float32)])
@pytest.mark.parametrize("direction", [0, 1])
def test_flatten_every_pair_of_source_and_destination_alignments(B, ctx, elem, dt, direction):
    """One slice for every pair (source offset, destination offset) inside a 16-byte granule,
    several lengths each (shorter than a granule, a few vectors, several chunks): the copy is
    exact and nothing outside the destination range is written."""
    per16 = 16 // elem
    lengths = [1, per16 - 1, per16, 3 * per16 + 1, 1024 // elem, 5 * (1024 // elem) + per16 + 3]
    room = -(-(max(lengths) + 4 * per16) // per16) * per16          # keeps every base 16-byte aligned
    combos = [(so, do, ln) for so in range(per16) for do in range(per16) for ln in lengths]
    n = len(combos)
    src = synth.normal_f32(61, 1, direction, 0, n * room, 1.0, "cuda").to(dt)
    dst = torch.zeros(n * room, dtype=dt, device="cuda")
    guard = 0x5A5A if elem == 2 else 0x5A5A5A5A
    dst.view(torch.int16 if elem == 2 else torch.int32).fill_(guard)
    slices = []
    for i, (so, do, ln) in enumerate(combos):
        # tensor i / bucket i start at element i * room of the two arrays (16-byte aligned)
        t_off, b_off = (so, do) if direction == 0 else (do, so)
        slices.append(B.so_slice(i, t_off, i, b_off, ln))
    tens, bucks = (src, dst) if direction == 0 else (dst, src)
    B.so_flatten(ctx, slices, [tens.data_ptr() + elem * i * room for i in range(n)],
                 [bucks.data_ptr() + elem * i * room for i in range(n)], elem, direction)
    torch.cuda.synchronize()
    want = torch.empty_like(dst)
    want.view(torch.int16 if elem == 2 else torch.int32).fill_(guard)
    for i, (so, do, ln) in enumerate(combos):
        want[i * room + do:i * room + do + ln] = src[i * room + so:i * room + so + ln]
    assert_bits_equal(dst, want, "copy over all alignment pairs")


def test_flatten_calls_queue_without_waiting(B, ctx):
    """Several gathers with different (and growing) slice tables are queued back to back; each
    must use its own table although the calls return before the copies have run."""
    jobs = []
    for k, nt in enumerate((3, 40, 7, 1500, 2)):
        numel = [((i * 2654435761 + k) % 997) + 1 for i in range(nt)]
        bucket = 1024
        total = sum(numel)
        slices, nb = B.so_layout_plan(numel, bucket)
        flat = synth.normal_f32(40 + k, 1, 0, 0, total, 1.0, "cuda")
        offs = np.cumsum([0] + numel)
        tensors = [flat[offs[i]:offs[i + 1]].clone() for i in range(nt)]
        buckets = torch.zeros(nb * bucket, dtype=torch.float32, device="cuda")
        B.so_flatten(ctx, slices, [t.data_ptr() for t in tensors],
                     [buckets.data_ptr() + 4 * bucket * j for j in range(nb)], 4, 0)
        jobs.append((flat, buckets, total))
    torch.cuda.synchronize()
    for k, (flat, buckets, total) in enumerate(jobs):
        assert_bits_equal(buckets[:total], flat, f"queued flatten {k}")
        assert not buckets[total:].any()


@pytest.mark.parametrize("gdt", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("limit", [0, 37])
def test_flatten_grad_stats_matches_oracle_and_feeds_the_guarded_step(B, ctx, gdt, limit):
    """Gathering gradient tensors into buckets and validating them in one pass (Sec. 4.3 + 4.4):
    the copy is exact, the statistics match the oracle's scalar loop (count exact, norm 1e-10)
    with and without NaN/Inf, and a guarded step that consumes the GPU-side result equals the
    host-validated step bit for bit.  Odd tensor sizes make most slices start at addresses that
    are not 16-byte aligned (element-wise path); `limit` cuts the gather into several launches."""
    numel = [5, 4096, 1, 10_007, 0, 8192, 333, 70_001, 2, 40_960]
    bucket = 24_000
    total = sum(numel)
    slices, nb = B.so_layout_plan(numel, bucket)
    code = dtype_code(torch.zeros(1, dtype=gdt))
    scale = 1.0 if gdt == torch.bfloat16 else 256.0
    sig = 1e-3 * scale
    inf, nan = (0x7F80, 0x7FC0) if gdt == torch.bfloat16 else (0x7C00, 0x7E00)
    hp = hp_struct(B)
    offs = np.cumsum([0] + numel)
    p0, m0, v0 = rand_state(nb * bucket, 77)
    if limit:
        B.so_set_limits(ctx, limit, 0)
    for poison, max_norm in ((False, 0.0), (False, 0.0625), (True, 0.0625)):
        flat = synth.normal_16bit(31, synth.STREAM_GRAD, int(poison), 0, total, sig, gdt, "cuda")
        if poison:
            raw = flat.view(torch.int16)
            raw[3], raw[4101], raw[total - 1] = inf, nan, (inf | 0x8000) - 0x10000
        tensors = [flat[offs[i]:offs[i + 1]].clone() for i in range(len(numel))]
        twins = []
        for _ in range(2):
            g = torch.zeros(nb * bucket, dtype=gdt, device="cuda")
            dbs = []
            for k in range(nb):
                n = min(bucket, total - k * bucket)
                sl = slice(k * bucket, k * bucket + n)
                db = DevBucket(B, p0[sl], gdt, m0=m0[sl], v0=v0[sl])
                dbs.append(db)
            twins.append((g, dbs))
        # fused: gather + statistics in one pass, then the guarded step
        g, dbs = twins[0]
        B.so_flatten_grad_stats(ctx, slices, [t.data_ptr() if t.numel() else 0 for t in tensors],
                                [d.g.data_ptr() for d in dbs], code, scale, max_norm)
        B.so_adam_step_guarded(ctx, [d.c for d in dbs], hp, 3)
        st, dec = B.so_grad_stats_fetch(ctx)
        got = torch.cat([d.g for d in dbs])
        assert_bits_equal(got, flat, "gathered gradients")
        inv = np.float32(1.0 / scale)
        want_s, want_c = oracle.grad_stats(bits16(flat), code, inv)
        assert st.nonfinite == want_c == (3 if poison else 0) and st.overflow == int(poison)
        assert abs(st.sumsq - want_s) <= NORM_REL * want_s
        assert dec.clip == oracle.clip_coef(math.sqrt(st.sumsq), max_norm)
        # separate: plain gather, standalone statistics, host validation, plain step
        g2, dbs2 = twins[1]
        B.so_flatten(ctx, slices, [t.data_ptr() if t.numel() else 0 for t in tensors],
                     [d.g.data_ptr() for d in dbs2], 2, 0)
        st2 = B.so_grad_stats(ctx, [d.c for d in dbs2], float(inv))
        assert st2.nonfinite == st.nonfinite and abs(st2.sumsq - st.sumsq) <= 1e-12 * st.sumsq
        dec2 = B.so_validate(st, max_norm, scale, 1.0)
        assert dec2.grad_scale == dec.grad_scale and dec2.action == dec.action
        if not poison:
            B.so_adam_step_multi(ctx, [d.c for d in dbs2], hp, 3, dec.grad_scale)
        for a, b in zip(dbs, dbs2):
            for x, y in zip(a.current(), b.current()):
                assert_bits_equal(x, y, "guarded step after the fused gather")
    B.so_set_limits(ctx, 0, 0)


def test_flatten_grad_stats_leaves_pending_speculative_statistics_alone(B, ctx):
    n = 50_000
    p, m, v = rand_state(n, 88)
    spec = DevBucket(B, p, alt=True, m0=m, v0=v)
    spec.g.copy_(synth.normal_16bit(32, synth.STREAM_GRAD, 0, 0, n, 1e-3, torch.bfloat16, "cuda"))
    spec.g.view(torch.int16)[17] = 0x7F80
    hp = hp_struct(B)
    B.so_adam_step(ctx, spec.c, hp, 1, 1.0, B.SO_SPEC_PINGPONG)
    numel = [3000, 4097]
    slices, nb = B.so_layout_plan(numel, 8192)
    flat = synth.normal_16bit(33, synth.STREAM_GRAD, 0, 0, sum(numel), 1e-3, torch.bfloat16, "cuda")
    tensors = [flat[:3000].clone(), flat[3000:].clone()]
    dst = torch.zeros(8192, dtype=torch.bfloat16, device="cuda")
    B.so_flatten_grad_stats(ctx, slices, [t.data_ptr() for t in tensors], [dst.data_ptr()], B.SO_GRAD_BF16, 1.0, 0.0)
    st, _ = B.so_grad_stats_fetch(ctx)
    s, c = oracle.grad_stats(bits16(flat), 0, 1.0)
    assert st.nonfinite == 0 and abs(st.sumsq - s) <= NORM_REL * s
    assert_bits_equal(dst[:sum(numel)], flat, "gather")
    sp = B.so_adam_step_stats(ctx)                      # the speculative step's own statistics
    s, c = oracle.grad_stats(bits16(spec.g), 0, 1.0)
    assert sp.nonfinite == c == 1 and abs(sp.sumsq - s) <= NORM_REL * s
    B.so_adam_rollback(ctx, spec.c)
    # empty gather: all-zero statistics, still a valid result for the guarded step
    B.so_flatten_grad_stats(ctx, [], [0], [0], B.SO_GRAD_BF16, 1.0, 1.0)
    st, dec = B.so_grad_stats_fetch(ctx)
    assert (st.sumsq, st.nonfinite, st.overflow, dec.action) == (0.0, 0, 0, B.SO_COMMIT)


# --------------------------------------------------------------------------------- streamer
@pytest.mark.parametrize("pinned", [True, False])
def test_stream_step_equals_resident_step(B, ctx, pinned):
    n, bucket = 1_000_003, 131_072
    p, m, v = rand_state(n, 900)
    g = synth.normal_16bit(14, synth.STREAM_GRAD, 0, 0, n, 1e-3, torch.bfloat16, "cuda")
    hp = hp_struct(B)
    res = DevBucket(B, p, m0=m, v0=v)
    res.g.copy_(g)
    hp_, hm_, hv_ = (t.cpu().pin_memory() if pinned else t.cpu() for t in (p, m, v))   # pageable works, slowly
    q = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    st = B.so_stream_state()
    st.host_param, st.host_exp_avg, st.host_exp_avg_sq = hp_.data_ptr(), hm_.data_ptr(), hv_.data_ptr()
    st.grad, st.param_lp = g.data_ptr(), q.data_ptr()
    st.n_total, st.bucket_elems, st.grad_dtype = n, bucket, B.SO_GRAD_BF16
    for t in (1, 2, 3):
        rep = B.so_stream_step(ctx, st, hp, t, 0.25)
        assert rep.buckets == -(-n // bucket) and rep.h2d_gbps > 0 and rep.d2h_gbps > 0
        B.so_adam_step(ctx, res.c, hp, t, 0.25)
    torch.cuda.synchronize()
    for x, y in zip((hp_, hm_, hv_), (res.p, res.m, res.v)):
        assert_bits_equal(x, y.cpu(), "stream vs resident")
    assert_bits_equal(q, res.q, "stream q")


@pytest.mark.parametrize("lg,own_staging", [(18, True), (22, True), (26, True), (22, False)])
def test_stream_step_bucket_sizes_with_poisoned_staging(B, ctx, lg, own_staging):
    """The streamed step at staged bucket sizes on both sides of the host link's saturation
    knee (2^18, 2^22, 2^26 elements; Sec. 4.3 studies bandwidth against transfer size): four full
    buckets and a partial one, so every staging slot is reused.  The staging slots are filled
    with NaN before every pass: a step that ran before its upload had landed, or an upload that
    overwrote a slot before its download had drained it, would leave NaN or stale values in the
    result, which must stay bit-identical to the resident step."""
    bucket = 1 << lg
    n = 4 * bucket + bucket // 3 + 5
    p, m, v = rand_state(n, 930 + lg)
    g = synth.normal_16bit(17, synth.STREAM_GRAD, lg, 0, n, 1e-3, torch.bfloat16, "cuda")
    hp = hp_struct(B)
    res = DevBucket(B, p, m0=m, v0=v)
    res.g.copy_(g)
    pins = [B.PinnedArray(n) for _ in range(3)]      # exact size, given back below (torch's pinned pool
    host = [a.t for a in pins]                       # would round up and keep the memory)
    for h, t in zip(host, (p, m, v)):
        h.copy_(t)
    del p, m, v
    q = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    st = B.so_stream_state()
    st.host_param, st.host_exp_avg, st.host_exp_avg_sq = (t.data_ptr() for t in host)
    st.grad, st.param_lp = g.data_ptr(), q.data_ptr()
    st.n_total, st.bucket_elems, st.grad_dtype = n, bucket, B.SO_GRAD_BF16
    staging = None
    if own_staging:
        staging = torch.empty(9 * bucket, dtype=torch.float32, device="cuda")
        st.staging, st.staging_bytes = staging.data_ptr(), 36 * bucket
    for t in (1, 2, 3):
        if staging is not None:
            staging.fill_(float("nan"))
        rep = B.so_stream_step(ctx, st, hp, t, 0.25)
        assert rep.buckets == 5
        B.so_adam_step(ctx, res.c, hp, t, 0.25)
        print(f"bucket 2^{lg}: step {t} {rep.total_ms:.1f} ms, H2D {rep.h2d_gbps:.1f} D2H {rep.d2h_gbps:.1f} GB/s")
    torch.cuda.synchronize()
    for x, y in zip(host, (res.p, res.m, res.v)):
        assert_bits_equal(x, y.cpu(), "stream vs resident")
    assert_bits_equal(q, res.q, "stream q")
    if own_staging:
        st.staging_bytes = 36 * bucket - 4
        with pytest.raises(B.SoError) as ei:
            B.so_stream_step(ctx, st, hp, 4, 0.25)
        assert ei.value.status == B.SO_ERR_INVALID_ARG
    host = None
    for a in pins:
        a.free()


# --------------------------------------------------------------------------------- cast (Sec. 4.5)
def _cast_inputs(n, seed):
    """fp32 values around every rounding case: all 65,536 upper halves with tie / just-off-tie
    lower halves (NaN, infinities, denormals, the largest finite values among them), then
    parameter-like normals at several scales."""
    upper = np.arange(65536, dtype=np.uint32)
    special = np.concatenate([((upper << 16) | lo) for lo in (0x0000, 0x7FFF, 0x8000, 0x8001, 0x0FFF, 0x1000, 0x1001)])
    x = np.empty(n, dtype=np.float32)
    k = min(n, special.size)
    x[:k] = special[:k].view(np.float32)
    if n > k:
        r = synth.normal_f32(seed, synth.STREAM_PARAM, 5, 0, n - k, 1.0, "cpu").numpy()
        x[k:] = r * np.float32(10.0) ** ((np.arange(n - k) % 13).astype(np.float32) - 8)
    return x


@pytest.mark.parametrize("lp", [0, 1])
@pytest.mark.parametrize("n", [0, 1, 5, 255, 256, 257, 7 * 65536 + 1531])
def test_cast_params_matches_the_oracle_bit_for_bit(B, ctx, n, lp):
    x = _cast_inputs(n, 77 + n % 11)
    want = oracle.cast_lp(x, lp)
    pd = torch.from_numpy(x).cuda()
    q = torch.full((n + 8,), 0x5A5A, dtype=torch.int16, device="cuda")
    B.so_cast_params(ctx, pd.data_ptr() if n else 0, q.data_ptr(), n, lp)
    torch.cuda.synchronize()
    got = q.cpu().numpy().view(np.uint16)
    nan = np.isnan(x)
    assert np.array_equal(got[:n][~nan], want[~nan])
    exp_mask, frac_mask = (0x7C00, 0x3FF) if lp else (0x7F80, 0x7F)
    assert np.all((got[:n][nan] & exp_mask) == exp_mask) and np.all((got[:n][nan] & frac_mask) != 0)
    assert np.all(got[n:] == 0x5A5A), "wrote past the end"
    # the same bits as the working copy a step leaves for the same parameters
    if n:
        d = DevBucket(B, torch.from_numpy(np.where(nan, np.float32(0.5), x)),
                      lp_dtype=torch.float16 if lp else torch.bfloat16)
        d.g.zero_()
        hp0 = B.hparams(0.0, 0.9, 0.999, 1e-8, 0.0)            # lr = 0: the step stores p unchanged ...
        fin = np.isfinite(x)                                    # ... where p is finite (0 x inf is NaN)
        B.so_adam_step(ctx, d.c, hp0, 1, 1.0)
        torch.cuda.synchronize()
        assert np.array_equal(bits16(d.q)[fin], want[fin])


@pytest.mark.parametrize("pinned,lp", [(True, 0), (True, 1), (False, 0)])
def test_stream_cast_params_equals_the_device_cast(B, ctx, pinned, lp):
    """fp32 parameters in host memory -> 16-bit working copy on the device, moved as fp32 and cast
    on the GPU (Sec. 4.5), at chunk sizes that leave one chunk, a ragged tail, and many reuses of
    the three staging slots; a streamed step in between leaves other data in those slots."""
    n = 3_300_007
    x = _cast_inputs(n, 91)
    want = oracle.cast_lp(x, lp)
    nan = np.isnan(x)
    pin = B.PinnedArray(n) if pinned else None
    host = pin.t if pinned else torch.empty(n)
    host.copy_(torch.from_numpy(x))
    q = torch.zeros(n + 8, dtype=torch.int16, device="cuda")
    for chunk in (1 << 22, 1 << 20, 1 << 18, 4096):
        q.fill_(0x5A5A)
        ms = B.so_stream_cast_params(ctx, host.data_ptr(), q.data_ptr(), n, chunk, lp)
        assert ms > 0
        got = q.cpu().numpy().view(np.uint16)
        assert np.array_equal(got[:n][~nan], want[~nan]), chunk
        assert np.all(got[n:] == 0x5A5A)
        if chunk == 1 << 20:        # a streamed step through the same slots
            m_, v_ = torch.zeros(n).pin_memory(), torch.zeros(n).pin_memory()
            p_ = torch.full((n,), 0.25).pin_memory()
            gs = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
            qs = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
            st = B.so_stream_state()
            st.host_param, st.host_exp_avg, st.host_exp_avg_sq = p_.data_ptr(), m_.data_ptr(), v_.data_ptr()
            st.grad, st.param_lp = gs.data_ptr(), qs.data_ptr()
            st.n_total, st.bucket_elems, st.grad_dtype = n, 1 << 19, B.SO_GRAD_BF16
            B.so_stream_step(ctx, st, hp_struct(B), 1, 1.0)
    assert B.so_stream_cast_params(ctx, host.data_ptr(), q.data_ptr(), 0, 4096, lp) == 0.0
    for bad_chunk in (0, 12):
        with pytest.raises(B.SoError) as ei:
            B.so_stream_cast_params(ctx, host.data_ptr(), q.data_ptr(), n, bad_chunk, lp)
        assert ei.value.status == B.SO_ERR_INVALID_ARG
    with pytest.raises(B.SoError) as ei:
        B.so_stream_cast_params(ctx, host.data_ptr(), q.data_ptr() + 2, n, 4096, lp)
    assert ei.value.status == B.SO_ERR_ALIGNMENT
    with pytest.raises(B.SoError) as ei:
        B.so_cast_params(ctx, q.data_ptr(), q.data_ptr(), 16, 7)
    assert ei.value.status == B.SO_ERR_INVALID_ARG
    host = None
    if pin:
        pin.free()


# --------------------------------------------------------------------------------- placement
@pytest.mark.parametrize("second_set", [False, True])
def test_arena_tune_places_the_arenas_inside_the_workspace(B, ctx, second_set):
    """so_arena_tune: the placement it returns lies inside the workspace, arenas do not overlap,
    it is by its own measurement never slower than the tight layout, the same seed gives the same
    candidates, and a step in the arenas it chose matches the oracle."""
    n = (1 << 22) + 1000
    plan = B.so_arena_plan(n)
    ws_bytes = (3 if second_set else 2) * plan.bytes + (64 << 20)
    ws = torch.empty(ws_bytes + 16, dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)                                            # NaN patterns: the call must clear them itself
    base = ws.data_ptr() + 6                                  # not even 16-byte aligned
    lay, alt, t_tight, t_tuned = B.so_arena_tune(ctx, base, ws_bytes, n, B.SO_GRAD_BF16, 12, 7, second_set)
    assert 0 < t_tuned <= t_tight
    spans = [(lay.param, 4 * n), (lay.grad, 2 * n), (lay.exp_avg, 4 * n), (lay.param_lp, 2 * n), (lay.exp_avg_sq, 4 * n)]
    if second_set:
        spans += [(alt.param, 4 * n), (alt.exp_avg, 4 * n), (alt.exp_avg_sq, 4 * n), (alt.param_lp, 2 * n)]
    spans.sort()
    assert all((base + o) % 16 == 0 for o, _ in spans)
    assert all(a[0] + a[1] <= b[0] for a, b in zip(spans, spans[1:])), spans
    assert spans[-1][0] + spans[-1][1] <= ws_bytes and lay.bytes == spans[-1][0] + spans[-1][1]
    # no timing asked for: the tight layout of so_arena_plan, shifted to the next 16-byte boundary
    lay0, alt0, z0, z1 = B.so_arena_tune(ctx, base, ws_bytes, n, B.SO_GRAD_BF16, 0, 7, second_set)
    assert (z0, z1) == (0.0, 0.0)
    assert [lay0.param, lay0.grad, lay0.exp_avg, lay0.param_lp, lay0.exp_avg_sq] == \
           [10 + x for x in (plan.param, plan.grad, plan.exp_avg, plan.param_lp, plan.exp_avg_sq)]
    # a step in the chosen arenas against the oracle
    def view(off, width, dt):
        o = 6 + off
        return ws[o:o + width * n].view(dt)
    p, m, v = (view(o, 4, torch.float32) for o in (lay.param, lay.exp_avg, lay.exp_avg_sq))
    g, q = view(lay.grad, 2, torch.bfloat16), view(lay.param_lp, 2, torch.bfloat16)
    p.copy_(synth.normal_f32(3, synth.STREAM_PARAM, 0, 0, n, 0.02, "cuda"))
    g.copy_(synth.normal_16bit(3, synth.STREAM_GRAD, 0, 0, n, 1e-3, torch.bfloat16, "cuda"))
    m.zero_(); v.zero_()
    ob = oracle.Bucket(p.cpu().numpy())
    bk = B.bucket_of(g, p, m, v, q)
    for t in (1, 2):
        B.so_adam_step(ctx, bk, hp_struct(B), t, 0.5)
        oracle.adamw_step(bits16(g), 0, ob.p, ob.m, ob.v, ob.q, t=t, s=np.float32(0.5), **HP)
    compare_state((p.cpu().numpy(), m.cpu().numpy(), v.cpu().numpy(), bits16(q)), ob, "tuned arenas: ")
    # errors
    with pytest.raises(B.SoError) as ei:
        B.so_arena_tune(ctx, base, plan.bytes - (4 << 20), n, B.SO_GRAD_BF16, 4, 1, second_set)
    assert ei.value.status == B.SO_ERR_INVALID_ARG
    with pytest.raises(B.SoError) as ei:
        B.so_arena_tune(ctx, base, ws_bytes, 0, B.SO_GRAD_BF16, 4, 1, second_set)
    assert ei.value.status == B.SO_ERR_INVALID_ARG
    d = DevBucket(B, torch.zeros(1024), alt=True)
    B.so_adam_step(ctx, d.c, hp_struct(B), 1, 1.0, B.SO_SPEC_PINGPONG)          # leaves statistics pending
    with pytest.raises(B.SoError) as ei:
        B.so_arena_tune(ctx, base, ws_bytes, n, B.SO_GRAD_BF16, 4, 1, second_set)
    assert ei.value.status == B.SO_ERR_STATE
    B.so_adam_step_stats(ctx)
    B.so_adam_commit(ctx, d.c)


def test_hybrid_step_equals_the_two_separate_steps(B, ctx):
    """Sec. 4.3 repartitioning: resident buckets stepped on a side stream while the host-resident
    buckets stream through.  Checked bit for bit against the two separate calls and, for the
    resident part, against the oracle."""
    n, bucket = 1_000_003, 131_072
    p, m, v = rand_state(n, 910)
    g = synth.normal_16bit(15, synth.STREAM_GRAD, 0, 0, n, 1e-3, torch.bfloat16, "cuda")
    hp = hp_struct(B)
    hybrid_host = [t.cpu().pin_memory() for t in (p, m, v)]
    plain_host = [t.cpu().pin_memory() for t in (p, m, v)]
    qs = [torch.zeros(n, dtype=torch.bfloat16, device="cuda") for _ in range(2)]

    def state(host, q):
        st = B.so_stream_state()
        st.host_param, st.host_exp_avg, st.host_exp_avg_sq = (t.data_ptr() for t in host)
        st.grad, st.param_lp = g.data_ptr(), q.data_ptr()
        st.n_total, st.bucket_elems, st.grad_dtype = n, bucket, B.SO_GRAD_BF16
        return st

    sizes = [300_001, 77, 524_288]
    pair, obs = [], []
    for j, nj in enumerate(sizes):
        pj, mj, vj = rand_state(nj, 920 + j)
        gj = synth.normal_16bit(16, synth.STREAM_GRAD, 0, j << 24, nj, 1e-3, torch.bfloat16, "cuda")
        both = []
        for _ in range(2):
            d = DevBucket(B, pj, m0=mj, v0=vj)
            d.g.copy_(gj)
            both.append(d)
        pair.append(both)
        obs.append((oracle_bucket(pj, mj, vj), bits16(gj)))
    for t in (1, 2):
        rep, res_ms = B.so_hybrid_step(ctx, state(hybrid_host, qs[0]), [d[0].c for d in pair], hp, t, 0.5)
        assert rep.buckets == -(-n // bucket) and res_ms > 0
        B.so_stream_step(ctx, state(plain_host, qs[1]), hp, t, 0.5)
        B.so_adam_step_multi(ctx, [d[1].c for d in pair], hp, t, 0.5)
        for ob, gb in obs:
            oracle.adamw_step(gb, 0, ob.p, ob.m, ob.v, ob.q, t=t, s=0.5, **HP)
    torch.cuda.synchronize()
    for x, y in zip(hybrid_host, plain_host):
        assert_bits_equal(x, y, "hybrid vs plain streamed state")
    assert_bits_equal(qs[0], qs[1], "hybrid vs plain streamed q")
    for (a, b), (ob, _) in zip(pair, obs):
        for name in ("p", "m", "v", "q"):
            assert_bits_equal(getattr(a, name), getattr(b, name), "hybrid vs plain resident " + name)
        compare_state(a.host_state(), ob, "hybrid resident: ")
    # nothing to stream: the call is an ordinary multi-bucket step
    empty = state(hybrid_host, qs[0])
    empty.n_total = 0
    B.so_hybrid_step(ctx, empty, [d[0].c for d in pair], hp, 3, 0.5)
    B.so_adam_step_multi(ctx, [d[1].c for d in pair], hp, 3, 0.5)
    torch.cuda.synchronize()
    for a, b in pair:
        assert_bits_equal(a.p, b.p, "hybrid with empty streamed part")
    # an invalid resident bucket is reported before anything is queued
    before = [t.clone() for t in hybrid_host]
    bad = B.so_bucket()
    for f, _ in B.so_bucket._fields_:
        setattr(bad, f, getattr(pair[0][0].c, f))
    bad.exp_avg = 0
    with pytest.raises(B.SoError):
        B.so_hybrid_step(ctx, state(hybrid_host, qs[0]), [bad], hp, 4, 0.5)
    torch.cuda.synchronize()
    for x, y in zip(hybrid_host, before):
        assert_bits_equal(x, y, "state after a rejected hybrid step")


def test_set_stream_and_two_contexts(B, ctx):
    """The context's work follows so_set_stream; two contexts on two streams do not disturb
    each other (each owns its tables, partial sums and results)."""
    n = 3 * 16384 + 77
    hp = hp_struct(B)
    side = torch.cuda.Stream()
    other = B.so_create(0, side.cuda_stream)
    sets = []
    for k in range(2):
        p, m, v = rand_state(n, 930 + k)
        d, ref = DevBucket(B, p, m0=m, v0=v), DevBucket(B, p, m0=m, v0=v)
        d.g.copy_(synth.normal_16bit(31 + k, synth.STREAM_GRAD, 0, 0, n, 1e-3, torch.bfloat16, "cuda"))
        ref.g.copy_(d.g)
        sets.append((d, ref))
    torch.cuda.synchronize()
    for t in (1, 2, 3):
        B.so_grad_stats_enqueue(ctx, [sets[0][0].c], 1.0, 0.05)
        B.so_grad_stats_enqueue(other, [sets[1][0].c], 1.0, 0.05)
        B.so_adam_step_guarded(ctx, [sets[0][0].c], hp, t)
        B.so_adam_step_guarded(other, [sets[1][0].c], hp, t)
    st0, dec0 = B.so_grad_stats_fetch(ctx)
    st1, dec1 = B.so_grad_stats_fetch(other)
    torch.cuda.synchronize()
    # the same work, one context, default stream, one bucket after the other
    for k, (d, ref) in enumerate(sets):
        for t in (1, 2, 3):
            B.so_grad_stats_enqueue(ctx, [ref.c], 1.0, 0.05)
            B.so_adam_step_guarded(ctx, [ref.c], hp, t)
        st, dec = B.so_grad_stats_fetch(ctx)
        assert (st.sumsq, st.nonfinite, dec.clip) == ((st0, st1)[k].sumsq, 0, (dec0, dec1)[k].clip)
        assert dec.clip < 1.0
        for name in ("p", "m", "v", "q"):
            assert_bits_equal(getattr(d, name), getattr(ref, name), f"context {k} {name}")
    # move the first context onto the side stream and back
    B.so_set_stream(ctx, side.cuda_stream)
    B.so_adam_step(ctx, sets[0][0].c, hp, 4, 0.5)
    side.synchronize()
    B.so_set_stream(ctx, torch.cuda.current_stream().cuda_stream)
    B.so_adam_step(ctx, sets[0][1].c, hp, 4, 0.5)
    torch.cuda.synchronize()
    assert_bits_equal(sets[0][0].p, sets[0][1].p, "after so_set_stream")
    B.so_destroy(other)


@pytest.mark.parametrize("mistake", ["epsilon inside the square root", "decoupled decay dropped",
                                     "bias correction one step late", "gradient multiplier ignored",
                                     "second moment from g instead of g^2"])
def test_parity_comparison_rejects_a_wrong_oracle(B, ctx, tmp_path, mistake):
    """The tolerance is tight enough to tell the method from a near miss: against an oracle with
    one planted mistake (planted on the CPU, in a copy of the oracle) the same comparison that
    passes everywhere else must fail."""
    import test_oracle_mutants as mut
    old, new = next((o, r) for name, o, r in mut.MUTANTS if name == mistake)
    text = open(mut.SRC).read()
    assert text.count(old) == 1
    wrong = mut._compile(text.replace(old, new), str(tmp_path / "wrong.so"))
    n = 100_003
    p, m, v = rand_state(n, 950)
    db = DevBucket(B, p, m0=m, v0=v)
    good, bad = oracle_bucket(p, m, v), oracle_bucket(p, m, v)
    hp = hp_struct(B)
    for t in range(1, 6):
        db.g.copy_(synth.normal_16bit(33, synth.STREAM_GRAD, t, 0, n, 1e-3, torch.bfloat16, "cuda"))
        B.so_adam_step(ctx, db.c, hp, t, 0.5)
        oracle.adamw_step(bits16(db.g), 0, good.p, good.m, good.v, good.q, t=t, s=0.5, **HP)
        with mut._Mutant(wrong):
            oracle.adamw_step(bits16(db.g), 0, bad.p, bad.m, bad.v, bad.q, t=t, s=0.5, **HP)
    compare_state(db.host_state(), good, "right oracle: ")
    with pytest.raises(AssertionError):
        compare_state(db.host_state(), bad, "wrong oracle: ")


def test_contexts_give_their_memory_back(B):
    """Create, use (statistics, step, flatten, streamer, hybrid: everything that allocates on
    first use) and destroy a context many times; device memory must not drain."""
    n = 50_000
    hp = hp_struct(B)
    d = DevBucket(B, torch.ones(n))
    host = [torch.zeros(n).pin_memory() for _ in range(3)]
    q = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    st = B.so_stream_state()
    st.host_param, st.host_exp_avg, st.host_exp_avg_sq = (t.data_ptr() for t in host)
    st.grad, st.param_lp = d.g.data_ptr(), q.data_ptr()
    st.n_total, st.bucket_elems, st.grad_dtype = n, 16384, B.SO_GRAD_BF16
    slices, nb = B.so_layout_plan([n], n)

    def cycle():
        c = B.so_create(0, torch.cuda.current_stream().cuda_stream)
        B.so_grad_stats(c, d.c, 1.0)
        B.so_adam_step(c, d.c, hp, 1, 1.0)
        B.so_flatten(c, slices, [d.p.data_ptr()], [d.m.data_ptr()], 4, 0)
        B.so_hybrid_step(c, st, [d.c], hp, 1, 1.0)
        B.so_train_reset(c, hp)
        B.so_train_capture(c, [d.c])
        B.so_train_replay(c)
        B.so_destroy(c)

    cycle()
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for _ in range(40):
        cycle()
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free0 - free1 < 32 << 20, f"{(free0 - free1) >> 20} MiB lost over 40 contexts"


# --------------------------------------------------------------------------------- errors
def test_argument_errors(B, ctx):
    n = 1024
    d = DevBucket(B, torch.zeros(n + 8))
    hp = hp_struct(B)
    bad = B.so_bucket()
    for f, _ in B.so_bucket._fields_:
        setattr(bad, f, getattr(d.c, f))
    bad.param = d.c.param + 4                       # misaligned
    bad.n = n
    with pytest.raises(B.SoError) as ei:
        B.so_adam_step(ctx, bad, hp, 1, 1.0)
    assert ei.value.status == B.SO_ERR_ALIGNMENT
    with pytest.raises(B.SoError) as ei:
        B.so_adam_step(ctx, d.c, hp, 0, 1.0)        # step < 1
    assert ei.value.status == B.SO_ERR_INVALID_ARG
    with pytest.raises(B.SoError) as ei:
        B.so_adam_step(ctx, d.c, hp, 1, float("nan"))
    assert ei.value.status == B.SO_ERR_INVALID_ARG
    with pytest.raises(B.SoError) as ei:
        B.so_adam_step(ctx, d.c, hp, 1, 1.0, B.SO_SPEC_PINGPONG)   # no alt arrays
    assert ei.value.status == B.SO_ERR_INVALID_ARG
    with pytest.raises(B.SoError) as ei:
        B.so_adam_commit(ctx, d.c)
    assert ei.value.status == B.SO_ERR_STATE
    fresh = B.so_create(0, None)
    with pytest.raises(B.SoError) as ei:
        B.so_adam_step_guarded(fresh, [d.c], hp, 1)
    assert ei.value.status == B.SO_ERR_STATE
    B.so_grad_stats_enqueue(fresh, [d.c], 1.0, 1.0)
    B.so_grad_stats(fresh, [d.c], 1.0)              # overwrites the GPU-side result ...
    with pytest.raises(B.SoError) as ei:            # ... so a guarded step may not use it
        B.so_adam_step_guarded(fresh, [d.c], hp, 1)
    assert ei.value.status == B.SO_ERR_STATE
    B.so_destroy(fresh)
    # hybrid step: a bad resident bucket is reported before anything of the streamed part is queued
    host = [torch.ones(n).pin_memory() for _ in range(3)]
    gs = torch.ones(n, dtype=torch.bfloat16, device="cuda")
    qs = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    st = B.so_stream_state()
    st.host_param, st.host_exp_avg, st.host_exp_avg_sq = (h.data_ptr() for h in host)
    st.grad, st.param_lp = gs.data_ptr(), qs.data_ptr()
    st.n_total, st.bucket_elems, st.grad_dtype = n, 256, B.SO_GRAD_BF16
    with pytest.raises(B.SoError) as ei:
        B.so_hybrid_step(ctx, st, [bad], hp, 1, 1.0)
    assert ei.value.status == B.SO_ERR_ALIGNMENT
    st.staging, st.staging_bytes = gs.data_ptr(), 16          # a workspace far too small
    with pytest.raises(B.SoError) as ei:
        B.so_stream_step(ctx, st, hp, 1, 1.0)
    assert ei.value.status == B.SO_ERR_INVALID_ARG
    with pytest.raises(B.SoError) as ei:
        B.so_flatten_grad_stats(ctx, [B.so_slice(0, 0, 0, 0, 8)], [gs.data_ptr()], [qs.data_ptr()], 7, 1.0, 0.0)
    assert ei.value.status == B.SO_ERR_INVALID_ARG
    with pytest.raises(B.SoError) as ei:
        B.so_flatten(ctx, [B.so_slice(0, 0, 0, 0, 8)], [d.p.data_ptr() + 2], [d.m.data_ptr()], 4, 0)
    assert ei.value.status == B.SO_ERR_ALIGNMENT                  # fp32 tensor at a 2-byte address
    torch.cuda.synchronize()
    assert all(bool((h == 1).all()) for h in host) and not qs.any()
    assert not d.p.any() and not d.m.any()          # nothing was modified
