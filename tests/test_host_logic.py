"""CPU-only checks of the library's host side: the shared library loads and exports every
function the header declares, the bucket layout planner, and the validation decision."""
import ctypes
import math
import os
import re

import numpy as np
import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    import paper_2509_21271_amd as pkg
    if not os.path.exists(pkg.LIB):
        pkg.build_library()
    from paper_2509_21271_amd import binding
    return binding


def test_library_exports_every_declared_symbol(B):
    inc = os.path.join(ROOT, "include")
    header = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(so_[a-z_0-9]+)\s*\(", header))
    assert len(declared) >= 24
    lib = ctypes.CDLL(B.LIB)
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared but not exported"
    assert declared == set(B.EXPORTS)
    assert "gfx950" in B.so_version()


def test_struct_sizes_match_header(B):
    assert ctypes.sizeof(B.so_bucket) == 9 * 8 + 8 + 4 * 4
    assert ctypes.sizeof(B.so_hparams) == 28
    assert ctypes.sizeof(B.so_stats) == 32
    assert ctypes.sizeof(B.so_decision) == 24
    assert ctypes.sizeof(B.so_slice) == 40
    assert ctypes.sizeof(B.so_arena_layout) == 48 and ctypes.sizeof(B.so_arena_alt) == 32


@pytest.mark.parametrize("numel,bucket", [([10, 5, 7], 8), ([1, 1, 1], 1), ([0, 9, 0, 3], 4),
                                          ([64], 8), ([3], 100), ([], 5), ([17, 31, 2, 2, 40], 16)])
def test_layout_plan_matches_definition(B, numel, bucket):
    slices, nb = B.so_layout_plan(numel, bucket)
    got = [(s.tensor, s.tensor_offset, s.bucket, s.bucket_offset, s.len) for s in slices]
    want, wnb = oracle.layout_plan(numel, bucket)
    assert got == want and nb == wnb


def test_layout_plan_of_the_benchmark_configs(B):
    import synth
    for i, nb_want in ((0, 1), (1, 5), (2, 27), (3, 81), (4, 117)):
        numel = [n for _, n in synth.tensor_list(i)]
        slices, nb = B.so_layout_plan(numel, synth.config(i)["bucket"])
        assert nb == nb_want
        assert sum(s.len for s in slices) == synth.total_params(i)
        bucket = synth.config(i)["bucket"]
        fill = {}
        for s in slices:
            assert s.bucket_offset == fill.get(s.bucket, 0)      # contiguous, in order
            fill[s.bucket] = s.bucket_offset + s.len
            assert fill[s.bucket] <= bucket
    assert synth.total_params(3) == 8_030_261_248
    assert synth.total_params(1) == 124_439_808


@pytest.mark.parametrize("n", [0, 1, 524_288, 524_289, 16_777_216, 8_030_261_248, 23_319_877_632])
def test_arena_plan_orders_p_g_m_q_v_on_2_mib_boundaries(B, n):
    lay = B.so_arena_plan(n)
    two_mib = 2 << 20
    offs = [lay.param, lay.grad, lay.exp_avg, lay.param_lp, lay.exp_avg_sq]
    sizes = [4 * n, 2 * n, 4 * n, 2 * n, 4 * n]
    assert offs[0] == 0 and offs == sorted(offs) and all(o % two_mib == 0 for o in offs)
    for (o, sz), nxt in zip(zip(offs, sizes), offs[1:] + [lay.bytes - two_mib]):
        assert o + sz <= nxt < o + sz + two_mib or sz == 0 and nxt == o       # tight: less than 2 MiB of padding
    assert lay.bytes == offs[-1] + -(-4 * n // two_mib) * two_mib + two_mib
    # the three fp32 arrays lie one fp32 plus one 16-bit arena apart
    assert lay.exp_avg - lay.param == lay.exp_avg_sq - lay.exp_avg == lay.grad + (lay.exp_avg - lay.grad)
    with pytest.raises(B.SoError):
        B.so_arena_plan(1 << 62)


@pytest.mark.parametrize("second_set", [False, True])
@pytest.mark.parametrize("n,spare", [(1, 0), (524_289, 0), (524_289, 1 << 30), (8_030_261_248, 0),
                                     (8_030_261_248, 80 << 30), (1_310_986_240, 60 << 30)])
def test_arena_candidates_never_overlap_or_leave_the_workspace(B, n, spare, second_set):
    """The placements so_arena_tune times: index 0 is so_arena_plan's layout, every other index a
    permutation of the arenas, packed or with gaps, inside the workspace, 2 MiB-aligned, without
    overlap, and a function of (seed, index) alone."""
    two_mib = 2 << 20
    plan = B.so_arena_plan(n)
    a4, a2 = plan.grad, plan.exp_avg - plan.grad
    packed = 3 * a4 + 2 * a2 + ((3 * a4 + a2) if second_set else 0)
    ws = packed + spare
    lay0, alt0 = B.so_arena_candidate(n, ws, 7, 0, second_set)
    assert [lay0.param, lay0.grad, lay0.exp_avg, lay0.param_lp, lay0.exp_avg_sq] == \
           [plan.param, plan.grad, plan.exp_avg, plan.param_lp, plan.exp_avg_sq]
    if second_set:
        first = plan.exp_avg_sq + a4
        assert [alt0.param, alt0.exp_avg, alt0.exp_avg_sq, alt0.param_lp] == [first, first + a4, first + 2 * a4, first + 3 * a4]
    seen = set()
    gapped = 0
    for index in range(1, 200):
        lay, alt = B.so_arena_candidate(n, ws, 7, index, second_set)
        spans = [(lay.param, 4 * n), (lay.grad, 2 * n), (lay.exp_avg, 4 * n), (lay.param_lp, 2 * n), (lay.exp_avg_sq, 4 * n)]
        if second_set:
            spans += [(alt.param, 4 * n), (alt.exp_avg, 4 * n), (alt.exp_avg_sq, 4 * n), (alt.param_lp, 2 * n)]
        assert all(o % two_mib == 0 for o, _ in spans)
        order = sorted(spans)
        assert all(x[0] + x[1] <= y[0] for x, y in zip(order, order[1:])), (index, order)
        assert order[-1][0] + order[-1][1] == lay.bytes <= ws
        is_packed = order[0][0] == 0 and all(y[0] - (x[0] + x[1]) < two_mib for x, y in zip(order, order[1:]))
        assert is_packed or (index % 2 == 0 and spare >= 512 * two_mib)
        gapped += not is_packed
        seen.add(tuple(o for o, _ in spans))
        again, _ = B.so_arena_candidate(n, ws, 7, index, second_set)
        assert bytes(again) == bytes(lay)
    assert len(seen) > (60 if n > 1 else 0)                  # many different placements among 199 indices
    assert gapped > 60 if spare >= 512 * two_mib else gapped == 0
    with pytest.raises(B.SoError):
        B.so_arena_candidate(n, packed - 1, 7, 3, second_set)
    with pytest.raises(B.SoError):
        B.so_arena_candidate(0, ws, 7, 3, second_set)


def test_layout_plan_rejects_bad_arguments(B):
    with pytest.raises(B.SoError):
        B.so_layout_plan([1, 2], 0)


@pytest.mark.parametrize("norm,max_norm,scale", [(0.5, 1.0, 1.0), (11.155, 1.0, 1.0), (89.6, 1.0, 1.0),
                                                 (3.0, 0.0, 65536.0), (1.0, 1.0, 1.0),
                                                 (1.0 - 1e-6, 1.0, 2.0), (7.0, 2.5, 1024.0)])
def test_validate_matches_oracle_clip(B, norm, max_norm, scale):
    st = B.so_stats(norm * norm, norm, 0, 0, 0)
    dec = B.so_validate(st, max_norm, scale, 1.0)
    clip = oracle.clip_coef(norm, max_norm)
    assert dec.clip == clip
    assert dec.grad_scale == np.float32(clip / scale)
    assert dec.action == (B.SO_ROLLBACK_REDO if clip < 1.0 else B.SO_COMMIT)
    assert dec.next_loss_scale == scale


def test_validate_overflow_halves_the_scale(B):
    st = B.so_stats(float("nan"), float("nan"), 3, 1, 0)
    dec = B.so_validate(st, 1.0, 65536.0, 1.0)
    assert dec.action == B.SO_ROLLBACK_SKIP and dec.next_loss_scale == 32768.0
    dec = B.so_validate(st, 1.0, 1.5, 1.0)
    assert dec.next_loss_scale == 1.0            # floor
    tr = oracle.Trainer([], lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, wd=0.0, loss_scale=1.5)
    tr.buckets = []
    g = [np.array([0x7F80], dtype=np.uint16)]
    tr.buckets = [None]
    assert not tr.iteration(g) and tr.loss_scale == 1.0


def test_plan_resident_is_the_smallest_n_of_the_inequality(B):
    """Brute force over n of the paper's repartitioning inequality (Sec. 4.3)."""
    import itertools
    for mg, so, mp, bwd, sr in itertools.product((0.0, 1.5, 20.0), (0.5, 7.0), (0.0, 3.0), (0.0, 2.0, 9.5),
                                                 (0.1, 1.0)):
        for nbk, cap in ((10, 10), (10, 3), (0, 5), (81, 200)):
            lhs, per = mg + so + mp, bwd + sr
            want = next((n for n in range(0, min(nbk, cap) + 1) if lhs <= n * per), min(nbk, cap))
            assert B.so_plan_resident(mg, so, mp, bwd, sr, nbk, cap) == want
    with pytest.raises(B.SoError):
        B.so_plan_resident(float("nan"), 1, 1, 1, 1, 4, 4)


def test_create_fails_cleanly_without_a_gpu(B):
    """No GPU, no fallback: creating a context must report an error, not crash or emulate."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(B.SoError):
        B.so_create(0, None)


def test_host_only_calls_reject_null_arguments(B):
    lib = ctypes.CDLL(B.LIB)
    lib.so_validate.restype = ctypes.c_int
    assert lib.so_validate(None, ctypes.c_double(1.0), ctypes.c_double(1.0), ctypes.c_double(1.0), None) == B.SO_ERR_INVALID_ARG
    lib.so_layout_plan.restype = ctypes.c_int
    assert lib.so_layout_plan(None, ctypes.c_size_t(0), ctypes.c_uint64(8), None, ctypes.c_size_t(0), None, None) == B.SO_ERR_INVALID_ARG
    lib.so_destroy.restype = ctypes.c_int
    assert lib.so_destroy(None) == B.SO_OK
    lib.so_last_error.restype = ctypes.c_char_p
    assert b"NULL" in lib.so_last_error(None)
    with pytest.raises(B.SoError):
        B.so_validate(B.so_stats(1.0, 1.0, 0, 0, 0), 1.0, 0.0, 1.0)      # loss scale must be > 0


# Hand-worked: start 8, growth after 2 clean iterations in a row, floor 1, ceiling 16.
# (overflow?, scale after the iteration)
LOSS_SCALE_WALK = [(0, 8.0), (0, 16.0), (0, 16.0), (0, 16.0), (1, 8.0), (0, 8.0), (1, 4.0), (1, 2.0),
                   (1, 1.0), (1, 1.0), (0, 1.0), (0, 2.0)]


def test_loss_scale_schedule_follows_the_hand_worked_walk(B):
    scale, clean = 8.0, 0
    for overflow, want in LOSS_SCALE_WALK:
        scale, clean = B.so_loss_scale_next(scale, overflow, clean, 2, 1.0, 16.0)
        assert scale == want
    # growth_interval 0: the scale never grows, and halving agrees with so_validate
    scale, clean = 65536.0, 0
    for it in range(1, 26):
        overflow = it % 5 == 0
        dec = B.so_validate(B.so_stats(1.0, 1.0, int(overflow), int(overflow), 0), 0.0, scale, 1.0)
        scale, clean = B.so_loss_scale_next(scale, overflow, clean, 0)
        assert scale == dec.next_loss_scale
    assert scale == 2048.0
    with pytest.raises(B.SoError):
        B.so_loss_scale_next(0.0, False, 0, 2)
