"""so_grad_stats_static -- the entry point that allocates nothing -- against so_grad_stats (bit
for bit: same grid, same order) and against the CPU oracle, on two calls in a row, the second
with a smaller input (so stale partials of the first call would show), with NaN/Inf, both
gradient types, empty input, and the size limit.  Collected last on purpose."""
import ctypes
import math
import struct

import numpy as np
import pytest
import torch

import oracle
import synth
from parity import DevBucket, bits16, dtype_code, NORM_REL

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2509_21271_amd import binding
    return binding


def _read_stats(out: torch.Tensor):
    """so_stats {double sumsq, norm; uint64 nonfinite; int32 overflow, reserved} from device bytes."""
    raw = out.cpu().numpy().tobytes()
    return struct.unpack("<ddQii", raw)[:4]


def _buckets(B, sizes, gdt, seed):
    out = []
    for i, n in enumerate(sizes):
        db = DevBucket(B, torch.zeros(n), gdt)
        if n:
            sig = 1e-3 if gdt == torch.bfloat16 else 40.0
            db.g.copy_(synth.normal_16bit(seed, synth.STREAM_GRAD, i, 0, n, sig, gdt, "cuda"))
        out.append(db)
    return out


@pytest.mark.parametrize("gdt", [torch.bfloat16, torch.float16])
def test_static_statistics_equal_the_context_call_twice_in_a_row(B, gdt):
    stream = torch.cuda.current_stream().cuda_stream
    inv = 1.0 if gdt == torch.bfloat16 else 1.0 / 64.0
    out = torch.zeros(32, dtype=torch.uint8, device="cuda")
    ctx = B.so_create(0, stream)
    big = _buckets(B, [0, 1, 8191, 8192, 8193, 0, 100_003, (1 << 23) + 5, 7, 40_000_000], gdt, 51)
    small = _buckets(B, [3, 12_345], gdt, 52)
    inf, nan = (0x7F80, 0x7FC0) if gdt == torch.bfloat16 else (0x7C00, 0x7E00)
    big[6].g.view(torch.int16)[100_002] = nan
    big[9].g.view(torch.int16)[39_999_999] = inf
    free0 = None
    for rnd, (dbs, bad_want) in enumerate(((big, 2), (small, 0), (big, 2))):
        torch.cuda.synchronize()
        if rnd == 1:
            free0 = torch.cuda.mem_get_info()[0]
        B.so_grad_stats_static([d.c for d in dbs], inv, stream, out.data_ptr())
        torch.cuda.synchronize()
        if rnd == 1:
            assert torch.cuda.mem_get_info()[0] == free0, "the call changed the amount of free device memory"
        sumsq, norm, bad, overflow = _read_stats(out)
        ref = B.so_grad_stats(ctx, [d.c for d in dbs], inv)
        assert (sumsq, norm, bad, overflow) == (ref.sumsq, ref.norm, ref.nonfinite, ref.overflow)
        tot, cnt = 0.0, 0
        for d in dbs:
            s, c = oracle.grad_stats(bits16(d.g), dtype_code(d.g), np.float32(inv))
            tot += s
            cnt += c
        assert bad == cnt == bad_want and overflow == (1 if cnt else 0)
        assert abs(sumsq - tot) <= NORM_REL * tot and abs(norm - math.sqrt(tot)) <= NORM_REL * math.sqrt(tot)
    B.so_destroy(ctx)


def test_static_statistics_empty_input_limit_and_errors(B):
    stream = torch.cuda.current_stream().cuda_stream
    out = torch.full((32,), 0xFF, dtype=torch.uint8, device="cuda")
    B.so_grad_stats_static([], 1.0, stream, out.data_ptr())
    torch.cuda.synchronize()
    assert _read_stats(out) == (0.0, 0.0, 0, 0)
    dbs = _buckets(B, [0, 0], torch.bfloat16, 53)
    out.fill_(0xFF)
    B.so_grad_stats_static([d.c for d in dbs], 1.0, stream, out.data_ptr())
    torch.cuda.synchronize()
    assert _read_stats(out) == (0.0, 0.0, 0, 0)
    # exactly the maximum number of non-empty buckets is accepted, one more is refused
    g = synth.normal_16bit(54, synth.STREAM_GRAD, 0, 0, 129 * 1024, 1e-3, torch.bfloat16, "cuda")
    many = []
    for i in range(129):
        b = B.so_bucket()
        b.grad, b.n, b.grad_dtype = g.data_ptr() + 2 * 1024 * i, 1000 + i, B.SO_GRAD_BF16
        many.append(b)
    B.so_grad_stats_static(many[:128], 1.0, stream, out.data_ptr())
    torch.cuda.synchronize()
    sumsq, norm, bad, overflow = _read_stats(out)
    want = sum(oracle.grad_stats(bits16(g[1024 * i:1024 * i + 1000 + i]), 0, 1.0)[0] for i in range(128))
    assert bad == 0 and abs(sumsq - want) <= NORM_REL * want
    with pytest.raises(B.SoError) as ei:
        B.so_grad_stats_static(many, 1.0, stream, out.data_ptr())
    assert ei.value.status == B.SO_ERR_UNSUPPORTED and "128" in str(ei.value)
    with pytest.raises(B.SoError) as ei:
        B.so_grad_stats_static(many[:2], 1.0, stream, 0)
    assert ei.value.status == B.SO_ERR_INVALID_ARG
    many[1].grad += 2
    with pytest.raises(B.SoError) as ei:
        B.so_grad_stats_static(many[:2], 1.0, stream, out.data_ptr())
    assert ei.value.status == B.SO_ERR_ALIGNMENT


def test_static_statistics_recorded_in_a_hip_graph_and_replayed(B):
    """What the entry point is for: recorded into a HIP graph (nothing may allocate there) and
    replayed, with the program's own eager work and synchronisations between the replays; every
    replay is checked against the context call on the gradients of that moment."""
    gdt = torch.bfloat16
    dbs = _buckets(B, [100_003, 0, 8192 * 3 + 1, 2_000_000], gdt, 55)
    out = torch.zeros(32, dtype=torch.uint8, device="cuda")
    ctx = B.so_create(0, torch.cuda.current_stream().cuda_stream)      # also resolves the scratch address
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.so_grad_stats_static([d.c for d in dbs], 0.5, torch.cuda.current_stream().cuda_stream, out.data_ptr())
    torch.cuda.synchronize()
    eager = torch.zeros(1 << 16, device="cuda")
    for rep in range(4):
        for i, d in enumerate(dbs):                      # new gradients in the same arrays
            if d.n:
                d.g.copy_(synth.normal_16bit(56 + rep, synth.STREAM_GRAD, i, 0, d.n, 1e-3, gdt, "cuda"))
        if rep == 2:
            dbs[3].g.view(torch.int16)[1_999_999] = 0x7F80
        eager.add_(1.0)
        torch.cuda.synchronize()
        out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        sumsq, norm, bad, overflow = _read_stats(out)
        ref = B.so_grad_stats(ctx, [d.c for d in dbs], 0.5)
        assert (sumsq, norm, bad, overflow) == (ref.sumsq, ref.norm, ref.nonfinite, ref.overflow), rep
        assert bad == (1 if rep == 2 else 0)
    assert float(eager[0]) == 4.0
    B.so_destroy(ctx)
