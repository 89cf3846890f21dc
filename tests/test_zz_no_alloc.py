"""The backward entry point that allocates nothing (hmar_attn_bwd_noalloc), through the C ABI,
against hmar_attn_bwd on the same inputs: two calls in a row, the second with a smaller input
and another schedule, then the first shape again (the fixed device array keeps the last call's
contents; every call must overwrite what it reads)."""
import ctypes

import pytest
import torch

import paper_2506_04421_amd as hm
import synth_inputs as si

pytestmark = pytest.mark.gpu


def _run_both(lib, sides, B, H, seed, dev):
    D = 64
    L = sum(s * s for s in sides)
    Q, K, V, dO = (t.to(dev) for t in si.draw((B, H, L, D), seed=seed, n_tensors=4))
    O, LSE = hm.hmar_attn_fwd(Q, K, V, sides)
    ref = hm.hmar_attn_bwd(Q, K, V, O, dO, LSE, sides)
    outs = [torch.full_like(Q, float("nan")) for _ in range(3)]
    arr = (ctypes.c_int32 * len(sides))(*sides)
    stream = torch.cuda.current_stream(dev).cuda_stream
    rc = lib.hmar_attn_bwd_noalloc(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), dO.data_ptr(),
                                   LSE.data_ptr(), outs[0].data_ptr(), outs[1].data_ptr(), outs[2].data_ptr(),
                                   arr, len(sides), B, H, D, 0.0, stream)
    assert rc == 0, hm.status_string(rc)
    torch.cuda.synchronize()
    for name, got, want in zip(("dQ", "dK", "dV"), outs, ref):
        assert torch.isfinite(got.float()).all(), (sides, name)
        assert torch.equal(got, want), (sides, name, (got.float() - want.float()).abs().max().item())


def test_no_alloc_backward_matches_the_workspace_backward_call_after_call():
    lib = hm.load_library()
    dev = torch.device("cuda:0")
    _run_both(lib, si.SIDES_256, 3, 5, seed=71, dev=dev)      # 10200 rows
    _run_both(lib, (2, 5, 3), 2, 3, seed=72, dev=dev)         # smaller input, other schedule
    _run_both(lib, si.SIDES_256, 3, 5, seed=73, dev=dev)      # the first schedule again, new data
    _run_both(lib, si.SIDES_256, 1, 2, seed=74, dev=dev)      # same schedule, fewer heads


def test_no_alloc_backward_recorded_into_a_graph_brings_its_own_tables():
    # the entry point's callers include code under graph capture: a graph recorded for one
    # schedule must replay correctly after calls for another schedule have used the same array,
    # and calls outside graphs must stay correct after replays
    lib = hm.load_library()
    dev = torch.device("cuda:0")
    D = 64
    _run_both(lib, (2, 5, 3), 1, 2, seed=80, dev=dev)             # the array's address is known from here on
    sides_a, B, H = (1, 2, 3, 4, 5, 6), 2, 3                       # a schedule first used inside the capture
    L = sum(s * s for s in sides_a)
    Q, K, V, dO = (t.to(dev) for t in si.draw((B, H, L, D), seed=81, n_tensors=4))
    O, LSE = hm.hmar_attn_fwd(Q, K, V, sides_a)
    ref = hm.hmar_attn_bwd(Q, K, V, O, dO, LSE, sides_a)
    outs = [torch.full_like(Q, float("nan")) for _ in range(3)]
    arr = (ctypes.c_int32 * len(sides_a))(*sides_a)
    torch.cuda.synchronize()
    side = torch.cuda.Stream(device=dev)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            rc = lib.hmar_attn_bwd_noalloc(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), dO.data_ptr(),
                                           LSE.data_ptr(), outs[0].data_ptr(), outs[1].data_ptr(), outs[2].data_ptr(),
                                           arr, len(sides_a), B, H, D, 0.0, side.cuda_stream)
    assert rc == 0, hm.status_string(rc)
    torch.cuda.synchronize()
    for rep in range(3):
        _run_both(lib, si.SIDES_256, 1, 3, seed=82 + rep, dev=dev)    # another schedule takes the array
        for t in outs:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, got, want in zip(("dQ", "dK", "dV"), outs, ref):
            assert torch.equal(got, want), (rep, name)
        _run_both(lib, si.SIDES_256, 1, 3, seed=90 + rep, dev=dev)    # and is still right after the replay
