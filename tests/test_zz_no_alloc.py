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
