"""Host-side checks of the C-ABI library: it loads without a GPU, exports what the header
declares, rejects bad arguments before any device work, and its tile schedule covers
exactly the oracle's explicit mask."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2506_04421_amd as hm
from paper_2506_04421_amd import binding
from oracle import hmar_attn_oracle as orc
import synth_inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

SCHEDULES = [si.SIDES_TINY, si.SIDES_256, si.SIDES_512, (1,), (7,), (16,), (1, 1, 1), (2, 5),
             (3, 1, 4, 1, 5), (12, 12), (1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 16), (20, 3, 20)]


def test_library_loads_and_exports_every_declared_symbol():
    lib = hm.load_library()
    header = open(os.path.join(ROOT, "include", "hmar_attn.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(hmar_[a-z_]+)\s*\(", header))
    assert {"hmar_attn_fwd", "hmar_attn_bwd", "hmar_attn_bwd_workspace_bytes", "hmar_status_string",
            "hmar_schedule_describe", "hmar_schedule_tiles"} <= declared
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings():
    assert hm.status_string(0) == "HMAR_OK"
    assert hm.status_string(1) == "HMAR_ERR_INVALID_ARG"
    assert hm.status_string(2) == "HMAR_ERR_UNSUPPORTED"
    assert hm.status_string(3) == "HMAR_ERR_WORKSPACE"
    assert hm.status_string(4) == "HMAR_ERR_HIP"
    assert "UNKNOWN" in hm.status_string(77)


@pytest.mark.parametrize("sides", SCHEDULES)
def test_describe_matches_oracle_schedule(sides):
    offs, pairs = hm.hmar_schedule_describe(sides)
    assert offs == orc.scale_offsets(sides)
    assert pairs == orc.allowed_pairs(sides)


@pytest.mark.parametrize("sides", SCHEDULES)
@pytest.mark.parametrize("which", [0, 1])
def test_tile_schedule_covers_exactly_the_mask(sides, which):
    mask = orc.markov_mask(sides)
    if which == 1:
        mask = mask.T           # owned rows are keys, visited rows are queries
    L = mask.shape[0]
    items, lo, hi = hm.hmar_schedule_tiles(sides, which)
    # per-row ranges are exactly the row's allowed set
    rebuilt = np.zeros_like(mask)
    for r in range(L):
        assert 0 <= lo[r] < hi[r] <= L
        rebuilt[r, lo[r]:hi[r]] = True
    assert np.array_equal(rebuilt, mask)
    # items partition the rows, own at most 128 rows, and visit the union of their rows' ranges
    owned = np.zeros(L, dtype=int)
    for (b, e, ob, oe) in items:
        assert 0 <= b < e <= L and e - b <= 128
        owned[b:e] += 1
        assert ob == min(lo[b:e]) and oe == max(hi[b:e])
        # every 64-wide tile the workgroup loads holds at least one allowed pair
        for t in range(ob, oe, 64):
            assert mask[b:e, t:min(t + 64, oe)].any()
    assert (owned == 1).all()
    # the kernels take a wavefront's extreme ranges from its first and last row: both bounds
    # must be non-decreasing along the rows
    assert all(lo[r] <= lo[r + 1] and hi[r] <= hi[r + 1] for r in range(L - 1))


def test_tile_counts_for_the_benchmark_schedules():
    # 64-row tiles executed per head by 32-row wavefronts: the useful/executed ratio the
    # design quotes (forward): 256px >= 0.80, 512px >= 0.90
    for sides, floor in ((si.SIDES_256, 0.80), (si.SIDES_512, 0.90)):
        items, lo, hi = hm.hmar_schedule_tiles(sides, 0)
        executed = 0
        for (b, e, ob, oe) in items:
            for w in range(b, e, 32):
                rows = range(w, min(w + 32, e))
                wlo = min(lo[r] for r in rows)
                whi = max(hi[r] for r in rows)
                for t in range(ob, oe, 64):
                    if t < whi and t + 64 > wlo:
                        executed += 32 * 64
        assert orc.allowed_pairs(sides) / executed >= floor


def _call_fwd(lib, Q=0x1000, K=0x2000, V=0x3000, O=0x4000, LSE=0x5000, sides=(1, 2), B=1, H=1, D=64, sm=0.0):
    arr = (ctypes.c_int32 * len(sides))(*sides) if sides is not None else None
    return lib.hmar_attn_fwd(Q, K, V, O, LSE, arr, len(sides) if sides is not None else 2, B, H, D, sm, None)


def test_forward_rejects_bad_arguments_before_touching_the_device():
    # fake but well-formed pointers: every call below must return before any device work
    lib = hm.load_library()
    assert _call_fwd(lib, Q=None) == 1
    assert _call_fwd(lib, LSE=None) == 1
    assert _call_fwd(lib, K=0x2004) == 1                 # misaligned
    assert _call_fwd(lib, sides=None) == 1
    assert _call_fwd(lib, sides=(1, 0, 3)) == 1
    assert _call_fwd(lib, sides=(1, -2)) == 1
    assert _call_fwd(lib, B=0) == 1
    assert _call_fwd(lib, H=-1) == 1
    assert _call_fwd(lib, sm=float("nan")) == 1
    assert _call_fwd(lib, D=128) == 2
    assert _call_fwd(lib, D=32) == 2
    assert _call_fwd(lib, sides=(1,) * 65) == 2          # more than HMAR_MAX_SCALES
    assert _call_fwd(lib, sides=(1025,)) == 2            # L beyond HMAR_MAX_SEQ_LEN


def test_backward_rejects_bad_arguments_and_small_workspace():
    lib = hm.load_library()
    sides = (1, 2, 3, 4)
    arr = (ctypes.c_int32 * 4)(*sides)
    need = hm.hmar_attn_bwd_workspace_bytes(sides, 2, 2, 64)
    assert need == 2 * (2 * 2 * 30 * 4)
    assert hm.hmar_attn_bwd_workspace_bytes(sides, 2, 2, 128) == 0
    p = [0x1000 * (i + 1) for i in range(9)]

    def call(ptrs=p, ws=0xA000, ws_bytes=need, D=64):
        return lib.hmar_attn_bwd(*ptrs, arr, 4, 2, 2, D, 0.0, ws, ws_bytes, None)

    assert call(ws_bytes=need - 1) == 3
    assert call(ws=None) == 3
    assert call(ws=0xA008) == 1
    assert call(D=16) == 2
    for i in range(9):
        q = list(p)
        q[i] = None
        assert call(ptrs=q) == 1


def test_binding_refuses_cpu_tensors_and_wrong_dtypes():
    import torch
    x = torch.zeros((1, 1, 5, 64), dtype=torch.bfloat16)
    with pytest.raises(hm.HmarError):
        hm.hmar_attn_fwd(x, x, x, (1, 2))
    assert os.path.exists(binding.LIB_PATH)


def test_binding_refuses_a_host_lse_before_any_library_call(monkeypatch):
    # a host pointer handed to a kernel would fault the GPU: the checks of the per-row fp32
    # tensors must fire in Python.  Device tensors are faked: no GPU is needed for this.
    import torch

    class FakeDeviceTensor:
        """Answers what the binding asks of a tensor, claiming to live on cuda:0."""
        def __init__(self, shape, dtype):
            self.shape, self.dtype, self.is_cuda = torch.Size(shape), dtype, True
            self.device = torch.device("cuda:0")
        def dim(self): return len(self.shape)
        def is_contiguous(self): return True
        def data_ptr(self): raise AssertionError("the library must not be reached")

    monkeypatch.setattr(binding, "_bf16_4d", lambda name, t, shape=None, device=None: t)
    q = FakeDeviceTensor((1, 1, 5, 64), torch.bfloat16)
    k = FakeDeviceTensor((1, 1, 5, 64), torch.bfloat16)
    host_lse = torch.zeros((1, 1, 5), dtype=torch.float32)
    with pytest.raises(hm.HmarError, match="LSE"):
        hm.hmar_attn_fwd_masked(q, k, k, (1, 2), hm.HMAR_MASK_MARKOV, O=q, LSE=host_lse)
    with pytest.raises(hm.HmarError, match="LSE"):
        hm.hmar_attn_step_fwd(q, k, k, 0, O=q, LSE=host_lse)
    with pytest.raises(hm.HmarError, match="LSE"):
        hm.hmar_attn_bwd(q, k, k, q, q, host_lse, (1, 2))
    # and a tensor on another device than Q's is refused by the real check
    monkeypatch.undo()
    with pytest.raises(hm.HmarError):
        binding._f32_stats("LSE", host_lse, (1, 1, 5), torch.device("cuda:0"))


@pytest.mark.parametrize("sides", [si.SIDES_TINY, si.SIDES_256, (2, 5), (3, 1, 4, 1, 5), (20, 3, 20)])
@pytest.mark.parametrize("direction", [0, 1])
def test_block_causal_tile_schedule_covers_exactly_the_var_mask(sides, direction):
    # `which` + 2 selects VAR's block-causal mask (Sec. "Background"): scale k sees every scale <= k
    mask = orc.block_causal_mask(sides)
    if direction == 1:
        mask = mask.T
    L = mask.shape[0]
    items, lo, hi = hm.hmar_schedule_tiles(sides, direction + 2)
    rebuilt = np.zeros_like(mask)
    for r in range(L):
        rebuilt[r, lo[r]:hi[r]] = True
    assert np.array_equal(rebuilt, mask)
    owned = np.zeros(L, dtype=int)
    for (b, e, ob, oe) in items:
        assert e - b <= 128 and ob == min(lo[b:e]) and oe == max(hi[b:e])
        owned[b:e] += 1
    assert (owned == 1).all()
    assert all(lo[r] <= lo[r + 1] and hi[r] <= hi[r + 1] for r in range(L - 1))


def test_step_and_masked_entry_points_reject_bad_arguments():
    lib = hm.load_library()
    arr = (ctypes.c_int32 * 2)(1, 2)
    p = [0x1000 * (i + 1) for i in range(5)]
    assert lib.hmar_attn_fwd_masked(*p, arr, 2, 7, 1, 1, 64, 0.0, None) == 1        # unknown mask kind
    assert lib.hmar_attn_fwd_masked(*p, arr, 2, -1, 1, 1, 64, 0.0, None) == 1
    assert lib.hmar_attn_step_fwd(*p, -1, 4, 1, 1, 64, 0.0, None) == 1
    assert lib.hmar_attn_step_fwd(*p, 4, 0, 1, 1, 64, 0.0, None) == 1
    assert lib.hmar_attn_step_fwd(*p, 4, 9, 1, 1, 32, 0.0, None) == 2
    assert lib.hmar_attn_step_fwd(None, *p[1:], 4, 9, 1, 1, 64, 0.0, None) == 1
    assert lib.hmar_attn_step_fwd(*p, 1 << 20, 9, 1, 1, 64, 0.0, None) == 2           # beyond HMAR_MAX_SEQ_LEN


def test_batched_steps_and_row_subsets_reject_bad_arguments():
    lib = hm.load_library()
    vp = ctypes.c_void_p
    def arrs(n, base=0x1000):
        return [(vp * n)(*[base * (j + 1) + 0x100 * i for i in range(n)]) for j in range(5)]
    i32 = ctypes.c_int32
    ok_prev, ok_cur = (i32 * 2)(1, 4), (i32 * 2)(4, 9)
    a = arrs(2)
    assert lib.hmar_attn_steps_fwd(*a, ok_prev, ok_cur, 0, 1, 1, 64, 0.0, None) == 1            # no steps
    assert lib.hmar_attn_steps_fwd(None, *a[1:], ok_prev, ok_cur, 2, 1, 1, 64, 0.0, None) == 1
    assert lib.hmar_attn_steps_fwd(*a, ok_prev, (i32 * 2)(4, 0), 2, 1, 1, 64, 0.0, None) == 1   # empty step
    assert lib.hmar_attn_steps_fwd(*a, (i32 * 2)(1, -4), ok_cur, 2, 1, 1, 64, 0.0, None) == 1
    bad = arrs(2); bad[3][1] = None
    assert lib.hmar_attn_steps_fwd(*bad, ok_prev, ok_cur, 2, 1, 1, 64, 0.0, None) == 1          # a null O
    mis = arrs(2); mis[1][0] = 0x2008
    assert lib.hmar_attn_steps_fwd(*mis, ok_prev, ok_cur, 2, 1, 1, 64, 0.0, None) == 1          # misaligned K
    assert lib.hmar_attn_steps_fwd(*a, ok_prev, ok_cur, 2, 1, 1, 128, 0.0, None) == 2
    assert lib.hmar_attn_steps_fwd(*a, ok_prev, ok_cur, 2, 1, 1, 64, float("inf"), None) == 1
    many = arrs(1025, base=0x100000)
    assert lib.hmar_attn_steps_fwd(*many, (i32 * 1025)(*([1] * 1025)), (i32 * 1025)(*([1] * 1025)), 1025,
                                   1, 1, 64, 0.0, None) == 2                                        # beyond HMAR_MAX_STEPS
    p = [0x1000 * (i + 1) for i in range(5)]
    rows = 0x9000
    assert lib.hmar_attn_step_fwd_rows(*p, None, 3, 4, 9, 1, 1, 64, 0.0, None) == 1
    assert lib.hmar_attn_step_fwd_rows(*p, rows, 0, 4, 9, 1, 1, 64, 0.0, None) == 1
    assert lib.hmar_attn_step_fwd_rows(*p, rows, 10, 4, 9, 1, 1, 64, 0.0, None) == 1           # more rows than the scale has
    assert lib.hmar_attn_step_fwd_rows(*p, rows + 2, 3, 4, 9, 1, 1, 64, 0.0, None) == 1        # misaligned index list
    assert lib.hmar_attn_step_fwd_rows(*p, rows, 3, 4, 9, 1, 1, 32, 0.0, None) == 2
    assert lib.hmar_attn_step_fwd_rows(*p, rows, 3, -1, 9, 1, 1, 64, 0.0, None) == 1


def test_no_alloc_backward_rejects_what_the_fixed_array_cannot_hold():
    lib = hm.load_library()
    p = [0x1000 * (i + 1) for i in range(9)]
    def call(sides, B, H, D=64):
        arr = (ctypes.c_int32 * len(sides))(*sides)
        return lib.hmar_attn_bwd_noalloc(*p, arr, len(sides), B, H, D, 0.0, None)
    assert call((91,), 1, 1) == 2                    # L = 8281 beyond HMAR_NOALLOC_MAX_SEQ_LEN
    assert call(si.SIDES_256, 64, 25) == 2           # 1 088 000 rows beyond HMAR_NOALLOC_MAX_ROWS
    assert call(si.SIDES_256, 1, 1, D=128) == 2
    assert call((1, 0), 1, 1) == 1
    q = list(p); q[6] = None
    arr = (ctypes.c_int32 * 2)(1, 2)
    assert lib.hmar_attn_bwd_noalloc(*q, arr, 2, 1, 1, 64, 0.0, None) == 1


COUNT_SCHEDULES = [(2, 6, 12, 20), (1, 3, 3, 7), (5,), (130, 70, 300), (1, 2, 6, 12, 20, 30, 56, 90, 156, 240)]


@pytest.mark.parametrize("counts", COUNT_SCHEDULES)
@pytest.mark.parametrize("which", [0, 1, 2, 3])
def test_tile_schedule_for_token_counts_covers_exactly_the_mask(counts, which):
    # `which` + 4: the sizes are token counts of scales that need not be square (Sec. "Background")
    mask = orc.block_causal_mask_from_counts(counts) if which & 2 else orc.markov_mask_from_counts(counts)
    if which & 1:
        mask = mask.T
    L = mask.shape[0]
    items, lo, hi = hm.hmar_schedule_tiles(counts, which + 4)
    assert len(lo) == L
    rebuilt = np.zeros_like(mask)
    for r in range(L):
        rebuilt[r, lo[r]:hi[r]] = True
    assert np.array_equal(rebuilt, mask)
    owned = np.zeros(L, dtype=int)
    for (b, e, ob, oe) in items:
        assert 0 <= b < e <= L and e - b <= 128 and ob == min(lo[b:e]) and oe == max(hi[b:e])
        owned[b:e] += 1
    assert (owned == 1).all()
    assert all(lo[r] <= lo[r + 1] and hi[r] <= hi[r + 1] for r in range(L - 1))


def test_counts_flag_in_the_entry_points():
    lib = hm.load_library()
    counts = (ctypes.c_int32 * 3)(2, 6, 12)
    p = [0x1000 * (i + 1) for i in range(5)]
    # 20 rows with counts, 4 + 36 + 144 = 184 rows with the same numbers read as sides
    assert hm.hmar_attn_bwd_workspace_bytes_masked((2, 6, 12), hm.HMAR_SCALE_COUNTS, 2, 3, 64) == 2 * (2 * 3 * 20 * 4)
    assert hm.hmar_attn_bwd_workspace_bytes_masked((2, 6, 12), hm.HMAR_MASK_MARKOV, 2, 3, 64) == 2 * (2 * 3 * 184 * 4)
    assert hm.hmar_attn_bwd_workspace_bytes_masked((2, 6, 12), hm.HMAR_MASK_BLOCK_CAUSAL | hm.HMAR_SCALE_COUNTS, 1, 1, 64) == 2 * 20 * 4
    assert hm.hmar_attn_bwd_workspace_bytes_masked((2, 6, 12), 0x200, 1, 1, 64) == 0          # unknown flag
    assert lib.hmar_attn_fwd_masked(*p, counts, 3, 0x200, 1, 1, 64, 0.0, None) == 1
    assert lib.hmar_attn_fwd_masked(*p, counts, 3, hm.HMAR_SCALE_COUNTS | 5, 1, 1, 64, 0.0, None) == 1
    big = (ctypes.c_int32 * 2)(1 << 20, 1)                                                      # L beyond HMAR_MAX_SEQ_LEN
    assert lib.hmar_attn_fwd_masked(*p, big, 2, hm.HMAR_SCALE_COUNTS, 1, 1, 64, 0.0, None) == 2
