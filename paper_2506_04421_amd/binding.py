"""ctypes binding of libhmar_attn.so: argument marshalling only.

Every step of the path (tile schedule, forward, backward) runs inside the library; this
module turns torch tensors into device pointers and a stream handle, checks dtypes and
shapes, and raises on a non-zero status.  There is no fallback: if the library has not
been built, importing the entry points fails with an error that says how to build it.
"""
from __future__ import annotations

import ctypes
import os
from typing import Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhmar_attn.so")

HMAR_OK = 0
_lib = None


class HmarError(RuntimeError):
    pass


def load_library() -> ctypes.CDLL:
    """dlopen the in-tree library (once) and declare the C signatures."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise HmarError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2506_04421_amd.build` "
            "(there is no CPU or PyTorch fallback for this path)")
    lib = ctypes.CDLL(LIB_PATH)
    i32, i64, f32, vp, sz = ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t
    pi32 = ctypes.POINTER(i32)
    lib.hmar_status_string.restype = ctypes.c_char_p
    lib.hmar_status_string.argtypes = [ctypes.c_int]
    lib.hmar_attn_fwd.restype = ctypes.c_int
    lib.hmar_attn_fwd.argtypes = [vp, vp, vp, vp, vp, pi32, i32, i32, i32, i32, f32, vp]
    lib.hmar_attn_fwd_masked.restype = ctypes.c_int
    lib.hmar_attn_fwd_masked.argtypes = [vp, vp, vp, vp, vp, pi32, i32, i32, i32, i32, i32, f32, vp]
    lib.hmar_attn_step_fwd.restype = ctypes.c_int
    lib.hmar_attn_step_fwd.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, f32, vp]
    pvp = ctypes.POINTER(vp)
    lib.hmar_attn_steps_fwd.restype = ctypes.c_int
    lib.hmar_attn_steps_fwd.argtypes = [pvp, pvp, pvp, pvp, pvp, pi32, pi32, i32, i32, i32, i32, f32, vp]
    lib.hmar_attn_step_fwd_rows.restype = ctypes.c_int
    lib.hmar_attn_step_fwd_rows.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, f32, vp]
    lib.hmar_attn_bwd_masked.restype = ctypes.c_int
    lib.hmar_attn_bwd_masked.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, pi32, i32, i32, i32, i32, i32, f32,
                                         vp, sz, vp]
    lib.hmar_attn_bwd_workspace_bytes.restype = sz
    lib.hmar_attn_bwd_workspace_bytes.argtypes = [pi32, i32, i32, i32, i32]
    lib.hmar_attn_bwd_workspace_bytes_masked.restype = sz
    lib.hmar_attn_bwd_workspace_bytes_masked.argtypes = [pi32, i32, i32, i32, i32, i32]
    lib.hmar_attn_bwd.restype = ctypes.c_int
    lib.hmar_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, pi32, i32, i32, i32, i32, f32, vp, sz, vp]
    lib.hmar_attn_bwd_noalloc.restype = ctypes.c_int
    lib.hmar_attn_bwd_noalloc.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, pi32, i32, i32, i32, i32, f32, vp]
    lib.hmar_schedule_describe.restype = ctypes.c_int
    lib.hmar_schedule_describe.argtypes = [pi32, i32, pi32, ctypes.POINTER(i64)]
    lib.hmar_schedule_tiles.restype = ctypes.c_int
    lib.hmar_schedule_tiles.argtypes = [pi32, i32, i32, pi32, i32, pi32, pi32, pi32]
    lib.hmar_profile_begin.restype = ctypes.c_int
    lib.hmar_profile_begin.argtypes = []
    lib.hmar_profile_end.restype = ctypes.c_int
    lib.hmar_profile_end.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
    lib.hmar_calibration_copy.restype = ctypes.c_int
    lib.hmar_calibration_copy.argtypes = [vp, vp, sz, vp]
    _lib = lib
    return lib


def status_string(code: int) -> str:
    return load_library().hmar_status_string(int(code)).decode()


def _check(code: int, what: str) -> None:
    if code != HMAR_OK:
        raise HmarError(f"{what} failed: {status_string(code)}")


_SIDES_CACHE = {}


def _sides_array(side_lens: Sequence[int], counts: bool = False):
    """(ctypes int32 array, count, L) of a schedule given as side lengths (or, with `counts`, as
    token counts per scale); cached, the hot path calls this per launch."""
    key = (tuple(side_lens), bool(counts))
    hit = _SIDES_CACHE.get(key)
    if hit is None:
        sides = [int(s) for s in key[0]]
        hit = ((ctypes.c_int32 * len(sides))(*sides), len(sides), sum(s if counts else s * s for s in sides))
        _SIDES_CACHE[key] = hit
    return hit


def _bf16_4d(name: str, t: torch.Tensor, shape=None, device=None):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise HmarError(f"{name} must be a device tensor")
    if device is not None and t.device != device:
        raise HmarError(f"{name} is on {t.device}, expected {device}: all tensors of a call share one device")
    if t.dtype != torch.bfloat16 or t.dim() != 4 or not t.is_contiguous():
        raise HmarError(f"{name} must be a contiguous bf16 tensor of shape [B, H, L, D]")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise HmarError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    return t


def _f32_stats(name: str, t: torch.Tensor, shape, device):
    """A per-row fp32 tensor (LSE): a host pointer handed to a kernel would fault the GPU."""
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.device != device:
        raise HmarError(f"{name} must be a device tensor on {device}")
    if t.dtype != torch.float32 or tuple(t.shape) != tuple(shape) or not t.is_contiguous():
        raise HmarError(f"{name} must be a contiguous fp32 tensor of shape {tuple(shape)}")
    return t


class _NoSwitch:
    def __enter__(self):
        return None

    def __exit__(self, *exc):
        return False


_NO_SWITCH = _NoSwitch()


def _on_device(device):
    """Context that makes `device` current for the call; free when it already is."""
    if torch.cuda.current_device() == (device.index if device.index is not None else torch.cuda.current_device()):
        return _NO_SWITCH
    return torch.cuda.device(device)


def _stream_handle(t: torch.Tensor) -> int:
    return torch.cuda.current_stream(t.device).cuda_stream


def hmar_schedule_describe(side_lens: Sequence[int]) -> Tuple[list, int]:
    """(prefix sums off[0..K], allowed (query, key) pairs per head); host only."""
    lib = load_library()
    arr, n, _ = _sides_array(side_lens)
    offs = (ctypes.c_int32 * (n + 1))()
    pairs = ctypes.c_int64(0)
    _check(lib.hmar_schedule_describe(arr, n, offs, ctypes.byref(pairs)), "hmar_schedule_describe")
    return list(offs), int(pairs.value)


def hmar_schedule_tiles(side_lens: Sequence[int], which: int):
    """(items [(own_begin, own_end, other_begin, other_end)], row_lo, row_hi); host only."""
    lib = load_library()
    arr, n, L = _sides_array(side_lens, bool(which & 4))
    cnt = ctypes.c_int32(0)
    _check(lib.hmar_schedule_tiles(arr, n, which, None, 0, ctypes.byref(cnt), None, None), "hmar_schedule_tiles")
    items = (ctypes.c_int32 * (4 * cnt.value))()
    lo = (ctypes.c_int32 * L)()
    hi = (ctypes.c_int32 * L)()
    _check(lib.hmar_schedule_tiles(arr, n, which, items, cnt.value, ctypes.byref(cnt), lo, hi), "hmar_schedule_tiles")
    flat = list(items)
    return [tuple(flat[4 * i:4 * i + 4]) for i in range(cnt.value)], list(lo), list(hi)


HMAR_MASK_MARKOV = 0
HMAR_MASK_BLOCK_CAUSAL = 1
HMAR_SCALE_COUNTS = 0x100      # OR into mask_kind: side_lens holds token counts per scale


def hmar_attn_fwd(Q, K, V, side_lens, sm_scale: float = 0.0, O=None, LSE=None):
    """Forward on the tensors' device and current stream.  Returns (O bf16, LSE fp32)."""
    return hmar_attn_fwd_masked(Q, K, V, side_lens, HMAR_MASK_MARKOV, sm_scale, O, LSE)


def hmar_attn_fwd_masked(Q, K, V, side_lens, mask_kind: int, sm_scale: float = 0.0, O=None, LSE=None):
    """Forward under the Markovian (0) or block-causal (1) mask; OR HMAR_SCALE_COUNTS into mask_kind
    to give token counts per scale instead of side lengths.  Returns (O bf16, LSE fp32)."""
    lib = load_library()
    _bf16_4d("Q", Q)
    B, H, L, D = Q.shape
    _bf16_4d("K", K, Q.shape, Q.device)
    _bf16_4d("V", V, Q.shape, Q.device)
    if O is None:
        O = torch.empty_like(Q)
    if LSE is None:
        LSE = torch.empty((B, H, L), dtype=torch.float32, device=Q.device)
    _bf16_4d("O", O, Q.shape, Q.device)
    _f32_stats("LSE", LSE, (B, H, L), Q.device)
    arr, n, L_sched = _sides_array(side_lens, bool(int(mask_kind) & HMAR_SCALE_COUNTS))
    if L_sched != L:
        raise HmarError("sequence length does not match the scale schedule")
    with _on_device(Q.device):
        code = lib.hmar_attn_fwd_masked(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), LSE.data_ptr(),
                                        arr, n, int(mask_kind), B, H, D, float(sm_scale), _stream_handle(Q))
    _check(code, "hmar_attn_fwd_masked")
    return O, LSE


def _step_tensors(Q, K, V, n_prev, O, LSE):
    _bf16_4d("Q", Q)
    B, H, n_cur, D = Q.shape
    _bf16_4d("K", K, (B, H, int(n_prev) + n_cur, D), Q.device)
    _bf16_4d("V", V, K.shape, Q.device)
    if O is None:
        O = torch.empty_like(Q)
    if LSE is None:
        LSE = torch.empty((B, H, n_cur), dtype=torch.float32, device=Q.device)
    _bf16_4d("O", O, Q.shape, Q.device)
    _f32_stats("LSE", LSE, (B, H, n_cur), Q.device)
    return O, LSE


def hmar_attn_step_fwd(Q, K, V, n_prev: int, sm_scale: float = 0.0, O=None, LSE=None):
    """One inference step: Q [B,H,n_cur,D] against K, V [B,H,n_prev+n_cur,D].  Returns (O, LSE)."""
    lib = load_library()
    O, LSE = _step_tensors(Q, K, V, n_prev, O, LSE)
    B, H, n_cur, D = Q.shape
    with _on_device(Q.device):
        code = lib.hmar_attn_step_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), LSE.data_ptr(),
                                      int(n_prev), n_cur, B, H, D, float(sm_scale), _stream_handle(Q))
    _check(code, "hmar_attn_step_fwd")
    return O, LSE


def hmar_attn_steps_fwd(Qs, Ks, Vs, n_prevs, sm_scale: float = 0.0, Os=None, LSEs=None):
    """Several independent inference steps in one call (see hmar_attn_step_fwd for one step's
    tensors).  Qs, Ks, Vs, n_prevs: equally long sequences.  Returns (list of O, list of LSE)."""
    lib = load_library()
    n = len(Qs)
    if n < 1 or not (len(Ks) == len(Vs) == len(n_prevs) == n):
        raise HmarError("hmar_attn_steps_fwd needs equally long, non-empty lists")
    Os = [None] * n if Os is None else list(Os)
    LSEs = [None] * n if LSEs is None else list(LSEs)
    B, H, _, D = Qs[0].shape
    for i in range(n):
        if tuple(Qs[i].shape[:2]) != (B, H) or Qs[i].shape[3] != D or Qs[i].device != Qs[0].device:
            raise HmarError("every step of a call has the same B, H, D and device")
        Os[i], LSEs[i] = _step_tensors(Qs[i], Ks[i], Vs[i], n_prevs[i], Os[i], LSEs[i])
    vp = ctypes.c_void_p * n
    i32 = ctypes.c_int32 * n
    with _on_device(Qs[0].device):
        code = lib.hmar_attn_steps_fwd(vp(*[t.data_ptr() for t in Qs]), vp(*[t.data_ptr() for t in Ks]),
                                       vp(*[t.data_ptr() for t in Vs]), vp(*[t.data_ptr() for t in Os]),
                                       vp(*[t.data_ptr() for t in LSEs]), i32(*[int(x) for x in n_prevs]),
                                       i32(*[int(q.shape[2]) for q in Qs]), n, B, H, D, float(sm_scale),
                                       _stream_handle(Qs[0]))
    _check(code, "hmar_attn_steps_fwd")
    return Os, LSEs


def hmar_attn_step_fwd_rows(Q, K, V, n_prev: int, rows: torch.Tensor, O, LSE, sm_scale: float = 0.0):
    """One refinement pass inside a scale: only the query rows listed in `rows` (device int32,
    distinct values in [0, n_cur)) are computed; the other rows of O and LSE stay as they are."""
    lib = load_library()
    O, LSE = _step_tensors(Q, K, V, n_prev, O, LSE)
    B, H, n_cur, D = Q.shape
    if (not isinstance(rows, torch.Tensor) or not rows.is_cuda or rows.device != Q.device or rows.dtype != torch.int32
            or rows.dim() != 1 or not rows.is_contiguous() or not 1 <= rows.numel() <= n_cur):
        raise HmarError("rows must be a contiguous device int32 vector of 1..n_cur row indices")
    with _on_device(Q.device):
        code = lib.hmar_attn_step_fwd_rows(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), LSE.data_ptr(),
                                           rows.data_ptr(), rows.numel(), int(n_prev), n_cur, B, H, D,
                                           float(sm_scale), _stream_handle(Q))
    _check(code, "hmar_attn_step_fwd_rows")
    return O, LSE


def hmar_attn_bwd_workspace_bytes(side_lens, B: int, H: int, D: int) -> int:
    lib = load_library()
    arr, n, _ = _sides_array(side_lens)
    return int(lib.hmar_attn_bwd_workspace_bytes(arr, n, B, H, D))


def hmar_attn_bwd_workspace_bytes_masked(side_lens, mask_kind: int, B: int, H: int, D: int) -> int:
    lib = load_library()
    arr, n, _ = _sides_array(side_lens, bool(int(mask_kind) & HMAR_SCALE_COUNTS))
    return int(lib.hmar_attn_bwd_workspace_bytes_masked(arr, n, int(mask_kind), B, H, D))


def hmar_attn_bwd(Q, K, V, O, dO, LSE, side_lens, sm_scale: float = 0.0,
                  dQ=None, dK=None, dV=None, workspace=None):
    """Backward on the tensors' device and current stream.  Returns (dQ, dK, dV) bf16."""
    return hmar_attn_bwd_masked(Q, K, V, O, dO, LSE, side_lens, HMAR_MASK_MARKOV, sm_scale, dQ, dK, dV, workspace)


def hmar_attn_bwd_masked(Q, K, V, O, dO, LSE, side_lens, mask_kind: int, sm_scale: float = 0.0,
                         dQ=None, dK=None, dV=None, workspace=None):
    """Backward under the Markovian (0) or block-causal (1) mask (HMAR_SCALE_COUNTS as in the
    forward).  Returns (dQ, dK, dV) bf16."""
    lib = load_library()
    _bf16_4d("Q", Q)
    B, H, L, D = Q.shape
    for name, t in (("K", K), ("V", V), ("O", O), ("dO", dO)):
        _bf16_4d(name, t, Q.shape, Q.device)
    _f32_stats("LSE", LSE, (B, H, L), Q.device)
    dQ = torch.empty_like(Q) if dQ is None else _bf16_4d("dQ", dQ, Q.shape, Q.device)
    dK = torch.empty_like(Q) if dK is None else _bf16_4d("dK", dK, Q.shape, Q.device)
    dV = torch.empty_like(Q) if dV is None else _bf16_4d("dV", dV, Q.shape, Q.device)
    arr, n, L_sched = _sides_array(side_lens, bool(int(mask_kind) & HMAR_SCALE_COUNTS))
    if L_sched != L:
        raise HmarError("sequence length does not match the scale schedule")
    if workspace is None:
        need = int(lib.hmar_attn_bwd_workspace_bytes_masked(arr, n, int(mask_kind), B, H, D))
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=Q.device)
    elif not isinstance(workspace, torch.Tensor) or not workspace.is_cuda or workspace.device != Q.device:
        raise HmarError("workspace must be a device tensor on the tensors' device")
    ws_bytes = workspace.numel() * workspace.element_size()
    with _on_device(Q.device):
        code = lib.hmar_attn_bwd_masked(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), dO.data_ptr(),
                                        LSE.data_ptr(), dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(),
                                        arr, n, int(mask_kind), B, H, D, float(sm_scale), workspace.data_ptr(),
                                        ws_bytes, _stream_handle(Q))
    _check(code, "hmar_attn_bwd_masked")
    return dQ, dK, dV


def hmar_attn_bwd_noalloc(Q, K, V, O, dO, LSE, side_lens, dQ, dK, dV, sm_scale: float = 0.0):
    """The backward without a workspace and without any allocation (not even of outputs: the
    caller passes dQ, dK, dV).  Markovian mask.  Returns (dQ, dK, dV)."""
    lib = load_library()
    _bf16_4d("Q", Q)
    B, H, L, D = Q.shape
    for name, t in (("K", K), ("V", V), ("O", O), ("dO", dO), ("dQ", dQ), ("dK", dK), ("dV", dV)):
        _bf16_4d(name, t, Q.shape, Q.device)
    _f32_stats("LSE", LSE, (B, H, L), Q.device)
    arr, n, L_sched = _sides_array(side_lens)
    if L_sched != L:
        raise HmarError("sequence length does not match the scale schedule")
    with _on_device(Q.device):
        code = lib.hmar_attn_bwd_noalloc(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), dO.data_ptr(),
                                         LSE.data_ptr(), dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(),
                                         arr, n, B, H, D, float(sm_scale), _stream_handle(Q))
    _check(code, "hmar_attn_bwd_noalloc")
    return dQ, dK, dV


KERNEL_NAMES = ("hmar_fwd_kernel", "hmar_dkdv_kernel", "hmar_dq_kernel")


def hmar_profile_begin() -> None:
    _check(load_library().hmar_profile_begin(), "hmar_profile_begin")


def hmar_profile_end():
    """{kernel name: (total ms, launches)} of the launches since hmar_profile_begin()."""
    ms = (ctypes.c_double * len(KERNEL_NAMES))()
    n = (ctypes.c_int64 * len(KERNEL_NAMES))()
    _check(load_library().hmar_profile_end(ms, n), "hmar_profile_end")
    return {KERNEL_NAMES[i]: (float(ms[i]), int(n[i])) for i in range(len(KERNEL_NAMES))}


def hmar_calibration_copy(dst: torch.Tensor, src: torch.Tensor) -> None:
    """Plain device copy kernel of known size (calibrates rocprofv3's HBM byte counters)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes or not (dst.is_cuda and src.is_cuda):
        raise HmarError("calibration copy needs two device tensors of equal byte size")
    _check(load_library().hmar_calibration_copy(dst.data_ptr(), src.data_ptr(), nbytes, _stream_handle(src)),
           "hmar_calibration_copy")
