#!/usr/bin/env python3
"""Interleaved A/B timing of builds of the library on one workload, one process, one GPU.

  python -m paper_2506_04421_amd.build --variant occ2 -DHMAR_TUNE_LDS_PAD_FWD=32768
  python -m paper_2506_04421_amd.tuning.ab_time 256px_b32_h24 main occ2

`main` is libhmar_attn.so, any other name libhmar_attn_<name>.so (see build.py).  Every build
runs forward and backward on the same three rotating buffer sets (larger than the last-level
cache), in rounds that alternate between the builds so that clock and temperature drift hit all
alike; the medians over the rounds are printed (forward, backward, and the two back to back on
the same buffers), with the first build as the reference.  Before
the timing, the outputs of every build are compared with the first one's (variants that skip
arithmetic or alias inputs differ by design: the comparison is printed, not asserted).
"""
from __future__ import annotations

import ctypes
import os
import statistics
import sys
import time

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
import synth_inputs as si                                   # noqa: E402
from paper_2506_04421_amd.build import LIB_PATH, variant_path   # noqa: E402


def _load(name: str) -> ctypes.CDLL:
    vp, i32, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
    pi32 = ctypes.POINTER(i32)
    lib = ctypes.CDLL(LIB_PATH if name == "main" else variant_path(name))
    lib.hmar_attn_fwd.restype = ctypes.c_int
    lib.hmar_attn_fwd.argtypes = [vp, vp, vp, vp, vp, pi32, i32, i32, i32, i32, f32, vp]
    lib.hmar_attn_bwd.restype = ctypes.c_int
    lib.hmar_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, pi32, i32, i32, i32, i32, f32, vp, sz, vp]
    lib.hmar_attn_bwd_workspace_bytes.restype = sz
    lib.hmar_attn_bwd_workspace_bytes.argtypes = [pi32, i32, i32, i32, i32]
    return lib


def main() -> int:
    if len(sys.argv) < 3:
        print(__doc__)
        return 2
    w = si.WORKLOADS[sys.argv[1]]
    names = sys.argv[2:]
    libs = {n: _load(n) for n in names}
    dev = torch.device("cuda:0")
    sides = (ctypes.c_int32 * len(w.sides))(*w.sides)
    g = torch.Generator(device=dev)
    g.manual_seed(1)
    sets = []
    for _ in range(3):
        q, k, v, do = (torch.randn((w.B, w.H, w.L, w.D), device=dev, generator=g).to(torch.bfloat16) for _ in range(4))
        sets.append([q, k, v, do, torch.empty_like(q), torch.empty((w.B, w.H, w.L), device=dev, dtype=torch.float32),
                     torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)])
    need = max(int(lib.hmar_attn_bwd_workspace_bytes(sides, len(w.sides), w.B, w.H, w.D)) for lib in libs.values())
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream().cuda_stream

    def fwd(lib, s):
        q, k, v, do, O, LSE, dq, dk, dv = s
        rc = lib.hmar_attn_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), O.data_ptr(), LSE.data_ptr(), sides,
                               len(w.sides), w.B, w.H, w.D, 0.0, stream)
        assert rc == 0, rc

    def bwd(lib, s):
        q, k, v, do, O, LSE, dq, dk, dv = s
        rc = lib.hmar_attn_bwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), O.data_ptr(), do.data_ptr(), LSE.data_ptr(),
                               dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), sides, len(w.sides), w.B, w.H, w.D, 0.0,
                               ws.data_ptr(), need, stream)
        assert rc == 0, rc

    ref = None
    for n, lib in libs.items():
        s = sets[0]
        for t in s[4:]:
            t.fill_(float("nan"))
        print("running", n, flush=True)          # names the build before its first launch
        fwd(lib, s)
        bwd(lib, s)
        torch.cuda.synchronize()
        outs = [t.float().clone() for t in s[4:]]
        if ref is None:
            ref = outs
        else:
            diffs = ", ".join(f"{nm} {(a - b).abs().max().item():.2e}" for nm, a, b in
                              zip(("O", "LSE", "dQ", "dK", "dV"), outs, ref))
            print(f"  {n} vs {names[0]}: max abs difference {diffs}", flush=True)
    for lib in libs.values():
        for s in sets:
            fwd(lib, s)
            bwd(lib, s)
    torch.cuda.synchronize()
    t0 = time.time()                                   # clocks settle under load
    while time.time() - t0 < 0.2:
        for s in sets:
            fwd(libs[names[0]], s)
        torch.cuda.synchronize()
    def step(lib, s):
        fwd(lib, s)
        bwd(lib, s)

    rounds, inner = 12, 9
    res = {n: {"fwd": [], "bwd": [], "step": []} for n in names}
    for _ in range(rounds):
        for n in names:
            for what, fn in (("fwd", fwd), ("bwd", bwd), ("step", step)):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for i in range(inner):
                    fn(libs[n], sets[i % 3])
                e1.record()
                torch.cuda.synchronize()
                res[n][what].append(e0.elapsed_time(e1) / inner * 1000)
    f0 = statistics.median(res[names[0]]["fwd"])
    b0 = statistics.median(res[names[0]]["bwd"])
    s0 = statistics.median(res[names[0]]["step"])
    for n in names:
        f = statistics.median(res[n]["fwd"])
        b = statistics.median(res[n]["bwd"])
        st = statistics.median(res[n]["step"])
        print(f"{w.name} {n:14s} fwd {f:7.1f} us ({(f / f0 - 1) * 100:+5.1f} %)  bwd {b:7.1f} us "
              f"({(b / b0 - 1) * 100:+5.1f} %)  fwd+bwd {st:7.1f} us ({(st / s0 - 1) * 100:+5.1f} %)", flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
