"""Timeline of the compress kernel's phases, per row, from a build with -DPICOSPEC_PHASE_CLOCKS.

    python -m paper_2603_19133_amd.phase_clocks [--rows 4096] [--V 151936] [--k 4096] [--dtype f32|bf16]

Builds a second copy of the library with the clocks compiled in (libpicospec_clocks.so next to the
regular one, which stays as it is), runs picospec_compress on random rows and prints, for a few
generations of rows, how long thread 0 of a workgroup spent between the phase boundaries (100 MHz
wall clock).  The stamped kernel stores 16 words per row behind the prob array, so this caller
allocates that array with room to spare.  A measuring aid: the stamps cost about 5 % of the kernel.
"""
from __future__ import annotations

import argparse
import ctypes as C
import os

import numpy as np
import torch

from . import build as _build

PHASES = [(1, "first loads landed"), (2, "key range of the sample"), (3, "threshold from the sample"),
          (4, "sample claimed"), (5, "streaming done"), (6, "statistics combined"),
          (7, "order: coarse histogram"), (8, "order: bin table"), (9, "order: fine histogram"),
          (10, "order: prefix, pivot"), (11, "order: gather"), (12, "order: rank in bin"),
          (13, "order: placed"), (14, "emission issued"), (15, "end")]


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--rows", type=int, default=4096)
    ap.add_argument("--V", type=int, default=151936)
    ap.add_argument("--k", type=int, default=4096)
    ap.add_argument("--dtype", choices=("f32", "bf16"), default="f32")
    a = ap.parse_args()
    lib_path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libpicospec_clocks.so")
    newest = max(os.path.getmtime(os.path.join(_build.CSRC, f)) for f in os.listdir(_build.CSRC))
    if not os.path.exists(lib_path) or os.path.getmtime(lib_path) < newest:
        _build.build(extra=["-DPICOSPEC_PHASE_CLOCKS"], out=lib_path)
    lib = C.CDLL(lib_path)
    _p, _i32, _i64, _f, _sz = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_size_t
    lib.picospec_compress.argtypes = [_p, C.c_int, _i64, _i32, _i32, _f, _i32, _f, _p, _p, _p, _p, _p, _p, _sz, _p]
    lib.picospec_compress.restype = C.c_int
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(1)
    dt = torch.float32 if a.dtype == "f32" else torch.bfloat16
    x = (torch.randn((a.rows, a.V), device=dev, generator=g) * 5).to(dt)
    extra = (a.rows * 16 * 8 + a.k * 4 - 1) // (a.k * 4) + 1            # rows of prob that hold the stamps
    idx = torch.empty((a.rows, a.k), dtype=torch.int32, device=dev)
    prob = torch.zeros((a.rows + extra, a.k), dtype=torch.float32, device=dev)
    cnt = torch.empty(a.rows, dtype=torch.int32, device=dev)
    mass, lse = torch.empty(a.rows, device=dev), torch.empty(a.rows, device=dev)
    for _ in range(3):
        rc = lib.picospec_compress(x.data_ptr(), 0 if a.dtype == "f32" else 1, a.V, a.rows, a.V, 1.0, a.k, 0.0,
                                   idx.data_ptr(), prob.data_ptr(), cnt.data_ptr(), mass.data_ptr(), lse.data_ptr(),
                                   None, 0, torch.cuda.current_stream().cuda_stream)
        if rc != 0:
            raise RuntimeError(f"picospec_compress rc={rc}")
    torch.cuda.synchronize()
    st = prob.view(-1)[a.rows * a.k:].view(torch.int64)[: a.rows * 16].view(a.rows, 16).cpu().numpy().astype(np.float64)
    t0 = st[:, 0].min()
    resident = 2 * torch.cuda.get_device_properties(0).multi_processor_count
    print(f"rows={a.rows} V={a.V} k={a.k} {a.dtype}: microseconds, mean (min .. max) over the rows of a generation")
    for gen in sorted({0, 1, (a.rows // resident) // 2, a.rows // resident - 1}):
        s = st[gen * resident:(gen + 1) * resident]
        if gen < 0 or not len(s):
            continue
        print(f"rows {gen * resident}..{gen * resident + len(s) - 1}: start {np.mean(s[:, 0] - t0) / 100:.1f} "
              f"({np.min(s[:, 0] - t0) / 100:.1f} .. {np.max(s[:, 0] - t0) / 100:.1f}), row time {np.mean(s[:, 15] - s[:, 0]) / 100:.1f}")
        last = 0
        for i, name in PHASES:
            d = (s[:, i] - s[:, last]) / 100
            print(f"   {name:28s} +{d.mean():6.2f} ({d.min():6.2f} .. {d.max():6.2f})")
            last = i
    print(f"row time, all rows: {np.mean(st[:, 15] - st[:, 0]) / 100:.2f} us; kernel span {(st[:, 15].max() - t0) / 100:.1f} us")
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
