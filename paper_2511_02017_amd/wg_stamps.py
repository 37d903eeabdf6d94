"""Per-workgroup time stamps of the final-token kernels (a measurement tool, not part of the library's interface).

    python -m paper_2511_02017_amd.build --stamps          # once: libtapout_stamps.so (same sources, -DTAPOUT_WG_STAMPS)
    python -m paper_2511_02017_amd.wg_stamps [workload] [option=value ...]

Runs rounds of a synthetic workload (default llama3) through tapout_round on the stamped build and prints, for the
last round, how long the workgroups of the slice kernel and of the locate kernel spent between their stamps: minimum,
median, 90th percentile, maximum over the workgroups, in microseconds.  The stamps stretch what they measure (each is a
scalar memory instruction its wavefront waits for): read the segments relative to each other; rocprofv3 and bench.py
time the library proper.
"""
from __future__ import annotations

import ctypes as C
import sys

import numpy as np
import torch

from . import binding, build, synth


def table(lib, which: int, n_wg: int, slots: int) -> np.ndarray:
    buf = np.zeros((n_wg, slots), dtype=np.uint64)
    lib.tapout_debug_wg_stamps.argtypes = [C.c_int, C.c_void_p, C.c_int]
    rc = lib.tapout_debug_wg_stamps(which, buf.ctypes.data, n_wg)
    if rc != 0:
        raise RuntimeError(f"tapout_debug_wg_stamps({which}) failed: {rc}")
    return buf.astype(np.int64)


def line(label: str, x: np.ndarray) -> str:
    if x.size == 0:
        return f"{label:44s} (none)"
    us = lambda v: v / 100.0
    return (f"{label:44s} min {us(x.min()):7.2f}  p50 {us(np.median(x)):7.2f}  p90 {us(np.percentile(x, 90)):7.2f}"
            f"  max {us(x.max()):7.2f}")


def main(argv) -> int:
    name = argv[0] if argv and "=" not in argv[0] else "llama3"
    opts = dict(kv.split("=") for kv in argv if "=" in kv)
    lib = binding.load_library(build.LIB_STAMPS)
    if not hasattr(lib, "tapout_debug_wg_stamps"):
        raise RuntimeError("the loaded library carries no time stamps (another build was loaded first)")
    w = synth.WORKLOADS[name]
    gen = synth.RoundGenerator(w, "cuda")
    policy = {"ucb1": binding.UCB1, "ts": binding.TS_BETA}[w.policy]
    tp = binding.Tapout(w.B, w.K, w.V, policy=policy)
    for k, v in opts.items():
        tp.set_option(k, int(v))
    rounds = [gen.round(r) for r in range(2)]
    arm = tp.bandit_select(w.B, u_ts=rounds[0].get("u_ts"))
    calls = [tp.prepare_round_call(r, arm, False, u_ts_next=r.get("u_ts")) for r in rounds]
    st = torch.cuda.current_stream().cuda_stream
    for i in range(21):
        calls[i % 2][0](st)
    torch.cuda.synchronize()

    nsl = (w.V + 2047) // 2048
    gx = (nsl + 3) // 4                                     # slice workgroups per sequence
    n_wg = w.B * gx
    print(f"{name}: V={w.V} B={w.B} K={w.K}; slice kernel: {n_wg} workgroups, {gx} per sequence; options {opts}")
    t = table(lib, 0, n_wg, 8)
    h = table(lib, 1, n_wg, 4)
    t0 = t[:, 0].min()
    ends = t[:, 3:7]
    wg_end = ends.max(axis=1)
    fused = h[:, 0].max() > t0                              # the accept decisions ran inside this launch
    print(line("slices: entry after the first entry", t[:, 0] - t0))
    print(line("slices: entry -> job known", t[:, 1] - t[:, 0]))
    print(line("slices: -> tables in LDS, rows requested", t[:, 2] - t[:, 1]))
    print(line("slices: -> loop done (per wavefront)", (ends - t[:, 2:3])[ends > 0]))
    print(line("slices: workgroup, entry -> last loop done", wg_end - t[:, 0]))
    print(line("slices: last loop done after first entry", wg_end - t0))
    if fused:
        print(line("  decisions: entry -> first data", h[:, 0] - t[:, 0]))
        print(line("  decisions: -> rows merged", h[:, 1] - h[:, 0]))
        print(line("  decisions: -> lse, log p, accept", h[:, 2] - h[:, 1]))
        print(line("  decisions: -> first rejection published", h[:, 3] - h[:, 2]))
        print(line("  decisions: -> job returned", t[:, 1] - h[:, 3]))
        last = (np.arange(n_wg) % gx) == gx - 1
        print(line("  entry -> job known, output-writing workgroups", (t[:, 1] - t[:, 0])[last]))
        print(line("  entry -> job known, the others", (t[:, 1] - t[:, 0])[~last]))

    loc = table(lib, 2, min(2 * w.B, 4096), 8)
    with_fin = loc[:w.B, 7].max() > 0 and 2 * w.B <= 4096   # the launch carried the draft epilogue's workgroups first
    lo = loc[w.B:2 * w.B] if with_fin else loc[:w.B]
    l0 = loc[:, 0][loc[:, 0] > 0].min()
    print(f"locate kernel: {w.B} workgroups" + (f" behind {w.B} of the draft epilogue" if with_fin else ""))
    print(line("locate: entry -> first data", lo[:, 1] - lo[:, 0]))
    print(line("locate: -> total weight known", lo[:, 2] - lo[:, 1]))
    print(line("locate: -> slice found", (lo[:, 3] - lo[:, 2])[lo[:, 3] > 0]))
    print(line("locate: -> token found", (lo[:, 4] - np.maximum(lo[:, 3], lo[:, 2]))[lo[:, 4] > 0]))
    print(line("locate: -> round ended", lo[:, 5] - lo[:, 4]))
    print(line("locate: workgroup total", lo[:, 5] - lo[:, 0]))
    if with_fin:
        fi = loc[:w.B]
        print(line("epilogue: workgroup total", fi[:, 7] - fi[:, 0]))
        print(line("launch: last workgroup done after first entry", np.maximum(fi[:, 7], lo[:, 5]) - l0))
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
