"""Where the time of the streaming expert kernels goes, per workgroup and per role.

Builds a second copy of the library whose expert_stream.hip is compiled with -DMOESD_STREAM_STAMPS (the library
proper is untouched), runs forwards of one benchmark shape through bench.py's runner (cold weight replicas) and prints,
for the gate/up and the down kernel of the last forward:

  * cycles per step of the loading waves (waiting for their loads, at the barrier, issuing the next slot) and of the
    multiplying waves (at the barrier, working),
  * when the 256 workgroups ended (percentiles) and the mean end time of each XCD.

Usage:  python3 -m paper_2505_19645_amd.stream_phases [--config qwen1.5-moe-a2.7b] [--T 64 ...]
"""
from __future__ import annotations

import argparse
import ctypes
import os
import subprocess
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FIELDS = ["t_start", "t_end", "load_wait", "load_barrier", "load_issue", "load_steps",
          "mult_barrier", "mult_work", "mult_steps", "tiles"]


def build_stamped() -> str:
    from paper_2505_19645_amd import build as hip_build
    hip_build.build(force=False)
    bdir = os.path.join(HERE, "_build")
    obj = os.path.join(bdir, "expert_stream_stamps.o")
    lib = os.path.join(bdir, "libmoesd_stamps.so")
    src = os.path.join(hip_build.CSRC, "expert_stream.hip")
    subprocess.run([hip_build.HIPCC] + hip_build.FLAGS + ["-DMOESD_STREAM_STAMPS", "-c", src, "-o", obj],
                   check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    others = [os.path.join(bdir, s + ".o") for s in hip_build.SOURCES if s != "expert_stream.hip"]
    subprocess.run([hip_build.HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + others + [obj], check=True)
    return lib


def report(stamps: np.ndarray, n_wg: int) -> None:
    for mode, name in ((0, "gate/up"), (1, "down")):
        s = {f: stamps[mode, :n_wg, i].astype(np.float64) for i, f in enumerate(FIELDS)}
        if s["mult_steps"].sum() == 0:
            continue
        ls, ms = s["load_steps"].sum(), s["mult_steps"].sum()
        t0 = s["t_start"].min()
        end = (s["t_end"] - t0) / 100.0   # the wall clock ticks at 100 MHz
        pct = np.percentile(end, [0, 10, 50, 90, 100])
        print(f"  {name:8s} {ms / n_wg:6.1f} steps and {s['tiles'].sum() / n_wg:5.1f} tiles per workgroup")
        print(f"           loading waves, cycles per step:     wait for loads {s['load_wait'].sum() / ls:6.0f}   barrier "
              f"{s['load_barrier'].sum() / ls:6.0f}   issue {s['load_issue'].sum() / ls:6.0f}")
        print(f"           multiplying waves, cycles per step: barrier {s['mult_barrier'].sum() / ms:6.0f}   work "
              f"{s['mult_work'].sum() / ms:6.0f}")
        print(f"           workgroup end times, us: min {pct[0]:.1f}  p10 {pct[1]:.1f}  median {pct[2]:.1f}  p90 {pct[3]:.1f}  "
              f"max {pct[4]:.1f}")
        print("           mean end time by XCD (workgroup id mod 8): " + " ".join(f"{end[x::8].mean():.1f}" for x in range(8)))


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="qwen1.5-moe-a2.7b")
    ap.add_argument("--T", type=int, nargs="+", default=[64])
    ap.add_argument("--steps", type=int, default=20)
    args = ap.parse_args()

    from paper_2505_19645_amd import binding
    binding.LIB_PATH = build_stamped()          # before the library is first loaded
    import torch
    import bench
    from paper_2505_19645_amd import synth
    shape = synth.PRESETS[args.config]
    host_w = synth.make_layer(shape, threads=16)
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    for T in args.T:
        run = bench.Runner(shape, host_w, bench.pick_replicas(shape, T))
        run.prepare(synth.make_tokens(shape, T, point=T))
        for i in range(args.steps):
            run.step(i)
        torch.cuda.synchronize()
        buf = np.zeros((2, 1024, len(FIELDS)), dtype=np.int64)
        rc = binding.lib().moesd_stream_stamps(buf.ctypes.data_as(ctypes.c_void_p), ctypes.c_size_t(buf.nbytes))
        if rc != 0:
            raise RuntimeError(f"moesd_stream_stamps: HIP error {rc}")
        print(f"{shape.name}, T = {T}, n_active = {int(run.n_active.item())}: last of {args.steps} forwards")
        report(buf, n_cu)


if __name__ == "__main__":
    main()
