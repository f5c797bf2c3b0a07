"""Where the fused projection kernel's time goes, measured on the kernel itself.

    python -m paper_2512_17910_amd.probe build            # on the CPU: the probe builds of the library
    python -m paper_2512_17910_amd.probe run --config 2   # on the GPU: one line per build
    python -m paper_2512_17910_amd.probe run --rows 1024  # the same with 128 of the 256 compute units busy
    python -m paper_2512_17910_amd.probe gaps --config 2  # on the GPU, product build: idle time between calls
    python -m paper_2512_17910_amd.probe mfma             # on the GPU: MFMAs alone, random operands in registers

A probe build (-DALORA_PROBE=bits, csrc/alora_gemm_bf16.hip) is the product kernel with time stamps, and
optionally with the main loop's global -> LDS copies (bit 1) and/or its LDS fragment reads (bit 2) left out, or
with every workgroup fetching the same operand tiles (bit 8), the MFMA sequence unchanged.  The results of those builds are wrong on purpose; they exist to show how long
the same instruction stream takes, and at what clock, with and without its data movement.  `run` starts one
process per build (two builds of the library cannot share a process) and prints, per build, the median time
of a workgroup's phases, the shader-clock cycles of its main loop and the clock that follows from the two.
`gaps` times the product kernel with host-side idle time between calls: a power limit that averaged over time
would let a kernel that follows idle time run faster.
"""
from __future__ import annotations

import argparse
import os
import subprocess
import sys
import time

HERE = os.path.dirname(os.path.abspath(__file__))
PROBE_DIR = os.path.join(HERE, "probe_builds")
VARIANTS = {4: "product instruction stream", 5: "no global->LDS copies in the main loop",
            6: "no LDS fragment reads in the main loop", 7: "neither: the MFMA sequence alone",
            12: "every workgroup fetches tile (0,0)'s operands: copies without L2 misses",
            20: "weights addressed as if stored tile by tile: one contiguous stream per workgroup"}
PHASES = ["entry", "ring issued, rows known", "expand + select done", "first slices landed", "main loop done",
          "stores issued", "stores drained"]


def probe_path(bits: int) -> str:
    return os.path.join(PROBE_DIR, f"libalora_qkv_probe{bits}.so")


def build() -> None:
    from . import build as b
    os.makedirs(PROBE_DIR, exist_ok=True)
    srcs = sorted(os.path.join(b.CSRC, f) for f in os.listdir(b.CSRC) if f.endswith(".hip"))
    for bits in VARIANTS:
        cmd = ["hipcc", *b.FLAGS, f"-DALORA_PROBE={bits}", "-o", probe_path(bits), *srcs]
        subprocess.run(cmd, check=True)
        print("built", probe_path(bits))
    exe = os.path.join(PROBE_DIR, "mfma_rate")
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-O3", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                    "-Wno-unused-command-line-argument", "-o", exe, os.path.join(HERE, "probe_src", "mfma_rate.hip")], check=True)
    print("built", exe)


def _batch(config: int, rows: int = 0):
    """The configuration's batch; with rows > 0 a batch of that many token rows (a multiple of 512) in the shapes
    of configuration 2, which occupies rows / 256 * 32 of the 256 compute units with one tile each."""
    import numpy as np
    from . import workloads as wl
    from .harness import DeviceBatch
    if rows:
        g = np.random.default_rng(5)
        segs = [wl.Segment(s, 0, 512, int(g.integers(0, 8)), int(g.integers(256, 512))) for s in range(rows // 512)]
        w = wl.assemble(f"8b-shapes-{rows}-rows", "bf16", 4096, 32, 8, 128, 8, 32, 16, segs, [512] * (rows // 512), seed=77)
    else:
        w = getattr(wl, f"config{config}")()
    return w, DeviceBatch(w, cache_fill=False)


def run_one(bits: int, config: int, calls: int, rows: int = 0) -> None:
    import ctypes
    import numpy as np
    import torch
    from . import binding as ab
    ab.use_probe_library(probe_path(bits))
    L = ab.lib()
    L.alora_probe_buffer_bytes.restype = ctypes.c_size_t
    L.alora_probe_set_buffer.argtypes = [ctypes.c_void_p]
    w, db = _batch(config, rows)
    if rows:
        ab.alora_qkv_set_tuning(3, 1)   # the tiling of configuration 2, whatever the row count
    nbytes = L.alora_probe_buffer_bytes()
    buf = torch.zeros(nbytes // 8, dtype=torch.int64, device="cuda")
    if L.alora_probe_set_buffer(buf.data_ptr()) != 0:
        raise RuntimeError("alora_probe_set_buffer failed")
    for _ in range(calls):
        ab.alora_qkv_forward(db.x, db.aid, db.start, db.W, db.A, db.B, db.q, db.kc, db.vc, db.slot, w.block_size,
                             db.dims, db.ws)
    torch.cuda.synchronize()
    raw = buf.cpu().numpy()
    n_wg = nbytes // 8 // 12
    st = raw[: n_wg * 8].reshape(n_wg, 8)
    cyc = raw[n_wg * 8:].reshape(n_wg, 4)
    live = (st[:, 0] > 0) & (st[:, 6] > 0)      # workgroups that ran the projection (not the grouping/shrink ones of a decode batch)
    st, cyc = st[live], cyc[live]
    us = (st[:, :7] - st[:, :1]) * 0.01          # the counter runs at 100 MHz
    d = np.diff(us, axis=1)
    loop_us = float(np.median(d[:, 3]))
    loop_cycles = float(np.median(cyc[cyc > 0]))
    span = float((st[:, 6].max() - st[:, 0].min()) * 0.01)
    phases = ", ".join(f"{PHASES[i]} -> {PHASES[i + 1]}: {np.median(d[:, i]):.2f}" for i in range(6))
    print(f"{w.name} probe {bits} ({VARIANTS[bits]}): {len(st)} workgroups, kernel span {span:.1f} us; "
          f"main loop {loop_us:.2f} us, {loop_cycles:.0f} shader cycles -> {loop_cycles / loop_us / 1e3:.3f} GHz; "
          f"median phase times in us: {phases}", flush=True)


def run(config: int, calls: int, rows: int = 0) -> None:
    for bits in VARIANTS:
        if not os.path.exists(probe_path(bits)):
            raise SystemExit(f"{probe_path(bits)} is missing: run `python -m paper_2512_17910_amd.probe build` first")
    for bits in VARIANTS:
        r = subprocess.run([sys.executable, "-m", "paper_2512_17910_amd.probe", "run-one", "--bits", str(bits),
                            "--config", str(config), "--calls", str(calls), "--rows", str(rows)],
                           cwd=os.path.dirname(HERE), timeout=300)
        if r.returncode != 0:      # nothing more on the GPU after a failed step
            raise SystemExit(r.returncode)


def gaps(config: int) -> None:
    import torch
    from . import binding as ab
    w, db = _batch(config)

    def call():
        ab.alora_qkv_forward(db.x, db.aid, db.start, db.W, db.A, db.B, db.q, db.kc, db.vc, db.slot, w.block_size,
                             db.dims, db.ws)
    for _ in range(50):
        call()
    torch.cuda.synchronize()
    for gap_us in (0, 100, 500, 1000, 3000, 0):
        n = 200 if gap_us < 1000 else 80
        ab.alora_qkv_profile_begin(n, every=1)
        torch.cuda.synchronize()
        for _ in range(n):
            call()
            if gap_us:
                torch.cuda.synchronize()
                t = time.perf_counter()
                while time.perf_counter() - t < gap_us * 1e-6:
                    pass
        torch.cuda.synchronize()
        ms, cnt = ab.alora_qkv_profile_end()
        print(f"cfg{config}: {gap_us:5d} us idle between calls: projection kernel {ms * 1e3:7.1f} us (mean of {cnt})",
              flush=True)


def main() -> None:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("what", choices=["build", "run", "run-one", "gaps", "mfma"])
    ap.add_argument("--config", type=int, default=2, choices=[2, 3, 4, 5, 6])
    ap.add_argument("--calls", type=int, default=30)
    ap.add_argument("--bits", type=int, default=4, choices=sorted(VARIANTS))
    ap.add_argument("--rows", type=int, default=0, help="run: a batch of this many rows in configuration 2's shapes instead")
    a = ap.parse_args()
    if a.what == "build":
        build()
    elif a.what == "run":
        run(a.config, a.calls, a.rows)
    elif a.what == "run-one":
        run_one(a.bits, a.config, a.calls, a.rows)
    elif a.what == "mfma":
        raise SystemExit(subprocess.run([os.path.join(PROBE_DIR, "mfma_rate")]).returncode)
    else:
        gaps(a.config)


if __name__ == "__main__":
    main()
