"""Package power and shader clock while a kernel runs, from the amdgpu driver's sysfs files.

The gate's profile leg (paper Sec. 3.1) reads a kernel's time against a ceiling.  On MI355X the ceiling of
a matrix-bound kernel is set by the package power limit: the shader clock is whatever the limit leaves,
and it depends on the operand values.  This module samples the two files an ordinary user can read,

    /sys/class/drm/card*/device/hwmon/hwmon*/power1_input    socket power in microwatts
    /sys/class/drm/card*/device/pp_dpm_sclk                  current shader clock (the starred line)

in a background thread, and, run as a program, writes the record kept under ``profiles/``:

    python3 -m paper_2605_28213_amd.telemetry [--seconds S]

which runs, for S seconds each and with a pause in between, (1) the expert state on the headline
workload, operands rotated over three sets, (2) the register-resident matrix-instruction probe on the
same operand values and (3) the same probe on zeros, and prints power, clock and throughput of each.
No arithmetic of the method lives here.
"""
from __future__ import annotations

import glob
import os
import re
import threading
import time
from typing import Callable, Dict, List, Optional


def _first(pattern: str) -> Optional[str]:
    hits = sorted(glob.glob(pattern))
    return hits[0] if hits else None


class Sampler:
    """Samples socket power (W) and shader clock (MHz) every `interval` seconds between start() and stop()."""

    def __init__(self, interval: float = 0.02, card: int = 0):
        dev = f"/sys/class/drm/card{card}/device"
        self.power_file = _first(dev + "/hwmon/hwmon*/power1_input") or _first(dev + "/hwmon/hwmon*/power1_average")
        self.cap_file = _first(dev + "/hwmon/hwmon*/power1_cap")
        self.sclk_file = dev + "/pp_dpm_sclk" if os.path.exists(dev + "/pp_dpm_sclk") else None
        self.interval = interval
        self.samples: List[tuple] = []          # (seconds since start, watts or None, MHz or None)
        self._stop = threading.Event()
        self._thread: Optional[threading.Thread] = None

    @property
    def available(self) -> bool:
        return self.power_file is not None or self.sclk_file is not None

    def power_cap_w(self) -> Optional[float]:
        try:
            return int(open(self.cap_file).read()) * 1e-6
        except Exception:
            return None

    def read_once(self):
        w = mhz = None
        try:
            w = int(open(self.power_file).read()) * 1e-6
        except Exception:
            pass
        try:
            m = re.search(r"(\d+)\s*Mhz\s*\*", open(self.sclk_file).read())
            mhz = float(m.group(1)) if m else None
        except Exception:
            pass
        return w, mhz

    def start(self) -> "Sampler":
        self.samples, t0 = [], time.perf_counter()
        self._stop.clear()

        def loop():
            while not self._stop.is_set():
                w, mhz = self.read_once()
                self.samples.append((time.perf_counter() - t0, w, mhz))
                self._stop.wait(self.interval)
        self._thread = threading.Thread(target=loop, daemon=True)
        self._thread.start()
        return self

    def stop(self) -> List[tuple]:
        self._stop.set()
        if self._thread is not None:
            self._thread.join()
        return self.samples

    @staticmethod
    def summary(samples: List[tuple], after: float = 0.0) -> Dict[str, Optional[float]]:
        """Mean and extremes of the samples taken later than `after` seconds."""
        ws = [w for t, w, _ in samples if t >= after and w is not None]
        cs = [c for t, _, c in samples if t >= after and c is not None]
        mean = lambda v: sum(v) / len(v) if v else None
        return {"samples": len(ws) or len(cs), "power_w_mean": mean(ws), "power_w_max": max(ws) if ws else None,
                "sclk_mhz_mean": mean(cs), "sclk_mhz_min": min(cs) if cs else None, "sclk_mhz_max": max(cs) if cs else None}


def run_for(seconds: float, launch: Callable[[], None], sync: Callable[[], None], batch: int = 20):
    """Calls launch() in batches for about `seconds`; returns (launches, wall seconds, power/clock samples)."""
    s = Sampler().start()
    t0 = time.perf_counter()
    n = 0
    while time.perf_counter() - t0 < seconds:
        for _ in range(batch):
            launch()
        sync()
        n += batch
    wall = time.perf_counter() - t0
    return n, wall, s.stop()


def main() -> None:
    import argparse

    import numpy as np
    import torch

    from . import gemm
    from . import inputs as gen

    ap = argparse.ArgumentParser()
    ap.add_argument("--seconds", type=float, default=6.0)
    args = ap.parse_args()
    assert torch.cuda.is_available()
    cfg = gen.CONFIGS["C2"]
    inp = gen.make_inputs(cfg, 0)
    stream = torch.cuda.Stream()
    sets = [(torch.from_numpy(inp.A.view(np.uint8).reshape(-1)).cuda(), torch.from_numpy(inp.B.view(np.uint8).reshape(-1)).cuda(),
             torch.empty(cfg.M * cfg.N * 2, dtype=torch.uint8, device="cuda")) for _ in range(3)]
    d = gemm.make_desc(cfg.M, cfg.N, cfg.K, cfg.in_dtype, cfg.out_dtype, cfg.layout_a, cfg.layout_b, stream=stream)
    wgs, iters = 1024, 400
    need = gemm.gemm_probe_mfma_operand_bytes(gemm.GEMM_BF16, wgs)
    sink = torch.zeros(wgs * 256, dtype=torch.float32, device="cuda")
    k = [0]
    flops = [0.0]

    d32 = gemm.make_desc(cfg.M, cfg.N, cfg.K, cfg.in_dtype, cfg.out_dtype, cfg.layout_a, cfg.layout_b, stream=stream,
                         flags=gemm.GEMM_FLAG_MFMA_32X32)

    def gemm_launch_with(desc):
        def f():
            A, B, C = sets[k[0] % 3]
            k[0] += 1
            assert gemm.gemm_run_ex(gemm.GEMM_K4_MFMA, desc, A, B, C) == gemm.GEMM_OK
        return f

    def probe(src, shape16=False):
        def f():
            if shape16:     # the 16x16x32 loop: twice the operand bytes per lane, the same flops in half the iterations
                rc, fl = gemm.gemm_probe_mfma16(gemm.GEMM_BF16, src, 2 * need, wgs, iters // 2, sink, sink.numel() * 4, stream)
            else:
                rc, fl = gemm.gemm_probe_mfma(gemm.GEMM_BF16, src, need, wgs, iters, sink, sink.numel() * 4, stream)
            assert rc == gemm.GEMM_OK
            flops[0] = fl
        return f

    cap = Sampler().power_cap_w()
    idle = Sampler().read_once()
    print(f"power cap {cap} W; idle: {idle[0]} W, {idle[1]} MHz")
    print("| what | launches | us per launch | TFLOP/s | of 2500 | socket W (mean / max after 1 s) | sclk MHz (mean, min-max after 1 s) |")
    print("|---|---|---|---|---|---|---|")
    zeros = torch.zeros(2 * need, dtype=torch.uint8, device="cuda")
    for name, fn, fl in (("K4 on the headline workload (16x16x32 instruction), 3 operand sets", gemm_launch_with(d), cfg.flops),
                         ("the same with the 32x32x16 instruction (GEMM_FLAG_MFMA_32X32)", gemm_launch_with(d32), cfg.flops),
                         ("16x16x32 probe on the headline operands' values", probe(sets[0][0], True), None),
                         ("32x32x16 probe on the headline operands' values", probe(sets[0][0]), None),
                         ("16x16x32 probe on zeros", probe(zeros, True), None),
                         ("32x32x16 probe on zeros", probe(zeros), None)):
        torch.cuda.synchronize()
        time.sleep(2.0)
        n, wall, samples = run_for(args.seconds, fn, stream.synchronize)
        per = wall / n
        tf = (fl if fl is not None else flops[0]) / per / 1e12
        s = Sampler.summary(samples, after=1.0)
        print(f"| {name} | {n} | {per * 1e6:.1f} | {tf:.0f} | {tf / 2500:.3f} | {s['power_w_mean']:.0f} / {s['power_w_max']:.0f} | "
              f"{s['sclk_mhz_mean']:.0f}, {s['sclk_mhz_min']:.0f}-{s['sclk_mhz_max']:.0f} |", flush=True)
        ramp = [(round(t, 2), w, c) for t, w, c in samples if t < 1.0][::5]
        print(f"<!-- first second of '{name}': (s, W, MHz) {ramp} -->")


if __name__ == "__main__":
    main()
