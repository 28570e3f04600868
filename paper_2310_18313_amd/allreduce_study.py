"""The FP8 gradient all-reduce of Sec. 2.1 run for N simulated ranks on one GPU, under the three scaling
strategies the communication ablation compares (Sec. 3.3): pre-scaling, post-scaling and auto-scaling.

Whatever the strategy, the result is a scaling tensor (payload, N * s_g) that stands for the mean gradient
(Eq. 6).  The strategies differ only in where the payloads sit inside the FP8 range, i.e. in the factor mu
of Eq. 3 that the per-rank scale is multiplied with:

  pre-scaling    every rank's gradient is divided by N before the sum: mu = 1/N.  The sum cannot
                 leave the range; small entries are lost.
  post-scaling   full-range payloads are summed and divided afterwards: mu = 1.  The sum clips.
  auto-scaling   mu follows the saturation statistic of the summed gradient (1/2 after an overflow, back
                 up to 2 over `ramp_steps` clean steps).

Everything that belongs to the method runs in the library's kernels (amax, cast, shared scale, re-quantise,
sum, the hand-over of the auto-scaling state from the summed gradient to the ranks, the error sums and counts);
this module only sequences the calls and turns the error sums into the figures the ablation plots.
"""
from __future__ import annotations

import math
from typing import List, Sequence

import numpy as np
import torch

from . import binding as B

STRATEGIES = ("pre", "post", "auto")


class Fp8AllReduce:
    """State of one simulated data-parallel group: per-rank FP8 payloads and metadata, the summed gradient."""

    def __init__(self, ctx: B.Context, n_ranks: int, total: int, fmt: int, cfg: B.AutoscaleCfg, strategy: str,
                 device: int = 0):
        if strategy not in STRATEGIES:
            raise ValueError(f"strategy must be one of {STRATEGIES}")
        if strategy == "pre" and n_ranks & (n_ranks - 1):
            raise ValueError("pre-scaling keeps scales powers of two only for a power-of-two number of ranks")
        self.ctx, self.n, self.fmt, self.cfg, self.strategy = ctx, n_ranks, fmt, cfg, strategy
        dev = f"cuda:{device}"
        size = max(total, 16)
        self.payload = [torch.zeros(size, dtype=torch.uint8, device=dev) for _ in range(n_ranks)]
        self.shared_payload = [torch.zeros(size, dtype=torch.uint8, device=dev) for _ in range(n_ranks)]
        self.meta = [ctx.new_meta(cfg) for _ in range(n_ranks)]
        self.shared_meta = [ctx.new_meta(cfg) for _ in range(n_ranks)]
        self.summed = torch.zeros(size, dtype=torch.uint8, device=dev)
        self.summed_meta = ctx.new_meta(cfg)
        self.shared = None

    def _plant_mu(self) -> None:
        if self.strategy == "auto":
            self.ctx.autoscale_broadcast(self.summed_meta, self.meta)
        else:
            mu_exp = -int(round(math.log2(self.n))) if self.strategy == "pre" else 0
            for m in self.meta:
                self.ctx.set_mu(m, mu_exp)

    def step(self, grads: Sequence[torch.Tensor]) -> None:
        """grads: one flat high-precision gradient buffer per rank.  Leaves the result in `summed`/`summed_meta`."""
        assert len(grads) == self.n
        c = self.ctx
        self._plant_mu()
        for r, g in enumerate(grads):
            c.amax_scale(g, self.fmt, self.meta[r], self.cfg)
            c.cast_fp8(g, self.payload[r], self.fmt, self.meta[r], self.cfg)
        self.shared = c.shared_scale(self.meta)
        for r in range(self.n):
            c.requantize_fp8(self.payload[r], self.fmt, self.meta[r], self.shared, self.shared_payload[r],
                             self.shared_meta[r])
        c.sum_fp8(self.shared_payload, self.fmt, self.shared, self.summed, self.summed_meta, self.cfg)

    def error_stats(self, mean_grad: torch.Tensor) -> np.ndarray:
        """SNR ingredients and underflow / overflow counts of the summed gradient against the true mean."""
        return self.ctx.quant_error_stats(mean_grad, self.summed, self.fmt, self.summed_meta)


def report(stats: np.ndarray, numels: List[int]) -> dict:
    """Presentation of the kernel's per-tensor sums and counts as the ablation plots them: totals over tensors as
    SNR in dB, underflow rate (of the non-zero reference entries), overflow rate."""
    sig, noi = float(stats["signal"].sum()), float(stats["noise"].sum())
    nz, n = int(stats["n_nonzero"].sum()), int(sum(numels))
    return {"snr_db": float("inf") if noi == 0 else 10 * math.log10(sig / noi) if sig > 0 else float("nan"),
            "underflow_rate": int(stats["n_underflow"].sum()) / max(nz, 1),
            "overflow_rate": int(stats["n_overflow"].sum()) / max(n, 1)}


def main(argv=None) -> None:
    """Prints SNR, underflow rate and overflow rate of the three strategies on synthetic per-rank gradients:
    rank r holds `signal` * s + noise_r, with s and noise_r drawn like the gradients of the chosen workload."""
    import argparse
    import json

    from . import synth

    ap = argparse.ArgumentParser(description=main.__doc__)
    ap.add_argument("--workload", default="gpt125m")
    ap.add_argument("--ranks", type=int, default=8)
    ap.add_argument("--steps", type=int, default=12)
    ap.add_argument("--fmt", choices=["e5m2", "e4m3"], default="e4m3")
    ap.add_argument("--signal", type=float, default=0.25, help="weight of the component all ranks share")
    ap.add_argument("--ramp-steps", type=int, default=8)
    ap.add_argument("--heavy-tails", action="store_true")
    ap.add_argument("--mu-rule", choices=["set-half", "halve"], default="set-half",
                    help="reading of the auto-scaling rule: set mu to 1/2 on overflow (default), or halve it on every "
                         "overflowing step down to 1/ranks")
    a = ap.parse_args(argv)
    wl = synth.workload(a.workload)
    if a.heavy_tails:
        wl.grad_kind = "student_t"
    lay = wl.layout
    fmt = B.E5M2 if a.fmt == "e5m2" else B.E4M3
    if a.mu_rule == "halve":
        cfg = B.autoscale_cfg(ramp_steps=a.ramp_steps, mu_rule=B.MU_HALVE, mu_min_exp=-max(1, int(math.ceil(math.log2(a.ranks)))))
    else:
        cfg = B.autoscale_cfg(ramp_steps=a.ramp_steps)
    ctx = B.Context(lay.tensors())
    size = max(lay.total, 16)
    common = torch.zeros(size, dtype=torch.float32, device="cuda:0")
    grads = [torch.zeros(size, dtype=torch.float32, device="cuda:0") for _ in range(a.ranks)]
    groups = {s: Fp8AllReduce(ctx, a.ranks, lay.total, fmt, cfg, s) for s in STRATEGIES}
    out = {}
    for step in range(1, a.steps + 1):
        synth.fill_gradients(common, wl, 999, step)
        for r, g in enumerate(grads):
            synth.fill_gradients(g, wl, 1000 + r, step)
            g.add_(common, alpha=a.signal)
        mean = torch.stack(grads).sum(dim=0) / a.ranks
        for s, grp in groups.items():
            grp.step(grads)
            out[s] = report(grp.error_stats(mean), lay.numels)
        del mean
    print(json.dumps({"workload": a.workload, "ranks": a.ranks, "fmt": a.fmt, "steps": a.steps, "signal": a.signal,
                      "heavy_tails": a.heavy_tails, "ramp_steps": a.ramp_steps, "mu_rule": a.mu_rule, "last_step": out}))


if __name__ == "__main__":
    main()
