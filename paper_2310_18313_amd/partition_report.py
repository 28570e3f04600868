"""Balance report of the whole-tensor greedy distribution (Sec. 2.3, Alg. 1) on the synthetic model layouts.

For every layout and GPU count: the per-GPU optimizer-state bytes (7 B/param: FP8 gradient, FP8 first moment,
FP16 second moment, FP16 master weight, FP8 weight copy) of the emptiest and the fullest GPU against the
ideal share, and how many tensors the fullest GPU holds.  Host only; uses the library's C function.

    python -m paper_2310_18313_amd.partition_report
"""
from __future__ import annotations

import numpy as np

from . import binding as B
from . import synth

STATE_BYTES_PER_PARAM = 7


def report(names=("flat1m", "gpt125m", "gpt7b", "gpt13b", "gpt175b_layer"), gpu_counts=(2, 8, 64)):
    rows = []
    for name in names:
        lay = synth.workload(name).layout
        sizes = np.array(lay.numels, dtype=np.int64) * STATE_BYTES_PER_PARAM
        for n in gpu_counts:
            owner, usage = B.greedy_partition(sizes, n)
            ideal = sizes.sum() / n
            fullest = int(np.argmax(usage))
            rows.append(dict(layout=name, gpus=n, tensors=lay.n_tensors, ideal_GB=ideal / 1e9, min_GB=usage.min() / 1e9,
                             max_GB=usage.max() / 1e9, max_over_ideal=usage.max() / ideal if ideal else float("nan"),
                             largest_tensor_GB=sizes.max() / 1e9, tensors_on_fullest=int(np.count_nonzero(owner == fullest))))
    return rows


def main() -> None:
    print(f"{'layout':14s} {'GPUs':>4s} {'tensors':>7s} {'ideal GB':>9s} {'min GB':>9s} {'max GB':>9s} {'max/ideal':>9s} "
          f"{'largest tensor GB':>17s} {'tensors on fullest':>18s}")
    for r in report():
        print(f"{r['layout']:14s} {r['gpus']:4d} {r['tensors']:7d} {r['ideal_GB']:9.4f} {r['min_GB']:9.4f} {r['max_GB']:9.4f} "
              f"{r['max_over_ideal']:9.3f} {r['largest_tensor_GB']:17.4f} {r['tensors_on_fullest']:18d}")


if __name__ == "__main__":
    main()
