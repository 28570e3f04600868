#!/usr/bin/env python3
"""Benchmark of the FP8 gradient cast + FP8 Adam step on one MI355X.

A "step" is one pass of the whole hot path over one model's flat tensors, all inputs resident in HBM:
    amax + scale      (read 2 B/param)
    FP8 cast          (read 2, write 1)
    fp8lm_adam_step_fp8: amax pass (read 2) + update pass (read 6, write 6)
= 19 algorithmic bytes per parameter.  The default path (`spec`) produces exactly these results but goes through
fp8lm_quantize_fp8, which reads a tensor once for amax and cast together when its power-of-two scale does not
change from the step before (17 bytes per parameter plus 3 for every element of a tensor that has to be cast
again); `--path jit` is the three entry points one after the other.  Successive steps take different gradient
buffers (independent draws), so that amax values move from step to step as they do in training.  The buffers are
placed so that two of the device's three HBM regions share the update pass's traffic (placement.RegionAllocator;
`--arena`: one plain allocation; the other of the two is run in a child process and printed beside the headline).
Prints one JSON line: parameters updated per second, the
achieved HBM bandwidth of the dominant kernel (the Adam update pass, 12 B/param) against the 8 TB/s
peak, the bandwidth that memory-only skeletons of the same kernels reach on the same buffers
("ceilings"), and the CPU oracle timed on the host cores for a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import subprocess
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

BYTES_PER_PARAM = {"amax": 2, "cast": 3, "adam_amax": 2, "adam_update": 12}   # "cast" is 4 on the fused path
HBM_PEAK_GBS = 8000.0


def cpu_baseline(wl, seed: int, budget_s: float = 20.0) -> dict:
    """The CPU oracle, as it stands, on a prefix of the workload sized for about `budget_s` seconds."""
    import numpy as np
    import torch
    import oracle as O
    from paper_2310_18313_amd import synth

    cores = max(1, min(os.cpu_count() or 1, 16))

    def sample_of(target_total: int):
        """Leading tensors of the workload, each cut to its first target/cores elements, until the
        target is reached: every thread then has a similar share whatever the tensor sizes are."""
        cap = max(1, target_total // cores)
        names, numels, acc = [], [], 0
        for nm, n in zip(wl.layout.names, wl.layout.numels):
            if n == 0:
                continue
            names.append(nm)
            numels.append(min(n, cap))
            acc += numels[-1]
            if acc >= target_total:
                break
        return synth.Workload("sample", synth.Layout(names, numels), wl.lr, wl.grad_kind, wl.sigma,
                              ramp_steps=wl.ramp_steps, hist_window=wl.hist_window)

    def run(sample_wl, cores=cores):
        lay = sample_wl.layout
        # deal tensors to threads, largest first, so every thread gets a similar share
        order = sorted(range(lay.n_tensors), key=lambda t: -lay.numels[t])
        shares = [[] for _ in range(cores)]
        loads = [0] * cores
        for t in order:
            k = loads.index(min(loads))
            shares[k].append(t)
            loads[k] += lay.numels[t]
        shares = [s for s in shares if s]
        grad = torch.zeros(lay.total, dtype=torch.bfloat16)
        w0 = torch.zeros(lay.total, dtype=torch.bfloat16)
        synth.fill_gradients(grad, sample_wl, seed, 1)
        synth.fill_weights(w0, lay, seed)
        gbits, wbits = synth.bits16(grad), synth.bits16(w0)
        cfg = O.default_cfg(ramp_steps=sample_wl.ramp_steps, hist_window=sample_wl.hist_window)
        # the threads share the flat buffers and write disjoint tensors of them
        bufs = dict(g8=np.zeros(lay.total, np.uint8), m=np.zeros(lay.total, np.uint8),
                    v=np.zeros(lay.total, np.uint16), w=np.zeros(lay.total, np.uint16),
                    wq=np.zeros(lay.total, np.uint8))
        jobs = []
        for ids in shares:
            tens = O.tensors_array([lay.tensors()[t] for t in ids])
            job = dict(bufs, tens=tens, metas=[O.new_meta(len(ids), cfg) for _ in range(5)])
            O.init_master(wbits, tens, job["w"], job["metas"][3])
            jobs.append(job)
        hp = O.AdamHparams(sample_wl.lr, 0.9, 0.95, 1e-8, 0.1, 1, 1, O.WCOPY_E4M3)

        def one(job):
            g, m, v, w, q = job["metas"]
            O.amax_scale(gbits, job["tens"], O.E5M2, g, cfg)
            O.cast_fp8(gbits, job["tens"], job["g8"], O.E5M2, g, cfg)
            O.adam_step_fp8(job["tens"], job["g8"], O.E5M2, g, job["m"], m, job["v"], v, job["w"], w, job["wq"], q, hp)

        t0 = time.perf_counter()
        with ThreadPoolExecutor(len(jobs)) as ex:
            list(ex.map(one, jobs))
        return time.perf_counter() - t0, lay.n_params, len(jobs)

    dt, n, _ = run(sample_of(1_000_000 * cores))        # calibration
    sample = sample_of(int(min(max(n / dt * budget_s, 1_000_000), 2e9)))
    dt, n, used = run(sample)
    lay = sample.layout
    one_wl = sample_of(int(min(max(n / dt / used * 4.0, 1_000_000), 2e8)))     # about 4 s on one thread
    dt1, n1, _ = run(one_wl, cores=1)
    return {"value": n / dt, "unit": "params/s", "cores": used, "kind": "oracle",
            "sample": f"first {lay.n_tensors} tensors of {wl.name}, each cut to at most {max(lay.numels)} elements "
                      f"({n} params), one step in {dt:.1f} s",
            "single_thread": {"value": n1 / dt1, "unit": "params/s", "sample": f"{n1} params in {dt1:.1f} s"}}


def measured_traffic(workload: str):
    """HBM bytes per launch of the dominant kernel as measured with rocprofv3 --pmc (FETCH_SIZE and
    WRITE_SIZE, scaled by a copy kernel of known size); None when no measurement is recorded."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}.txt")
    try:
        for line in open(path):
            parts = line.split("#")[0].split()
            if len(parts) == 2 and parts[0] == "adam_update":
                return float(parts[1])
    except OSError:
        pass
    return None


def placement_compare(args, spread: bool) -> dict:
    """The chosen path once more in the other placement: one plain arena (v | gradient source | w | m | FP8 gradient |
    copy, one allocation) when the headline ran region-aware, and the other way round.  In a process of its own, begun
    after this one has given its device memory back: where a plain allocation lands depends on what the process
    allocated and freed before, and the figure wanted is that of a fresh process.  Printed beside the headline."""
    cmd = [sys.executable, os.path.abspath(__file__), "--only-path", "--no-cpu-baseline", "--no-ceilings",
           "--workload", args.workload, "--seed", str(args.seed), "--path", args.path, "--steps", str(min(args.steps, 10)),
           "--warmup", str(args.warmup), "--grad-buffers", str(args.grad_buffers), "--exact", str(args.exact),
           "--stats", str(args.stats)] + ([] if spread else ["--arena"]) + (["--wcopy-over-grad"] if args.wcopy_over_grad else [])
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=400)
    lines = [ln for ln in res.stdout.splitlines() if ln.startswith("{")]
    if res.returncode != 0 or len(lines) != 1:
        raise RuntimeError(f"the run in the other placement failed (exit {res.returncode}): {res.stderr.strip().splitlines()[-1:]}")
    d = json.loads(lines[0])
    upd = d["kernels"]["adam_update"]
    return {"command": " ".join(["bench.py"] + cmd[2:]), "placement": d["config"]["placement"], "steps": d["steps"],
            "ms_per_step": round(d["ms_per_step"], 3), "params_per_s": d["value"], "adam_update_avg_ms": upd["avg_ms"],
            "adam_update_frac_of_peak": d["roofline"]["frac"]}


def _region_map_arena(ctx, lay) -> dict:
    """Where in device memory do the streams of the update pass have to lie?  One allocation over nearly all of the
    device; the update-shaped memory skeleton (fp8lm_memory_skeleton: 12 bytes per element, reads and writes mixed,
    no arithmetic) is timed (a) with 2^29 elements, its 16-bit streams at the start and its 8-bit streams d GiB
    further on, (b) at the workload's full size with the five streams at chosen offsets, (c) reads alone."""
    import torch
    from paper_2310_18313_amd import binding as B
    G = 1 << 30
    gib = (torch.cuda.mem_get_info(0)[0] >> 30) - 8
    arena = torch.zeros(gib * G, dtype=torch.uint8, device="cuda:0")

    def timed(shape, bufs, n, reps=3):
        ctx.memory_skeleton(shape, bufs, n)
        torch.cuda.synchronize()
        ctx.set_timing(True)
        ctx.get_timing()
        for _ in range(reps):
            ctx.memory_skeleton(shape, bufs, n)
        k, ms = ctx.get_timing()["skeleton"]
        ctx.set_timing(False)
        return round(ms / k, 3)

    def win(off_gib, nbytes):
        return arena[int(off_gib * G): int(off_gib * G) + nbytes]

    def i16(t):
        return t.view(torch.int16)

    n = 1 << 29
    pair = {}
    for d in range(4, gib - 2, 4):
        b = win(d, 3 * n)
        pair[d] = timed(B.SKEL_UPDATE, [b[:n], b[n:2 * n], i16(win(0, 2 * n)), i16(win(1, 2 * n)), b[2 * n:]], n)
    P = lay.total // 4096 * 4096
    s16, s8 = 2 * P / G, P / G
    full = {}
    if 3 * s16 + 3 * s8 < gib - 100:

        def upd(v, w, m, g, q):
            return timed(B.SKEL_UPDATE, [win(g, P), win(m, P), i16(win(v, 2 * P)), i16(win(w, 2 * P)), win(q, P)], P)

        for base in range(0, int(gib - 2 * s16 - 3 * s8), 24):
            full[f"packed v w m g8 wq from +{base} GiB"] = upd(base, base + s16, base + 2 * s16, base + 2 * s16 + s8,
                                                             base + 2 * s16 + 2 * s8)
        full["one arena from +0 in the order v, gradient source, w, m, g8, wq"] = upd(0, 2 * s16, 3 * s16, 3 * s16 + s8, 3 * s16 + 2 * s8)
        full["one arena from +0 in the order v, wq, gradient source, w, g8, m (what --arena allocates)"] = upd(0, 2 * s16 + s8, 3 * s16 + 2 * s8, 3 * s16 + s8, s16)
        full["v wq / w m g8: second group from +100 GiB"] = upd(0, 100, 100 + s16, 100 + s16 + s8, s16)
        full["v m / w g8 wq: second group from +100 GiB"] = upd(0, 100, s16, 100 + s16, 100 + s16 + s8)
        full["v / w / m g8 wq at +0, +100, +200 GiB"] = upd(0, 100, 200, 200 + s8, 200 + 2 * s8)
        # the pass's reads alone and its writes alone (6 bytes per element each), in one region and over two
        for tag, shape in (("reads alone", B.SKEL_UPDATE_READS), ("writes alone", B.SKEL_UPDATE_WRITES)):
            full[f"{tag}, all streams from +0 GiB"] = timed(shape, [win(2 * s16, P), win(2 * s16 + s8, P), i16(win(0, 2 * P)),
                                                                    i16(win(s16, 2 * P)), win(2 * s16 + 2 * s8, P)], P)
            full[f"{tag}, v wq / w m g8: second group from +100 GiB"] = timed(
                shape, [win(100 + s16 + s8, P), win(100 + s16, P), i16(win(0, 2 * P)), i16(win(100, 2 * P)), win(s16, P)], P)
    reads = {o: timed(B.SKEL_READ16, [i16(win(o, 8 * G))], 4 * G) for o in range(0, gib - 8, 40)}
    return {"device_GiB_used": gib, "params": P,
            "update_skeleton_ms_2^29_elements_16bit_streams_at_0_8bit_streams_at_GiB": pair,
            "update_skeleton_ms_full_size": full, "read16_ms_8GiB_at_GiB": reads}


def region_map(lay) -> dict:
    """bench.py --region-map: the table over one allocation of nearly all device memory, then one written buffer in
    three placements."""
    import torch
    from paper_2310_18313_amd import binding as B
    from paper_2310_18313_amd.placement import StripedArena, probe_ms
    G = 1 << 30
    ctx = B.Context(lay.tensors())
    out = _region_map_arena(ctx, lay)           # its allocation is gone when it returns
    gc.collect()
    torch.cuda.empty_cache()
    P = out["params"]

    def timed(shape, bufs, n, reps=3):
        ctx.memory_skeleton(shape, bufs, n)
        torch.cuda.synchronize()
        ctx.set_timing(True)
        ctx.get_timing()
        for _ in range(reps):
            ctx.memory_skeleton(shape, bufs, n)
        k, ms = ctx.get_timing()["skeleton"]
        ctx.set_timing(False)
        return round(ms / k, 3)

    # One written buffer: beside the buffer that is read, 100 GiB further on, and in 1 GiB pieces that alternate between
    # two regions (placement.StripedArena).  Where the plain allocations lie is looked up with the probe.
    striped = {}
    if 7 * P < (torch.cuda.mem_get_info(0)[0] - 110 * G):
        src = torch.zeros(2 * P, dtype=torch.uint8, device="cuda:0")
        same = torch.zeros(P, dtype=torch.uint8, device="cuda:0")
        spacer = torch.empty(100 * G, dtype=torch.uint8, device="cuda:0")
        other = torch.zeros(P, dtype=torch.uint8, device="cuda:0")
        del spacer
        torch.cuda.empty_cache()
        n_pr = 1 << 28
        t_same, t_other = probe_ms(ctx, src, same, n_pr), probe_ms(ctx, src, other, n_pr)
        st8 = StripedArena(ctx, P).tensor(0, P)
        where = lambda t: "in the source's region" if 12 * n_pr / (t * 1e-3) < 5.5e12 else "in another region"
        for tag, dst in ((f"plain allocation made right after the source: {where(t_same)} (probe {t_same:.3f} ms)", same),
                         (f"plain allocation made 100 GiB later: {where(t_other)} (probe {t_other:.3f} ms)", other),
                         ("pieces of 1 GiB alternating between two regions", st8)):
            striped[tag] = {"cast_shape_ms": timed(B.SKEL_CAST, [src.view(torch.int16), dst], P),
                            "write8_ms": timed(B.SKEL_WRITE8, [dst], P),
                            "read8x2_with_half_the_source_ms": timed(B.SKEL_READ8X2, [dst, src[:P]], P)}
    out["one_written_buffer_13B_layout"] = striped
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="gpt13b")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-budget", type=float, default=20.0, help="seconds of oracle work the cpu_baseline leg aims for")
    ap.add_argument("--chunk", type=int, default=0)
    ap.add_argument("--blocks-per-cu", type=int, default=0)
    ap.add_argument("--single-pass-min-chunks", type=int, default=-1,
                    help="chunks per workgroup below which tensors are finished by a second launch (0: never)")
    ap.add_argument("--exact", type=int, default=1)
    ap.add_argument("--stats", type=int, default=0)
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run the library's plain 128-bit copy kernel over 4 GiB (m -> FP8 gradient buffer) three times: "
                         "a kernel of known size that profiler counters are scaled by")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the memory-only skeletons of the four kernels that are timed on the same buffers after the step")
    ap.add_argument("--path", choices=["spec", "jit", "fused", "spec-fused", "spec-m2", "single"], default="spec",
                    help="jit: amax pass + cast + two-pass Adam (19 B/param, the three entry points as they are); "
                         "spec: the same results through fp8lm_quantize_fp8, which casts with the predicted scale while "
                         "measuring the amax and casts again only the tensors whose scale changed (17 B/param + redone "
                         "tensors); fused: same results, the cast also does the Adam step's first pass (18 B/param, one "
                         "GPU only); spec-fused: both (16 B/param + redone tensors); spec-m2: spec, and the Adam step "
                         "through fp8lm_adam_step_fp8_m2, which drops the read-only pass for a second first-moment buffer "
                         "(same results; 15 B/param + redone tensors; state 7 instead of 6 B/param); single: delayed "
                         "gradient scaling + predicted first-moment scale (15 B/param, results differ: looser scales)")
    ap.add_argument("--grad-buffers", type=int, default=3,
                    help="number of gradient source buffers with independent draws that successive steps rotate through")
    ap.add_argument("--allreduce-steps", type=int, default=0, metavar="N",
                    help="also time the shared-scale re-quantise kernel and the N-rank FP8 sum (Eq. 4-6) on this layout")
    ap.add_argument("--only-path", action="store_true",
                    help="time the chosen path only: not the other paths, not the repeat in the other placement")
    ap.add_argument("--arena", action="store_true",
                    help="carve all buffers out of one plain allocation, one after the other.  Default: the two halves "
                         "of the update pass's traffic are placed in different HBM regions by placement.RegionAllocator "
                         "(plain allocations, checked by timing; spacers up to the next region are held briefly)")
    ap.add_argument("--spread", action="store_true", help="what the default does (kept for older command lines)")
    ap.add_argument("--region-map", action="store_true",
                    help="instead of the benchmark: time the update-shaped memory skeleton with its streams at chosen "
                         "places of one allocation over nearly all device memory, and print the table as JSON")
    ap.add_argument("--wcopy-over-grad", action="store_true",
                    help="write the E4M3 weight copy over the FP8 gradient (wcopy == grad): one buffer fewer, same bytes moved")
    ap.add_argument("--no-placement-compare", "--no-spread-compare", dest="no_placement_compare", action="store_true",
                    help="do not repeat the measurement in the other placement (one plain arena, or with --arena the "
                         "region-aware one) after the headline run")
    ap.add_argument("--arena-order", default="", help="comma-separated buffer names (v,grad,w,m,g8,wq) in the order they are "
                    "carved out of the one allocation")
    ap.add_argument("--graph", action="store_true",
                    help="also record one step into a HIP graph and time its replays (small workloads are bound by "
                         "launch latency; the hyper-parameters, step number included, are baked into the graph)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2310_18313_amd import binding as B
    from paper_2310_18313_amd import synth
    from paper_2310_18313_amd.state import OptimizerState

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    B.lib()  # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    wl = synth.workload(args.workload)
    lay = wl.layout
    P = lay.n_params
    cfg = B.autoscale_cfg(ramp_steps=wl.ramp_steps, hist_window=wl.hist_window)
    if args.region_map:
        print(json.dumps(region_map(lay)), flush=True)
        return 0
    st = OptimizerState(lay.tensors(), lay.total, cfg, 0, B.E5M2, B.WCOPY_E4M3, spread=not args.arena,
                        grad_buffer=True, n_grad_buffers=max(1, args.grad_buffers),
                        arena_order=args.arena_order.split(",") if args.arena_order else None,
                        second_m=(args.path == "spec-m2" or (not args.only_path and not args.wcopy_over_grad)),
                        wcopy_over_grad=args.wcopy_over_grad)
    if args.chunk or args.blocks_per_cu or args.single_pass_min_chunks >= 0:
        st.ctx.set_tuning(args.chunk or 16384, args.blocks_per_cu or 16,
                          (1 << 30) if args.single_pass_min_chunks < 0 else args.single_pass_min_chunks)
    grad = st.grad
    placement = {"allocation": "two groups in different HBM regions" if st.spread else
                 ("one arena" if args.arena else "plain, one allocation per buffer (regions not told apart)"),
                 **st.placement}
    if st.spread:
        from paper_2310_18313_amd.placement import verify_spread
        placement["check_v_vs_w"] = verify_spread(st.ctx, st.v, st.w)      # overwrites both
        st.v.zero_()
        st.w.zero_()
    synth.fill_weights(grad, lay, args.seed)          # reuse the buffer for the initial weights
    st.init_master(grad)
    torch.cuda.synchronize()
    # gradient sources: independent draws that successive steps rotate through (allocated with the state)
    grad.zero_()
    grads = st.grads
    for k, gbuf in enumerate(grads):
        synth.fill_gradients(gbuf, wl, args.seed, 1 + k)
    torch.cuda.synchronize()

    base_bytes = {"jit": 19, "fused": 18, "single": 15, "spec": 17, "spec-fused": 16, "spec-m2": 15}   # before anything is redone
    mode_of = {"jit": B.MSCALE_EXACT_PASS, "fused": B.MSCALE_FROM_CAST, "single": B.MSCALE_PREDICTED,
               "spec": B.MSCALE_EXACT_PASS, "spec-fused": B.MSCALE_FROM_CAST, "spec-m2": B.MSCALE_EXACT_PASS}
    step_no = [0]

    def run_steps(path, n):
        """n steps of one path; the very first step of the run is always just in time (it seeds the history)."""
        for _ in range(n):
            step_no[0] += 1
            hp = B.adam_hparams(wl.lr, step_no[0], exact=args.exact, stats=args.stats, m_scale_mode=mode_of[path])
            st.step(grads[step_no[0] % len(grads)], hp, delayed=(path == "single" and step_no[0] > 1),
                    speculative=path.startswith("spec"), pair_m=(path == "spec-m2"))

    def timed(path, n):
        """(seconds, per-kernel timing, bytes per parameter and step actually moved, speculation totals of the region)."""
        torch.cuda.synchronize()
        before, before_m = st.ctx.speculation_stats(), st.ctx.speculation_stats(moment=True)
        st.ctx.set_timing(True)
        st.ctx.get_timing()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_steps(path, n)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        tm = st.ctx.get_timing()
        st.ctx.set_timing(False)
        after, after_m = st.ctx.speculation_stats(), st.ctx.speculation_stats(moment=True)
        spec = {k: after[k] - before[k] for k in after}
        spec.update({"moment_" + k: after_m[k] - before_m[k] for k in after_m})
        # a tensor cast twice costs its 2 B/element read and 1 B/element write (3 + 1 with the moment read) once more;
        # a first moment computed twice its two 1 B/element reads and its 1 B/element write
        redo_bytes = ((4 if path == "spec-fused" else 3) * spec["elems_redone"] + 3 * spec["moment_elems_redone"]) / n
        return dt, tm, base_bytes[path] + redo_bytes / P, spec

    run_steps(args.path, args.warmup)
    dt, timing, bytes_per_param, spec_totals = timed(args.path, args.steps)
    other_paths = {}
    if not args.only_path:
        for path in ("jit", "spec", "fused", "spec-fused", "spec-m2", "single"):
            if path == "spec-m2" and st.m_other is None:
                continue
            if path != args.path:
                run_steps(path, 2)
                n = min(args.steps, 10)
                odt, _, obytes, _ = timed(path, n)
                other_paths[path] = {"ms_per_step": round(odt / n * 1e3, 3), "params_per_s": P / (odt / n),
                                     "bytes_per_param_step": round(obytes, 3)}

    ms_per_step = dt / args.steps * 1e3
    kernels = {}
    for name, bpp in BYTES_PER_PARAM.items():
        n, ms = timing[name]
        if not n:
            continue
        if name == "adam_amax" and args.path == "spec-m2":
            # no read-only pass on this path: what is timed under this id is the repair of failed moment speculations
            kernels["moment_repair"] = {"avg_ms": round(ms / args.steps, 4), "launches": n}
            continue
        if name == "cast":
            # the cast is timed per step: a speculative step launches it twice (all tensors, then the ones to redo)
            per_step = ms / args.steps
            moved = (base_bytes[args.path] + (4 if args.path == "spec-fused" else 3) * spec_totals["elems_redone"] / args.steps / P
                     - {"jit": 16, "fused": 14, "single": 12, "spec": 14, "spec-fused": 12, "spec-m2": 12}[args.path])
            kernels[name] = {"avg_ms": round(per_step, 4), "launches": n, "bytes_per_param": round(moved, 3),
                             "GBps": round(moved * P / (per_step * 1e-3) / 1e9, 1)}
            continue
        avg = ms / n
        kernels[name] = {"avg_ms": round(avg, 4), "launches": n, "bytes_per_param": bpp,
                         "GBps": round(bpp * P / (avg * 1e-3) / 1e9, 1)}
    dom = "adam_update"
    achieved = kernels[dom]["GBps"]
    out = {
        "metric": "params updated/sec + achieved HBM GB/s (% of peak), FP8 cast+Adam step",
        "value": P / (dt / args.steps),
        "unit": "params/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": wl.name, "tensors": lay.n_tensors, "params": P, "grad_fmt": "e5m2",
                   "m_fmt": "e4m3", "v": "fp16 scaled", "master": "fp16 scaled", "wcopy": "e4m3",
                   "exact_div_sqrt": bool(args.exact), "path": args.path,
                   "bytes_per_param_step": round(bytes_per_param, 3), "algorithmic_bytes_per_param_step": 19,
                   "gradient_buffers": len(grads), "wcopy_over_grad": bool(args.wcopy_over_grad), "state_bytes_per_param": st.state_bytes_per_param + (1 if args.path == "spec-m2" else 0),
                   "placement": placement},
        "step_GBps": round(bytes_per_param * P / (dt / args.steps) / 1e9, 1),
        "step_frac_of_peak": round(bytes_per_param * P / (dt / args.steps) / 1e9 / HBM_PEAK_GBS, 4),
        "kernels": kernels,
        "speculation": ({"steps": spec_totals["calls"], "tensors_cast_twice_per_step": round(spec_totals["tensors_redone"] / max(1, spec_totals["calls"]), 2),
                         "share_of_elements_cast_twice": round(spec_totals["elems_redone"] / max(1, spec_totals["calls"]) / P, 4),
                         **({"moments_computed_twice_per_step": round(spec_totals["moment_tensors_redone"] / max(1, spec_totals["moment_calls"]), 2),
                             "share_of_moment_elements_computed_twice": round(spec_totals["moment_elems_redone"] / max(1, spec_totals["moment_calls"]) / P, 4)}
                            if args.path == "spec-m2" else {})}
                        if args.path.startswith("spec") else None),
        "other_paths": other_paths,
        "roofline": {"kernel": "adam_update_kernel", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": measured_traffic(wl.name)},
    }
    if args.graph:
        hp = B.adam_hparams(wl.lr, step_no[0] + 1, exact=args.exact, m_scale_mode=mode_of[args.path])
        delayed = args.path == "single"
        graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            st.step(grad, hp, delayed=delayed, speculative=args.path.startswith("spec"))
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        out["graph_replay_ms_per_step"] = (time.perf_counter() - t0) / args.steps * 1e3
    want_ceilings = not args.no_ceilings and lay.total >= (1 << 20)
    if args.calibration_copy:
        nbytes = min(lay.total // 16 * 16, 1 << 32)
        st.ctx.set_timing(True)
        st.ctx.get_timing()
        for _ in range(3):
            st.ctx.copy_bytes(st.m, st.g8, nbytes)
        n, ms = st.ctx.get_timing()["copy"]
        st.ctx.set_timing(False)
        out["calibration_copy"] = {"bytes_read": nbytes, "bytes_written": nbytes, "avg_ms": round(ms / n, 4),
                                   "GBps": round(2 * nbytes / (ms / n * 1e-3) / 1e9, 1)}
    if args.allreduce_steps:
        N = args.allreduce_steps
        ranks = [st.g8] + [st.g8.clone() for _ in range(N - 1)]
        metas = [st.g_meta] * N
        shared = st.ctx.shared_scale(metas)
        summed = torch.zeros_like(st.g8)
        out_meta = st.ctx.new_meta(cfg)
        st.ctx.set_timing(True)
        st.ctx.get_timing()
        for _ in range(5):
            st.ctx.requantize_fp8(ranks[0], B.E5M2, st.g_meta, shared, summed, out_meta)
            st.ctx.sum_fp8(ranks, B.E5M2, shared, summed, out_meta, cfg)
        tm = st.ctx.get_timing()
        st.ctx.set_timing(False)
        rq, sm = tm["requantize"][1] / tm["requantize"][0], tm["sum"][1] / tm["sum"][0]
        extra = {"ranks": N,
                 "requantize": {"avg_ms": round(rq, 4), "bytes_per_param": 2, "GBps": round(2 * P / (rq * 1e-3) / 1e9, 1)},
                 "sum": {"avg_ms": round(sm, 4), "bytes_per_param": N + 1, "GBps": round((N + 1) * P / (sm * 1e-3) / 1e9, 1)}}
        del ranks, summed
    else:
        extra = None
    if want_ceilings:
        # Memory-only skeletons of the four kernels (same grid, tile walk, access widths and cache policies, XORs for
        # arithmetic) over the same buffers, whole tiles only: the bandwidth this access pattern reaches on this
        # machine.  Last, because they overwrite the state.
        n_el = lay.total // 4096 * 4096
        shapes = {"amax": (B.SKEL_READ16, [grad]), "cast": (B.SKEL_CAST, [grad, st.g8]),
                  "adam_amax": (B.SKEL_READ8X2, [st.g8, st.m]),
                  "adam_update": (B.SKEL_UPDATE, [st.g8, st.m, st.v, st.w, st.wq]),
                  "update_reads_only": (B.SKEL_UPDATE_READS, [st.g8, st.m, st.v, st.w, st.wq]),
                  "update_writes_only": (B.SKEL_UPDATE_WRITES, [st.g8, st.m, st.v, st.w, st.wq]),
                  "write16": (B.SKEL_WRITE16, [grad]), "write8": (B.SKEL_WRITE8, [st.g8])}
        ceilings = {}
        for name, (shape, bufs) in shapes.items():
            views = [t.view(torch.int16) if t.element_size() == 2 else t for t in bufs]
            st.ctx.memory_skeleton(shape, views, n_el)
            st.ctx.set_timing(True)
            st.ctx.get_timing()
            for _ in range(5):
                st.ctx.memory_skeleton(shape, views, n_el)
            n, ms = st.ctx.get_timing()["skeleton"]
            st.ctx.set_timing(False)
            bpe = B.SKEL_BYTES_PER_ELEM[shape]
            ceilings[name] = {"avg_ms": round(ms / n, 4), "bytes_per_elem": bpe,
                              "GBps": round(bpe * n_el / (ms / n * 1e-3) / 1e9, 1)}
            if name in kernels:
                kernels[name]["frac_of_skeleton"] = round(ceilings[name]["avg_ms"] / kernels[name]["avg_ms"], 4)
        path_ms = sum(ceilings[k]["avg_ms"] for k in ("amax", "cast", "adam_amax", "adam_update"))
        ceilings["step_of_skeletons_ms"] = round(path_ms, 3)        # the pass structure of the jit path, memory only
        # what sharing the memory between the two directions costs the update shape: its reads alone plus its writes
        # alone, against both in one kernel
        ceilings["update_mixing_cost"] = round(ceilings["adam_update"]["avg_ms"] / (
            ceilings["update_reads_only"]["avg_ms"] + ceilings["update_writes_only"]["avg_ms"]), 4)
        out["ceilings"] = ceilings
        if args.path == "jit":
            out["step_frac_of_skeletons"] = round(path_ms / ms_per_step, 4)
        elif args.path == "spec":       # no separate amax pass; tensors cast twice are not in the skeleton sum
            out["step_frac_of_skeletons"] = round((path_ms - ceilings["amax"]["avg_ms"]) / ms_per_step, 4)
    shapes = bufs = views = gbuf = None       # every view of the arena has to go before its memory does
    del st, grad, grads, shapes, bufs, views, gbuf
    gc.collect()
    torch.cuda.empty_cache()
    if not (args.no_placement_compare or args.only_path) and lay.total >= (1 << 28):
        key = "region_aware_allocation" if args.arena else "plain_arena_allocation"
        try:
            out[key] = placement_compare(args, spread=args.arena)
        except (RuntimeError, MemoryError, subprocess.SubprocessError, ValueError, KeyError) as e:       # the headline is printed whatever happens to this extra
            out[key] = {"error": str(e).splitlines()[0][:200]}
        torch.cuda.empty_cache()
    if extra:
        out["allreduce_steps"] = extra
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, args.seed, budget_s=args.cpu_budget)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
