#!/usr/bin/env python3
"""Benchmark of the Moshpit group-averaging hot path on one MI355X.

A step is one pass of the whole hot path over one synthetic peer-state matrix:
device-side generation of the failure masks for the workload's rounds, one
group-mean kernel per round (axis cycling t mod d), and one dist-to-mean
reduction of the resulting state.  Consecutive steps continue the round counter
and work on the evolving state (timing depends on masks and addresses, not on
values).  The state is resident in HBM before the timed region starts.

Prints ONE JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak bandwidth, GB/s (1 GB = 1e9 B)
METRIC = "peer-state averaging GB/s per round and % of MI355X HBM peak; rounds/sec"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def live_in_groups(masks: np.ndarray, M: int, d: int, t0: int) -> np.ndarray:
    """L_t per round: peers that take part and whose group has >= 2 participants
    (the rows a round reads once and writes once).  Pure bookkeeping on the
    mask bytes; axis a = t mod d has row stride M^a."""
    out = np.zeros(len(masks), dtype=np.int64)
    N = masks.shape[1]
    for r, row in enumerate(masks):
        a = (t0 + r) % d
        S = M ** a
        grid = row.reshape(N // (S * M), M, S).astype(np.int64)   # [upper digits][digit a][lower digits]
        k = grid.sum(axis=1)
        out[r] = int(k[k >= 2].sum())
    return out


def read_traffic(path: str):
    """HBM bytes per launch of the dominant kernel from a committed rocprofv3
    --pmc summary (a line `traffic_bytes_per_launch: <number>`), or None."""
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=4, help="workload 1..5 (default: the largest, 4)")
    ap.add_argument("--cpu-cols", type=int, default=-1,
                    help="columns of the state the CPU oracle is timed on (0 = skip, -1 = auto)")
    ap.add_argument("--no-copy-probe", action="store_true")
    ap.add_argument("--no-fused", action="store_true", help="skip the fused multi-round measurement")
    ap.add_argument("--tuning", type=str, default="", help="cols,unroll,nontemporal[,block,waves_per_cu] override for sweeps")
    ap.add_argument("--row-pad", type=int, default=0, help="extra elements between rows (row_stride = P + pad)")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (all peers are virtual peers in one GPU's HBM); "
              "--gpus must be 1", file=sys.stderr)
        return 2

    import torch
    from paper_2103_03239_amd import binding, inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    w = inputs.CONFIGS[args.config]
    s = w.elem_size
    log(f"[bench] workload {w.name}: N={w.N} (M={w.M}, d={w.d}) P={w.P} "
        f"{'f32' if w.dtype == 0 else 'bf16'} state {w.N * w.P * s / 2**30:.2f} GiB, {w.rounds} rounds/step")
    t_gen = time.time()
    # rows start on 128-byte boundaries (only workload 3 needs padding for that: 24 elements)
    row_stride = inputs.aligned_row_stride(w.P, w.dtype) + args.row_pad
    X = inputs.make_state(w, dev, row_stride=row_stride)
    torch.cuda.synchronize()
    log(f"[bench] state generated in {time.time() - t_gen:.1f}s")

    sched = binding.Schedule(kind=w.kind, p=w.p, seed=w.mask_seed, down_rounds=w.down)
    m = binding.Moshpit(w.N, w.P, w.M, w.d, w.dtype)
    m.bind_state(X)
    if args.tuning:
        m.set_tuning(*(int(v) for v in args.tuning.split(",")))

    total_steps = args.warmup + args.steps
    all_masks = m.schedule_mask(sched, 0, total_steps * w.rounds)
    L = live_in_groups(all_masks, w.M, w.d, 0)
    round_bytes = 2.0 * s * w.P * L                      # algorithmic bytes of every round
    dist_bytes = float(w.N) * w.P * s                    # the distortion reads the state once

    # cpu baseline input: first columns of the INITIAL state (copied before the GPU changes it)
    cpu_cols = args.cpu_cols
    if cpu_cols < 0:
        cpu_cols = min(w.P, max(1024, (2 ** 31) // w.N))   # ~2^31 doubles = 16 GiB of fp64 at most
    X_cpu = X[:, :cpu_cols].to("cpu") if cpu_cols > 0 else None

    def step(k: int):
        _, ms = m.run(k * w.rounds, w.rounds, sched, want_times=True)
        dist = m.dist_to_mean()
        return ms, dist

    for k in range(args.warmup):
        step(k)
    torch.cuda.synchronize()
    round_ms = []
    dists = []
    t0 = time.perf_counter()
    for k in range(args.warmup, total_steps):
        ms, dist = step(k)
        round_ms.append(ms)
        dists.append(dist)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    round_ms = np.array(round_ms, dtype=np.float64)               # [steps, rounds]
    timed_bytes = round_bytes[args.warmup * w.rounds:].reshape(args.steps, w.rounds)
    step_bytes = float(timed_bytes.sum()) + args.steps * dist_bytes
    value = step_bytes / elapsed / 1e9
    ms_per_step = elapsed / args.steps * 1e3
    k1_bytes_per_launch = float(timed_bytes.mean())
    k1_ms_per_launch = float(round_ms.mean())
    k1_gbps = k1_bytes_per_launch / (k1_ms_per_launch * 1e-3) / 1e9
    per_axis = {}
    for a in range(w.d):
        sel = [(r % w.d) == a for r in range(w.rounds)]          # steps start at multiples of rounds
        if (w.rounds % w.d) != 0:
            sel = None
        if sel is not None:
            sel = np.array(sel)
            per_axis[f"axis{a}_gbps"] = round(float(timed_bytes[:, sel].sum() / (round_ms[:, sel].sum() * 1e-3) / 1e9), 1)
    log(f"[bench] {args.steps} steps in {elapsed:.3f}s; group-mean kernel {k1_gbps:.0f} GB/s "
        f"({100 * k1_gbps / HBM_PEAK_GBPS:.1f}% of peak), step {value:.0f} GB/s; dist/P after last step "
        f"{dists[-1] / w.P:.3e}")

    # the same steps with fused multi-round passes (bit-identical results, fewer passes over HBM)
    fused = None
    if not args.no_fused:
        fsteps = max(2, args.steps // 2)
        for k in range(total_steps, total_steps + 1):
            m.run(k * w.rounds, w.rounds, sched, flags=binding.RUN_FUSED)
        m.sync()
        f_masks = m.schedule_mask(sched, (total_steps + 1) * w.rounds, fsteps * w.rounds)
        f_bytes = float((2.0 * s * w.P * live_in_groups(f_masks, w.M, w.d, (total_steps + 1) * w.rounds)).sum())
        tf = time.perf_counter()
        for k in range(total_steps + 1, total_steps + 1 + fsteps):
            m.run(k * w.rounds, w.rounds, sched, flags=binding.RUN_FUSED)
        m.sync()
        f_elapsed = time.perf_counter() - tf
        fused = {"ms_per_step": round(f_elapsed / fsteps * 1e3, 4),
                 "rounds_per_s": round(w.rounds * fsteps / f_elapsed, 2),
                 "effective_gbps": round(f_bytes / f_elapsed / 1e9, 1),
                 "speedup_vs_single_rounds": round((float(round_ms.sum()) / args.steps) / (f_elapsed / fsteps * 1e3), 3),
                 "note": "rounds only (no dist-to-mean); effective = single-round algorithmic bytes / time, "
                         "may exceed the HBM peak because a fused pass touches HBM once for several rounds"}
        log(f"[bench] fused passes: {fused['ms_per_step']} ms per {w.rounds} rounds, effective "
            f"{fused['effective_gbps']} GB/s, {fused['speedup_vs_single_rounds']}x the single-round kernels")

    # averaging in random groups of M peers (the simplified scheme of Thm 3.2): same kernel, rows
    # addressed through a seeded permutation; every peer takes part, so a round moves 2*s*N*P bytes
    random_groups = None
    if not args.no_fused and w.N <= 65536:
        stream = torch.cuda.current_stream(dev)
        for t in range(2):
            m.random_groups_round(t, 77, w.M)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        m.sync()
        reps = 8
        e0.record(stream)
        for t in range(2, 2 + reps):
            m.random_groups_round(t, 77, w.M)
        e1.record(stream)
        torch.cuda.synchronize()
        rg_ms = e0.elapsed_time(e1) / reps
        random_groups = {"group_size": w.M, "ms_per_round": round(rg_ms, 4),
                         "gbps": round(2.0 * s * w.N * w.P / (rg_ms * 1e-3) / 1e9, 1),
                         "note": "includes the permutation kernel of every round"}
        log(f"[bench] random groups of {w.M}: {rg_ms:.3f} ms per round, {random_groups['gbps']} GB/s")

    # Alg. 1 with chunk-index keys: integer grouping kernels + the peer-list instantiation of the
    # group-mean kernel; bytes counted as 2*s*P per participating peer
    dynamic = None
    if not args.no_fused and w.N <= 65536:
        stream = torch.cuda.current_stream(dev)
        dy_masks = all_masks[: w.rounds]
        m.dynamic_reset()
        for t in range(2):
            m.dynamic_round(t, 55, dy_masks[t])
        m.sync()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for t in range(w.rounds):
            m.dynamic_round(2 + t, 55, dy_masks[t])
        e1.record(stream)
        torch.cuda.synchronize()
        dy_ms = e0.elapsed_time(e1) / w.rounds
        dy_bytes = 2.0 * s * w.P * float(dy_masks.sum()) / w.rounds
        dynamic = {"ms_per_round": round(dy_ms, 4), "gbps": round(dy_bytes / (dy_ms * 1e-3) / 1e9, 1),
                   "note": "includes the key/grouping kernels and the host-to-device copy of each round's mask"}
        log(f"[bench] chunk-index-key round: {dy_ms:.3f} ms per round, {dynamic['gbps']} GB/s")

    # Moshpit SGD communication iteration (Alg. 2): the round averages theta - gamma*g; every
    # participating peer reads theta and g and writes theta: 3*s*P bytes
    sgd = None
    if not args.no_fused:
        G = torch.empty((w.N, row_stride), dtype=X.dtype, device=dev)[:, : w.P]   # laid out like the state
        G.normal_(0.0, 1.0)
        stream = torch.cuda.current_stream(dev)
        sg_masks = all_masks[: w.rounds]
        for t in range(2):
            m.sgd_round(t, G, 1e-3, sg_masks[t])
        m.sync()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for t in range(w.rounds):
            m.sgd_round(t, G, 1e-3, sg_masks[t])
        e1.record(stream)
        torch.cuda.synchronize()
        sg_ms = e0.elapsed_time(e1) / w.rounds
        sg_bytes = 3.0 * s * w.P * float(sg_masks.sum()) / w.rounds
        sgd = {"ms_per_round": round(sg_ms, 4), "gbps": round(sg_bytes / (sg_ms * 1e-3) / 1e9, 1),
               "note": "theta <- group mean of (theta - gamma*g); includes the host-to-device copy of each round's mask"}
        log(f"[bench] Moshpit SGD round: {sg_ms:.3f} ms per round, {sgd['gbps']} GB/s")
        del G

    # returning peers copy an up-to-date peer's parameters (App. on a dynamic number of peers):
    # 2*s*P bytes per returning peer; masks of consecutive rounds of the workload's schedule
    refresh = None
    if not args.no_fused and all_masks.shape[0] >= 2:
        stream = torch.cuda.current_stream(dev)
        pairs = [(all_masks[r - 1], all_masks[r]) for r in range(1, min(all_masks.shape[0], 1 + w.rounds))]
        returning = sum(int(((b == 1) & (a == 0)).sum()) for a, b in pairs if int(((a == 1) & (b == 1)).sum()) > 0)
        if returning > 0:
            m.refresh(1, 88, pairs[0][0], pairs[0][1])
            m.sync()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for r, (a, b) in enumerate(pairs):
                m.refresh(1 + r, 88, a, b)
            e1.record(stream)
            torch.cuda.synchronize()
            rf_ms = e0.elapsed_time(e1) / len(pairs)
            rf_bytes = 2.0 * s * w.P * returning / len(pairs)
            refresh = {"ms_per_refresh": round(rf_ms, 4), "returning_peers": round(returning / len(pairs), 1),
                       "gbps": round(rf_bytes / (rf_ms * 1e-3) / 1e9, 1),
                       "note": "donor draw + row copies; includes the host-to-device copy of the two masks"}
            log(f"[bench] refresh of returning peers: {rf_ms:.3f} ms, {refresh['gbps']} GB/s")

    copy_gbps = None
    if not args.no_copy_probe:
        nbytes = min(w.N * w.P * s, 8 * 2 ** 30)
        nbytes -= nbytes % 16
        src = torch.empty(nbytes, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        stream = torch.cuda.current_stream(dev)
        for _ in range(2):
            binding.copy_probe(dst, src, stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(5):
            binding.copy_probe(dst, src, stream)
        e1.record(stream)
        torch.cuda.synchronize()
        copy_gbps = 5 * 2.0 * nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del src, dst
        log(f"[bench] plain copy kernel: {copy_gbps:.0f} GB/s (read+write)")

    cpu = None
    if X_cpu is not None:
        from oracle import moshpit_oracle as orc
        threads = min(16, os.cpu_count() or 1)
        ref = X_cpu.to(torch.float64).numpy()
        del X_cpu
        slab = max(1, -(-cpu_cols // threads))
        # whole steps of the same workload, continuing the round counter, until ~10 s of CPU work
        cpu_s, cpu_bytes, cpu_steps = 0.0, 0.0, 0
        while cpu_s < 10.0 and cpu_steps < 64:
            t_first = cpu_steps * w.rounds
            masks_k = orc.schedule_masks(w.kind, w.p, w.mask_seed, w.down, w.N, t_first, w.rounds)
            t1 = time.perf_counter()
            orc.run(ref, w.M, w.d, t_first, w.rounds, masks_k, threads=threads, slab=slab)
            cpu_s += time.perf_counter() - t1
            cpu_bytes += float((2.0 * s * cpu_cols * live_in_groups(masks_k, w.M, w.d, t_first)).sum())
            cpu_steps += 1
        cpu = {"value": round(cpu_bytes / cpu_s / 1e9, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
               "sample": f"{cpu_steps} steps x {w.rounds} rounds of {w.name} on the first {cpu_cols} of {w.P} "
                         f"columns (all {w.N} peers, fp64 state), {cpu_s:.2f} s of oracle time",
               "rounds_per_s_full_width": round(cpu_steps * w.rounds / cpu_s * cpu_cols / w.P, 4)}
        log(f"[bench] cpu oracle: {cpu['value']} GB/s on {threads} threads ({cpu_s:.1f}s, {cpu_steps} steps)")
        if args.config in (1, 2):
            # the small workloads also on ONE host thread (about 5 s)
            one_s, one_bytes, one_steps = 0.0, 0.0, 0
            while one_s < 5.0 and one_steps < 64:
                t_first = (cpu_steps + one_steps) * w.rounds
                masks_k = orc.schedule_masks(w.kind, w.p, w.mask_seed, w.down, w.N, t_first, w.rounds)
                t1 = time.perf_counter()
                orc.run(ref, w.M, w.d, t_first, w.rounds, masks_k, threads=1, slab=cpu_cols)
                one_s += time.perf_counter() - t1
                one_bytes += float((2.0 * s * cpu_cols * live_in_groups(masks_k, w.M, w.d, t_first)).sum())
                one_steps += 1
            cpu["one_thread_gbps"] = round(one_bytes / one_s / 1e9, 3)
            log(f"[bench] cpu oracle on one thread: {cpu['one_thread_gbps']} GB/s ({one_s:.1f}s, {one_steps} steps)")

    traffic = read_traffic(os.path.join(ROOT, "profiles", f"group_mean_cfg{args.config}.txt"))
    out = {
        "metric": METRIC,
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if w.dtype == 0 else "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "N": w.N, "M": w.M, "d": w.d, "P": w.P, "rounds_per_step": w.rounds,
                   "failure_kind": w.kind, "failure_p": w.p, "state_bytes": w.N * w.P * s,
                   "row_stride_elems": row_stride,
                   "step": "mask generation + rounds x group-mean + 1 dist-to-mean"},
        "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBPS, 2),
        "rounds_per_s": round(w.rounds * args.steps / elapsed, 2),
        "group_mean_gbps": round(k1_gbps, 1),
        "group_mean_ms_per_round": round(k1_ms_per_launch, 4),
        "group_mean_rounds_per_s": round(1e3 / k1_ms_per_launch, 2),
        "group_mean_ms_min_median_max": [round(float(round_ms.min()), 4), round(float(np.median(round_ms)), 4),
                                         round(float(round_ms.max()), 4)],
        "group_mean_pct_of_copy_probe": None if copy_gbps is None else round(100 * k1_gbps / copy_gbps, 1),
        **per_axis,
        "copy_probe_gbps": None if copy_gbps is None else round(copy_gbps, 1),
        "dist_to_mean_per_param": dists[-1] / w.P,
        "roofline": {"bound": "hbm", "achieved": round(k1_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(k1_gbps / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "kernel": "group_mean_kernel", "bytes_per_launch": k1_bytes_per_launch,
                     "ms_per_launch": round(k1_ms_per_launch, 5)},
        "fused": fused,
        "random_groups": random_groups,
        "dynamic_keys": dynamic,
        "sgd_round": sgd,
        "refresh": refresh,
        "cpu_baseline": cpu,
    }
    m.close()
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
