#!/usr/bin/env python3
"""Benchmark of the Moshpit group-averaging hot path on one MI355X.

A step is one pass of the whole hot path over one synthetic peer-state matrix:
device-side generation of the failure masks for the workload's rounds, one
group-mean kernel per round (axis cycling t mod d), and one dist-to-mean
reduction of the resulting state.  Consecutive steps continue the round counter
and work on the evolving state (timing depends on masks and addresses, not on
values).  The state is resident in HBM before the timed region starts.

The headline (value, config, roofline, cpu_baseline) is workload 4, the
configuration the target is quoted on.  The same line carries a `workloads`
object with a shorter measurement of the other four workload shapes: averaging
kernel GB/s and fraction of the HBM peak, rounds/s, the fused pass, the
distortion kernel, the CPU oracle beside it, the parity error on a column
sample and (workload 2) the distortion after every round next to the oracle's.

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


def sample_columns(P: int, count: int, seed: int) -> np.ndarray:
    """First and last columns plus random ones, sorted and unique."""
    rng = np.random.default_rng(seed)
    cols = set(range(min(P, 8))) | set(range(max(0, P - 8), P))
    cols |= set(rng.integers(0, P, size=max(0, count - len(cols))).tolist())
    return np.array(sorted(cols), dtype=np.int64)


def row_errors(got: np.ndarray, want: np.ndarray) -> float:
    norm = np.linalg.norm(want, axis=1)
    err = np.linalg.norm(got - want, axis=1)
    return float((err / np.where(norm > 0, norm, 1.0)).max())


def time_oracle(orc, ref, w, threads, budget_s, step0=0):
    """Whole steps of the workload on the oracle's fp64 copy `ref`, continuing the round
    counter, until about budget_s seconds of oracle time.  Returns (GB/s in the GPU's
    algorithmic bytes, seconds, steps)."""
    cols = ref.shape[1]
    slab = max(1, -(-cols // threads)) if threads > 1 else cols
    spent, nbytes, steps = 0.0, 0.0, 0
    while spent < budget_s and steps < 64:
        t_first = (step0 + steps) * w.rounds
        masks_k = orc.schedule_masks(w.kind, w.p, w.mask_seed, w.down, w.N, t_first, w.rounds)
        t1 = time.perf_counter()
        orc.run(ref, w.M, w.d, t_first, w.rounds, masks_k, threads=threads, slab=slab)
        spent += time.perf_counter() - t1
        nbytes += float((2.0 * w.elem_size * cols * live_in_groups(masks_k, w.M, w.d, t_first)).sum())
        steps += 1
    return nbytes / spent / 1e9, spent, steps


def measure(cfg: int, steps: int, warmup: int, cpu_cols: int, cpu_budget_s: float, tuning: str, row_pad: int,
            full_oracle_curve: bool, extras: bool, copy_probe: bool, sgd_iteration: bool = True):
    """One workload: generate the state, run warm-up and timed steps, the fused variant,
    the distortion kernel, the parity sample and the CPU oracle.  Returns a dict of results."""
    import torch
    from oracle import moshpit_oracle as orc
    from paper_2103_03239_amd import binding, inputs

    dev = torch.device("cuda:0")
    w = inputs.CONFIGS[cfg]
    s = w.elem_size
    log(f"[bench] workload {w.name}: N={w.N} (M={w.M}, d={w.d}) P={w.P} "
        f"{'f32' if w.dtype == 0 else 'bf16'} state {w.N * w.P * s / 2**30:.2f} GiB, {w.rounds} rounds/step")
    t_gen = time.time()
    # rows start on 128-byte boundaries (only workload 3 needs padding for that: 24 elements)
    row_stride = inputs.aligned_row_stride(w.P, w.dtype) + row_pad
    X = inputs.make_state(w, dev, row_stride=row_stride,
                          progress=lambda done, n: log(f"[bench] state rows {done}/{n}") if n > 1024 else None)
    torch.cuda.synchronize()
    log(f"[bench] state generated in {time.time() - t_gen:.1f}s")
    stream = torch.cuda.current_stream(dev)

    sched = binding.Schedule(kind=w.kind, p=w.p, seed=w.mask_seed, down_rounds=w.down)
    m = binding.Moshpit(w.N, w.P, w.M, w.d, w.dtype)
    m.bind_state(X)
    if tuning:
        m.set_tuning(*(int(v) for v in tuning.split(",")))

    total_steps = warmup + steps
    all_masks = m.schedule_mask(sched, 0, total_steps * w.rounds)
    L = live_in_groups(all_masks, w.M, w.d, 0)
    round_bytes = 2.0 * s * w.P * L                      # algorithmic bytes of every round
    dist_bytes = float(w.N) * w.P * s                    # the distortion reads the state once

    # inputs of the CPU legs, copied from the INITIAL state before the GPU changes it
    if cpu_cols < 0:
        cpu_cols = min(w.P, max(1024, (2 ** 31) // w.N))   # ~2^31 doubles = 16 GiB of fp64 at most
    X_cpu = X[:, :cpu_cols].to("cpu") if cpu_cols > 0 else None
    cols = sample_columns(w.P, 256, seed=cfg)
    cols_dev = torch.from_numpy(cols).to(dev)
    sample_ref = X.index_select(1, cols_dev).to("cpu").to(torch.float64).numpy().copy()
    X_full = X.to("cpu") if full_oracle_curve else None

    # first step from the fresh state: distortion after every round, parity on the column sample
    dist_first, _ = m.run(0, w.rounds, sched, want_dist=True)
    sample_got = X.index_select(1, cols_dev).to("cpu").to(torch.float64).numpy()
    masks0 = all_masks[: w.rounds]
    orc.run(sample_ref, w.M, w.d, 0, w.rounds, masks0, threads=8, slab=64)
    parity = row_errors(sample_got, sample_ref)
    log(f"[bench] first step: dist/P {dist_first[0] / w.P:.4e} -> {dist_first[-1] / w.P:.4e}; "
        f"max row error vs oracle on {len(cols)} columns {parity:.2e}")

    def step(k: int):
        _, ms = m.run(k * w.rounds, w.rounds, sched, want_times=True)
        dist = m.dist_to_mean()
        return ms, dist

    for k in range(1, max(warmup, 1)):
        step(k)
    first_timed = max(warmup, 1)
    total_steps = first_timed + steps
    if total_steps * w.rounds > len(all_masks):
        all_masks = m.schedule_mask(sched, 0, total_steps * w.rounds)
        round_bytes = 2.0 * s * w.P * live_in_groups(all_masks, w.M, w.d, 0)
    torch.cuda.synchronize()
    round_ms = []
    t0 = time.perf_counter()
    for k in range(first_timed, total_steps):
        ms, _ = step(k)
        round_ms.append(ms)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    round_ms = np.array(round_ms, dtype=np.float64)               # [steps, rounds]
    timed_bytes = round_bytes[first_timed * w.rounds: total_steps * w.rounds].reshape(steps, w.rounds)
    step_bytes = float(timed_bytes.sum()) + steps * dist_bytes
    value = step_bytes / elapsed / 1e9
    k1_bytes_per_launch = float(timed_bytes.mean())
    k1_ms_per_launch = float(round_ms.mean())
    k1_gbps = k1_bytes_per_launch / (k1_ms_per_launch * 1e-3) / 1e9
    per_axis = {}
    if w.rounds % w.d == 0:                                       # steps start at multiples of rounds
        for a in range(w.d):
            sel = np.array([(r % w.d) == a for r in range(w.rounds)])
            per_axis[f"axis{a}_gbps"] = round(float(timed_bytes[:, sel].sum() / (round_ms[:, sel].sum() * 1e-3) / 1e9), 1)
    log(f"[bench] {steps} steps in {elapsed:.3f}s; group-mean kernel {k1_gbps:.0f} GB/s "
        f"({100 * k1_gbps / HBM_PEAK_GBPS:.1f}% of peak), step {value:.0f} GB/s")

    # rounds only, queued back to back with no per-round events and one wait at the end
    next_step = total_steps
    rsteps = max(steps, 4)
    m.sync()
    tr = time.perf_counter()
    for k in range(next_step, next_step + rsteps):
        m.run(k * w.rounds, w.rounds, sched)
    m.sync()
    r_elapsed = time.perf_counter() - tr
    next_step += rsteps
    rounds_per_s_queued = w.rounds * rsteps / r_elapsed

    # the same steps with fused multi-round passes (bit-identical results, fewer passes over HBM)
    fsteps = max(2, steps // 2)
    m.run(next_step * w.rounds, w.rounds, sched, flags=binding.RUN_FUSED)
    m.sync()
    next_step += 1
    f_masks = m.schedule_mask(sched, next_step * w.rounds, fsteps * w.rounds)
    f_bytes = float((2.0 * s * w.P * live_in_groups(f_masks, w.M, w.d, next_step * w.rounds)).sum())
    tf = time.perf_counter()
    for k in range(next_step, next_step + fsteps):
        m.run(k * w.rounds, w.rounds, sched, flags=binding.RUN_FUSED)
    m.sync()
    f_elapsed = time.perf_counter() - tf
    next_step += fsteps
    fused = {"ms_per_step": round(f_elapsed / fsteps * 1e3, 4),
             "rounds_per_s": round(w.rounds * fsteps / f_elapsed, 2),
             "effective_gbps": round(f_bytes / f_elapsed / 1e9, 1),
             "speedup_vs_single_rounds": round((float(round_ms.sum()) / steps) / (f_elapsed / fsteps * 1e3), 3),
             "note": "rounds only (no dist-to-mean); effective = single-round algorithmic bytes / time, "
                     "may exceed the HBM peak because a fused pass touches HBM once for several rounds"}
    log(f"[bench] fused passes: {fused['ms_per_step']} ms per {w.rounds} rounds, effective "
        f"{fused['effective_gbps']} GB/s, {fused['speedup_vs_single_rounds']}x the single-round kernels")

    # the distortion kernels alone (device input, device output, no host synchronisation)
    out_dev = torch.zeros(1, dtype=torch.float64, device=dev)
    binding.dist_to_mean_static(X, out_dev, stream)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(5):
        binding.dist_to_mean_static(X, out_dev, stream)
    e1.record(stream)
    torch.cuda.synchronize()
    k3_ms = e0.elapsed_time(e1) / 5
    k3_gbps = dist_bytes / (k3_ms * 1e-3) / 1e9

    res = {
        "w": w, "row_stride": row_stride, "value": value, "elapsed": elapsed, "steps": steps,
        "warmup": first_timed, "k1_gbps": k1_gbps, "k1_bytes_per_launch": k1_bytes_per_launch,
        "k1_ms_per_launch": k1_ms_per_launch, "round_ms": round_ms, "per_axis": per_axis,
        "rounds_per_s_queued": rounds_per_s_queued, "fused": fused, "k3_gbps": k3_gbps, "k3_ms": k3_ms,
        "dist_first": dist_first, "parity": parity, "parity_cols": len(cols),
    }

    if extras:
        res.update(measure_extras(m, X, w, all_masks, row_stride, dev, sgd_iteration))

    if copy_probe:
        nbytes = min(w.N * w.P * s, 8 * 2 ** 30)
        nbytes -= nbytes % 16
        src = torch.empty(nbytes, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(2):
            binding.copy_probe(dst, src, stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(5):
            binding.copy_probe(dst, src, stream)
        e1.record(stream)
        torch.cuda.synchronize()
        res["copy_gbps"] = 5 * 2.0 * nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del src, dst
        log(f"[bench] plain copy kernel: {res['copy_gbps']:.0f} GB/s (read+write)")

    m.close()
    del X
    torch.cuda.empty_cache()

    if full_oracle_curve:
        ref_full = X_full.to(torch.float64).numpy()
        del X_full
        t1 = time.perf_counter()
        res["dist_oracle"] = orc.run(ref_full, w.M, w.d, 0, w.rounds, masks0, want_dist=True, threads=16,
                                     slab=max(256, w.P // 64))
        log(f"[bench] oracle distortion curve on the whole state in {time.perf_counter() - t1:.1f}s")
        del ref_full

    if X_cpu is not None:
        threads = min(16, os.cpu_count() or 1)
        ref = X_cpu.to(torch.float64).numpy()
        del X_cpu
        gbps, cpu_s, cpu_steps = time_oracle(orc, ref, w, threads, cpu_budget_s)
        cpu = {"value": round(gbps, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
               "sample": f"{cpu_steps} steps x {w.rounds} rounds of {w.name} on the first {cpu_cols} of {w.P} "
                         f"columns (all {w.N} peers, fp64 state), {cpu_s:.2f} s of oracle time",
               "rounds_per_s_full_width": round(cpu_steps * w.rounds / cpu_s * cpu_cols / w.P, 4)}
        log(f"[bench] cpu oracle: {cpu['value']} GB/s on {threads} threads ({cpu_s:.1f}s, {cpu_steps} steps)")
        if cfg in (1, 2):
            one_gbps, one_s, one_steps = time_oracle(orc, ref, w, 1, min(cpu_budget_s, 3.0), step0=cpu_steps)
            cpu["one_thread_gbps"] = round(one_gbps, 3)
            log(f"[bench] cpu oracle on one thread: {cpu['one_thread_gbps']} GB/s ({one_s:.1f}s, {one_steps} steps)")
        res["cpu"] = cpu
    return res


def measure_extras(m, X, w, all_masks, row_stride, dev, sgd_iteration=True):
    """The widened entry points on the same state (random groups, chunk-index keys, the
    Moshpit SGD step, the refresh of returning peers)."""
    import torch
    s = w.elem_size
    stream = torch.cuda.current_stream(dev)
    out = {}

    def timed(fn, reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        m.sync()
        e0.record(stream)
        for r in range(reps):
            fn(r)
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    # averaging in random groups of M peers (the simplified scheme of Thm 3.2): same kernel, rows
    # addressed through a seeded permutation; every peer takes part, so a round moves 2*s*N*P bytes
    for t in range(2):
        m.random_groups_round(t, 77, w.M)
    rg_ms = timed(lambda r: m.random_groups_round(2 + r, 77, w.M), 8)
    out["random_groups"] = {"group_size": w.M, "ms_per_round": round(rg_ms, 4),
                            "gbps": round(2.0 * s * w.N * w.P / (rg_ms * 1e-3) / 1e9, 1),
                            "note": "includes the permutation kernels of every round"}
    log(f"[bench] random groups of {w.M}: {rg_ms:.3f} ms per round, {out['random_groups']['gbps']} GB/s")

    # Alg. 1 with chunk-index keys: integer grouping kernels + the peer-list instantiation of the
    # group-mean kernel; bytes counted as 2*s*P per participating peer
    dy_masks = all_masks[: w.rounds]
    m.dynamic_reset()
    for t in range(2):
        m.dynamic_round(t, 55, dy_masks[t])
    dy_ms = timed(lambda r: m.dynamic_round(2 + r, 55, dy_masks[r]), w.rounds)
    dy_bytes = 2.0 * s * w.P * float(dy_masks.sum()) / w.rounds
    out["dynamic_keys"] = {"ms_per_round": round(dy_ms, 4), "gbps": round(dy_bytes / (dy_ms * 1e-3) / 1e9, 1),
                           "note": "includes the key/grouping kernels and the host-to-device copy of each round's mask"}
    log(f"[bench] chunk-index-key round: {dy_ms:.3f} ms per round, {out['dynamic_keys']['gbps']} GB/s")

    # Moshpit SGD communication iteration (Alg. 2): the round averages theta - gamma*g; every
    # participating peer reads theta and g and writes theta: 3*s*P bytes
    G = torch.empty((w.N, row_stride), dtype=X.dtype, device=dev)[:, : w.P]   # laid out like the state
    G.normal_(0.0, 1.0)
    sg_masks = all_masks[: w.rounds]
    for t in range(2):
        m.sgd_round(t, G, 1e-3, sg_masks[t])
    sg_ms = timed(lambda r: m.sgd_round(r, G, 1e-3, sg_masks[r]), w.rounds)
    sg_bytes = 3.0 * s * w.P * float(sg_masks.sum()) / w.rounds
    out["sgd_round"] = {"ms_per_round": round(sg_ms, 4), "gbps": round(sg_bytes / (sg_ms * 1e-3) / 1e9, 1),
                        "note": "theta <- group mean of (theta - gamma*g); includes the host-to-device copy of each round's mask"}
    log(f"[bench] Moshpit SGD round: {sg_ms:.3f} ms per round, {out['sgd_round']['gbps']} GB/s")
    # a whole iteration of Moshpit SGD (local step + the workload's rounds): fused, the local step is
    # applied while the first pass loads its tiles; round by round it rides on the first round's kernel
    if sgd_iteration:
        from paper_2103_03239_amd import binding
        sched = binding.Schedule(kind=w.kind, p=w.p, seed=w.mask_seed, down_rounds=w.down)
        m.sgd_run(0, w.rounds, G, 1e-3, sched, flags=binding.RUN_FUSED)
        it_fused = timed(lambda r: m.sgd_run((r + 1) * w.rounds, w.rounds, G, 1e-3, sched, flags=binding.RUN_FUSED), 3)
        it_plain = timed(lambda r: m.sgd_run((r + 4) * w.rounds, w.rounds, G, 1e-3, sched), 3)
        out["sgd_iteration"] = {"rounds": w.rounds, "ms_fused": round(it_fused, 4), "ms_round_by_round": round(it_plain, 4),
                                "note": "theta - gamma*g for the peers present in the first round, then the rounds"}
        log(f"[bench] Moshpit SGD iteration with {w.rounds} rounds: {it_fused:.3f} ms fused, {it_plain:.3f} ms round by round")
    del G

    # returning peers copy an up-to-date peer's parameters (App. on a dynamic number of peers):
    # 2*s*P bytes per returning peer; masks of consecutive rounds of the workload's schedule
    out["refresh"] = None
    pairs = [(all_masks[r - 1], all_masks[r]) for r in range(1, min(all_masks.shape[0], 1 + w.rounds))]
    returning = sum(int(((b == 1) & (a == 0)).sum()) for a, b in pairs if int(((a == 1) & (b == 1)).sum()) > 0)
    if returning > 0:
        m.refresh(1, 88, pairs[0][0], pairs[0][1])
        rf_ms = timed(lambda r: m.refresh(1 + r, 88, pairs[r][0], pairs[r][1]), len(pairs))
        rf_bytes = 2.0 * s * w.P * returning / len(pairs)
        out["refresh"] = {"ms_per_refresh": round(rf_ms, 4), "returning_peers": round(returning / len(pairs), 1),
                          "gbps": round(rf_bytes / (rf_ms * 1e-3) / 1e9, 1),
                          "note": "donor draw + row copies; includes the host-to-device copy of the two masks"}
        log(f"[bench] refresh of returning peers: {rf_ms:.3f} ms, {out['refresh']['gbps']} GB/s")
    return out


def summary(res) -> dict:
    """The per-workload entry of the `workloads` object."""
    w = res["w"]
    out = {
        "N": w.N, "M": w.M, "d": w.d, "P": w.P, "dtype": "f32" if w.dtype == 0 else "bf16",
        "rounds_per_step": w.rounds, "steps": res["steps"],
        "group_mean_gbps": round(res["k1_gbps"], 1),
        "group_mean_frac_of_hbm_peak": round(res["k1_gbps"] / HBM_PEAK_GBPS, 4),
        "group_mean_ms_per_round": round(res["k1_ms_per_launch"], 5),
        **res["per_axis"],
        "step_gbps": round(res["value"], 1),
        "rounds_per_s": round(res["rounds_per_s_queued"], 1),
        "fused_ms_per_step": res["fused"]["ms_per_step"],
        "fused_speedup_vs_single_rounds": res["fused"]["speedup_vs_single_rounds"],
        "dist_to_mean_gbps": round(res["k3_gbps"], 1),
        "dist_per_param_by_round": [float(v / w.P) for v in res["dist_first"]],
        "max_row_error_vs_oracle": res["parity"], "parity_sample_columns": res["parity_cols"],
        "oracle_gbps": res["cpu"]["value"] if "cpu" in res else None,
        "oracle_cores": res["cpu"]["cores"] if "cpu" in res else None,
        "oracle_sample": res["cpu"]["sample"] if "cpu" in res else None,
    }
    if "dist_oracle" in res:
        out["oracle_dist_per_param_by_round"] = [float(v / w.P) for v in res["dist_oracle"]]
    if w.N * w.P * w.elem_size < 2 ** 28:
        out["note"] = "state fits the on-chip caches and a round is launch-bound: not an HBM figure"
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=4, help="headline workload 1..5 (default: the largest, 4)")
    ap.add_argument("--cpu-cols", type=int, default=-1,
                    help="columns of the state the CPU oracle is timed on (0 = skip, -1 = auto)")
    ap.add_argument("--no-copy-probe", action="store_true")
    ap.add_argument("--no-fused", action="store_true", help="skip the widened entry points (random groups, SGD, refresh)")
    ap.add_argument("--no-sgd-iteration", action="store_true",
                    help="skip the Moshpit SGD iteration leg (its first pass is the fused kernel with a gradient read: "
                         "leave it out when that kernel's plain passes are profiled)")
    ap.add_argument("--no-workloads", action="store_true", help="skip the short measurements of the other workloads")
    ap.add_argument("--tuning", type=str, default="", help="cols,unroll,nontemporal[,block,waves_per_cu] override for sweeps")
    ap.add_argument("--row-pad", type=int, default=0, help="extra elements between rows (row_stride = P + pad)")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (all peers are virtual peers in one GPU's HBM); "
              "--gpus must be 1", file=sys.stderr)
        return 2

    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2

    head = measure(args.config, args.steps, args.warmup, args.cpu_cols, 10.0, args.tuning, args.row_pad,
                   full_oracle_curve=(args.config == 2), extras=not args.no_fused, copy_probe=not args.no_copy_probe,
                   sgd_iteration=not args.no_sgd_iteration)
    w = head["w"]
    s = w.elem_size

    workloads = {w.name: summary(head)}
    if not args.no_workloads:
        for cfg in (1, 2, 3, 5):
            if cfg == args.config:
                continue
            res = measure(cfg, 4, 1, -1 if args.cpu_cols != 0 else 0, 3.0, "", 0, full_oracle_curve=(cfg == 2),
                          extras=False, copy_probe=False)
            workloads[res["w"].name] = summary(res)

    traffic = read_traffic(os.path.join(ROOT, "profiles", f"group_mean_cfg{args.config}.txt"))
    round_ms = head["round_ms"]
    copy_gbps = head.get("copy_gbps")
    out = {
        "metric": METRIC,
        "value": round(head["value"], 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": head["warmup"],
        "ms_per_step": round(head["elapsed"] / args.steps * 1e3, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if w.dtype == 0 else "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "N": w.N, "M": w.M, "d": w.d, "P": w.P, "rounds_per_step": w.rounds,
                   "failure_kind": w.kind, "failure_p": w.p, "state_bytes": w.N * w.P * s,
                   "row_stride_elems": head["row_stride"],
                   "step": "mask generation + rounds x group-mean + 1 dist-to-mean"},
        "pct_of_hbm_peak": round(100 * head["value"] / HBM_PEAK_GBPS, 2),
        "rounds_per_s": round(w.rounds * args.steps / head["elapsed"], 2),
        "group_mean_gbps": round(head["k1_gbps"], 1),
        "group_mean_ms_per_round": round(head["k1_ms_per_launch"], 4),
        "group_mean_rounds_per_s": round(1e3 / head["k1_ms_per_launch"], 2),
        "group_mean_ms_min_median_max": [round(float(round_ms.min()), 4), round(float(np.median(round_ms)), 4),
                                         round(float(round_ms.max()), 4)],
        "group_mean_pct_of_copy_probe": None if copy_gbps is None else round(100 * head["k1_gbps"] / copy_gbps, 1),
        **head["per_axis"],
        "copy_probe_gbps": None if copy_gbps is None else round(copy_gbps, 1),
        "dist_to_mean_gbps": round(head["k3_gbps"], 1),
        "dist_per_param_by_round_first_step": [float(v / w.P) for v in head["dist_first"]],
        "max_row_error_vs_oracle": head["parity"],
        "roofline": {"bound": "hbm", "achieved": round(head["k1_gbps"], 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(head["k1_gbps"] / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "kernel": "group_mean_kernel", "bytes_per_launch": head["k1_bytes_per_launch"],
                     "ms_per_launch": round(head["k1_ms_per_launch"], 5)},
        "fused": head["fused"],
        "random_groups": head.get("random_groups"),
        "dynamic_keys": head.get("dynamic_keys"),
        "sgd_round": head.get("sgd_round"),
        "sgd_iteration": head.get("sgd_iteration"),
        "refresh": head.get("refresh"),
        "cpu_baseline": head.get("cpu"),
        "workloads": workloads,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
