#!/usr/bin/env python3
"""Throughput of the EF21 hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--only C2]

A step is one EF21 iteration (Algorithm 2: local gradients, Top-k of the difference, update of
g_i and g, model step) over the synthetic workload.  The headline line is configuration C2
(n = 20 workers, d = 2000, m = 5000 dense rows each, k = 20), the one that exercises every stage;
the other configurations (C0, C1 Top-k alone, C3 CSR, C4 supplied gradients at network scale) are
reported inside "workloads" of the same JSON line.  Inputs are resident in HBM before timing starts.
Prints ONE JSON line on stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E, vendor figure
PROFILES = os.path.join(ROOT, "profiles")
KERNEL_SOURCES = os.path.join(ROOT, "paper_2106_05203_amd", "csrc")


def source_fingerprint() -> str:
    """Hash of the kernel sources: a profile summary taken at other sources does not describe this library."""
    import hashlib
    h = hashlib.sha256()
    for name in sorted(os.listdir(KERNEL_SOURCES)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(KERNEL_SOURCES, name), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(key: str):
    """HBM bytes per launch of a dominant kernel from the rocprofv3 --pmc summary under profiles/ (FETCH_SIZE +
    WRITE_SIZE scaled by a plain copy's readings; the summary holds the commands).  The summaries carry
    machine-readable lines `traffic <key> <bytes>` and `kernel-sources <fingerprint>`; one taken at other kernel
    sources than this tree's is refused (None, and a line on stderr), not quoted."""
    if not os.path.isdir(PROFILES):
        return None
    for name in sorted(os.listdir(PROFILES)):
        if not name.endswith("_pmc.md"):
            continue
        text = open(os.path.join(PROFILES, name)).read().split("\n")
        stamp = [ln.split()[1] for ln in text if ln.startswith("kernel-sources ") and len(ln.split()) > 1]
        for ln in text:
            f = ln.split()
            if len(f) == 3 and f[0] == "traffic" and f[1] == key:
                if not stamp or stamp[0] != source_fingerprint():
                    log(f"profiles/{name} was taken at kernel sources {stamp[0] if stamp else '?'}, this tree is "
                        f"{source_fingerprint()}: its traffic figure for {key} is NOT quoted")
                    return None
                return float(f[2])
    return None


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


REPEATS = 5


class Timed:
    """`warmup` untimed calls, then REPEATS loops of exactly `steps` calls, each loop between two
    synchronisations and two HIP events on the current stream.  ms per step: median and minimum over the loops,
    by the host clock (wall) and by the events (ev)."""

    def __init__(self, torch, fn, steps: int, warmup: int, repeats: int = None):
        repeats = REPEATS if repeats is None else repeats
        for i in range(warmup):
            fn(i)
        torch.cuda.synchronize()
        walls, evs = [], []
        at = warmup
        for _ in range(repeats):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t0 = time.perf_counter()
            e0.record()
            for i in range(steps):
                fn(at + i)
            e1.record()
            torch.cuda.synchronize()
            walls.append((time.perf_counter() - t0) * 1e3 / steps)
            evs.append(e0.elapsed_time(e1) / steps)
            at += steps
        walls.sort()
        evs.sort()
        self.wall, self.wall_min = walls[len(walls) // 2], walls[0]
        self.ev, self.ev_min = evs[len(evs) // 2], evs[0]
        self.repeats, self.steps = repeats, steps

    def fields(self, clock: str = "wall") -> dict:
        med, low = (self.wall, self.wall_min) if clock == "wall" else (self.ev, self.ev_min)
        return {"ms_per_step": round(med, 5), "ms_per_step_min": round(low, 5),
                "timing": f"median and min of {self.repeats} loops of {self.steps} steps, "
                          + ("host clock around synchronised loops" if clock == "wall" else "HIP events")}


def kernel_times(torch, h, fn, steps: int):
    """Per-kernel-class average duration (ms per launch) from HIP events inside the library."""
    h.set_timing(True)
    for i in range(steps):
        fn(i)
    t = h.get_timing(reset=True)
    h.set_timing(False)
    return {name: ms / cnt for name, (ms, cnt) in t.items()}, {name: cnt / steps for name, (ms, cnt) in t.items()}


def roofline(bytes_per_launch: float, ms: float, kernel: str, traffic=None) -> dict:
    achieved = bytes_per_launch / (ms * 1e-3) / 1e9
    return {"bound": "hbm", "kernel": kernel, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
            "frac_by_traffic": None if traffic is None else round(traffic / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "algorithmic_bytes_per_launch": int(bytes_per_launch), "avg_launch_ms": round(ms, 5)}


def dev(torch, a, dtype=None):
    import numpy as np
    return torch.from_numpy(np.ascontiguousarray(a if dtype is None else a.astype(dtype))).cuda()


# ------------------------------------------------------------------------------------------ workloads
def bench_dense(torch, binding, workloads, name: str, steps: int, warmup: int):
    import numpy as np
    c = workloads.CONFIGS[name]
    n, d, m, k = c["n"], c["d"], c["m"], c["k"]
    log(f"{name}: generating dense logistic regression n={n} d={d} m={m}")
    W = workloads.logreg_dense(n, d, m, seed=c["seed"])
    A, y = dev(torch, W.A), dev(torch, W.y)
    h = binding.EF21(n, d, k, c["gamma"])
    h.set_problem_dense(A, y, c["lam"])
    x0 = torch.zeros(d, device="cuda")
    h.set_state(x0, h.local_grad(x0), None)          # g_i^0 = grad f_i(x^0)
    t = Timed(torch, lambda i: h.step(), steps, warmup)
    wall = t.wall
    per_kernel, launches = kernel_times(torch, h, lambda i: h.step(), steps)
    out = {"value": round(1e3 / wall, 2), "unit": "EF21 iterations/s", **t.fields(),
           "ms_per_step_events": round(t.ev, 5), "kernel_ms": {k_: round(v, 5) for k_, v in per_kernel.items()},
           "iteration_algorithmic_bytes": 4 * n * m * d + 4 * n * m + 12 * n * d + 24 * n * k + 12 * d}
    if "grad_main" in per_kernel:
        out["roofline"] = roofline(4.0 * n * m * d + 4.0 * n * m + 4.0 * d, per_kernel["grad_main"],
                                   "logreg_dense_fused_kernel (grad_main)", measured_traffic(f"{name}/grad_main"))
    else:                 # (a run that measures the one-launch iteration only)
        out["roofline"] = roofline(out["iteration_algorithmic_bytes"], per_kernel["small_step"],
                                   "small_step_kernel (the whole iteration)", None)
    out["iteration_frac_of_hbm_peak"] = round(out["iteration_algorithmic_bytes"] / (wall * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    if name == "C2":      # the same problem under Algorithm 3 (EF21+): two Top-k selections and the choice per worker
        tp = Timed(torch, lambda i: h.step(None, binding.PLUS), steps, warmup)
        pk, pl = kernel_times(torch, h, lambda i: h.step(None, binding.PLUS), steps)
        out["ef21_plus"] = {"value": round(1e3 / tp.wall, 2), "unit": "EF21+ iterations/s", **tp.fields(),
                            "kernel_ms_per_step": {k_: round(v * pl[k_], 5) for k_, v in pk.items()},
                            "plain_compressor_chosen_last_step": int(h.get_choices()[0].sum().item())}
    if name == "C2":      # and under Algorithm 4 (the original EF, the comparison method), errors started at zero
        h.set_state(x0, torch.zeros((n, d), device="cuda"), None)
        te = Timed(torch, lambda i: h.step(None, binding.CLASSIC_EF), steps, warmup)
        out["classic_ef"] = {"value": round(1e3 / te.wall, 2), "unit": "EF iterations/s", **te.fields()}
    if name == "C2":      # and under Algorithm 5: minibatches of m/8 rows per worker, drawn without replacement, a
        tau = m // 8      # fresh one every iteration (eight batches prepared in HBM, the draw is the caller's)
        rng = np.random.default_rng(c["seed"] + 5)
        batches = [dev(torch, np.stack([rng.choice(m, size=tau, replace=False) for _ in range(n)]), np.int32)
                   for _ in range(8)]
        h.set_state(x0, torch.zeros((n, d), device="cuda"), None)

        def sto(i):
            h.set_minibatch(batches[i % 8])
            h.step()
        ts = Timed(torch, sto, steps, warmup)
        wall_s = ts.wall
        pk, _ = kernel_times(torch, h, sto, steps)
        h.set_minibatch(None)
        gbytes = 4.0 * n * tau * d + 8.0 * n * tau + 4.0 * d
        out["ef21_stochastic"] = {"value": round(1e3 / wall_s, 2), "unit": "Algorithm 5 iterations/s", "tau": tau,
                                  **ts.fields(), "grad_main_ms": round(pk["grad_main"], 5),
                                  "grad_main_GBps": round(gbytes / (pk["grad_main"] * 1e-3) / 1e9, 1)}
    if name == "C0":      # launch-bound: beside the three kernels of the default, the one-launch iteration,
        t1 = Timed(torch, lambda i: h.step(None, binding.ONE_LAUNCH), steps, warmup)
        out["one_launch"] = {"value": round(1e3 / t1.wall, 2), "unit": "EF21 iterations/s", **t1.fields()}
        # and the same iterations replayed from a HIP graph of 10 captured steps
        out["hip_graph_10_steps"] = graph_replay(torch, h, steps)
    return out, (W, h)


def device_info(torch) -> dict:
    """What the runtime reports about the GPU the numbers were taken on."""
    pr = torch.cuda.get_device_properties(0)
    out = {"name": pr.name, "compute_units": pr.multi_processor_count,
           "memory_GiB": round(pr.total_memory / 2 ** 30, 1)}
    for key, attr in (("arch", "gcnArchName"), ("l2_cache_MiB", "L2_cache_size"), ("wavefront", "warp_size"),
                      ("lds_per_cu_KiB", "shared_memory_per_multiprocessor")):
        v = getattr(pr, attr, None)
        if v is not None:
            out[key] = round(v / 2 ** 20, 1) if key == "l2_cache_MiB" else (round(v / 1024) if key == "lds_per_cu_KiB" else v)
    return out


def hbm_ceiling(torch, binding, gib: int = 1, reps: int = 10):
    """What the simplest kernels get out of this GPU's HBM: one read of `gib` GiB, and a copy of it."""
    src = torch.zeros(gib << 28, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    sink = torch.zeros(1, device="cuda")
    nbytes = src.numel() * 4
    out = {}
    for name, fn, moved in (("read", lambda: binding.ef21_hbm_read(src, sink), nbytes),
                            ("copy", lambda: binding.ef21_hbm_copy(dst, src), 2 * nbytes)):
        for _ in range(2):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        out[f"{name}_GBps"] = round(moved / (e0.elapsed_time(e1) / reps * 1e-3) / 1e9, 1)
    out["note"] = f"plain kernels on {gib} GiB: a read with non-temporal loads; a copy (read + written bytes counted)"
    return out


def graph_replay(torch, h, steps: int, per_graph: int = 10):
    """ef21_step only enqueues kernels, so it can be captured: ms per iteration when `per_graph` steps are
    captured into one HIP graph and the graph is replayed (reported beside the eager figure, never as it)."""
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        h.use_current_stream()
        h.step()
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for _ in range(per_graph):
                h.step()
        replays = max(1, steps // per_graph)
        graph.replay()
        side.synchronize()
        times = []
        for _ in range(REPEATS):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(side)
            for _ in range(replays):
                graph.replay()
            e1.record(side)
            side.synchronize()
            times.append(e0.elapsed_time(e1) / (replays * per_graph))
    h.use_current_stream()
    times.sort()
    ms = times[len(times) // 2]
    return {"ms_per_step": round(ms, 5), "ms_per_step_min": round(times[0], 5), "value": round(1e3 / ms, 2),
            "unit": "EF21 iterations/s",
            "timing": f"median and min of {REPEATS} loops of {replays} replays of {per_graph} captured steps, HIP events"}


def bench_topk(torch, binding, workloads, steps: int, warmup: int):
    c = workloads.CONFIGS["C1"]
    n, d = c["n"], c["d"]
    log(f"C1: generating 4 x [{n}][{d}] Top-k inputs")
    pool = [dev(torch, workloads.topk_rows(n, d, seed=s)) for s in range(4)]     # 320 MB > 256 MB cache
    res = {}
    for k in c["ks"]:
        idx = torch.empty((n, k), dtype=torch.int32, device="cuda")
        val = torch.empty((n, k), dtype=torch.float32, device="cuda")
        t = Timed(torch, lambda i: binding.ef21_topk(pool[i % 4], k, idx, val), steps, warmup)
        th = Timed(torch, lambda i: binding.ef21_topk(pool[0], k, idx, val), steps, warmup)
        ev, ev_hot = t.ev, th.ev
        bytes_call = 4.0 * n * d + 8.0 * n * k
        res[f"k={k}"] = {
            "value": round(n * d / (ev * 1e-3), 1), "unit": "Top-k elements/s", "ms_per_call": round(ev, 5),
            "ms_per_call_min": round(t.ev_min, 5), "ms_per_call_host_clock": round(t.wall, 5),
            "timing": t.fields("ev")["timing"],
            "call_frac_of_hbm_peak": round(bytes_call / (ev * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "same_buffer_every_call": {"value": round(n * d / (ev_hot * 1e-3), 1), "ms_per_call": round(ev_hot, 5)},
        }
    # the roofline of the workload: the whole call (collect + count + emit) against the bytes of one read of
    # the rows and one write of the pairs, at the k where it is worst
    worst = min((kk for kk in res), key=lambda kk: res[kk]["call_frac_of_hbm_peak"])
    kw = int(worst.split("=")[1])
    res["roofline"] = roofline(4.0 * n * d + 8.0 * n * kw, res[worst]["ms_per_call"],
                               f"ef21_topk call, {worst} (all kernels of the call)", None)
    return res


def bench_csr(torch, binding, workloads, steps: int, warmup: int):
    import numpy as np
    c = workloads.CONFIGS["C3"]
    n, d, m, k, nnz = c["n"], c["d"], c["m"], c["k"], c["nnz_per_row"]
    log(f"C3: generating CSR logistic regression n={n} d={d} m={m} nnz/row={nnz}")
    W = workloads.logreg_csr(n, d, m, nnz, seed=c["seed"])
    rp, col, val, y = dev(torch, W.rowptr), dev(torch, W.col), dev(torch, W.val), dev(torch, W.y)
    h = binding.EF21(n, d, k, c["gamma"])
    h.set_problem_csr(rp, col, val, y, m, c["lam"])
    x0 = torch.zeros(d, device="cuda")
    h.set_state(x0, h.local_grad(x0), None)
    t = Timed(torch, lambda i: h.step(), steps, warmup)
    wall = t.wall
    per_kernel, launches = kernel_times(torch, h, lambda i: h.step(), steps)
    total_nnz = n * m * nnz
    it_bytes = 8 * total_nnz + 8 * (n * m + 1) + 4 * n * m + 12 * n * d + 24 * n * k + 12 * d
    out = {"value": round(1e3 / wall, 2), "unit": "EF21 iterations/s", **t.fields(),
           "kernel_ms": {k_: round(v, 5) for k_, v in per_kernel.items()}, "iteration_algorithmic_bytes": it_bytes,
           "iteration_frac_of_hbm_peak": round(it_bytes / (wall * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    # the gradient takes two passes (two launches of the grad_main class): its algorithmic bytes against both
    out["roofline"] = roofline(8.0 * total_nnz + 8.0 * (n * m + 1) + 4.0 * n * m + 4.0 * n * d,
                               per_kernel["grad_main"] * launches["grad_main"],
                               "csrr_dot_kernel + csc_grad_kernel (grad_main, both passes)",
                               measured_traffic("C3/grad_main"))
    h.close()
    return out, W


def bench_grads(torch, binding, workloads, steps: int, warmup: int):
    c = workloads.CONFIGS["C4"]
    n, d, k = c["n"], c["d"], c["k"]
    log(f"C4: generating Student-t gradients n={n} d={d}")
    # "drawn fresh each step": a pool of NP independent gradient sets made on the device (358 MB each, every one
    # larger than the caches), cycled.  (A short pool of rotated copies of one set makes the selection threshold
    # jump with the pool's period, which independent draws do not.)
    NP = 8
    pool = workloads.student_t_grads_on_device(n, d, NP, seed=c["seed"])
    h = binding.EF21(n, d, k, c["gamma"])
    t = Timed(torch, lambda i: h.step(pool[i % NP]), steps, warmup)
    wall = t.wall
    per_kernel, launches = kernel_times(torch, h, lambda i: h.step(pool[i % NP]), steps)
    it_bytes = 8 * n * d + 12 * d + 24 * n * k
    out = {"value": round(1e3 / wall, 2), "unit": "EF21 iterations/s (gradients supplied)", **t.fields(),
           "kernel_ms": {k_: round(v, 5) for k_, v in per_kernel.items()}, "iteration_algorithmic_bytes": it_bytes,
           "iteration_frac_of_hbm_peak": round(it_bytes / (wall * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
           "topk_elements_per_s": round(n * d / (sum(v for k_, v in per_kernel.items() if k_.startswith("topk")) * 1e-3), 1)}
    # the comparison method on the same gradients: Algorithm 4 rewrites its whole state e_i every round
    h.set_state(torch.zeros(d, device="cuda"), torch.zeros((n, d), device="cuda"), None)
    te = Timed(torch, lambda i: h.step(pool[i % NP], binding.CLASSIC_EF), steps, warmup, repeats=3)
    out["classic_ef"] = {"value": round(1e3 / te.wall, 2), "unit": "EF iterations/s (gradients supplied)", **te.fields()}
    # Algorithm 3 on the same gradients: two Top-k selections, the distortions and the mean of the rows, each a
    # pass of its own over the long rows
    h.set_state(torch.zeros(d, device="cuda"), torch.zeros((n, d), device="cuda"), None)
    tp = Timed(torch, lambda i: h.step(pool[i % NP], binding.PLUS), max(10, steps // 2), max(3, warmup // 2), repeats=3)
    pk, pl = kernel_times(torch, h, lambda i: h.step(pool[i % NP], binding.PLUS), max(10, steps // 2))
    out["ef21_plus"] = {"value": round(1e3 / tp.wall, 2), "unit": "EF21+ iterations/s (gradients supplied)",
                        **tp.fields(),
                        "kernel_ms_per_step": {k_: round(v * pl[k_], 5) for k_, v in pk.items()},
                        "plain_compressor_chosen_last_step": int(h.get_choices()[0].sum().item())}
    # Fresh draws every step are EF21+'s worst case: g_i says nothing about the next gradient, every worker takes the
    # plain compressor and its whole row of g_i is rewritten.  Gradients that change slowly (one set plus 5 % of
    # another), as along a training run, let the Markov compressor win: the state then changes in k places per row.
    slow = [pool[0] + 0.05 * pool[j] for j in range(1, 5)]
    h.set_state(torch.zeros(d, device="cuda"), torch.zeros((n, d), device="cuda"), None)
    ts = Timed(torch, lambda i: h.step(slow[i % 4], binding.PLUS), max(10, steps // 2), max(5, warmup // 2), repeats=3)
    out["ef21_plus"]["slowly_varying_gradients"] = {
        "value": round(1e3 / ts.wall, 2), "unit": "EF21+ iterations/s (gradients supplied)", **ts.fields(),
        "plain_compressor_chosen_last_step": int(h.get_choices()[0].sum().item())}
    del slow
    dom = "topk_collect" if "topk_collect" in per_kernel else "topk_row"
    out["roofline"] = roofline(8.0 * n * d, per_kernel[dom], f"{dom} (reads grad and g_i once)",
                               measured_traffic(f"C4/{dom}"))
    h.close()
    return out


def cpu_baseline_dense(workloads, W, name: str, budget_s: float = 12.0):
    """The oracle as it stands, single-threaded, on full-size inputs of the headline workload."""
    import numpy as np
    from oracle import ef21_oracle as oracle
    c = workloads.CONFIGS[name]
    P = oracle.LogRegDense(W.A, W.y, c["lam"])
    x0 = np.zeros(P.d)
    st = oracle.init_state(x0, P.grads(x0), c["k"], init="grad", storage_f32=True)
    t0 = time.perf_counter()
    its = 0
    while True:
        oracle.iteration(st, P.grads, c["k"], c["gamma"], storage_f32=True)
        its += 1
        el = time.perf_counter() - t0
        if el > budget_s or its >= c["iters"]:
            break
    return {"value": round(its / el, 4), "unit": "EF21 iterations/s", "cores": 1, "kind": "oracle",
            "sample": f"{its} of the {c['iters']} iterations of {name} at full size ({el:.1f} s)"}


def cpu_baseline_csr(workloads, W, budget_s: float = 8.0, max_its: int = 20):
    """The oracle on C3 at full size, cut to at most `max_its` iterations or `budget_s` seconds."""
    import numpy as np
    from oracle import ef21_oracle as oracle
    c = workloads.CONFIGS["C3"]
    P = oracle.LogRegCSR(W.rowptr, W.col, W.val, W.y, c["n"], c["m"], c["d"], c["lam"])
    x0 = np.zeros(P.d)
    st = oracle.init_state(x0, P.grads(x0), c["k"], init="grad", storage_f32=True)
    t0 = time.perf_counter()
    its = 0
    while True:
        oracle.iteration(st, P.grads, c["k"], c["gamma"], storage_f32=True)
        its += 1
        el = time.perf_counter() - t0
        if el > budget_s or its >= max_its:
            break
    return {"value": round(its / el, 4), "unit": "EF21 iterations/s", "cores": 1, "kind": "oracle",
            "sample": f"{its} of the {c['iters']} iterations of C3 at full size ({el:.1f} s)"}


def cpu_baseline_grads(workloads, workers: int = 2):
    """The oracle on C4 at full d: one iteration with supplied gradients (the stable full sort of 11.2 million
    magnitudes per worker takes seconds), on `workers` of the n workers; the rate is scaled to all n."""
    import numpy as np
    from oracle import ef21_oracle as oracle
    c = workloads.CONFIGS["C4"]
    n, d, k = c["n"], c["d"], c["k"]
    grads = workloads.student_t_grads(workers, d, seed=c["seed"]).astype(np.float64)
    st = oracle.EF21State(np.zeros(d), np.zeros((workers, d)), np.zeros(d))
    t0 = time.perf_counter()
    oracle.iteration(st, lambda x: grads, k, c["gamma"], storage_f32=True)
    el = time.perf_counter() - t0
    return {"value": round(1.0 / (el * n / workers), 5), "unit": "EF21 iterations/s (gradients supplied)", "cores": 1,
            "kind": "oracle",
            "sample": f"1 iteration at full d on {workers} of the {n} workers ({el:.1f} s), scaled to {n} workers"}


def cpu_baseline_topk(workloads):
    import numpy as np
    from oracle import ef21_oracle as oracle
    c = workloads.CONFIGS["C1"]
    V = workloads.topk_rows(2, c["d"], seed=0).astype(np.float64)
    t0 = time.perf_counter()
    for row in V:
        oracle.topk(row, 1000)
    el = time.perf_counter() - t0
    return {"value": round(2 * c["d"] / el, 1), "unit": "Top-k elements/s", "cores": 1, "kind": "oracle",
            "sample": f"2 of the 20 rows of C1 (d = {c['d']}), k = 1000 ({el:.1f} s)"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--repeats", type=int, default=5, help="timed loops of --steps steps each (median and min reported)")
    ap.add_argument("--only", default="", help="comma list of C0,C1,C2,C3,C4 (C2, the headline, always runs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--print-fingerprint", action="store_true", help="print the hash of the kernel sources and exit")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run five plain device-to-device copies of 1 GiB (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.print_fingerprint:
        print(source_fingerprint())
        return 0
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (workers are rows of a batch; there are no collectives); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2106_05203_amd import binding, workloads
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    if args.calibrate_copy:
        src = torch.full((1 << 28,), 1.0, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "5 device-to-device copies", "bytes_read_each": src.numel() * 4,
                          "bytes_written_each": src.numel() * 4}), flush=True)
        return 0
    binding.load_library()
    which = set(filter(None, args.only.split(","))) or {"C0", "C1", "C2", "C3", "C4"}
    K, Wm = args.steps, args.warmup

    global REPEATS
    REPEATS = max(1, args.repeats)
    ceiling = hbm_ceiling(torch, binding)
    head, (W2, h2) = bench_dense(torch, binding, workloads, "C2", K, Wm)
    extra = {}
    cpu = None
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on C2")
        cpu = cpu_baseline_dense(workloads, W2, "C2")
    h2.close()
    del W2
    if "C0" in which:
        extra["C0"], (W0, h0) = bench_dense(torch, binding, workloads, "C0", K, Wm)
        h0.close()
        if not args.no_cpu_baseline:
            extra["C0"]["cpu_baseline"] = cpu_baseline_dense(workloads, W0, "C0")
    if "C1" in which:
        extra["C1"] = bench_topk(torch, binding, workloads, K, Wm)
        if not args.no_cpu_baseline:
            extra["C1"]["cpu_baseline"] = cpu_baseline_topk(workloads)
    if "C3" in which:
        extra["C3"], W3 = bench_csr(torch, binding, workloads, K, Wm)
        if not args.no_cpu_baseline:
            log("timing the CPU oracle on C3")
            extra["C3"]["cpu_baseline"] = cpu_baseline_csr(workloads, W3)
        del W3
    if "C4" in which:
        extra["C4"] = bench_grads(torch, binding, workloads, K, Wm)
        if not args.no_cpu_baseline:
            log("timing the CPU oracle on C4")
            extra["C4"]["cpu_baseline"] = cpu_baseline_grads(workloads)

    # the roofline fraction of every measured workload's dominant kernel, and the worst of them beside the headline's
    by_workload = {"C2": head["roofline"]}
    for name in ("C1", "C3", "C4"):
        if name in extra and "roofline" in extra[name]:
            by_workload[name] = extra[name]["roofline"]
    worst_name = min(by_workload, key=lambda w_: by_workload[w_]["frac"])
    iteration_fracs = {"C2": head["iteration_frac_of_hbm_peak"]}
    for name in ("C3", "C4"):
        if name in extra:
            iteration_fracs[name] = extra[name]["iteration_frac_of_hbm_peak"]

    c2 = workloads.CONFIGS["C2"]
    line = {
        "metric": "EF21 iterations/s (whole iteration: local gradients, Top-k, state update, aggregation, model step)",
        "value": head["value"], "unit": "iterations/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": head["ms_per_step"], "ms_per_step_min": head["ms_per_step_min"], "timing": head["timing"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"C2: EF21, logistic regression + nonconvex regulariser, n={c2['n']} workers, "
                               f"d={c2['d']}, m={c2['m']} dense fp32 rows per worker, Top-k k={c2['k']}, "
                               f"gamma={c2['gamma']}, lambda={c2['lam']}", "n": c2["n"], "d": c2["d"], "m": c2["m"],
                   "k": c2["k"]},
        "roofline": head["roofline"],
        "roofline_worst": {"workload": worst_name, **by_workload[worst_name],
                           "note": "lowest fraction among the dominant kernels of the workloads measured in this run "
                                   "(algorithmic bytes / HIP-event time / 8 TB/s); the headline's is the best of them"},
        "roofline_frac_by_workload": {w_: r_["frac"] for w_, r_ in by_workload.items()},
        "iteration_frac_of_hbm_peak_by_workload": iteration_fracs,
        "kernel_sources": source_fingerprint(),
        "hbm_measured_ceiling": ceiling,
        "device": device_info(torch),
        "cpu_baseline": cpu,
        "kernel_ms": head["kernel_ms"],
        "iteration_frac_of_hbm_peak": head["iteration_frac_of_hbm_peak"],
        "ef21_plus": head.get("ef21_plus"),
        "classic_ef": head.get("classic_ef"),
        "ef21_stochastic": head.get("ef21_stochastic"),
        "workloads": extra,
    }
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
