#!/usr/bin/env python3
"""Benchmark of the GradiVeQ codec hot path on one MI355X.

One "step" = the whole compressed aggregation of one training iteration (Section 2,
Eqs. 2-4): N x gvq_compress (one per simulated worker), gvq_aggregate, gvq_decompress, on
synthetic gradients that are already resident in HBM.  The basis is fitted once before
the timed region (gvq_fit_basis, reported separately: the paper refreshes it once per
L_t + L_c iterations).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload vgg16] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix rate
FP64_MFMA_PEAK_TFLOPS = 78.6  # MI355X published fp64 matrix rate


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # A process's first few dozen steps run 1 - 9 % slower than the rest (the GPU settles on its clocks): the defaults
    # measure the steady state; one step is 0.06 - 2.4 ms, so the whole run still takes about a second.
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="vgg16", help="a workload name, or \"all\" for one line per workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="after the timed region, run gvq_aggregate with ONE input three times: a plain "
                         "copy of S*k floats, the known-size kernel that HBM byte counters are scaled by")
    ap.add_argument("--fit-gradients", type=int, default=None,
                    help="override L (gradients the basis is fitted on)")
    ap.add_argument("--skip-fit", action="store_true",
                    help="import a seeded random orthonormal basis instead of fitting one (counter runs: the "
                         "long-slice fit enqueues tens of thousands of small kernels)")
    ap.add_argument("--no-next-rows", action="store_true",
                    help="leave out the timings of the ring step, the monitor, flatten, the first-slice-sampling fit "
                         "and the rank selection (profiler runs: their launches would mix with those of the timed steps "
                         "and of the pooled fit in per-kernel statistics)")
    ap.add_argument("--option", action="append", default=[], metavar="INDEX=VALUE",
                    help="gvq_set_option(INDEX, VALUE) before the run (launch tuning, for A/B timings); repeatable")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (the N workers are simulated as N "
                 "device buffers on it); --gpus above 1 is not supported.")

    import torch

    from paper_1811_03617_amd import WORKLOADS, gvq

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)
    for o in args.option:
        index, value = (int(v) for v in o.split("="))
        gvq.gvq_set_option(index, value)
    # "all": one JSON line per workload (the whole table of measurements from one command); the default is the
    # headline workload alone, ONE line
    names = list(WORKLOADS) if args.workload == "all" else [args.workload]
    for name in names:
        print(json.dumps(run_workload(name, args)), flush=True)


def run_workload(name, args):
    import numpy as np
    import torch

    from paper_1811_03617_amd import WORKLOADS, gvq, synth

    dev = "cuda:0"
    w = WORKLOADS[name]
    L = args.fit_gradients or w.L
    es = 2 if w.dtype == "bf16" else 4
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32

    # ---- inputs, resident in HBM ------------------------------------------------------
    basis = gvq.Basis(w.M, w.d, w.k, w.block_offsets(), w.dtype)
    S = basis.S
    workers = synth.worker_gradients(w, dev)
    fit_grads = [] if args.skip_fit else synth.fit_gradients(w, dev, L=L)
    comps = [torch.empty(S * w.k, device=dev, dtype=torch.float32) for _ in range(w.N)]
    total = torch.empty(S * w.k, device=dev, dtype=torch.float32)
    out = torch.empty(w.M, device=dev, dtype=tdt)
    torch.cuda.synchronize()

    def ev():
        return torch.cuda.Event(enable_timing=True)

    first_slice_ms = select_k_ms = ks = None

    # ---- basis refresh (timed on its own) -----------------------------------------------
    if args.skip_fit:
        rng = np.random.default_rng(w.seed)
        U0 = np.stack([np.linalg.qr(rng.standard_normal((w.d, w.k)))[0] for _ in range(w.n_blocks)])
        basis.import_(U0.astype(np.float32), np.zeros((w.n_blocks, w.d), np.float32))
        sweeps, fit_ms = None, float("nan")
    else:
        basis.fit(fit_grads)
        sweeps = basis.fit_status()
        e0, e1 = ev(), ev()
        e0.record()
        basis.fit(fit_grads)
        e1.record()
        torch.cuda.synchronize()
        fit_ms = e0.elapsed_time(e1)
        if not args.no_next_rows:
            # Section 3's own sampling: the basis of every block from the L samples of its first slice (L < d here:
            # the L x L sample-Gram route); then the pooled fit again, untimed, so that the steps run on its basis
            basis.fit(fit_grads, first_slice_only=True)
            e0, e1 = ev(), ev()
            e0.record()
            basis.fit(fit_grads, first_slice_only=True)
            e1.record()
            torch.cuda.synchronize()
            first_slice_ms = e0.elapsed_time(e1)
            basis.fit(fit_grads)
            torch.cuda.synchronize()
            # Eq. 5: the smallest k per basis whose leading eigenvalues hold 1 - lambda of the total (lambda = 0.01 as
            # in Section 4), from the eigenvalues on the device; the time includes the copy of the B results
            basis.select_k(0.01)
            t0 = time.perf_counter()
            ks = basis.select_k(0.01)
            select_k_ms = (time.perf_counter() - t0) * 1e3
    del fit_grads

    def step(events=None):
        if events is not None:
            events[0].record()
        for g, c in zip(workers, comps):
            basis.compress(g, w.N, c)
        if events is not None:
            events[1].record()
        basis.aggregate(comps, total)
        if events is not None:
            events[2].record()
        basis.decompress(total, out)
        if events is not None:
            events[3].record()

    # The GPU takes its time to settle on its clocks after the idle moments of set-up: a quarter of a second of the
    # same work first (untimed, whatever --warmup says), so that a short run measures the same machine as a long one.
    settle_until = time.perf_counter() + 0.25
    while time.perf_counter() < settle_until:
        for _ in range(10):
            step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    marks = [[ev() for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(marks[i])
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps

    comp_ms = sum(m[0].elapsed_time(m[1]) for m in marks) / args.steps / w.N   # per launch
    agg_ms = sum(m[1].elapsed_time(m[2]) for m in marks) / args.steps
    dec_ms = sum(m[2].elapsed_time(m[3]) for m in marks) / args.steps
    dev_ms = marks[0][0].elapsed_time(marks[-1][3]) / args.steps

    # ---- algorithmic traffic (bytes every kernel must move at least once) -----------------
    comp_bytes = S * (w.d * es + 4 * w.k)                 # one compress launch
    agg_bytes = (w.N + 1) * S * 4 * w.k
    dec_bytes = S * (4 * w.k + w.d * es)
    path_bytes = w.N * comp_bytes + agg_bytes + dec_bytes
    grad_bytes = w.N * w.M * es

    ms_per_step = max(wall_ms, dev_ms)
    value = grad_bytes / ms_per_step / 1e6                # GB/s of gradient through the path
    eff = path_bytes / ms_per_step / 1e6

    # per-step device times (first event of a step to its last) and a plain copy through the same
    # library (gvq_aggregate of ONE vector), the practical ceiling of this memory system for a 1:1 stream
    step_ms = sorted(m[0].elapsed_time(m[3]) for m in marks)
    c0, c1 = ev(), ev()
    basis.aggregate(comps[:1], total)
    c0.record()
    for _ in range(10):
        basis.aggregate(comps[:1], total)
    c1.record()
    torch.cuda.synchronize()
    copy_gbs = 2 * S * 4 * w.k * 10 / c0.elapsed_time(c1) / 1e6

    if args.calibration_copy:
        for _ in range(3):
            basis.aggregate(comps[:1], total)
        torch.cuda.synchronize()

    # ---- the rows beyond Eqs. 2-4, each timed on its own (not part of `value`) -------------------------------
    next_rows = None

    def per_call_ms(fn, n=10):
        fn(); fn()
        a0, a1 = ev(), ev()
        a0.record()
        for i in range(n):
            fn(i)
        a1.record()
        torch.cuda.synchronize()
        return a0.elapsed_time(a1) / n

    if not args.no_next_rows:
        # Algorithm 1's ring step: compress a worker's gradient and add the partial sum that came in (fused)
        ring_ms = per_call_ms(lambda i=0: basis.compress_segment(workers[i % w.N], w.N, 0, S, comps[(i + 1) % 2], comps[i % 2]))
        # Eq. 6 monitor: per-basis squared residual of one gradient (three launches)
        loss_dev = torch.empty(w.n_blocks, device=dev, dtype=torch.float64)
        loss_ms = per_call_ms(lambda i=0: basis.local_loss(workers[i % w.N], w.N, loss_dev))
        # Fig. 2a flattening of the largest layer of this size class: a fully connected layer, [F][D][1][1]
        lay_F = 4096 if w.M >= 4096 * 4096 else 64
        lay_D = min(w.M, 1 << 26) // lay_F
        lay = workers[0][:lay_F * lay_D]
        flat_dev = torch.empty_like(lay)
        code = gvq.BF16 if w.dtype == "bf16" else gvq.F32
        flat_ms = per_call_ms(lambda i=0: gvq.gvq_flatten_conv(lay, flat_dev, lay_F, lay_D, 1, 1, code))
        unflat_ms = per_call_ms(lambda i=0: gvq.gvq_unflatten_conv(flat_dev, out[:lay_F * lay_D], lay_F, lay_D, 1, 1, code))
        next_rows = {"ring_step_ms": round(ring_ms, 4),
                     "ring_step_GBs": round((comp_bytes + S * 4 * w.k) / ring_ms / 1e6, 1),
                     "local_loss_ms": round(loss_ms, 4), "local_loss_gradient_GBs": round(w.M * es / loss_ms / 1e6, 1),
                     "flatten_layer": f"[{lay_F}][{lay_D}][1][1]",
                     "flatten_GBs": round(2 * lay_F * lay_D * es / flat_ms / 1e6, 1),
                     "unflatten_GBs": round(2 * lay_F * lay_D * es / unflat_ms / 1e6, 1)}
        step()   # leaves comps / total / out as the timed steps did
        torch.cuda.synchronize()

    # reconstruction quality (the paper's loss ||ghat - g||^2 / ||g||^2), as a sanity number
    gsum = torch.zeros(w.M, device=dev, dtype=torch.float64)
    for g in workers:
        gsum += g.double()
    loss = float(((out.double() - gsum) ** 2).sum() / (gsum ** 2).sum())
    del gsum

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(w.name, {}).get("compress_bytes_per_launch")
        except Exception:
            traffic = None

    res = {
        "metric": "GB/s fp32 gradient through compress+aggregate+decompress; % of HBM peak",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if w.dtype == "f32" else "bf16 storage, f32 arithmetic",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: M={w.M} d={w.d} k={w.k} N={w.N} L={L} bases={w.n_blocks} "
                               f"store={w.dtype}"},
        "hbm_effective_GBs": round(eff, 1),
        "pct_of_hbm_peak": round(100.0 * eff / HBM_PEAK_GBS, 2),
        "path_algorithmic_bytes": path_bytes,
        "ms_per_step_min": round(step_ms[0], 4), "ms_per_step_median": round(step_ms[len(step_ms) // 2], 4),
        "copy_kernel_GBs": round(copy_gbs, 1),
        "kernels_ms": {"compress_per_launch": round(comp_ms, 4), "aggregate": round(agg_ms, 4),
                       "decompress": round(dec_ms, 4)},
        "kernels_GBs": {"compress": round(comp_bytes / comp_ms / 1e6, 1),
                        "aggregate": round(agg_bytes / agg_ms / 1e6, 1),
                        "decompress": round(dec_bytes / dec_ms / 1e6, 1)},
        "fit": None if args.skip_fit else {"ms": round(fit_ms, 3), "L": L, "jacobi_sweeps": sweeps,
                                            "input_GBs": round(L * w.M * es / fit_ms / 1e6, 1)},
        "reconstruction_loss": loss,
        "next_rows": next_rows,
        "roofline": {"bound": "hbm", "kernel": "compress", "achieved": round(comp_bytes / comp_ms / 1e6, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(comp_bytes / comp_ms / 1e6 / HBM_PEAK_GBS, 4),
                     "algorithmic_bytes_per_launch": comp_bytes, "traffic": traffic,
                     # the counters need the profiler around the process: this number is the committed
                     # result of that run (command in the named file), not a measurement of this run
                     "traffic_source": None if traffic is None else
                     "profiles/hbm_traffic.json (rocprofv3 FETCH_SIZE/WRITE_SIZE runs, see profiles/*_hbm_traffic.md)"},
    }
    # the basis refresh against its own roofline: d x d Gram sums on the fp64 matrix pipe (only the
    # symmetric half of the 16 x 16 blocks is multiplied), input read once from HBM
    if not args.skip_fit:
        full = w.M // w.d
        blocks16 = (w.d + 15) // 16
        fit_flop = 2.0 * L * full * 256 * (blocks16 * (blocks16 + 1) // 2)
        fit_in_bytes = float(L) * w.M * es
        mfma_s, hbm_s = fit_flop / (FP64_MFMA_PEAK_TFLOPS * 1e12), fit_in_bytes / (HBM_PEAK_GBS * 1e9)
        if mfma_s >= hbm_s:
            res["fit"]["roofline"] = {"bound": "mfma", "achieved": round(fit_flop / fit_ms / 1e9, 2),
                                      "peak": FP64_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                                      "frac": round(fit_flop / fit_ms / 1e9 / FP64_MFMA_PEAK_TFLOPS, 4),
                                      "note": "whole refresh (moments + eigensolver) against the moments' flop"}
        else:
            res["fit"]["roofline"] = {"bound": "hbm", "achieved": round(fit_in_bytes / fit_ms / 1e6, 1),
                                      "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                      "frac": round(fit_in_bytes / fit_ms / 1e6 / HBM_PEAK_GBS, 4),
                                      "note": "whole refresh (moments + eigensolver) against the input bytes"}
        if first_slice_ms is not None:
            res["fit"]["first_slice_sampling_ms"] = round(first_slice_ms, 3)
            res["fit"]["select_k"] = {"lambda": 0.01, "ms": round(select_k_ms, 3),
                                      "k_min": int(min(ks)), "k_max": int(max(ks))}
    # slices longer than 128 elements multiply on the bf16 matrix pipe (three products of bf16 terms per
    # fp32 product): should that ever take longer at its peak than the bytes take at the HBM peak, the
    # pipe is the roofline
    if w.d > 128:
        split_flop = 3 * 2.0 * S * w.d * w.k
        if split_flop / (MFMA_BF16_PEAK_TFLOPS * 1e12) > comp_bytes / (HBM_PEAK_GBS * 1e9):
            res["roofline"] = {"bound": "mfma", "kernel": "compress", "achieved": round(split_flop / comp_ms / 1e9, 2),
                               "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                               "frac": round(split_flop / comp_ms / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4),
                               "algorithmic_flop_per_launch": split_flop, "traffic": None}

    # ---- the float64 oracle on the host cores, same inputs, bounded sample --------------------
    if not args.no_cpu_baseline:
        import oracle
        U32, mu32, _ = basis.export()
        U64, mu64 = U32.astype(np.float64), mu32.astype(np.float64)
        offs = w.block_offsets()
        threads = oracle.num_threads()

        def run_oracle(ns):
            """compress x N + aggregate + decompress on the first ns slices."""
            hosts = [synth.to_numpy(g[: min(w.M, ns * w.d)]) for g in workers]
            sub_offs = None
            if offs is not None:
                sub_offs = [o for o in offs if o < ns] + [ns]
            Us, mus = (U64, mu64) if offs is None else (U64[: len(sub_offs) - 1], mu64[: len(sub_offs) - 1])
            t = time.perf_counter()
            ys = [oracle.compress(h, Us, mus, w.N, dtype=w.dtype, offsets=sub_offs) for h in hosts]
            Y = oracle.aggregate(ys)
            oracle.decompress(Y, Us, mus, hosts[0].shape[0], offsets=sub_offs)
            return time.perf_counter() - t

        probe = min(S, 1 << 13)
        t_probe = run_oracle(probe)
        ns = int(min(S, max(probe, probe * 15.0 / max(t_probe, 1e-6))))   # aim at ~15 s
        t_cpu = run_oracle(ns)
        sample_bytes = w.N * min(w.M, ns * w.d) * es
        res["cpu_baseline"] = {"value": round(sample_bytes / t_cpu / 1e9, 3), "unit": "GB/s",
                               "cores": threads, "kind": "oracle",
                               "sample": f"first {ns} of {S} slices of all {w.N} workers "
                                         f"({sample_bytes / 1e9:.2f} GB of gradient), {t_cpu:.1f} s"}
        # the same oracle on ONE thread, on a sample sized for ~4 s
        oracle.set_threads(1)
        ns1 = int(min(S, max(1 << 10, ns * 4.0 / max(t_cpu, 1e-6) / max(threads, 1))))
        t1 = run_oracle(ns1)
        oracle.set_threads(threads)
        res["cpu_baseline"]["value_1_thread"] = round(w.N * min(w.M, ns1 * w.d) * es / t1 / 1e9, 3)
        res["cpu_baseline"]["sample_1_thread"] = f"first {ns1} slices, {t1:.1f} s"
    basis.close()
    del workers, comps, total, out
    return res


if __name__ == "__main__":
    main()
