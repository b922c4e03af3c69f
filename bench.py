#!/usr/bin/env python3
"""Throughput of the hypergradient hot path on one MI355X.

A step is one whole Neumann hypergradient (upper gradient on the validation batch,
forward/backward cache on the train batch, K Hessian-vector products with the
recurrence v <- v - alpha H v, and the mixed second-order VJP into lambda) of the
metric workload: per-parameter L2-decay hyperparameters on the 4-linear-layer GELU MLP
3072-1024-1024-1024-10 (d = 5 256 202), bf16 GEMM operands with fp32 accumulation,
train/val batches of 256, K = 5, alpha = 0.01.  Inputs are synthetic (seeded Gaussian
mixture) and resident in HBM before the timed region.

Prints one JSON line.  Besides the contract keys it carries
  roofline        the launch with the largest share of the step: the weight-gradient instantiation of
                  the fused GEMM whose epilogue applies one step of the Neumann sum to the parameter-
                  sized vectors (all layers in one launch).  It is bandwidth-bound (reduction = batch
                  = 256): algorithmic bytes per launch (20 per parameter) over the launch duration
                  from HIP events recorded by the library, against the HBM peak
  rfwd_link / rbwd_link  one link of the R-forward / R-backward chain (the kernel instantiation with the
                  largest total in the rocprofv3 trace is the R-forward link: 15 launches a step)
  gemm_aggregate  every launch of the GEMM kernel template against the bf16 MFMA peak
  hvp             the per-Hessian-vector-product figures of the metric
  other_configs   the same measurement (median and minimum per call, HVP rate, the launch kind with the
                  largest share and its roofline fraction) on the other benchmark configurations
  cpu_baseline    the fp64 numpy oracle timed on the host cores for the same workload
and, for context, the finite-difference, bilevel-step and three-level-chain rates.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0
PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0


def algorithmic_flops(dims, B):
    """grad = 6 B sum(P) - 2 B n0 n1; HVP = 12 B sum(P) - 8 B n0 n1 (weight matrices only)."""
    P = sum(dims[i] * dims[i + 1] for i in range(len(dims) - 1))
    first = dims[0] * dims[1]
    return 6.0 * B * P - 2.0 * B * first, 12.0 * B * P - 8.0 * B * first


def pmc_traffic_bytes_per_launch(config, which="gemm_fused_kernel"):
    """HBM-side bytes per launch from a committed counter summary (all GEMM launches, or the
    weight-gradient/Neumann instantiation alone), or None when there is no summary for this
    workload or the kernel sources have changed since it was taken."""
    import profile_summary
    path = os.path.join(ROOT, "profiles", f"{which}_config{config}_pmc.txt")
    if not os.path.exists(path):
        return None
    fields = {}
    for line in open(path):
        if ":" in line:
            k, v = line.split(":", 1)
            fields[k.strip()] = v.strip()
    if fields.get("source_hash") != profile_summary.source_hash():
        return None
    try:
        return float(fields["traffic_bytes_per_launch"])
    except (KeyError, ValueError):
        return None


def load_workload(wk, orc_module, index):
    """The seeded workload; config 1 places w at the exact ridge solution (an input of the path)."""
    wl = wk.config(index)
    if wl.w is None:
        import numpy as np
        wl.w = orc_module.ridge_solve(wl.X_tr, wl.t_tr, wl.lam.astype(np.float64)).astype(np.float32)
    return wl


class Runner:
    """One workload resident on the GPU, with the timing loops of this file."""

    def __init__(self, wl, torch, binding):
        self.torch, self.wl = torch, wl
        self.b = binding.from_workload(wl, device="cuda:0")
        self.w, self.lam = torch.as_tensor(wl.w).cuda(), torch.as_tensor(wl.lam).cuda()
        self.out = torch.empty(self.b.n_hyper, dtype=torch.float32, device="cuda")

    def neumann(self, K=None):
        wl = self.wl
        self.b.betty_hypergrad_neumann(self.w, self.lam, wl.K if K is None else K, wl.alpha, out=self.out)

    def timed(self, fn, steps, warmup):
        """Mean seconds per call over `steps` calls issued back to back (the throughput figure)."""
        torch = self.torch
        torch.cuda.synchronize()
        # the calls are issued with the handle's stream current, so the binding adds no
        # cross-stream ordering events around them
        with torch.cuda.stream(self.b.stream):
            for _ in range(warmup):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / steps

    def per_call(self, fn, steps, warmup):
        """Median and minimum seconds of single calls, each between two events on the handle's stream."""
        torch = self.torch
        with torch.cuda.stream(self.b.stream):
            for _ in range(warmup):
                fn()
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
            for e0, e1 in ev:
                e0.record()
                fn()
                e1.record()
            torch.cuda.synchronize()
        ms = [e0.elapsed_time(e1) for e0, e1 in ev]
        return statistics.median(ms) * 1e-3, min(ms) * 1e-3

    def launch_kinds(self, n_prof=5):
        """Per launch kind: launches, milliseconds, algorithmic flops and bytes per step, from the
        library's event bracketing of every launch of a few extra steps."""
        b = self.b
        b.profile(True)
        with self.torch.cuda.stream(b.stream):
            for _ in range(n_prof):
                self.neumann()
            recs = b.profile_records()
        b.profile(False)
        by_kind = {}
        for kind, ms, flops, nbytes in recs:
            a = by_kind.setdefault(kind, [0.0, 0.0, 0.0, 0.0])
            a[0] += 1.0 / n_prof; a[1] += ms / n_prof; a[2] += flops / n_prof; a[3] += nbytes / n_prof
        return by_kind

    def close(self):
        self.b.close()


def kind_roofline(kind, v, peak_tflops):
    """Roofline entry of one launch kind: parameter-shaped update launches against HBM, GEMM launches
    against the MFMA peak of the operand type."""
    launches, ms, flops, nbytes = v
    if kind.startswith("gemm_update") and nbytes > 0:
        gbs = nbytes / (ms * 1e-3) / 1e9
        return {"kind": kind, "bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": gbs / PEAK_HBM_GBS, "launches_per_step": launches, "avg_launch_us": ms / launches * 1e3}
    if flops > 0:
        tf = flops / (ms * 1e-3) / 1e12
        return {"kind": kind, "bound": "mfma", "achieved": tf, "peak": peak_tflops, "unit": "TFLOP/s",
                "frac": tf / peak_tflops, "launches_per_step": launches, "avg_launch_us": ms / launches * 1e3}
    if nbytes > 0:
        gbs = nbytes / (ms * 1e-3) / 1e9
        return {"kind": kind, "bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": gbs / PEAK_HBM_GBS, "launches_per_step": launches, "avg_launch_us": ms / launches * 1e3}
    return {"kind": kind, "bound": None, "launches_per_step": launches, "avg_launch_us": ms / launches * 1e3}


def measure_other(index, wk, orc_module, torch, binding, steps, warmup):
    wl = load_workload(wk, orc_module, index)
    r = Runner(wl, torch, binding)
    t_mean = r.timed(r.neumann, steps, warmup)
    t_k0 = r.timed(lambda: r.neumann(0), max(5, steps // 4), 3)
    med, mn = r.per_call(r.neumann, steps, 3)
    kinds = r.launch_kinds(3)
    r.close()
    B = wl.X_tr.shape[0]
    _, hvp_flops = algorithmic_flops(wl.dims, B)
    t_hvp = (t_mean - t_k0) / wl.K
    peak = PEAK_BF16_TFLOPS if wl.prec == "bf16" else PEAK_FP32_MFMA_TFLOPS
    top = max(kinds.items(), key=lambda kv: kv[1][1])
    note = None
    if wl.prec == "bf16" and wl.act == "relu":
        note = "mixed: forward products on fp32 operands (ReLU mask decided at fp32 accuracy), all other GEMMs bf16"
    return {"workload": f"config {index}: {wl.name}, d={wl.d}, batch {B}/{wl.X_val.shape[0]}, Neumann K={wl.K} alpha={wl.alpha}",
            "dtype": "bf16" if wl.prec == "bf16" else "f32", "precision_note": note,
            "hypergradients_per_s": 1.0 / t_mean, "ms_per_step": t_mean * 1e3,
            "median_ms": med * 1e3, "min_ms": mn * 1e3, "steps": steps,
            "hvp": {"ms": t_hvp * 1e3, "algorithmic_gflop": hvp_flops / 1e9, "tflops": hvp_flops / t_hvp / 1e12,
                    "frac_of_mfma_peak": hvp_flops / t_hvp / 1e12 / peak, "mfma_peak_tflops": peak},
            "top_launch_kind": kind_roofline(top[0], top[1], peak),
            "share_of_step_by_kind": {k: v[1] / sum(x[1] for x in kinds.values()) for k, v in kinds.items()}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=4, help="workload index (4 = the metric workload)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the measurements on configurations 1, 2, 3 and 5")
    ap.add_argument("--only-neumann", action="store_true",
                    help="run only the timed Neumann steps (no K=0, finite-difference or event-bracketed "
                         "legs): the form used under the hardware counters")
    ap.add_argument("--method", default="neumann", choices=["neumann", "fd", "cg"],
                    help="with --only-neumann: the variant whose steps are run (for profiles of the other variants)")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run one plain device-to-device copy of this many MiB (a known-size kernel "
                         "to calibrate hardware byte counters against when profiling)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on exactly one GPU (no collectives or sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2207_02849_amd import binding
    from paper_2207_02849_amd import workloads as wk

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    if args.calib_copy_mib > 0:
        src = torch.ones(args.calib_copy_mib * (1 << 20) // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    orc = None
    if args.config == 1 or (not args.only_neumann and not (args.no_other_configs and args.no_cpu_baseline)):
        from oracle import betty_oracle as orc          # config 1's w (the exact ridge solution) and the CPU baseline
    wl = load_workload(wk, orc, args.config)
    run = Runner(wl, torch, binding)
    b, w, lam, out = run.b, run.w, run.lam, run.out
    K, alpha = wl.K, wl.alpha

    if args.only_neumann:
        fn = {"neumann": run.neumann,
              "fd": lambda: b.betty_hypergrad_fd(w, lam, K, alpha, wl.eps_scale, out=out),
              "cg": lambda: b.betty_hypergrad_cg(w, lam, K, out=out)}[args.method]
        t_step = run.timed(fn, args.steps, args.warmup)
        print(json.dumps({"metric": "hypergradients/s", "method": args.method, "value": 1.0 / t_step,
                          "ms_per_step": t_step * 1e3, "steps": args.steps, "warmup": args.warmup,
                          "config": {"workload": wl.name}}))
        return
    t_step = run.timed(run.neumann, args.steps, args.warmup)
    n_side = max(10, args.steps // 4)
    med, mn = run.per_call(run.neumann, args.steps, 3)
    t_k0 = run.timed(lambda: run.neumann(0), n_side, 5)
    t_fd = None
    if wl.hp == "l2":
        t_fd = run.timed(lambda: b.betty_hypergrad_fd(w, lam, K, alpha, wl.eps_scale, out=out), n_side, 5)

    # the step around the path (one unrolled lower SGD step, the hypergradient, one Adam step)
    mom = torch.zeros_like(w)
    am, av = torch.zeros(b.n_hyper, device="cuda"), torch.zeros(b.n_hyper, device="cuda")
    w_work, lam_work = w.clone(), lam.clone()
    counter = [0]

    def bilevel():
        counter[0] += 1
        b.betty_lower_sgd_step(w_work, lam_work, mom, 1e-3, 0.9, 0.0)
        b.betty_hypergrad_neumann(w_work, lam_work, K, alpha, out=out)
        b.betty_upper_adam_step(lam_work, out, am, av, counter[0], 1e-5)
    t_bilevel = run.timed(bilevel, n_side, 5)

    # the three-level chain (reweight -> pretrain -> finetune) on the same architecture and batch sizes
    t_chain = None
    if wl.d < 5e7 and len(wl.dims) > 2:
        pre_wl, ft_wl = wk.chain3(seed=0, dims=wl.dims, act=wl.act, prec=wl.prec, batch=wl.X_tr.shape[0],
                                  hidden=100, rho=0.007, sigma=2.0, K=K, alpha=alpha)
        bp = binding.from_workload(pre_wl, stream=b.stream)
        bf = binding.from_workload(ft_wl, stream=b.stream)
        cw, cth, cv = (torch.as_tensor(x).cuda() for x in (pre_wl.w, pre_wl.lam, ft_wl.w))
        cout = torch.empty(bp.n_hyper, dtype=torch.float32, device="cuda")
        t_chain = run.timed(lambda: bp.betty_hypergrad_chain3(bf, cw, cth, cv, K, alpha, K, alpha, out=cout), n_side, 5)
        bp.close()
        bf.close()

    B = wl.X_tr.shape[0]
    grad_flops, hvp_flops = algorithmic_flops(wl.dims, B)
    t_hvp = (t_step - t_k0) / K if K > 0 else float("nan")
    peak = PEAK_BF16_TFLOPS if wl.prec == "bf16" else PEAK_FP32_MFMA_TFLOPS

    # per-kernel durations from HIP events around every launch of a few extra steps
    by_kind = run.launch_kinds(5)
    zero = [0.0, 0.0, 0.0, 0.0]
    upd, fin = by_kind.get("gemm_update", zero), by_kind.get("gemm_update_final", zero)
    # every launch of the GEMM kernel, whether its epilogue carries the Neumann update or not
    gemm = [sum(by_kind.get(k, zero)[i] for k in ("gemm", "gemm_rfwd", "gemm_rbwd", "gemm_update", "gemm_update_final"))
            for i in range(4)]
    gemm_tflops = gemm[2] / (gemm[1] * 1e-3) / 1e12 if gemm[1] > 0 else 0.0
    # vector phase of the recurrence: it lives in the epilogue of the weight-gradient launch, so its
    # rate is quoted over the whole fused launch (20 algorithmic bytes per parameter)
    vec_gbs = upd[3] / (upd[1] * 1e-3) / 1e9 if upd[1] > 0 else 0.0
    total_ms = sum(v[1] for v in by_kind.values())
    phases = {k: {"launches_per_step": v[0], "ms_per_step": v[1], "share_of_step": v[1] / total_ms}
              for k, v in by_kind.items()}

    traffic_all = pmc_traffic_bytes_per_launch(args.config)
    traffic_upd = pmc_traffic_bytes_per_launch(args.config, "gemm_fused_kernel_wgrad_neumann")
    result = {
        "metric": "hypergradients/s, MLP Neumann K=5; HVP % of MFMA peak",
        "value": 1.0 / t_step,
        "unit": "hypergradients/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": t_step * 1e3,
        "median_ms": med * 1e3,
        "min_ms": mn * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if wl.prec == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"config {args.config}: {wl.name}, d={wl.d}, batch {B}/{wl.X_val.shape[0]}, "
                               f"Neumann K={K} alpha={alpha}"},
        "roofline": {
            "bound": "hbm",
            "kernel": "gemm_fused_kernel<64x64 tile, epilogue WGRAD_NEUMANN>: all layers' weight-gradient "
                      "products of one Hessian-vector product with the Neumann step on s, g, lambda and "
                      "the operand copies in the epilogue (longest launch of the step, and with its INIT and "
                      "final siblings the largest share of it; the instantiation with the largest total in the "
                      "trace is the 7.7 us R-forward link, see rfwd_link)",
            "achieved": vec_gbs,
            "peak": PEAK_HBM_GBS,
            "unit": "GB/s",
            "frac": vec_gbs / PEAK_HBM_GBS,
            "traffic": traffic_upd,
            "launches_per_step": upd[0],
            "avg_launch_us": (upd[1] / upd[0] * 1e3) if upd[0] else None,
            "algorithmic_bytes_per_launch": (upd[3] / upd[0]) if upd[0] else None,
        },
        "rfwd_link": kind_roofline("gemm_rfwd", by_kind["gemm_rfwd"], peak) if "gemm_rfwd" in by_kind else None,
        "rbwd_link": kind_roofline("gemm_rbwd", by_kind["gemm_rbwd"], peak) if "gemm_rbwd" in by_kind else None,
        "gemm_aggregate": {
            "bound": "mfma",
            "kernel": "gemm_fused_kernel (all instantiations; every GEMM launch of one hypergradient)",
            "achieved": gemm_tflops,
            "peak": peak,
            "unit": "TFLOP/s",
            "frac": gemm_tflops / peak,
            "traffic": traffic_all,
            "launches_per_step": gemm[0],
            "avg_launch_us": gemm[1] / gemm[0] * 1e3 if gemm[0] else None,
            "avg_launch_gflop": gemm[2] / gemm[0] / 1e9 if gemm[0] else None,
        },
        "hvp": {"ms": t_hvp * 1e3, "algorithmic_gflop": hvp_flops / 1e9,
                "tflops": hvp_flops / t_hvp / 1e12, "frac_of_bf16_mfma_peak": hvp_flops / t_hvp / 1e12 / peak},
        "phases": phases,
        "fd_hypergradients_per_s": (1.0 / t_fd) if t_fd else None,
        # the finite-difference variant forms its products from fp32 operands (the difference of two
        # gradients eps apart needs fp32 accuracy), so fp32 MFMA is the roof of its GEMMs: one upper
        # gradient plus 2K lower gradients, each a forward, a backward and a weight-gradient pass
        "fd": None if not t_fd else {
            "ms": t_fd * 1e3, "algorithmic_gflop": (2 * K + 1) * grad_flops / 1e9,
            "tflops": (2 * K + 1) * grad_flops / t_fd / 1e12,
            "frac_of_fp32_mfma_peak": (2 * K + 1) * grad_flops / t_fd / 1e12 / PEAK_FP32_MFMA_TFLOPS},
        "bilevel_upper_steps_per_s": {"value": 1.0 / t_bilevel,
                                      "step": "1 lower momentum-SGD step + Neumann hypergradient + Adam step on lambda"},
        "chain3_hypergradients_per_s": None if t_chain is None else {
            "value": 1.0 / t_chain,
            "step": f"three-level chain on the same architecture: Neumann K={K} best-response product on the "
                    "proximal finetuning problem, then on the reweighting pretraining problem"},
    }
    run.close()
    del run, b, w, lam, out, w_work, lam_work, mom, am, av
    torch.cuda.empty_cache()

    if not args.no_other_configs:
        others = {}
        for idx in (1, 2, 3, 5):
            if idx == args.config:
                continue
            others[f"config{idx}"] = measure_other(idx, wk, orc, torch, binding, steps=20 if idx == 5 else 100,
                                                   warmup=3 if idx == 5 else 10)
            torch.cuda.empty_cache()
        result["other_configs"] = others

    if not args.no_cpu_baseline:
        from threadpoolctl import threadpool_info
        y_tr = wl.y_tr
        if y_tr is None and wl.y_clean is not None:
            y_tr = orc.apply_label_noise(wl.y_clean, wl.noise_words, wl.noise_alt, wl.noise_p)[0]
        prob = orc.Problem(dims=wl.dims, act=wl.act, loss=wl.loss, hp=wl.hp, has_bias=wl.has_bias,
                           X_tr=wl.X_tr, X_val=wl.X_val, y_tr=y_tr, y_val=wl.y_val, t_tr=wl.t_tr,
                           t_val=wl.t_val, wnet_hidden=wl.wnet_hidden)
        reps, t_cpu = 0, 0.0
        t0 = time.perf_counter()
        while reps < 1 or (time.perf_counter() - t0 < 10.0 and reps < 8):
            orc.hypergrad_neumann(prob, wl.w, wl.lam, K, alpha)
            reps += 1
        t_cpu = (time.perf_counter() - t0) / reps
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        result["cpu_baseline"] = {"value": 1.0 / t_cpu, "unit": "hypergradients/s", "cores": os.cpu_count(),
                                  "blas_threads": threads, "kind": "oracle (numpy fp64, BLAS matmul)",
                                  "sample": f"{reps} whole hypergradient(s) of the same workload (fp64 numpy oracle)"}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
