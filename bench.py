#!/usr/bin/env python3
"""Throughput of SAMA's per-iteration hot path on one MI355X: meta-steps/sec.

One "step" = one pass of the whole hot path at unroll U (default 1): U x sama_base_step + one sama_meta_step
(direct-gradient pass, adaptation + norm, two +-eps passes, finite-difference combine, meta-Adam, nudge) on
synthetic batches that are resident in HBM before the timed region starts.

Prints ONE JSON line.  `roofline` is for the dominant kernel (measured in a separate instrumented replay of the
same steps with HIP events on the launch stream, so that the event records do not slow the timed region);
`roofline.kernels` lists every kernel family.  `cpu_baseline` is the float64 oracle on the host cores on a
bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PEAK_BF16_TFLOPS = 2500.0      # dense bf16 MFMA
PEAK_FP32_MATRIX_TFLOPS = 157.3


def measured_traffic(cfg_id, family):
    """HBM-side bytes per launch of a kernel family, as the two rocprofv3 --pmc runs of this command measured them
    (FETCH_SIZE and WRITE_SIZE, calibrated on the library's own copy kernel): read from the line
    `traffic_bytes_per_launch <family> = <bytes>` of profiles/bench_workload<k>_hbm_traffic.md, which the profile summary
    carries next to its table.  None where no such profile exists (other workloads, other launch options)."""
    import re
    path = os.path.join(ROOT, "profiles", f"bench_workload{cfg_id}_hbm_traffic.md")
    try:
        m = re.search(r"traffic_bytes_per_launch\s+" + re.escape(family) + r"\s*=\s*([0-9.eE+]+)", open(path).read())
    except OSError:
        return None
    return float(m.group(1)) if m else None


def fwd_flops(wl, batch):
    """Algorithmic flops of one forward pass of the base learner on `batch` samples (2 flops per MAC)."""
    if wl.kind == "mlp":
        return sum(2.0 * batch * wl.dims[i] * wl.dims[i + 1] for i in range(len(wl.dims) - 1))
    L, d, heads, ffn, S, V, C = wl.dims
    M = batch * S
    per_layer = 2.0 * M * d * 3 * d + 2.0 * M * d * d + 2 * 2.0 * M * d * ffn + 2 * 2.0 * batch * heads * S * S * (d // heads)
    return L * per_layer + 2.0 * batch * d * C


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", type=int, default=5, help="BASELINE.json config number 1..5")
    ap.add_argument("--unroll", type=int, default=1)
    ap.add_argument("--fast-meta-pass", type=int, default=0)
    ap.add_argument("--fast-base-pass", type=int, default=0,
                    help="1: the base step contracts with the bf16 working copy alone (ordinary mixed precision) instead of the "
                         "two-term split of the fp32 master weights; not the configuration the parity tests prove")
    ap.add_argument("--corr-hidden", type=int, default=0,
                    help="label correction (Sec. 4.1) with a corrector of this hidden width; 0 = the headline data-reweighting workload")
    ap.add_argument("--aux", action="store_true",
                    help="auxiliary-task reweighting (Sec. 4.3) instead of the headline workload: the 12-layer encoder with a "
                         "50304-token masked-token head, 16 finetuning + 16 auxiliary sequences per base step")
    ap.add_argument("--length-mix", action="store_true",
                    help="encoder workloads: padded batches with a seeded length mix (key-padding mask); padded tokens are "
                         "still computed, so the rate is that of full sequences")
    ap.add_argument("--graph", action="store_true",
                    help="capture each iteration (unroll base steps + meta step) into a HIP graph once per synthetic batch and time "
                         "replays instead of eager calls")
    ap.add_argument("--no-unroll10", action="store_true", help="skip the extra timed region at unroll 10 (the paper's operating point)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-roofline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from datagen import make_workload, init_theta, init_lambda, init_lambda_corr, make_aux_workload, make_aux_batch, AUX_TASK
    import paper_2310_05674_amd as pkg

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.graph:                                          # capture needs a stream other than the default one
        run_stream = torch.cuda.Stream(device=dev)
        torch.cuda.set_stream(run_stream)
    cfg_id = args.workload
    nb = 4                                                  # distinct synthetic batches cycled through
    if args.aux:
        if args.corr_hidden:
            sys.exit("bench.py: --aux and --corr-hidden cannot be combined")
        cfg_id = AUX_TASK["base"]
        wl = make_aux_workload(n_train=AUX_TASK["batch"] * nb, n_meta=AUX_TASK["meta_batch"] * nb)
    else:
        wl0 = make_workload(cfg_id, n_train=8, n_meta=8)        # shapes only
        wl = make_workload(cfg_id, n_train=min(wl0.batch * nb, 12800) if cfg_id != 1 else None,
                           n_meta=min(wl0.meta_batch * nb, 1280) if cfg_id != 1 else None)
    th0, lam0 = init_theta(wl), init_lambda(wl)
    if args.corr_hidden > 0:
        lam0 = np.concatenate([lam0, init_lambda_corr(wl, args.corr_hidden)])
    cfg = pkg.SamaConfig.make(wl.kind, wl.dims, H=wl.H, max_batch=wl.batch, max_meta_batch=wl.meta_batch,
                              base_lr=wl.base_lr, meta_lr=wl.meta_lr, alpha=wl.alpha, beta1=wl.beta1, beta2=wl.beta2,
                              adam_eps=wl.adam_eps, fast_meta_pass=args.fast_meta_pass, fast_base_pass=args.fast_base_pass, corr_hidden=args.corr_hidden,
                              **(dict(aux_mlm=1, max_aux_batch=AUX_TASK["n_pt"], max_aux_masked=AUX_TASK["n_pt"] * (AUX_TASK["dims"][4] // 5 + 1)) if args.aux else {}))
    s = pkg.Sama(cfg, th0, lam0)
    n, n16 = s.n, s.lib.sama_gemm_param_count(__import__("ctypes").byref(cfg))
    batches = []
    if args.length_mix and (wl.kind != "encoder" or args.aux):
        raise SystemExit("--length-mix applies to the encoder workloads 3..5 (not to --aux)")
    from datagen import seq_lengths
    len_train = seq_lengths(wl.seed + 11, len(wl.y_train), wl.dims[4]) if args.length_mix else None
    len_meta = seq_lengths(wl.seed + 12, len(wl.y_meta), wl.dims[4]) if args.length_mix else None
    dl = lambda a: None if a is None else torch.as_tensor(np.ascontiguousarray(a), device=dev)
    for k in range(nb):
        it, im = wl.train_batch(k), wl.meta_batch_idx(k)
        batches.append((s.batch(torch.as_tensor(np.ascontiguousarray(wl.x_train[it]), device=dev),
                                torch.as_tensor(wl.y_train[it].astype(np.int32), device=dev),
                                seq_len=dl(None if len_train is None else len_train[it])),
                        s.batch(torch.as_tensor(np.ascontiguousarray(wl.x_meta[im]), device=dev),
                                torch.as_tensor(wl.y_meta[im].astype(np.int32), device=dev),
                                seq_len=dl(None if len_meta is None else len_meta[im]))))

    aux = []
    if args.aux:
        S = wl.dims[4]
        for k in range(nb):
            ids, seq, pos, tgt = make_aux_batch(wl, k, AUX_TASK["n_pt"])
            t = lambda a: torch.as_tensor(np.ascontiguousarray(a).astype(np.int32), device=dev)
            aux.append(s.aux_batch(t(ids), t(seq.astype(np.int64) * S + pos), t(tgt)))

    def step(k):
        tb, mb = batches[k % nb]
        if args.aux:
            for _ in range(args.unroll):
                s.aux_base_step(tb, aux[k % nb])
            s.aux_meta_step(aux[k % nb], mb)
            return
        for _ in range(args.unroll):
            s.base_step(tb)
        s.meta_step(tb, mb)

    if args.aux:
        s.aux_base_step(batches[0][0], aux[0])
    else:
        s.base_step(batches[0][0])                          # one step of Adam history before anything is timed
    step_eager = step
    if args.graph:
        step_eager(0)                                       # lazy set-up (second stream, kernel attributes) outside the captures
        torch.cuda.synchronize(dev)
        graphs = []
        for k in range(nb):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=run_stream, capture_error_mode="thread_local"):
                step_eager(k)
            graphs.append(g)

        def step(k):                                        # noqa: F811
            graphs[k % nb].replay()
    for k in range(args.warmup):
        step(k)
    torch.cuda.synchronize(dev)
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(args.warmup + k)
    torch.cuda.synchronize(dev)
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    status = s.get_state("COUNTERS").cpu().numpy()
    skipped = int(status[2])

    # The paper's operating point (App. B: unroll step 10): ten base steps per meta step, timed after the headline region
    unroll10 = None
    if args.unroll == 1 and not args.no_unroll10:
        def step10(k):
            tb, mb = batches[k % nb]
            for _ in range(10):
                (s.aux_base_step(tb, aux[k % nb]) if args.aux else s.base_step(tb))
            (s.aux_meta_step(aux[k % nb], mb) if args.aux else s.meta_step(tb, mb))
        step10(0)
        torch.cuda.synchronize(dev)
        k10 = max(2, min(5, args.steps // 4))
        t1 = time.perf_counter()
        for k in range(k10):
            step10(1 + k)
        torch.cuda.synchronize(dev)
        e10 = time.perf_counter() - t1
        unroll10 = {"unroll": 10, "value": k10 / e10, "unit": "meta-steps/s", "ms_per_step": 1e3 * e10 / k10, "steps": k10, "warmup": 1,
                    "base_steps_per_s": 10 * k10 / e10, "launch": "eager"}

    out = {
        "metric": "SAMA meta-steps/sec on 1 MI355X", "value": args.steps / elapsed, "unit": "meta-steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.bf16 else "f32", "data": "synthetic",
        "config": {"workload": ("auxiliary-task reweighting (Sec. 4.3; not a BASELINE.json config), {} auxiliary sequences / {} masked "
                                "positions per base step: ".format(AUX_TASK["n_pt"], aux[0].n_mask) if args.aux else
                                f"BASELINE.json configs[{cfg_id - 1}]: ") +
                   ("MLP " + "-".join(map(str, wl.dims)) if wl.kind == "mlp" else
                    "encoder L={} d={} heads={} ffn={} S={} V={} C={}".format(*wl.dims)),
                   "params": int(n), "train_batch": wl.batch, "meta_batch": wl.meta_batch, "unroll": args.unroll,
                   "launch": "hip graph replay" if args.graph else "eager", "padding": "length mix" if args.length_mix else "none", "wnet_hidden": wl.H, "corr_hidden": args.corr_hidden, "n_lambda": int(s.nl), "meta_pass": "bf16" if args.fast_meta_pass else "split hi+lo", "base_pass": "bf16" if args.fast_base_pass else "split hi+lo",
                   "last_step_skipped": bool(skipped),
                   "workspace_bytes": int(s.lib.sama_workspace_bytes(__import__("ctypes").byref(cfg)))},
    }

    # ---------------------------------------------------------------- per-kernel roofline (instrumented replay)
    if not args.no_roofline:
        prof_steps = min(args.steps, 5)
        # The timed region above overlaps the weight-gradient GEMMs and the per-layer optimizer / adaptation slices with
        # the backward chain on a second stream.  Per-kernel figures are about the kernels, so the instrumented replay
        # keeps every launch on one stream (a tuning hook of the library): no two kernels share the machine.
        import ctypes
        s.lib.sama_dev_side_stream(ctypes.c_int32(0))
        s.profile(True)
        for k in range(prof_steps):
            step_eager(k)
        torch.cuda.synchronize(dev)
        fam = s.profile_read()
        s.profile(False)
        s.lib.sama_dev_side_stream(ctypes.c_int32(1))
        kernels = {}
        for name, (cnt, ms, units) in fam.items():
            avg_us = 1e3 * ms / cnt
            ent = {"launches_per_step": cnt / prof_steps, "avg_us": avg_us, "ms_per_step": ms / prof_steps}
            if name.startswith("gemm_bf16") or name.startswith("attention"):
                # The library counts a two-term (hi + lo) launch as the contraction over the concatenated operand it
                # executes, 2 M N (2K); the algorithmic work of the method is 2 M N K per GEMM, whatever the split.
                alg = 0.5 * units if name.endswith("_hilo") else units
                ent.update(bound="mfma", achieved=alg / (ms * 1e-3) / 1e12, peak=PEAK_BF16_TFLOPS, unit="TFLOP/s")
                if name.endswith("_hilo"):
                    ent["executed"] = {"achieved": units / (ms * 1e-3) / 1e12, "frac": units / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                                       "note": "matrix-core work as issued: both halves of the split weights"}
            elif name == "gemm_f32":
                ent.update(bound="mfma", achieved=units / (ms * 1e-3) / 1e12, peak=PEAK_FP32_MATRIX_TFLOPS, unit="TFLOP/s")
            elif units > 0:   # every other family is priced in algorithmic bytes
                ent.update(bound="hbm", achieved=units / (ms * 1e-3) / 1e9, peak=PEAK_HBM_GBS, unit="GB/s")
            if "achieved" in ent:
                ent["frac"] = ent["achieved"] / ent["peak"]
            kernels[name] = ent
        dom = max(kernels, key=lambda k: kernels[k]["ms_per_step"])
        d = kernels[dom]
        U = args.unroll
        paper_flops = (3 * U + 5) * fwd_flops(wl, wl.batch)   # three-pass count of Sec. 3.3 (train and meta batches are equal here)
        if args.aux:   # base steps run over ft + auxiliary sequences and the vocabulary head; the +- passes over the auxiliary ones
            n_pt, head = AUX_TASK["n_pt"], 2.0 * aux[0].n_mask * wl.dims[1] * wl.dims[5]
            paper_flops = (3 * U * (fwd_flops(wl, wl.batch + n_pt) + head) + 3 * fwd_flops(wl, wl.meta_batch)
                           + 2 * (fwd_flops(wl, n_pt) + head))
        ew = [kernels[k] for k in ("adam", "adapt_norm", "perturb_lo", "residual_lo", "nudge") if k in kernels]
        ew_bytes = sum(k["achieved"] * 1e9 * k["ms_per_step"] * 1e-3 for k in ew)
        ew_ms = sum(k["ms_per_step"] for k in ew)
        default_launch = args.unroll == 1 and not (args.fast_meta_pass or args.fast_base_pass or args.aux or args.corr_hidden or args.length_mix)
        out["roofline"] = {
            "replay": "per-kernel durations from an instrumented replay with every launch on one stream; the timed steps "
                      "run the weight-gradient GEMMs and per-layer update slices on a second stream",
            "kernel": dom, "bound": d.get("bound"), "achieved": d.get("achieved"), "peak": d.get("peak"),
            "unit": d.get("unit"), "frac": d.get("frac"),
            "work": "algorithmic: 2 M N K per GEMM (bytes the method must move for the HBM-bound families)",
            "executed": d.get("executed"),   # hi + lo families: the matrix-core work as issued, 2 M N (2K); else null
            "traffic": measured_traffic(cfg_id, dom) if default_launch else None,
            "avg_us": d["avg_us"],
            "elementwise_chain": {"bound": "hbm", "achieved": ew_bytes / (ew_ms * 1e-3) / 1e9 if ew_ms > 0 else None,
                                  "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                  "frac": ew_bytes / (ew_ms * 1e-3) / 1e9 / PEAK_HBM_GBS if ew_ms > 0 else None,
                                  "ms_per_step": ew_ms, "bytes_per_param": ew_bytes / n},
            "step_algorithmic": {"flops_per_step": paper_flops, "achieved": paper_flops / (ms_per_step * 1e-3) / 1e12,
                                 "unit": "TFLOP/s", "peak": PEAK_BF16_TFLOPS if wl.bf16 else PEAK_FP32_MATRIX_TFLOPS},
            "kernels": kernels,
        }
    if unroll10 is not None:
        out["unroll10"] = unroll10

    # ---------------------------------------------------------------- oracle on the host cores (bounded sample)
    if not args.no_cpu_baseline:
        from oracle import models
        from oracle.reweight import SamaOracle
        # One oracle iteration costs a + b * batch seconds (a: the elementwise chain over the n parameters and the fixed
        # overheads, b: the passes over one sample).  Workloads 1-3 are timed at the benched batch itself; for 4 and 5
        # that takes minutes, so a and b are measured at two small batch sizes and the benched batch is priced with them.
        sizes = {1: [wl.batch], 2: [wl.batch], 3: [wl.batch], 4: [1, 3], 5: [1, 2]}[cfg_id]
        reps = {1: 20, 2: 10, 3: 2}.get(cfg_id, 1)
        times = []
        for cb in sizes:
            cm = min(cb, wl.meta_batch)
            it, im = wl.train_batch(0)[:cb], wl.meta_batch_idx(0)[:cm]
            x, y, xm, ym = wl.x_train[it], wl.y_train[it], wl.x_meta[im], wl.y_meta[im]
            if args.length_mix:
                x, xm = models.with_lengths(x, len_train[it]), models.with_lengths(xm, len_meta[im])
            if args.aux:
                from oracle.auxtask import AuxTaskOracle
                orc = AuxTaskOracle(models.make_model(wl.kind, wl.dims, mlm=True), th0, lam0, base_lr=wl.base_lr,
                                    meta_lr=wl.meta_lr, alpha=wl.alpha)
                pt = make_aux_batch(wl, 0, cb)
                orc.base_step((x, y), pt)                                     # history (untimed)
                t0 = time.perf_counter()
                for _ in range(args.unroll):
                    orc.base_step((x, y), pt)
                orc.meta_step(pt, (xm, ym))
            else:
                orc = SamaOracle(models.make_model(wl.kind, wl.dims), th0, lam0, base_lr=wl.base_lr, meta_lr=wl.meta_lr,
                                 alpha=wl.alpha, corr_hidden=args.corr_hidden,
                                 n_classes=wl.dims[-1] if args.corr_hidden > 0 else None)
                orc.base_step(x, y)                                           # history (untimed)
                t0 = time.perf_counter()
                for _ in range(reps):
                    for _ in range(args.unroll):
                        orc.base_step(x, y)
                    orc.meta_step(x, y, xm, ym)
            times.append((time.perf_counter() - t0) / reps)
            del orc
        try:
            import threadpoolctl
            threads = max((p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()), default=1)
        except Exception:
            threads = os.cpu_count()
        if len(sizes) == 1:
            tcpu = times[0]
            sample = (f"{reps} iteration(s) (unroll {args.unroll}) of the float64 NumPy oracle at the benched train/meta batch "
                      f"{wl.batch}/{wl.meta_batch}: {tcpu:.3f} s each")
        else:
            b_ = (times[1] - times[0]) / (sizes[1] - sizes[0])
            a_ = times[0] - b_ * sizes[0]
            tcpu = a_ + b_ * wl.batch
            sample = (f"one iteration (unroll {args.unroll}) of the float64 NumPy oracle at train = meta batch {sizes[0]} and {sizes[1]}: "
                      f"{times[0]:.2f} s and {times[1]:.2f} s, i.e. {a_:.2f} s + {b_:.2f} s per sample; the benched batch "
                      f"{wl.batch}/{wl.meta_batch} priced with that line: {tcpu:.1f} s per iteration")
        out["cpu_baseline"] = {"value": 1.0 / tcpu, "unit": "meta-steps/s", "cores": int(threads), "kind": "oracle", "sample": sample}
    s.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
