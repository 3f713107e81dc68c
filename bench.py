#!/usr/bin/env python3
"""Benchmark of one learner's training step on one MI355X.

A step is one pass of the whole hot path over one synthetic batch: blstm_forward,
softmax_xent_fwd_bwd, blstm_backward, the learner's sgd_step and its adpsgd_mix with a ring
neighbour's replica held in the same HBM (the last two as one pass over the weights: sgd_mix_pair
without a gradient for the neighbour, bit-identical to the two calls).  Inputs are resident in HBM before the timed region.

Prints ONE JSON line:
  value            frames/s of the whole job (wall clock around K steps, synchronised on both sides);
  step_ms          median and minimum of the K steps timed one by one with events on the launch stream;
  kernel_classes   per-class durations from HIP events the library records on the launch stream;
  roofline         the kernel that takes the largest share of the step, by kernel name, against the
                   bf16 MFMA peak; roofline_gemm: the product class with the largest share; roofline_recurrent:
                   the slower of the two persistent recurrent kernels;
  adpsgd_mix ...   the streaming kernels against HBM bandwidth;
  other_workloads  the same step on the large-batch, 6x1024 and 6x512 workloads, briefly (8 timed steps each);
  cpu_baseline     the float64 oracle timed on this machine's host cores on the same workload.
HBM traffic figures ("traffic") are read from profiles/hbm_traffic_<workload>.txt, which records the
hash of the kernel sources it was measured with; they are null when the sources have changed since.
"""
from __future__ import annotations

import argparse
import glob
import hashlib
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA = 2.5e15      # FLOP/s, dense
PEAK_FP32_MFMA = 157.3e12
PEAK_HBM = 8.0e12            # B/s

# kernel name behind each timing class of the library (one class = one kernel function, by shape several instantiations)
KERNEL_OF_CLASS = {
    "recurrent_fwd_persistent": "rec_fwd_kernel", "recurrent_bwd_persistent": "rec_bwd_kernel",
    "gemm_wgrad": "gemm_group_kernel", "softmax_rows": "softmax_rows_bf16_regs_kernel",
    "gemm_input_projection": "gemm_kernel", "gemm_bottleneck": "gemm_kernel", "gemm_logits": "gemm_kernel",
    "gemm_softmax_bwd": "gemm_kernel", "gemm_dgrad": "gemm_kernel", "gemm_recurrent_fwd": "gemm_kernel",
    "gemm_recurrent_bwd": "gemm_kernel", "cell_fwd": "cell_fwd_kernel", "cell_bwd": "cell_bwd_kernel",
}


def source_hash():
    """Hash of the kernel sources: measured HBM traffic is only quoted for the sources it was measured with."""
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_1904_04956_amd", "csrc", "*"))):
        with open(f, "rb") as fh:
            h.update(os.path.basename(f).encode())
            h.update(fh.read())
    return h.hexdigest()[:16]


def measured_traffic(workload, batch):
    """{class: HBM bytes per launch} from profiles/hbm_traffic_<workload>.txt, {} if absent or measured on other sources.

    The file holds lines `sources <hash>`, `batch <B>` and `bytes_per_launch <class> <bytes>` besides its prose."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    if not os.path.exists(path):
        return {}
    out, ok_src, ok_batch = {}, False, False
    for line in open(path):
        w = line.split()
        if len(w) >= 2 and w[0] == "sources":
            ok_src = w[1] == source_hash()
        elif len(w) >= 2 and w[0] == "batch":
            ok_batch = int(w[1]) == batch
        elif len(w) >= 3 and w[0] == "bytes_per_launch":
            out[w[1]] = float(w[2])
    return out if (ok_src and ok_batch) else {}


def flops_by_class(T, B, D, H, L, P, V, softmax_wgrad_deferred=False):
    """Algorithmic FLOP of one step per kernel class (2 FLOP per multiply-add).

    softmax_wgrad_deferred: dW_s runs in the backward pass's grouped weight-gradient launch
    (BLSTM_OPT_DEFER_SOFTMAX_WGRAD) instead of in softmax_xent_fwd_bwd."""
    M = T * B
    Z = P if P > 0 else 2 * H
    din = [D] + [2 * H] * (L - 1)
    f = {}
    f["gemm_input_projection"] = sum(2 * M * 8 * H * d for d in din)
    f["gemm_recurrent_fwd"] = L * (T - 1) * 2 * (2 * B * 4 * H * H)
    f["gemm_bottleneck"] = 2 * M * 2 * H * P
    f["gemm_logits"] = 2 * M * V * Z
    f["gemm_softmax_bwd"] = 2 * 2 * M * V * Z
    f["gemm_recurrent_bwd"] = L * (T - 1) * 2 * (2 * B * 4 * H * H)
    # the persistent kernels do a whole layer (both directions, all frames) per launch
    f["recurrent_fwd_persistent"] = f["gemm_recurrent_fwd"]
    f["recurrent_bwd_persistent"] = f["gemm_recurrent_bwd"]
    f["gemm_wgrad"] = sum(2 * M * 8 * H * d for d in din) + L * 2 * (T - 1) * B * 8 * H * H + 2 * M * P * 2 * H
    f["gemm_dgrad"] = sum(2 * M * 8 * H * d for d in din[1:]) + 2 * M * 2 * H * P
    if softmax_wgrad_deferred:
        f["gemm_softmax_bwd"] -= 2 * M * V * Z
        f["gemm_wgrad"] += 2 * M * V * Z
    return f


def flop_per_frame(D, H, L, P, V):
    """Forward + backward FLOP per frame: 2 * (3 * MACs - the input-gradient product of layer 1)."""
    Z = P if P > 0 else 2 * H
    din = [D] + [2 * H] * (L - 1)
    macs = sum(2 * 4 * H * (d + H) for d in din) + (2 * H * P if P > 0 else 0) + Z * V
    return 2 * (3 * macs - 2 * 4 * H * D)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="paper4x512")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true", help="skip the per-kernel-class event pass")
    ap.add_argument("--rec-sync", type=int, default=-1, help="exchange protocol of the persistent kernels (library default if < 0)")
    ap.add_argument("--rec-path", type=int, default=0, help="1 = one launch per frame")
    ap.add_argument("--mix-replicas", type=int, default=16, help="replicas of the separate adpsgd_mix measurement")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short runs of the other workloads (large batch, 6x1024, 6x512) reported under other_workloads")
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="first copy 1 GiB three times with a plain copy kernel (reference for HBM counters under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (one learner per GPU, no collectives); use --gpus 1")

    import numpy as np
    import torch
    from paper_1904_04956_amd import binding as bl
    from paper_1904_04956_amd import inputs
    from paper_1904_04956_amd.harness import Learner

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    w = inputs.WORKLOADS[args.workload]
    d = w.dims()
    if args.batch > 0:
        d["B"] = args.batch
    T, B = d["T"], d["B"]
    bf = w.mode == 1

    if args.traffic_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    lrn = Learner(mode=w.mode, recurrent_path=args.rec_path, **d)
    if args.rec_sync >= 0:
        bl.blstm_set_option(lrn.ctx, bl.BLSTM_OPT_RECURRENT_SYNC, args.rec_sync)
    theta = inputs.make_theta(lrn.n, w.seed, bf16=bf)
    x, labels = inputs.make_batch(T, B, d["D"], d["V"], w.seed, bf16=bf)
    lrn.set_theta(theta)
    lrn.set_batch(x, labels)
    # the ring neighbour's replica: same buffers a second learner would hold
    nb_theta = lrn.theta.clone()
    nb_shadow = lrn.shadow.clone() if lrn.shadow is not None else None
    masters = [lrn.theta, nb_theta]
    shadows = [lrn.shadow, nb_shadow] if nb_shadow is not None else None

    def step():
        lrn.calgrad()
        # Eq. 4 for this learner: its own update (Eq. 1c), then the average with the neighbour's replica as it stands,
        # in one pass over the weights (same bits as sgd_step followed by adpsgd_mix)
        bl.sgd_mix_pair(lrn.theta, nb_theta, lrn.shadow, nb_shadow, lrn.grad, None, lrn.n, w.lr, lrn.momentum, lrn.velocity, None)
        lrn.weights_changed()

    for _ in range(args.warmup):
        step()
    lrn.check_status()                       # synchronises; raises if a persistent kernel gave up a wait
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    lrn.check_status()
    ms_per_step = 1e3 * dt / args.steps
    frames_per_s = T * B * args.steps / dt
    loss = lrn.loss_value()
    # the same steps one by one, each bracketed by events on the launch stream
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for a, b in evs:
        a.record(); step(); b.record()
    torch.cuda.synchronize()
    each = [a.elapsed_time(b) for a, b in evs]
    # for reference: the same step with the update and the averaging as the two separate calls (same bits, 10 B more per parameter)
    def step_two_calls():
        lrn.calgrad()
        lrn.apply(w.lr)
        bl.adpsgd_mix(masters, shadows, lrn.n, 2, [1, 0])
        lrn.weights_changed()
    for _ in range(2):
        step_two_calls()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step_two_calls()
    torch.cuda.synchronize()
    two_call_ms = 1e3 * (time.perf_counter() - t0) / args.steps
    fpf = flop_per_frame(d["D"], d["H"], d["L"], d["P"], d["V"])
    peak = PEAK_BF16_MFMA if bf else PEAK_FP32_MFMA

    out = {
        "metric": "training frames/sec (fwd+bwd+update) on 1 MI355X", "value": frames_per_s, "unit": "frames/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if bf else "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: {d['L']}x{d['H']} BLSTM, D={d['D']}, T={T}, B={B}, P={d['P']}, V={d['V']}, "
                               f"step = forward + softmax-xent + backward + sgd_step + adpsgd_mix with one neighbour replica (update and average in one pass)",
                   "global_batch": B, "seq_len": T, "lr": w.lr},
        "step_ms": {"median": statistics.median(each), "min": min(each), "timed": "each step between two events on the launch stream"},
        "ms_per_step_two_call_form": two_call_ms,
        "flop_per_frame": fpf,
        "pct_of_mfma_peak": 100.0 * frames_per_s * fpf / peak,
        "final_loss": loss,
    }

    # ---- per-kernel-class durations: HIP events recorded by the library on the launch stream ----
    traffic = measured_traffic(w.name, B)
    if not args.no_profile:
        bl.blstm_profile_enable(lrn.ctx, 1)
        nprof = min(args.steps, 10)
        for _ in range(nprof):
            lrn.calgrad()
        torch.cuda.synchronize()
        prof = bl.blstm_profile_read(lrn.ctx)
        bl.blstm_profile_enable(lrn.ctx, 0)
        fl = flops_by_class(T, B, d["D"], d["H"], d["L"], d["P"], d["V"], softmax_wgrad_deferred=lrn.defer_softmax_wgrad)
        classes = {}
        for name, (ms, cnt) in prof.items():
            if cnt == 0:
                continue
            ent = {"ms_per_step": ms / nprof, "launches_per_step": cnt / nprof, "avg_launch_us": 1e3 * ms / cnt}
            if fl.get(name, 0) > 0:
                ent["tflops"] = fl[name] / (ms / nprof * 1e-3) / 1e12
            classes[name] = ent
        out["kernel_classes"] = classes

        def roofline_of(name):
            c = classes[name]
            flop_launch = fl[name] / c["launches_per_step"]
            achieved = flop_launch / (c["avg_launch_us"] * 1e-6) / 1e12
            return {"kernel": KERNEL_OF_CLASS.get(name, name), "class": name, "bound": "mfma", "achieved": achieved, "peak": peak / 1e12,
                    "unit": "TFLOP/s", "frac": achieved * 1e12 / peak, "traffic": traffic.get(name),
                    "flop_per_launch": flop_launch, "avg_launch_us": c["avg_launch_us"], "share_of_step": c["ms_per_step"] / ms_per_step}

        with_flop = {k: v for k, v in classes.items() if fl.get(k, 0) > 0}
        # time per kernel NAME: the product classes share one kernel function only nominally (different instantiations),
        # so the dominant kernel is looked for among the classes that are one kernel each
        single = {k: v for k, v in with_flop.items() if KERNEL_OF_CLASS.get(k) != "gemm_kernel"}
        if single:
            out["roofline"] = roofline_of(max(single, key=lambda k: single[k]["ms_per_step"]))
        gemm = {k: v for k, v in with_flop.items() if k.startswith("gemm_")}
        if gemm:
            out["roofline_gemm"] = roofline_of(max(gemm, key=lambda k: gemm[k]["ms_per_step"]))
        # the persistent recurrent kernels (latency chains): the slower of the two, whichever kernel leads the step
        rec = {k: v for k, v in with_flop.items() if k.startswith("recurrent_")}
        if rec:
            out["roofline_recurrent"] = roofline_of(max(rec, key=lambda k: rec[k]["ms_per_step"]))

    # ---- the averaging kernel on R replicas of this model, against HBM bandwidth ----------------
    R = args.mix_replicas
    if R >= 2 and R % 2 == 0:
        reps = [lrn.theta, nb_theta] + [torch.empty_like(lrn.theta).uniform_(-0.1, 0.1) for _ in range(R - 2)]
        shs = None
        if bf:
            shs = [lrn.shadow, nb_shadow] + [torch.empty_like(lrn.shadow) for _ in range(R - 2)]
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        for it in range(3):
            bl.adpsgd_mix(reps, shs, lrn.n, R, bl.adpsgd_ring_partner(R, it))
        nmix = 20
        ev[0].record()
        for it in range(nmix):
            bl.adpsgd_mix(reps, shs, lrn.n, R, bl.adpsgd_ring_partner(R, it))
        ev[1].record()
        torch.cuda.synchronize()
        mix_ms = ev[0].elapsed_time(ev[1]) / nmix
        bytes_per = R * lrn.n * (8 + (2 if bf else 0))
        gbs = bytes_per / (mix_ms * 1e-3) / 1e9
        pair_traffic = traffic.get("adpsgd_mix_pair")
        out["adpsgd_mix"] = {"kernel": "mix_kernel", "replicas": R, "params": lrn.n, "ms": mix_ms, "bound": "hbm", "achieved": gbs,
                             "peak": PEAK_HBM / 1e9, "unit": "GB/s", "frac": gbs * 1e9 / PEAK_HBM, "bytes_per_launch": bytes_per,
                             "traffic": pair_traffic * R / 2 if pair_traffic else None}
        # the same replicas through the R-way average of the synchronous strategy (Fig. 3a)
        for it in range(2):
            bl.sync_average(reps, shs, lrn.n, R)
        ev[0].record()
        for it in range(nmix):
            bl.sync_average(reps, shs, lrn.n, R)
        ev[1].record()
        torch.cuda.synchronize()
        sync_ms = ev[0].elapsed_time(ev[1]) / nmix
        out["sync_average"] = {"replicas": R, "ms": sync_ms, "bound": "hbm", "achieved": bytes_per / (sync_ms * 1e-3) / 1e9,
                               "peak": PEAK_HBM / 1e9, "unit": "GB/s", "frac": bytes_per / (sync_ms * 1e-3) / PEAK_HBM,
                               "bytes_per_launch": bytes_per}
        del reps, shs
    # Eq. 4 for the learner and its neighbour in one pass (update of both + average), against the two-call form
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    nb_grad = lrn.grad.clone()
    for it in range(3):
        bl.sgd_mix_pair(lrn.theta, nb_theta, lrn.shadow, nb_shadow, lrn.grad, nb_grad, lrn.n, 0.0)
    ev[0].record()
    for it in range(20):
        bl.sgd_mix_pair(lrn.theta, nb_theta, lrn.shadow, nb_shadow, lrn.grad, nb_grad, lrn.n, 0.0)
    ev[1].record()
    torch.cuda.synchronize()
    pair_ms = ev[0].elapsed_time(ev[1]) / 20
    pair_bytes = 2 * lrn.n * (12 + (2 if bf else 0))
    out["sgd_mix_pair"] = {"ms": pair_ms, "bound": "hbm", "achieved": pair_bytes / (pair_ms * 1e-3) / 1e9, "peak": PEAK_HBM / 1e9,
                           "unit": "GB/s", "frac": pair_bytes / (pair_ms * 1e-3) / PEAK_HBM, "bytes_per_launch": pair_bytes,
                           "note": "one pass for both replicas' sgd_step and their adpsgd_mix (lr = 0 here so the weights stay put)"}
    lrn.close()
    # ... and the one-sided form the step above uses (this learner's update + the average with the neighbour as it stands)
    for it in range(3):
        bl.sgd_mix_pair(lrn.theta, nb_theta, lrn.shadow, nb_shadow, lrn.grad, None, lrn.n, 0.0)
    ev[0].record()
    for it in range(20):
        bl.sgd_mix_pair(lrn.theta, nb_theta, lrn.shadow, nb_shadow, lrn.grad, None, lrn.n, 0.0)
    ev[1].record()
    torch.cuda.synchronize()
    one_ms = ev[0].elapsed_time(ev[1]) / 20
    one_bytes = lrn.n * (20 + (4 if bf else 0))
    out["sgd_mix_one_sided"] = {"ms": one_ms, "bound": "hbm", "achieved": one_bytes / (one_ms * 1e-3) / 1e9, "peak": PEAK_HBM / 1e9,
                                "unit": "GB/s", "frac": one_bytes / (one_ms * 1e-3) / PEAK_HBM, "bytes_per_launch": one_bytes,
                                "traffic": traffic.get("sgd_mix_one_sided"),
                                "note": "the update-and-average pass of the timed step (lr = 0 here)"}
    del lrn, nb_theta, nb_shadow, nb_grad, masters, shadows
    torch.cuda.empty_cache()

    # ---- the other workloads, briefly: the same step (forward .. adpsgd_mix with a neighbour), 3 warm-up + 8 timed steps ----
    if not args.no_other_workloads and args.workload == "paper4x512" and args.batch == 0:
        others = {}
        for name in ("largebatch", "wide6x1024", "paper6x512"):
            ow = inputs.WORKLOADS[name]
            od = ow.dims()
            ol = Learner(mode=ow.mode, **od)
            ol.set_theta(inputs.make_theta(ol.n, ow.seed, bf16=ow.mode == 1))
            ox, olab = inputs.make_batch(od["T"], od["B"], od["D"], od["V"], ow.seed, bf16=ow.mode == 1)
            ol.set_batch(ox, olab)
            onb, onbs = ol.theta.clone(), ol.shadow.clone()

            def ostep():
                ol.calgrad()
                bl.sgd_mix_pair(ol.theta, onb, ol.shadow, onbs, ol.grad, None, ol.n, ow.lr, ol.momentum, ol.velocity, None)
                ol.weights_changed()

            for _ in range(3):
                ostep()
            ol.check_status()
            t0 = time.perf_counter()
            for _ in range(8):
                ostep()
            torch.cuda.synchronize()
            odt = (time.perf_counter() - t0) / 8
            ol.check_status()
            ofpf = flop_per_frame(od["D"], od["H"], od["L"], od["P"], od["V"])
            others[name] = {"workload": f"{od['L']}x{od['H']} BLSTM, D={od['D']}, T={od['T']}, B={od['B']}, P={od['P']}, V={od['V']}",
                            "ms_per_step": 1e3 * odt, "frames_per_s": od["T"] * od["B"] / odt,
                            "pct_of_mfma_peak": 100.0 * od["T"] * od["B"] / odt * ofpf / PEAK_BF16_MFMA, "steps": 8, "warmup": 3,
                            "final_loss": ol.loss_value()}
            ol.close()
            del ol, onb, onbs
            torch.cuda.empty_cache()
        out["other_workloads"] = others

    # ---- the oracle on this machine's host cores: the same workload, whole batch, best of three steps ------------
    if not args.no_cpu_baseline:
        from oracle import blstm_oracle as orc
        try:
            from threadpoolctl import threadpool_info, threadpool_limits
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            threadpool_limits = None
            cores = os.cpu_count()

        def oracle_step(dm, th64, nb64, xx, ll, lr):
            _, g = orc.loss_and_grad(dm, th64, xx, ll)
            th64, _ = orc.sgd_step(th64, g, lr)
            return orc.adpsgd_mix([th64, nb64], [1, 0])

        dm = orc.Dims(**d)
        th64 = theta.astype(np.float64)
        nb64 = th64.copy()
        times = []
        budget0 = time.perf_counter()
        for _ in range(3):
            t0 = time.perf_counter()
            th64, nb64 = oracle_step(dm, th64, nb64, x, labels, w.lr)
            times.append(time.perf_counter() - t0)
            if time.perf_counter() - budget0 > 25.0:      # bounded: about half a minute at most
                break
        best = min(times)
        out["cpu_baseline"] = {"value": T * B / best, "unit": "frames/s", "cores": cores, "kind": "oracle",
                               "sample": f"best of {len(times)} whole steps (loss, gradient, SGD update, pair averaging) of the same "
                                         f"workload, all {B} sequences, float64 numpy, {best:.2f} s per step"}
        # one thread, the tiny workload (the case the oracle finishes in milliseconds)
        if threadpool_limits is not None:
            tw = inputs.WORKLOADS["tiny"]
            tdm = orc.Dims(**tw.dims())
            tth = inputs.make_theta(orc.param_count(tdm), tw.seed).astype(np.float64)
            tx, tl = inputs.make_batch(tw.T, tw.B, tw.D, tw.V, tw.seed)
            with threadpool_limits(limits=1):
                tt = []
                tnb = tth.copy()
                for _ in range(5):
                    t0 = time.perf_counter()
                    tth, tnb = oracle_step(tdm, tth, tnb, tx, tl, tw.lr)
                    tt.append(time.perf_counter() - t0)
            out["cpu_baseline"]["tiny_workload_one_thread"] = {"value": tw.T * tw.B / min(tt), "unit": "frames/s", "cores": 1,
                                                               "sample": f"best of 5 whole steps of the tiny workload, {min(tt) * 1e3:.1f} ms per step"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
