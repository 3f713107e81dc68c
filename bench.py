#!/usr/bin/env python3
"""Benchmark of one learner's training step on one MI355X.

A step is one pass of the whole hot path over one synthetic batch: blstm_forward,
softmax_xent_fwd_bwd, blstm_backward, sgd_step and one adpsgd_mix with a ring neighbour's
replica held in the same HBM.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line: frames/s of the whole job, the roofline of the kernel class that
takes the most time (HIP events on the launch stream, recorded inside the library), and the
float64 oracle timed on this machine's host cores on a bounded sample of the same workload.
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

PEAK_BF16_MFMA = 2.5e15      # FLOP/s, dense
PEAK_FP32_MFMA = 157.3e12
PEAK_HBM = 8.0e12            # B/s

# HBM bytes per launch (fetch + write) of kernel classes, from rocprofv3 --pmc runs of this script
# (FETCH_SIZE and WRITE_SIZE, each scaled by its reading for the 1 GiB copy of --traffic-calibration);
# the runs and figures are in profiles/hbm_traffic_paper4x512.txt.  Keyed by (workload, batch, class).
MEASURED_HBM_BYTES_PER_LAUNCH = {
    ("paper4x512", 256, "recurrent_bwd_persistent"): (2 * 74703.8 + 129024.0) * 1024,
    ("paper4x512", 256, "recurrent_fwd_persistent"): (2 * 64671.3 + 86016.1) * 1024,
    ("paper4x512", 256, "gemm_logits"): (2 * 51944.5 + 336000.0) * 1024,
    # nine launches per step: dW_x of layers 0-3 and dW_p (one kernel name, five launches), four dU_h
    ("paper4x512", 256, "gemm_wgrad"): (2 * (5 * 75956.3 + 4 * 92284.0) + (5 * 13228.6 + 4 * 16384.0)) * 1024 / 9,
}
MEASURED_MIX_BYTES_PER_PAIR = {"paper4x512": (2 * 119318.0 + 357967.2) * 1024}   # one launch on two replicas


def flops_by_class(T, B, D, H, L, P, V):
    """Algorithmic FLOP of one step per kernel class (2 FLOP per multiply-add), and launches."""
    M = T * B
    Z = P if P > 0 else 2 * H
    din = [D] + [2 * H] * (L - 1)
    f = {}
    f["gemm_input_projection"] = (sum(2 * M * 8 * H * d for d in din), L)
    f["gemm_recurrent_fwd"] = (L * (T - 1) * 2 * (2 * B * 4 * H * H), L * (T - 1))
    f["gemm_bottleneck"] = (2 * M * 2 * H * P, 1 if P > 0 else 0)
    f["gemm_logits"] = (2 * M * V * Z, 1)
    f["gemm_softmax_bwd"] = (2 * 2 * M * V * Z, 2)
    f["gemm_recurrent_bwd"] = (L * (T - 1) * 2 * (2 * B * 4 * H * H), L * (T - 1))
    # the persistent kernels do a whole layer (both directions, all frames) per launch
    f["recurrent_fwd_persistent"] = (f["gemm_recurrent_fwd"][0], L)
    f["recurrent_bwd_persistent"] = (f["gemm_recurrent_bwd"][0], L)
    f["gemm_wgrad"] = (sum(2 * M * 8 * H * d for d in din) + L * 2 * (T - 1) * B * 8 * H * H + 2 * M * P * 2 * H,
                       2 * L + (1 if P > 0 else 0))
    f["gemm_dgrad"] = (sum(2 * M * 8 * H * d for d in din[1:]) + 2 * M * 2 * H * P, L - 1 + (1 if P > 0 else 0))
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
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="first copy 1 GiB three times with a plain copy kernel (reference for HBM counters under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (one learner per GPU, no collectives); use --gpus 1")

    import numpy as np
    import torch
    from paper_1904_04956_amd import binding as bl
    from paper_1904_04956_amd import inputs
    from paper_1904_04956_amd.harness import Learner, mix

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
        lrn.apply(w.lr)
        bl.adpsgd_mix(masters, shadows, lrn.n, 2, [1, 0])
        lrn.weights_changed()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = 1e3 * dt / args.steps
    frames_per_s = T * B * args.steps / dt
    lrn.check_status()
    loss = lrn.loss_value()
    fpf = flop_per_frame(d["D"], d["H"], d["L"], d["P"], d["V"])
    peak = PEAK_BF16_MFMA if bf else PEAK_FP32_MFMA

    out = {
        "metric": "training frames/sec (fwd+bwd+update) on 1 MI355X",
        "value": frames_per_s, "unit": "frames/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf else "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: {d['L']}x{d['H']} BLSTM, D={d['D']}, T={T}, B={B}, P={d['P']}, V={d['V']}, "
                               f"step = forward + softmax-xent + backward + sgd_step + adpsgd_mix with one neighbour replica",
                   "global_batch": B, "seq_len": T, "lr": w.lr},
        "flop_per_frame": fpf,
        "pct_of_mfma_peak": 100.0 * frames_per_s * fpf / peak,
        "final_loss": loss,
    }

    # ---- per-kernel-class durations: HIP events recorded by the library on the launch stream ----
    # (everything on one stream for this pass: events around a launch that shares the device with the
    #  second stream's products would time the sharing, not the kernel)
    if not args.no_profile:
        bl.blstm_profile_enable(lrn.ctx, 1)
        nprof = min(args.steps, 10)
        for _ in range(nprof):
            lrn.calgrad()
        torch.cuda.synchronize()
        prof = bl.blstm_profile_read(lrn.ctx)
        bl.blstm_profile_enable(lrn.ctx, 0)
        fl = flops_by_class(T, B, d["D"], d["H"], d["L"], d["P"], d["V"])
        classes = {}
        for name, (ms, cnt) in prof.items():
            if cnt == 0:
                continue
            ent = {"ms_per_step": ms / nprof, "launches_per_step": cnt / nprof, "avg_launch_us": 1e3 * ms / cnt}
            if name in fl and fl[name][0] > 0:
                ent["tflops"] = fl[name][0] / (ms / nprof * 1e-3) / 1e12
            classes[name] = ent
        out["kernel_classes"] = classes
        def roofline_of(name):
            launches = classes[name]["launches_per_step"]
            flop_launch = fl[name][0] / launches
            achieved = flop_launch / (classes[name]["avg_launch_us"] * 1e-6) / 1e12
            key = (w.name, B, name)
            return {"kernel": name, "bound": "mfma", "achieved": achieved, "peak": peak / 1e12, "unit": "TFLOP/s",
                    "frac": achieved * 1e12 / peak, "traffic": MEASURED_HBM_BYTES_PER_LAUNCH.get(key),
                    "flop_per_launch": flop_launch, "avg_launch_us": classes[name]["avg_launch_us"]}

        with_flop = {k: v for k, v in classes.items() if k in fl and fl[k][0] > 0}
        if with_flop:
            # the class that takes the most time, and the plain product class that takes the most time
            out["roofline"] = roofline_of(max(with_flop, key=lambda k: with_flop[k]["ms_per_step"]))
            gemm = {k: v for k, v in with_flop.items() if k.startswith("gemm_")}
            if gemm:
                out["roofline_gemm"] = roofline_of(max(gemm, key=lambda k: gemm[k]["ms_per_step"]))

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
        out["adpsgd_mix"] = {"replicas": R, "params": lrn.n, "ms": mix_ms, "bound": "hbm", "achieved": gbs,
                             "peak": PEAK_HBM / 1e9, "unit": "GB/s", "frac": gbs * 1e9 / PEAK_HBM,
                             "bytes_per_launch": bytes_per,
                             "traffic": (MEASURED_MIX_BYTES_PER_PAIR[w.name] * R / 2
                                         if w.name in MEASURED_MIX_BYTES_PER_PAIR and B == w.dims()["B"] else None)}
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

    # ---- the oracle on this machine's host cores, on a bounded sample of the same workload ------
    if not args.no_cpu_baseline:
        from oracle import blstm_oracle as orc
        Bs = min(B, 64)
        dd = dict(d); dd["B"] = Bs
        dm = orc.Dims(**dd)
        th64 = theta.astype(np.float64)
        nb64 = th64.copy()
        nsteps, cdt = 0, 0.0
        t0 = time.perf_counter()
        while nsteps < 2 or (cdt < 12.0 and nsteps < 50):     # about 12 s of oracle steps on the sample
            _, g = orc.loss_and_grad(dm, th64, x[:, :Bs], labels[:, :Bs])
            th64, _ = orc.sgd_step(th64, g, w.lr)
            th64, nb64 = orc.adpsgd_mix([th64, nb64], [1, 0])
            nsteps += 1
            cdt = time.perf_counter() - t0
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()
        out["cpu_baseline"] = {"value": T * Bs * nsteps / cdt, "unit": "frames/s", "cores": cores, "kind": "oracle",
                               "sample": f"{nsteps} steps (loss, gradient, SGD update, pair averaging) of the same model on the "
                                         f"first {Bs} of {B} sequences, float64 numpy, {cdt:.1f} s"}
    lrn.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
