#!/usr/bin/env python3
"""Throughput of one AlexNet SGD training step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--batch 128] [--no-cpu-baseline]

A step is one pass of the whole hot path over one synthetic minibatch whose
stored uint8 pictures are already resident in HBM: on-device preprocessing
(mean subtract, random crop, flip) of minibatch k+1 on a side stream,
overlapped with forward + backward + momentum update of minibatch k on the
compute stream.  Prints ONE JSON line: images/s, the MFMA roofline of the
dominant kernel (measured with HIP events on the stream the kernels run on) and
the float64 oracle timed on the host cores of the same machine.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

PEAK_FP32_MFMA_TFLOPS = 157.3  # MI355X dense fp32 matrix peak: 256 CU x 256 flop/clk x 2.4 GHz
PEAK_BF16_MFMA_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak
# Memory-side traffic of the GEMM launches of one fp32 batch-128 step, bytes per launch (23 launches):
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE scaled by a 1 GiB elementwise copy, from
# profiles/train_step_alexnet_b128_fp32_counters.txt.  Not measured for other configurations.
GEMM_TRAFFIC_FP32_B128 = 329756789
PEAK_HBM_GBS = 8000.0


def cpu_baseline(sample_batch: int):
    """The float64 oracle, as it stands, on the host cores: one full training
    step (preprocess + forward + backward + update) on `sample_batch` pictures."""
    import numpy as np
    import synthetic_inputs as S
    from helpers import oracle_spec, to64
    from oracle import alexnet_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    spec = oracle_spec(S.ALEXNET, sample_batch, seed=S.SEED_BASE + 3)
    params = to64(S.make_params(O.param_shapes(spec), S.SEED_BASE + 3))
    mom = {k: np.zeros_like(v) for k, v in params.items()}
    raw, labels = S.make_raw_batch(sample_batch, 3, 256, 256, 1000, S.SEED_BASE + 3)
    mean = S.make_mean_image(3, 256, 256, S.SEED_BASE + 7)
    t0 = time.perf_counter()
    ox, oy, fl = O.crop_flip_params(spec, 0)
    x = O.preprocess(raw, mean, ox, oy, fl, 227, 227)
    O.train_step(spec, params, mom, x, labels, 0)
    dt = time.perf_counter() - t0
    return {"value": sample_batch / dt, "unit": "images/s", "cores": threads, "kind": "oracle",
            "sample": f"one float64 numpy training step (preprocess+fwd+bwd+update) on {sample_batch} images, {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=128)
    ap.add_argument("--precision", choices=["fp32", "bf16"], default="fp32",
                    help="arithmetic of the matrix products (bf16: operands rounded, fp32 accumulation)")
    ap.add_argument("--cpu-sample", type=int, default=256)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-overlap", action="store_true", help="run preprocessing on the compute stream")
    ap.add_argument("--no-exchange", action="store_true", help="skip timing the two-replica exchange kernels")
    ap.add_argument("--no-host-loader", action="store_true",
                    help="skip the run fed from host memory through the loading thread (reported beside `value`)")
    ap.add_argument("--kernel-table", action="store_true", help="also print the per-kernel table to stderr")
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="also run three plain 1 GiB elementwise copies (under rocprofv3 --pmc they calibrate FETCH_SIZE / "
                         "WRITE_SIZE: each reads and writes exactly 2^30 bytes)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (two replicas share one GPU in its "
              "data-parallel test); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synthetic_inputs as S
    from paper_1412_2302_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP library has no CPU path", file=sys.stderr)
        sys.exit(1)

    wl, batch = S.ALEXNET, args.batch
    bf16 = args.precision == "bf16"
    peak = PEAK_BF16_MFMA_TFLOPS if bf16 else PEAK_FP32_MFMA_TFLOPS
    net = B.AlexNet(wl, batch, seed=S.SEED_BASE + 3, precision=1 if bf16 else 0)
    net.set_params(S.make_params(net.shapes, S.SEED_BASE + 3))
    # a small pool of distinct minibatches resident in HBM, cycled through
    pool = 4
    raws, labels = [], []
    for i in range(pool):
        r, l = S.make_raw_batch(batch, 3, 256, 256, 1000, S.SEED_BASE + 3 + i)
        raws.append(torch.from_numpy(r).cuda())
        labels.append(torch.from_numpy(l).cuda())
    mean = torch.from_numpy(S.make_mean_image(3, 256, 256, S.SEED_BASE + 7)).cuda()

    compute = torch.cuda.Stream()
    side = compute if args.no_overlap else torch.cuda.Stream()
    ready = [torch.cuda.Event(), torch.cuda.Event()]   # slot s holds a preprocessed batch
    freed = [torch.cuda.Event(), torch.cuda.Event()]   # the step reading slot s has finished
    torch.cuda.synchronize()

    def run(nsteps: int, first_step: int):
        """Enqueues nsteps pipelined steps; slot (k % 2) holds minibatch k."""
        with torch.cuda.stream(side):
            net.preprocess(raws[first_step % pool], mean, first_step, first_step % 2, stream=side)
            ready[first_step % 2].record(side)
        for k in range(first_step, first_step + nsteps):
            s = k % 2
            if k + 1 < first_step + nsteps:
                if k > first_step:  # the step that read slot 1-s must be done before it is overwritten
                    side.wait_event(freed[1 - s])
                net.preprocess(raws[(k + 1) % pool], mean, k + 1, 1 - s, stream=side)
                ready[1 - s].record(side)
            compute.wait_event(ready[s])
            net.train_step(labels[k % pool], k, slot=s, stream=compute)
            freed[s].record(compute)

    if args.traffic_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)  # an elementwise kernel (copy_ would go through the DMA engines)
        torch.cuda.synchronize()
        del src, dst

    run(args.warmup, 0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps, args.warmup)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    net.check(stream=compute)
    loss = float(net.loss.cpu().item())
    ms_per_step = dt / args.steps * 1e3
    value = batch * args.steps / dt

    # ---- per-kernel durations with HIP events on the launch streams (same work, second pass) ----
    prof_steps = min(args.steps, 10)
    B.profile_begin()
    run(prof_steps, args.warmup + args.steps)
    torch.cuda.synchronize()
    entries = B.profile_end()
    gemm = [e for e in entries if ":gemm" in e["name"]]
    other = [e for e in entries if ":gemm" not in e["name"]]
    gemm_ms = sum(e["total_ms"] for e in gemm)
    gemm_calls = sum(e["calls"] for e in gemm)
    gemm_flops = sum(e["flops"] for e in gemm)
    all_ms = sum(e["total_ms"] for e in entries)
    achieved = gemm_flops / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
    roofline = {
        "kernel": ("ax::gemm_bf16_kernel (bf16 MFMA" if bf16 else "ax::gemm_kernel (fp32 MFMA")
                  + " implicit-GEMM: conv fwd/bwd-data/bwd-weight and dense layers)",
        "bound": "mfma", "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s",
        "frac": round(achieved / peak, 4),
        "traffic": GEMM_TRAFFIC_FP32_B128 if (not bf16 and batch == 128) else None,
        "launches_per_step": gemm_calls // prof_steps,
        # flops the launches execute for the layers: 2 x multiply-adds of the operation for the direct
        # convolutions and the dense layers, and the 36 channel products of the transformed 3x3 layers
        # (2.6x fewer multiply-adds than their direct form, so this is below the step's 4.136 GFLOP/image)
        "flops_per_launch": gemm_flops / max(gemm_calls, 1),
        "flops_by_definition_per_launch": 4.136e9 * batch / max(gemm_calls // prof_steps, 1),
        # the same launch time against the direct-form count of the layers (2 x multiply-adds of the definition):
        # above the peak where the transformed layers do the work with fewer multiplies
        "achieved_by_definition": round(4.136e9 * batch * prof_steps / (gemm_ms * 1e-3) / 1e12, 2) if gemm_ms > 0 else None,
        "frac_by_definition": round(4.136e9 * batch * prof_steps / (gemm_ms * 1e-3) / 1e12 / peak, 4) if gemm_ms > 0 else None,
        "note": "achieved/frac count the flops the launches execute (matrix-core utilisation); the 3x3 and 5x5 layers "
                "run as 36 products of F(4x4,3x3)-transformed tiles with 2.6x fewer multiplies than their definition",
        "avg_launch_ms": gemm_ms / max(gemm_calls, 1),
        "share_of_kernel_time": round(gemm_ms / all_ms, 4) if all_ms > 0 else None,
    }
    table = []
    for e in sorted(entries, key=lambda e: -e["total_ms"]):
        ms = e["total_ms"] / e["calls"]
        row = {"name": e["name"], "calls_per_step": e["calls"] / prof_steps, "avg_ms": round(ms, 4)}
        if e["flops"] > 0:
            row["tflops"] = round(e["flops"] / e["calls"] / (ms * 1e-3) / 1e12, 2)
        if e["bytes"] > 0:
            row["gbs"] = round(e["bytes"] / e["calls"] / (ms * 1e-3) / 1e9, 1)
        table.append(row)
    if args.kernel_table:
        for row in table:
            print(json.dumps(row), file=sys.stderr)
    bw = [e for e in other if e["bytes"] > 0]
    bw_ms = sum(e["total_ms"] for e in bw)
    hbm = {"achieved": round(sum(e["bytes"] for e in bw) / (bw_ms * 1e-3) / 1e9, 1) if bw_ms > 0 else None,
           "peak": PEAK_HBM_GBS, "unit": "GB/s", "ms_per_step": round(bw_ms / prof_steps, 4),
           "note": "all bandwidth-bound kernels together (LRN, pool, update, reductions, preprocess)"}

    # ---- the two-replica exchange kernels alone (bandwidth-bound; not part of `value`) ----
    exchange = None
    if not args.no_exchange:
        peer = B.AlexNet(wl, batch, seed=S.SEED_BASE + 4, precision=1 if bf16 else 0)
        peer.set_params(S.make_params(peer.shapes, S.SEED_BASE + 3))
        torch.cuda.synchronize()
        B.profile_begin()
        for _ in range(10):
            B.average_replicas(net, peer, stream=compute)
        for _ in range(10):
            B.average_gradients_update(net, peer, stream=compute)
        torch.cuda.synchronize()
        ex = {e["name"]: e for e in B.profile_end()}
        def _rate(name):
            e = ex[name]
            ms = e["total_ms"] / e["calls"]
            return {"avg_ms": round(ms, 4), "gbs": round(e["bytes"] / e["calls"] / (ms * 1e-3) / 1e9, 1)}
        exchange = {"average_replicas": _rate("average"), "average_gradients_update": _rate("avg_grad_update"),
                    "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "note": "average_replicas = two launches (parameters, momentum), 16 B/param each; the "
                            "gradient-exchange update is one launch of 40 B/param and replaces two updates + the average"}
        peer.close()

    # ---- the same steps fed from host memory by the loading thread (PCIe inclusive; never `value`) ----
    host_loader = None
    if not args.no_host_loader:
        count = 4 * batch
        himg = torch.from_numpy(np.concatenate([S.make_raw_batch(batch, 3, 256, 256, 1000, S.SEED_BASE + 3 + i)[0]
                                                for i in range(4)]))
        hlab = torch.from_numpy(np.concatenate([S.make_raw_batch(batch, 3, 256, 256, 1000, S.SEED_BASE + 3 + i)[1]
                                                for i in range(4)]))
        loader = B.Loader(net, himg, hlab, depth=3, copy_stream=side)
        torch.cuda.synchronize()

        lab = loader.stage(0, mean, side, compute)
        t1 = 0.0
        for k in range(args.warmup + args.steps):
            if k == args.warmup:
                torch.cuda.synchronize()
                t1 = time.perf_counter()
            nxt = loader.stage(k + 1, mean, side, compute)  # one more is staged than trained: harmless
            net.train_step(lab, k, slot=k % 2, stream=compute)
            loader.done(k, compute)
            lab = nxt
        torch.cuda.synchronize()
        dt_l = time.perf_counter() - t1
        net.check(stream=compute)
        host_loader = {"value": round(batch * args.steps / dt_l, 1), "unit": "images/s",
                       "ms_per_step": round(dt_l / args.steps * 1e3, 4),
                       "note": f"{count} stored pictures in pageable host memory -> pinned staging (3 sets) -> "
                               "host-to-device copies on the side stream -> on-device preprocessing; "
                               "PCIe inclusive"}
        loader.close()

    out = {
        "metric": "AlexNet train images/sec at batch 128 on 1 MI355X; conv MFMA utilisation %",
        "value": round(value, 1), "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": f"full AlexNet training step, {args.precision}, batch {batch}: uint8 3x256x256 pictures in HBM, "
                               "on-device mean-subtract/crop/flip on a side stream, conv1-5 + LRN + pools + fc6-8 "
                               "with dropout, softmax cross-entropy, momentum/weight-decay update",
                   "batch": batch, "overlap_preprocess": not args.no_overlap, "final_loss": round(loss, 5)},
        "mfma_utilisation_pct": round(100 * achieved / peak, 2),
        "step_flops": 4.136e9 * batch,
        "step_mfma_frac": round(4.136e9 * batch / (ms_per_step * 1e-3) / 1e12 / peak, 4),
        "roofline": roofline,
        "hbm_kernels": hbm,
        "exchange": exchange,
        "host_loader": host_loader,
        "kernels": table[:12],
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.cpu_sample)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
