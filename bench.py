#!/usr/bin/env python3
"""Throughput of one AlexNet SGD training step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--batch 128] [--precision fp32|bf16]

A step is one pass of the whole hot path over one synthetic minibatch whose
stored uint8 pictures are already resident in HBM: on-device preprocessing
(mean subtract, random crop, flip) of minibatch k+1 on a side stream,
overlapped with forward + backward + momentum update of minibatch k on the
compute stream.  Prints ONE JSON line: images/s of the headline configuration
(fp32, batch 128), the MFMA roofline of its dominant kernel (measured with HIP
events on the stream the kernels run on), every bandwidth-bound kernel against
the HBM peak, the same step at batch 256 in fp32 and with bf16 products, each
convolution alone (forward, data gradient, weight gradient), the two-replica
exchange kernels, the loading thread, and the float64 oracle timed on the host
cores of the same machine.
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
PEAK_HBM_GBS = 8000.0
STEP_FLOPS_PER_IMAGE = 4.136e9  # 2 x multiply-adds of the definition: three passes of every layer, no conv1 data gradient
# Memory-side traffic of the GEMM launches, bytes per launch, as summarised from rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE runs of this very script by paper_1412_2302_amd/pmc_summary.py (scaled by a 1 GiB elementwise copy).
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "gemm_traffic.json")
# kernels that belong to the matrix path of a layer: the products themselves, the tile transforms around them,
# split-k reductions and the re-packing of weights
MATRIX_PATH = ("gemm", "gemm_bf16", "wino_in", "wino_out", "wino_dy", "wino_dx", "wino_filter", "wino_dw",
               "slab_finish", "reduce_slabs", "fc_finish", "run_repack", "phase_pack", "weight_transpose")


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


def _kernel_of(name: str) -> str:
    return name.rsplit(":", 1)[-1]


def _traffic(key: str):
    """Measured HBM bytes per GEMM launch for configuration `key`, if a counter summary of it is committed."""
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f).get(key)
    except (OSError, ValueError):
        rec = None
    if not rec:
        return None, "not measured: no rocprofv3 --pmc summary of this configuration under profiles/"
    return rec["bytes_per_launch"], rec.get("source", "profiles/gemm_traffic.json")


class Pipeline:
    """One replica fed from a small pool of stored minibatches resident in HBM; preprocessing of minibatch k+1
    on the side stream overlaps the training step of minibatch k on the compute stream."""

    def __init__(self, torch, B, S, batch, precision, overlap=True):
        self.torch, self.B, self.batch = torch, B, batch
        self.net = B.AlexNet(S.ALEXNET, batch, seed=S.SEED_BASE + 3, precision=precision)
        self.net.set_params(S.make_params(self.net.shapes, S.SEED_BASE + 3))
        self.pool = 4
        self.raws, self.labels = [], []
        for i in range(self.pool):
            r, l = S.make_raw_batch(batch, 3, 256, 256, 1000, S.SEED_BASE + 3 + i)
            self.raws.append(torch.from_numpy(r).cuda())
            self.labels.append(torch.from_numpy(l).cuda())
        self.mean = torch.from_numpy(S.make_mean_image(3, 256, 256, S.SEED_BASE + 7)).cuda()
        self.compute = torch.cuda.Stream()
        self.side = torch.cuda.Stream() if overlap else self.compute
        self.ready = [torch.cuda.Event(), torch.cuda.Event()]   # slot s holds a preprocessed batch
        self.freed = [torch.cuda.Event(), torch.cuda.Event()]   # the step reading slot s has finished
        torch.cuda.synchronize()

    def run(self, nsteps: int, first_step: int):
        """Enqueues nsteps pipelined steps; slot (k % 2) holds minibatch k."""
        net, side, compute, pool = self.net, self.side, self.compute, self.pool
        net.preprocess(self.raws[first_step % pool], self.mean, first_step, first_step % 2, stream=side)
        self.ready[first_step % 2].record(side)
        for k in range(first_step, first_step + nsteps):
            s = k % 2
            if k + 1 < first_step + nsteps:
                if k > first_step:  # the step that read slot 1-s must be done before it is overwritten
                    side.wait_event(self.freed[1 - s])
                net.preprocess(self.raws[(k + 1) % pool], self.mean, k + 1, 1 - s, stream=side)
                self.ready[1 - s].record(side)
            compute.wait_event(self.ready[s])
            net.train_step(self.labels[k % pool], k, slot=s, stream=compute)
            self.freed[s].record(compute)

    def close(self):
        self.net.close()


def measure(torch, B, S, batch, bf16, steps, warmup, overlap=True, keep=False):
    """Times `steps` pipelined training steps, then the same steps again under the library's event profiler.
    Returns (record, pipeline or None)."""
    pipe = Pipeline(torch, B, S, batch, 1 if bf16 else 0, overlap)
    net = pipe.net
    peak = PEAK_BF16_MFMA_TFLOPS if bf16 else PEAK_FP32_MFMA_TFLOPS
    pipe.run(warmup, 0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pipe.run(steps, warmup)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    net.check(stream=pipe.compute)
    loss = float(net.loss.cpu().item())
    ms_per_step = dt / steps * 1e3

    # ---- per-kernel durations with HIP events on the launch streams (same work, second pass) ----
    prof_steps = min(steps, 10)
    B.profile_begin()
    pipe.run(prof_steps, warmup + steps)
    torch.cuda.synchronize()
    entries = B.profile_end()
    gemm = [e for e in entries if _kernel_of(e["name"]) in ("gemm", "gemm_bf16")]
    gemm_ms = sum(e["total_ms"] for e in gemm)
    gemm_calls = sum(e["calls"] for e in gemm)
    gemm_flops = sum(e["flops"] for e in gemm)
    gemm_bytes = sum(e["bytes"] for e in gemm)
    matrix_ms = sum(e["total_ms"] for e in entries if _kernel_of(e["name"]) in MATRIX_PATH)
    all_ms = sum(e["total_ms"] for e in entries)
    achieved = gemm_flops / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
    step_flops = STEP_FLOPS_PER_IMAGE * batch
    key = f"{'bf16' if bf16 else 'fp32'}_b{batch}"
    traffic, traffic_source = _traffic(key)
    launches = gemm_calls // prof_steps
    roofline = {
        "kernel": ("ax::gemm_bf16_kernel (bf16 MFMA" if bf16 else "ax::gemm_kernel (fp32 MFMA")
                  + " implicit-GEMM: conv fwd/bwd-data/bwd-weight, the 36 products of the tile-transformed layers,"
                    " dense layers)",
        "bound": "mfma", "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s",
        "frac": round(achieved / peak, 4),
        "traffic": traffic, "traffic_source": traffic_source,
        # operand tensors read once + result written once, per launch, as the library's profiler counts them
        "algorithmic_bytes_per_launch": round(gemm_bytes / max(gemm_calls, 1)),
        "traffic_over_algorithmic": round(traffic / (gemm_bytes / max(gemm_calls, 1)), 3) if traffic else None,
        "launches_per_step": launches,
        # flops the launches execute for the layers: 2 x multiply-adds of the operation for the direct
        # convolutions and the dense layers, and the 36 channel products of the transformed layers
        # (2.6x fewer multiply-adds than their direct form)
        "flops_per_launch": gemm_flops / max(gemm_calls, 1),
        "avg_launch_ms": gemm_ms / max(gemm_calls, 1),
        "gemm_ms_per_step": round(gemm_ms / prof_steps, 4),
        # the step's flops by definition over everything the matrix path of the layers runs: products, tile
        # transforms, split-k reductions, weight re-packing (transformed layers do the work with fewer multiplies,
        # so this is the honest "by definition" rate: the transforms' time is in the denominator)
        "matrix_path_ms_per_step": round(matrix_ms / prof_steps, 4),
        "definition_tflops_over_matrix_path": round(step_flops * prof_steps / (matrix_ms * 1e-3) / 1e12, 2) if matrix_ms else None,
        "definition_frac_over_matrix_path": round(step_flops * prof_steps / (matrix_ms * 1e-3) / 1e12 / peak, 4) if matrix_ms else None,
        "note": "achieved/frac = flops the GEMM launches execute / their time (matrix-core utilisation)",
        "share_of_kernel_time": round(gemm_ms / all_ms, 4) if all_ms > 0 else None,
    }
    # ---- every bandwidth-bound kernel against the HBM peak (algorithmic bytes / launch time) ----
    by_kernel = {}
    for e in entries:
        if e["bytes"] <= 0 or _kernel_of(e["name"]) in ("gemm", "gemm_bf16"):
            continue
        k = by_kernel.setdefault(_kernel_of(e["name"]), {"calls": 0, "ms": 0.0, "bytes": 0.0})
        k["calls"] += e["calls"]; k["ms"] += e["total_ms"]; k["bytes"] += e["bytes"]
    hbm_rows = []
    for name, k in sorted(by_kernel.items(), key=lambda kv: -kv[1]["ms"]):
        gbs = k["bytes"] / (k["ms"] * 1e-3) / 1e9 if k["ms"] > 0 else 0.0
        hbm_rows.append({"kernel": name, "launches_per_step": round(k["calls"] / prof_steps, 2),
                         "mb_per_step": round(k["bytes"] / prof_steps / 1e6, 2),
                         "us_per_step": round(k["ms"] / prof_steps * 1e3, 1), "gbs": round(gbs, 1),
                         "frac": round(gbs / PEAK_HBM_GBS, 4)})
    bw_ms = sum(k["ms"] for k in by_kernel.values())
    hbm = {"peak": PEAK_HBM_GBS, "unit": "GB/s",
           "achieved": round(sum(k["bytes"] for k in by_kernel.values()) / (bw_ms * 1e-3) / 1e9, 1) if bw_ms else None,
           "ms_per_step": round(bw_ms / prof_steps, 4),
           "note": "algorithmic bytes (each tensor read or written once) / HIP-event time of the launches; "
                   "the update of the dense layers runs beside a convolution GEMM",
           "kernels": hbm_rows}
    table = []
    for e in sorted(entries, key=lambda e: -e["total_ms"]):
        ms = e["total_ms"] / e["calls"]
        row = {"name": e["name"], "calls_per_step": e["calls"] / prof_steps, "avg_ms": round(ms, 4)}
        if e["flops"] > 0:
            row["tflops"] = round(e["flops"] / e["calls"] / (ms * 1e-3) / 1e12, 2)
        elif e["bytes"] > 0:
            row["gbs"] = round(e["bytes"] / e["calls"] / (ms * 1e-3) / 1e9, 1)
        table.append(row)
    rec = {"value": round(batch * steps / dt, 1), "unit": "images/s", "ms_per_step": round(ms_per_step, 4),
           "steps": steps, "warmup": warmup, "batch": batch, "dtype": "bf16" if bf16 else "f32",
           "final_loss": round(loss, 5),
           "step_flops": step_flops,
           "step_mfma_frac": round(step_flops / (ms_per_step * 1e-3) / 1e12 / peak, 4),
           "roofline": roofline, "hbm_kernels": hbm, "kernels": table}
    if keep:
        return rec, pipe
    pipe.close()
    return rec, None


def conv_stack(torch, B, S, batch=128):
    """Workload 2: each convolution alone at batch 128 (channel-last tensors, packed weights: no layout
    conversion in the timed calls), forward, data gradient (conv1's too) and weight gradient.  The time of a
    pass is the sum of every kernel the call launches (tile transforms and split-k reductions included), the
    flops are 2 x multiply-adds of the definition."""
    net = B.AlexNet(S.ALEXNET, batch)
    out, total_ms, total_flops = [], 0.0, 0.0
    c, h = 3, 227
    for li, (cout, k, stride, pad, groups, _l, pool) in enumerate(S.ALEXNET["conv"], start=1):
        ho = (h + 2 * pad - k) // stride + 1
        flops = 2.0 * batch * ho * ho * cout * (c // groups) * k * k
        g = torch.Generator(device="cuda").manual_seed(S.SEED_BASE + 2 + li)
        x = torch.randn(batch * h * h * c, device="cuda", generator=g)
        dy = torch.randn(batch * ho * ho * cout, device="cuda", generator=g)
        w = torch.randn(cout, c // groups, k, k, device="cuda", generator=g) * 0.01
        wf, wb = net.pack_conv_weight(li, w)
        y, dx, dwf = torch.empty_like(dy), torch.empty_like(x), torch.empty_like(wf)
        db = torch.empty(cout, device="cuda")
        calls = {"fwd": lambda: net.conv_forward_nhwc(li, x, wf, None, False, y),
                 "bwd_data": lambda: net.conv_backward_data_nhwc(li, dy, wb, dx, wf=wf),
                 "bwd_weight": lambda: net.conv_backward_weight_nhwc(li, x, dy, dwf, db)}
        row = {"layer": f"conv{li}", "gflop_per_pass": round(flops / 1e9, 2)}
        for name, fn in calls.items():
            for _ in range(2):
                fn()
            torch.cuda.synchronize()
            reps = 5
            B.profile_begin()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            ent = B.profile_end()  # the weight-gradient call also sums the bias gradient
            ms = sum(e["total_ms"] for e in ent) / reps
            gemm_ms = sum(e["total_ms"] for e in ent if _kernel_of(e["name"]) == "gemm") / reps
            gemm_fl = sum(e["flops"] for e in ent if _kernel_of(e["name"]) == "gemm") / reps
            row[name] = {"ms": round(ms, 4), "tflops_by_definition": round(flops / (ms * 1e-3) / 1e12, 1),
                         "gemm_ms": round(gemm_ms, 4),
                         "gemm_tflops_executed": round(gemm_fl / (gemm_ms * 1e-3) / 1e12, 1) if gemm_ms else None}
            total_ms += ms
            total_flops += flops
        out.append(row)
        c, h = cout, ((ho - 3) // 2 + 1 if pool else ho)
    net.close()
    return {"batch": batch, "dtype": "f32", "layers": out, "total_ms": round(total_ms, 3),
            "total_gflop_by_definition": round(total_flops / 1e9, 1),
            "tflops_by_definition": round(total_flops / (total_ms * 1e-3) / 1e12, 1),
            "peak": PEAK_FP32_MFMA_TFLOPS,
            "note": "fwd + bwd-data + bwd-weight of conv1-5, each alone on N(0,1) tensors; conv2-5 run as F(4x4,3x3) "
                    "tile transforms around 36 products, so the rate by definition may pass the fp32 MFMA peak while "
                    "gemm_tflops_executed (what the matrix cores do) stays below it"}


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
    ap.add_argument("--no-extra-configs", action="store_true",
                    help="skip the batch-256 fp32 / bf16 steps and the convolutions alone")
    ap.add_argument("--only-step", action="store_true",
                    help="the timed steps and their kernel profile only (what a rocprofv3 run should see)")
    ap.add_argument("--only-conv-stack", action="store_true",
                    help="only the convolutions alone (workload 2), for a rocprofv3 run of that workload")
    ap.add_argument("--kernel-table", action="store_true", help="also print the per-kernel table to stderr")
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="also run three plain 1 GiB elementwise copies (under rocprofv3 --pmc they calibrate FETCH_SIZE / "
                         "WRITE_SIZE: each reads and writes exactly 2^30 bytes)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (two replicas share one GPU in its "
              "data-parallel test); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    if args.only_step:
        args.no_exchange = args.no_host_loader = args.no_extra_configs = args.no_cpu_baseline = True

    import numpy as np
    import torch
    import synthetic_inputs as S
    from paper_1412_2302_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP library has no CPU path", file=sys.stderr)
        sys.exit(1)

    wl, batch = S.ALEXNET, args.batch
    bf16 = args.precision == "bf16"

    if args.traffic_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)  # an elementwise kernel (copy_ would go through the DMA engines)
        torch.cuda.synchronize()
        del src, dst

    if args.only_conv_stack:
        print(json.dumps({"conv_stack": conv_stack(torch, B, S)}))
        return

    rec, pipe = measure(torch, B, S, batch, bf16, args.steps, args.warmup, overlap=not args.no_overlap, keep=True)
    net, compute, side, mean = pipe.net, pipe.compute, pipe.side, pipe.mean
    if args.kernel_table:
        for row in rec["kernels"]:
            print(json.dumps(row), file=sys.stderr)

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
            gbs = e["bytes"] / e["calls"] / (ms * 1e-3) / 1e9
            return {"avg_ms": round(ms, 4), "gbs": round(gbs, 1), "frac": round(gbs / PEAK_HBM_GBS, 4)}
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
        lsteps = max(args.steps, 40)  # a short run measures the pipeline filling, not its steady state
        for k in range(args.warmup + lsteps):
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
        host_loader = {"value": round(batch * lsteps / dt_l, 1), "unit": "images/s",
                       "ms_per_step": round(dt_l / lsteps * 1e3, 4), "steps": lsteps,
                       "vs_resident": round(batch * lsteps / dt_l / rec["value"], 4),
                       "note": f"{count} stored pictures in pageable host memory -> pinned staging (3 sets) -> "
                               "host-to-device copies on the side stream -> on-device preprocessing; "
                               "PCIe inclusive"}
        loader.close()
    pipe.close()
    del pipe, net
    torch.cuda.empty_cache()

    # ---- the other configurations, measured by the same code in the same run ----
    extra = {}
    if not args.no_extra_configs:
        sub_steps, sub_warm = min(args.steps, 10), min(args.warmup, 3)
        for name, (b2, bf2) in {"batch256_fp32": (256, False), "batch256_bf16": (256, True)}.items():
            if (b2, bf2) == (batch, bf16):
                continue
            r, _ = measure(torch, B, S, b2, bf2, sub_steps, sub_warm)
            r["kernels"] = r["kernels"][:8]
            extra[name] = r
            torch.cuda.empty_cache()
        extra["conv_stack"] = conv_stack(torch, B, S)

    out = {
        "metric": "AlexNet train images/sec at batch 128 on 1 MI355X; conv MFMA utilisation %",
        "value": rec["value"], "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": rec["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": rec["dtype"], "data": "synthetic",
        "config": {"workload": f"full AlexNet training step, {args.precision}, batch {batch}: uint8 3x256x256 pictures in HBM, "
                               "on-device mean-subtract/crop/flip on a side stream, conv1-5 + LRN + pools + fc6-8 "
                               "with dropout, softmax cross-entropy, momentum/weight-decay update",
                   "batch": batch, "overlap_preprocess": not args.no_overlap, "final_loss": rec["final_loss"]},
        "mfma_utilisation_pct": round(100 * rec["roofline"]["frac"], 2),
        "step_flops": rec["step_flops"],
        "step_mfma_frac": rec["step_mfma_frac"],
        "roofline": rec["roofline"],
        "hbm_kernels": rec["hbm_kernels"],
        "exchange": exchange,
        "host_loader": host_loader,
        "kernels": rec["kernels"][:12],
    }
    out.update(extra)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.cpu_sample)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
