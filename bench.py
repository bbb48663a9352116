#!/usr/bin/env python3
"""Benchmark of the layer-quantization hot path on one MI355X.

A "step" is one pass of the whole path over one layer whose inputs are already
in HBM: Hessian accumulation (X X^T), damping, Cholesky + inverse, grid,
column scores + order, permutation, shared-Hinv elimination, column loop, emit.
The default workload is the ResNet-50-shaped 3x3 convolution 256->256
(W 256 x 2304, X 2304 x 25088, 4-bit per-row grids, 1 % damping).

Prints ONE JSON line (see the keys below).  `roofline` is for the kernel that
dominates the step (the fp64 MFMA X X^T kernel), timed live with HIP events on
the library's stream; `cpu_baseline` is the fp64 CPU oracle timed on this
machine's host cores.
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

PEAK_FP64_MFMA_TFLOPS = 78.6   # MI355X dense fp64 matrix peak
PEAK_HBM_GBS = 8000.0
PEAK_INT8_MFMA_TOPS = 5000.0    # MI355X dense int8 matrix peak (5.0 POP/s)


def _blob_hash(path: str) -> str:
    """git's blob hash of a file's current contents."""
    import hashlib
    data = open(path, "rb").read()
    return hashlib.sha1(b"blob %d\0" % len(data) + data).hexdigest()


def measured_traffic(kernel: str, workload: str):
    """HBM bytes per launch of `kernel` on `workload` from the counter runs recorded in profiles/traffic.json
    (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, each scaled by what the same counter reads for a plain device
    copy of known size).  None when no record exists or when the kernel's source file has changed since the
    counters were read (the record carries the file's git blob hash)."""
    try:
        records = json.load(open(os.path.join(ROOT, "profiles", "traffic.json")))["records"]
    except (OSError, ValueError, KeyError):
        return None
    for r in records:
        if r.get("kernel") == kernel and r.get("workload") == workload:
            try:
                if _blob_hash(os.path.join(ROOT, r["source"])) == r["source_blob"]:
                    return float(r["bytes_per_launch"])
            except OSError:
                pass
    return None


def _median(v):
    v = sorted(v)
    n = len(v)
    return v[n // 2] if n % 2 else 0.5 * (v[n // 2 - 1] + v[n // 2])


def sweep(model: str, steps: int, warmup: int, concurrency: int, iid: bool, int8: bool, batch_small: bool) -> int:
    """Whole-model sweep: every layer of a ResNet-50- or YOLOv5s-shaped network (4-bit, per-row grids,
    128 images), each layer fed as the network would feed it: a k x k or strided convolution accumulates
    its Hessian straight from its seeded ReLU-Gaussian input maps (fobq_hessian_accumulate_conv, a bounded
    number of images per call), a 1 x 1 convolution of stride 1 and the classifier from X (d_col x N).
    Weights and inputs come from the seeded counter-based generator of workloads.py, evaluated on the
    device; everything is resident in HBM before anything is timed.  `iid` = the earlier variant that feeds
    every layer an unfolded matrix of independent activations (no spatial correlation between taps).

    Two measurements, each the MEDIAN over `steps` whole-model runs after `warmup`: (1) one layer after the
    other on one context (`sequential_ms`); (2) up to `concurrency` layers in flight on as many contexts /
    streams (layers are independent of each other; most of a layer is a chain of short dependent launches
    that leaves the GPU nearly idle, so layers overlap): `ms_per_step`, the whole-model time.
    After the timed region every layer is run once more and checked on the device: `perm` is a permutation,
    Q = scale * (code - zero), codes within the grid, and the loss the path reports equals
    1/2 tr(dW H_d dW^T) evaluated from the path's own Hessian; a miss fails the run."""
    import torch

    import paper_2509_05576_amd as fobq
    import workloads

    fobq.load_library()
    layers = workloads.sweep_layers(model)
    pad_budget = 1 << 28                           # floats in the padded copy of one accumulate_conv call (1 GiB)
    chunk_elems = 1 << 28                          # elements of X per accumulate call (1 GiB)
    Ws, Ins, per_call = [], [], []
    for spec in layers:
        Ws.append(spec.make_w_device())
        if iid or spec.conv is None:
            Ins.append(workloads.device_normal_f32((spec.d_col, spec.n), 1.0, spec.seed,
                                                   workloads.STREAM_ACT + 16 * spec.layer_index, relu=True))
            per_call.append(max(32, (chunk_elems // spec.d_col) // 32 * 32))
        else:
            Ins.append(spec.make_input_device())
            images, side, ch, k, pad = spec.conv
            per_img = (side + 2 * pad) ** 2 * ch
            per_call.append(max(1, min(images, pad_budget // per_img - 1)))
    torch.cuda.synchronize()
    total_weights = sum(spec.weights for spec in layers)
    input_bytes = sum(int(t.numel()) * 4 for t in Ins)

    def hessian(ctx, spec, inp, pc, H_out=None):
        if inp.dim() == 4:
            ctx.hessian_conv(inp, spec.conv[3], spec.stride, spec.conv[4], images_per_call=pc, H_out=H_out)
        else:
            ctx.hessian(inp, chunk=pc, H_out=H_out)

    # layers of up to 256 columns go through fobq_quantize_layers_batched, all of them in one call: their
    # Hessians are accumulated one by one into buffers of their own, then every stage of the path is one launch
    # for the whole batch
    small = [i for i, spec in enumerate(layers) if batch_small and spec.d_col <= 256]
    big = [i for i in range(len(layers)) if i not in set(small)]
    Hs = {i: torch.empty((layers[i].d_col, layers[i].d_col), dtype=torch.float64, device="cuda") for i in small}
    outs = [None] * len(layers)
    batch_outs = None

    def run_small_batch(ctx):
        nonlocal batch_outs
        if small:
            batch_outs = ctx.quantize_layers_batched([Ws[i] for i in small], [Hs[i] for i in small], bits=layers[small[0]].bits,
                                                     group=0, damp=layers[small[0]].damp, outs=batch_outs)
            for i, o in zip(small, batch_outs):
                outs[i] = o

    hmode = fobq.HESSIAN_INT8_SLICES if int8 else fobq.HESSIAN_FP64
    # (1) one layer at a time; per-layer time = median over the runs (a batched layer: its Hessian's time plus
    # its share of the batched call)
    ctx = fobq.Ctx(0)
    ctx.set_hessian_mode(hmode)
    layer_ms = [[] for _ in layers]
    seq_runs, batch_ms = [], []
    for it in range(warmup + steps):
        torch.cuda.synchronize()
        t_run = time.perf_counter()
        for i, (spec, W, inp, pc) in enumerate(zip(layers, Ws, Ins, per_call)):
            t0 = time.perf_counter()
            if i in Hs:
                hessian(ctx, spec, inp, pc, H_out=Hs[i])
            else:
                hessian(ctx, spec, inp, pc)
                outs[i] = ctx.quantize_layer(W, bits=spec.bits, group=spec.group, damp=spec.damp, out=outs[i])
            torch.cuda.synchronize()
            if it >= warmup:
                layer_ms[i].append((time.perf_counter() - t0) * 1e3)
        t0 = time.perf_counter()
        run_small_batch(ctx)
        torch.cuda.synchronize()
        if it >= warmup:
            batch_ms.append((time.perf_counter() - t0) * 1e3)
            seq_runs.append((time.perf_counter() - t_run) * 1e3)
    workspace_seq = ctx.workspace_bytes()
    share = _median(batch_ms) / len(small) if small else 0.0
    per_layer = [{"layer": spec.name, "d_row": spec.d_row, "d_col": spec.d_col, "n": spec.n,
                  "input": "maps" if inp.dim() == 4 else "X", "batched": i in Hs,
                  "ms": round(_median(ms) + (share if i in Hs else 0.0), 3)}
                 for i, (spec, inp, ms) in enumerate(zip(layers, Ins, layer_ms))]

    # validity of every layer, on the device, from the path's own Hessian
    checked = 0
    for i, (spec, W, inp, pc) in enumerate(zip(layers, Ws, Ins, per_call)):
        d = spec.d_col
        if i in Hs:
            H, o = Hs[i], outs[i]            # the batched call's own inputs and outputs
        else:
            H = torch.empty((d, d), dtype=torch.float64, device="cuda")
            hessian(ctx, spec, inp, pc, H_out=H)
            o = ctx.quantize_layer(W, bits=spec.bits, group=spec.group, damp=spec.damp, out=outs[i])
        torch.cuda.synchronize()
        perm = o.perm.long()
        ok_perm = bool(torch.equal(torch.sort(perm).values, torch.arange(d, device="cuda")))
        codes = o.codes.to(torch.float64)
        Q = o.Q.to(torch.float64)
        sc, ze = o.scales.to(torch.float64), o.zeros.to(torch.float64)
        ok_q = bool(torch.allclose(Q, sc * (codes - ze), rtol=1e-6, atol=1e-12)) and int(o.codes.max()) <= 2 ** spec.bits - 1
        lam = spec.damp * float(torch.diagonal(H).mean())
        dW = W.to(torch.float64) - Q
        expect = 0.5 * float(((dW @ H) * dW).sum()) + 0.5 * lam * float((dW * dW).sum())
        got = float(o.loss[0])
        ok_loss = abs(got - expect) <= 1e-6 * abs(expect)
        if not (ok_perm and ok_q and ok_loss):
            print(f"bench.py: sweep check failed on {spec.name}: perm {ok_perm}, Q {ok_q}, loss {got} vs {expect}",
                  file=sys.stderr)
            return 1
        checked += 1
    ctx.close()

    # (2) the whole model, several layers in flight
    K = max(1, concurrency)
    streams = [torch.cuda.Stream() for _ in range(K)]
    ctxs = [fobq.Ctx(0, stream=st.cuda_stream) for st in streams]
    for c in ctxs:
        c.set_hessian_mode(hmode)

    # layers are independent, so the in-flight pass may take them in any order: widest first -- a wide layer is a
    # long chain of short launches that leaves the GPU nearly idle, and started early it runs beside the Hessians of
    # the layers that follow instead of alone at the end (network order: 65.6 / 85.2 ms, widest first: 61.6 / 80.8)
    flight_order = sorted(range(len(layers)), key=lambda i: -layers[i].d_col)

    def whole_model():
        busy = [False] * K
        for slot, i in enumerate(flight_order):
            spec, W, inp, pc = layers[i], Ws[i], Ins[i], per_call[i]
            k = slot % K
            if busy[k]:
                ctxs[k].finish()
                busy[k] = False
            if i in Hs:
                hessian(ctxs[k], spec, inp, pc, H_out=Hs[i])
                continue
            hessian(ctxs[k], spec, inp, pc)
            outs[i] = ctxs[k].quantize_layer(W, bits=spec.bits, group=spec.group, damp=spec.damp, out=outs[i], wait=False)
            busy[k] = True
        for k in range(K):
            if busy[k]:
                ctxs[k].finish()
        torch.cuda.synchronize()            # every Hessian of the batched layers is complete
        run_small_batch(ctxs[0])

    runs = []
    for it in range(warmup + steps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        whole_model()
        torch.cuda.synchronize()
        if it >= warmup:
            runs.append((time.perf_counter() - t0) * 1e3)
    workspace_flight = sum(c.workspace_bytes() for c in ctxs)
    for c in ctxs:
        c.close()
    med = _median(runs)
    line = {"metric": f"whole-model quantization time, {model}-shaped network ({len(layers)} layers)",
            "value": round(total_weights / (med * 1e-3), 1), "unit": "weights/s", "n_gpus": 1, "steps": steps,
            "warmup": warmup, "ms_per_step": round(med, 3), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "f64", "data": "synthetic",
            "config": {"workload": f"sweep_{model}: all layers, 4-bit per-row, damp 0.01, 128 images, "
                                   + ("every layer from an unfolded matrix of independent activations"
                                      if iid else "k x k and strided convolutions from their input maps"),
                       "hessian_arithmetic": "int8 slices where d_col >= 384 (stride-1 k x k convolutions with a multiple of 64 channels by tap "
                                             "offsets), else fp64 MFMA" if int8 else "fp64 MFMA",
                       "weights": total_weights, "layers_in_flight": K, "input_bytes": input_bytes},
            "whole_model_seconds": round(med * 1e-3, 4), "runs_ms": [round(r, 2) for r in runs],
            "sequential_ms": round(_median(seq_runs), 3), "sequential_runs_ms": [round(r, 2) for r in seq_runs],
            "layers_checked": checked, "layers_batched": len(small),
            "batched_call_ms": round(_median(batch_ms), 3) if small else None,
            "workspace_bytes": {"one_context": workspace_seq, "contexts_in_flight": workspace_flight},
            "per_layer": per_layer}
    print(json.dumps(line))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c2_resnet50_3x3")
    ap.add_argument("--block", type=int, default=0, help="0 = blocked (default), 1 = unblocked rank-1 path")
    ap.add_argument("--chunk", type=int, default=0, help="calibration columns per accumulate call (0 = all)")
    ap.add_argument("--from-maps", action="store_true",
                    help="conv workloads: accumulate the Hessian straight from the feature maps "
                         "(fobq_hessian_accumulate_conv) instead of the unfolded X")
    ap.add_argument("--concurrency", type=int, default=16,
                    help="whole-model sweeps: layers in flight at once (one context and stream each)")
    ap.add_argument("--hessian", choices=("i8", "f64"), default="i8",
                    help="how X X^T is formed: i8 = exact int8 slice products on the matrix cores where the mode "
                         "applies (d_col >= 384, n >= 512 per call; H within 3e-13 of the fp64 sum), f64 = fp64 "
                         "matrix instructions")
    ap.add_argument("--no-batch", action="store_true",
                    help="whole-model sweeps: quantize the layers of up to 256 columns one by one instead of all of "
                         "them in one fobq_quantize_layers_batched call")
    ap.add_argument("--iid", action="store_true",
                    help="whole-model sweeps: feed every layer an unfolded matrix of independent activations "
                         "instead of the convolutions' input maps (the earlier variant, kept for comparison)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--obq-rows", type=int, default=0,
                    help="with the CPU baseline: also run the per-row OBQ baseline (own inverse Hessian per row) "
                         "of the oracle on this many rows and report its cost and loss next to FastOBQ's")
    ap.add_argument("--also-from-maps", action="store_true",
                    help="convolution workloads: after the headline run, time the same layer once more with its Hessian "
                         "accumulated from the feature maps and report it as `same_layer_from_feature_maps`")
    ap.add_argument("--copy-probe", action="store_true",
                    help="run one plain device copy of X first (known bytes; calibrates HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (across GPUs the method would shard by whole layers, "
              "and inside a layer by calibration columns and by rows of W); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2509_05576_amd as fobq
    import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU fallback", file=sys.stderr)
        return 2
    if args.workload in ("sweep_resnet50", "sweep_yolov5s"):
        return sweep(args.workload[len("sweep_"):], max(5, min(args.steps, 9)), min(args.warmup, 2), args.concurrency,
                     args.iid, args.hessian == "i8", not args.no_batch)
    fobq.load_library()
    spec = workloads.configs()[args.workload]
    W = spec.make_w()
    X = spec.make_x()
    Wd = torch.from_numpy(W).cuda()
    Xd = torch.from_numpy(X).cuda()
    Md = None
    if args.from_maps:
        if spec.conv is None:
            print(f"bench.py: workload {spec.name} is not a convolution", file=sys.stderr)
            return 2
        Md = torch.from_numpy(spec.make_maps()).cuda()
    torch.cuda.synchronize()

    if args.copy_probe:
        probe = Xd.clone()          # reads and writes X.numel() * 4 bytes
        torch.cuda.synchronize()
        del probe

    ctx = fobq.Ctx(0)
    ctx.set_hessian_mode(fobq.HESSIAN_INT8_SLICES if args.hessian == "i8" else fobq.HESSIAN_FP64)
    out = None

    def step():
        nonlocal out
        if Md is not None:
            ctx.hessian_conv(Md, spec.conv[3], spec.stride, spec.conv[4])
        else:
            ctx.hessian(Xd, chunk=args.chunk or None)
        out = ctx.quantize_layer(Wd, bits=spec.bits, group=spec.group, damp=spec.damp, block=args.block, out=out)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # Timed region: HIP events around the dominant kernel's stage only (every timed interval is two event
    # records on the library's stream, a few microseconds of launch gap each; nine stages would add about
    # 1 % to a step).  The split over all stages comes from a second, untimed pass of the same steps.
    dominant = "columns" if args.block == 1 else "xxt"
    fobq.fobq_profile_enable(ctx.handle, fobq.FOBQ_PROFILE_STAGE(fobq.STAGES.index(dominant)))
    fobq.fobq_profile_reset(ctx.handle)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    timed = ctx.stage_ms()
    fobq.fobq_profile_enable(ctx.handle, True)
    fobq.fobq_profile_reset(ctx.handle)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    stages = ctx.stage_ms()
    stages[dominant] = timed[dominant]
    fobq.fobq_profile_enable(ctx.handle, False)

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    weights = spec.d_row * spec.d_col
    value = weights / (ms_per_step * 1e-3)

    # dominant kernel: the X X^T kernel, one launch per accumulate call
    xxt_ms, xxt_launches = stages["xxt"]
    launches_per_step = xxt_launches / args.steps
    n_per_launch = spec.n / launches_per_step
    flops_per_launch = spec.d_col * (spec.d_col + 1) * n_per_launch     # one triangle: d(d+1)/2 entries x 2N flop
    avg_ms = xxt_ms / xxt_launches
    form = ctx.hessian_form()              # what the library took for this shape and input
    int8 = form != fobq.FORM_FP64
    offsets = form == fobq.FORM_INT8_TAP_OFFSETS
    if int8:
        # integer-slice formulation: 19 int8 slice products per entry the kernel forms, against the dense int8 peak.
        # Entries: the lower triangle, d (d + 1) / 2 -- or, for a convolution taken by tap offsets, the two block
        # rows of c channels that hold every offset, 2 c d (the rest of H comes from them by corrections).
        channels = spec.conv[2] if (offsets and spec.conv is not None) else 0
        entries2 = 4.0 * channels * spec.d_col if offsets else float(spec.d_col) * (spec.d_col + 1)    # 2 x entries
        ops_per_launch = 19.0 * entries2 * n_per_launch
        achieved = ops_per_launch / (avg_ms * 1e-3) / 1e12
        roofline = {"kernel": "xxt_i8_kernel", "bound": "mfma", "achieved": round(achieved, 1), "peak": PEAK_INT8_MFMA_TOPS,
                    "unit": "TOP/s", "frac": round(achieved / PEAK_INT8_MFMA_TOPS, 4),
                    "traffic": measured_traffic("xxt_i8_kernel", spec.name) if launches_per_step == 1 and not args.from_maps else None,
                    "avg_launch_ms": round(avg_ms, 4), "algorithmic_ops_per_launch": ops_per_launch,
                    "slice_products": 19, "entries_formed": "two block rows (tap offsets)" if offsets else "lower triangle",
                    "fp64_equivalent_TFLOPs": round(flops_per_launch / (avg_ms * 1e-3) / 1e12, 2),
                    "fp64_equivalent_over_fp64_mfma_peak": round(flops_per_launch / (avg_ms * 1e-3) / 1e12 / PEAK_FP64_MFMA_TFLOPS, 3)}
        # What the int8 matrix cores sustain on this machine, outside the timed region: the kernel's inner loop
        # with its operands fixed in LDS (no fetches, no barriers).  The rate depends on the operand bytes -- the
        # chip holds its power limit by slowing the matrix pipes -- so `frac` (against the published peak) has a
        # ceiling well below 1 that no kernel change moves; `frac_of_sustained` is against the probe on operands
        # distributed like this workload's digits.
        probe = {name: round(ctx.probe_int8_matrix_rate(kind), 1)
                 for name, kind in (("equal_bytes", fobq.PROBE_EQUAL_BYTES), ("random_bytes", fobq.PROBE_RANDOM_BYTES),
                                    ("relu_normal_digits", fobq.PROBE_RELU_DIGITS))}
        roofline["sustained_matrix_rate_TOPs"] = probe
        roofline["frac_of_sustained"] = round(achieved / probe["relu_normal_digits"], 4)
    else:
        achieved = flops_per_launch / (avg_ms * 1e-3) / 1e12
        roofline = {"kernel": "xxt_kernel", "bound": "mfma", "achieved": round(achieved, 3),
                    "peak": PEAK_FP64_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_FP64_MFMA_TFLOPS, 4),
                    "traffic": measured_traffic("xxt_kernel", spec.name) if launches_per_step == 1 and not args.from_maps else None,
                    "avg_launch_ms": round(avg_ms, 4),
                    "algorithmic_flops_per_launch": flops_per_launch}

    stage_ms = {k: round(v[0] / args.steps, 4) for k, v in stages.items()}
    R, d = spec.d_row, spec.d_col
    if args.block == 1:
        # the literal rank-1 path: step_kernel (one launch per column) dominates and is HBM-bound.  The
        # launches are timed together (HIP events around the stage on the library's stream), so launch gaps
        # are included.  Two byte counts per layer: the algorithmic one of the streaming formulation with
        # fp32 weights, 4 R d^2 + (8/3) d^3 (W read + write, upper triangle of the fp64 running inverse read +
        # write) -- `achieved` and `frac` -- and what this kernel really moves, whose running weights are
        # fp64: 8 R d^2 + (8/3) d^3 (`moved_*`).  One launch = one column.
        bytes_per_launch = (4.0 * R * d * d + 8.0 / 3.0 * d ** 3) / d
        moved_per_launch = (8.0 * R * d * d + 8.0 / 3.0 * d ** 3) / d
        col_ms, _ = stages["columns"]
        avg_ms = col_ms / (args.steps * d)
        ach = bytes_per_launch / (avg_ms * 1e-3) / 1e9
        moved = moved_per_launch / (avg_ms * 1e-3) / 1e9
        roofline = {"kernel": "step_kernel", "bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(ach / PEAK_HBM_GBS, 4), "traffic": measured_traffic("step_kernel", spec.name),
                    "avg_launch_ms": round(avg_ms, 6), "algorithmic_bytes_per_launch": bytes_per_launch,
                    "moved_bytes_per_launch": moved_per_launch, "moved_GBs": round(moved, 1),
                    "moved_frac": round(moved / PEAK_HBM_GBS, 4)}
    # The other contractions of the path, from the stage events of the second pass (each stage is many short
    # dependent launches, so these are stage-level rates, launch gaps included), against the fp64 matrix
    # peak: shared-Hinv elimination d^3 / 3 flop (symmetric trailing updates), column loop R d^2 (deferred
    # compensation), Cholesky + triangular inverse + L^-T L^-1 d^3.
    secondary = []
    if args.block != 1:
        for name, stage_names, flops in (("eliminate (elim_iter_kernel)", ("eliminate",), d ** 3 / 3.0),
                                         ("columns (col_block_kernel)", ("columns",), float(R) * d * d),
                                         ("cholesky + inverse (chol_iter_kernel, gemm64_kernel)",
                                          ("cholesky", "inverse"), float(d) ** 3)):
            ms = sum(stages[n][0] for n in stage_names) / args.steps
            if ms > 0:
                tf = flops / (ms * 1e-3) / 1e12
                secondary.append({"stage": name, "bound": "mfma", "algorithmic_flops": flops, "ms": round(ms, 4),
                                  "achieved": round(tf, 3), "peak": PEAK_FP64_MFMA_TFLOPS, "unit": "TFLOP/s",
                                  "frac": round(tf / PEAK_FP64_MFMA_TFLOPS, 4)})
    workspace = ctx.workspace_bytes()

    # --also-from-maps: the same layer with its Hessian accumulated from the input maps of the convolution instead of
    # the unfolded X (what a caller that holds the maps would do): reported beside the headline, never as `value`.
    # Off by default, so that the kernels of a default run are those of the headline path alone.
    from_maps = None
    if spec.conv is not None and not args.from_maps and args.block != 1 and args.chunk == 0 and args.also_from_maps:
        Mm = torch.from_numpy(spec.make_maps()).cuda()
        out_m = None

        def step_maps():
            nonlocal out_m
            ctx.hessian_conv(Mm, spec.conv[3], spec.stride, spec.conv[4])
            out_m = ctx.quantize_layer(Wd, bits=spec.bits, group=spec.group, damp=spec.damp, block=args.block, out=out_m)

        for _ in range(args.warmup):
            step_maps()
        torch.cuda.synchronize()
        tm0 = time.perf_counter()
        for _ in range(args.steps):
            step_maps()
        torch.cuda.synchronize()
        ms_maps = (time.perf_counter() - tm0) * 1e3 / args.steps
        form_m = ctx.hessian_form()
        from_maps = {"ms_per_step": round(ms_maps, 4), "value": round(weights / (ms_maps * 1e-3), 1), "unit": "weights/s",
                     "hessian_arithmetic": {fobq.FORM_FP64: "fp64 MFMA", fobq.FORM_INT8_SLICES: "int8 slices",
                                            fobq.FORM_INT8_TAP_OFFSETS: "int8 slices of two block rows, the other blocks by tap offsets"}[form_m],
                     "codes_equal_to_the_run_from_X": bool(torch.equal(out_m.codes, out.codes))}
        del Mm

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        t = time.perf_counter()
        ref = oracle.quantize_layer(W, X=X, bits=spec.bits, group=spec.group, damp_rel=spec.damp)
        cpu_s = time.perf_counter() - t
        codes = out.codes.cpu().numpy().astype(np.int64)
        cpu = {"value": round(weights / cpu_s, 1), "unit": "weights/s", "cores": oracle.num_threads(),
               "kind": "oracle", "sample": f"the whole {spec.name} layer once ({cpu_s:.1f} s): H, inverse, order, column loop",
               "seconds": round(cpu_s, 2), "codes_differ_vs_gpu": float((codes != ref.codes).mean())}
        if args.obq_rows > 0:
            # the paper's comparison (OBQ vs FastOBQ, Tables 1-2 "Time") on this synthetic layer, CPU oracle only
            nr = min(args.obq_rows, spec.d_row)
            t = time.perf_counter()
            ob = oracle.obq_rows(W, ref.Hinv, spec.bits, spec.group, ref.scales, ref.zeros, rows=(0, nr))
            obq_s = time.perf_counter() - t
            dW = W[:nr].astype(np.float64) - ref.Q[:nr]
            fast_loss = 0.5 * float(np.einsum("ij,jk,ik->", dW, ref.H_damped, dW))
            cpu["obq"] = {"rows": nr, "seconds": round(obq_s, 2),
                          "est_layer_seconds": round(obq_s * spec.d_row / nr, 1),
                          "obq_over_fastobq_time": round(obq_s * spec.d_row / nr / cpu_s, 1),
                          "obq_over_fastobq_gpu_time": round(obq_s * spec.d_row / nr / (ms_per_step * 1e-3), 1),
                          "fastobq_over_obq_loss_same_rows": round(fast_loss / float(ob.lossrow[:nr].sum()), 4)}
            if spec.d_col <= 4096:
                # the same baseline on the GPU (fobq_obq_rows: one workgroup per row), same rows, same Hinv
                Hinv_dev = torch.from_numpy(ref.Hinv).cuda()
                ctx.obq_rows(Wd, Hinv_dev, bits=spec.bits, group=spec.group, rows=(0, 1))
                torch.cuda.synchronize()
                t = time.perf_counter()
                g_codes, _, g_order, g_loss = ctx.obq_rows(Wd, Hinv_dev, bits=spec.bits, group=spec.group, rows=(0, nr))
                torch.cuda.synchronize()
                g_s = time.perf_counter() - t
                same = (g_order[:nr].cpu().numpy() == ob.order[:nr]).all(axis=1)
                cpu["obq"]["gpu"] = {"rows": nr, "seconds": round(g_s, 4),
                                     "rows_with_the_oracles_order": int(same.sum()),
                                     "codes_differ_vs_oracle": float((g_codes[:nr].cpu().numpy().astype(np.int64) != ob.codes[:nr]).mean()),
                                     "loss_rel_diff": float(abs(float(g_loss[:nr].sum()) - float(ob.lossrow[:nr].sum())) / float(ob.lossrow[:nr].sum())),
                                     "note": "one workgroup per row, rows side by side; a row's d x d inverse sits in LDS up to d = 128, "
                                             "in device memory beyond (then the kernel streams d^3 x 16 bytes per row)"}

    line = {
        "metric": "weights quantized per second, whole layer path"
                  + (" (ResNet-50 3x3 shape)" if spec.name == "c2_resnet50_3x3" else f" ({spec.name})"),
        "value": round(value, 1), "unit": "weights/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64 (X X^T: exact int8 slice products, int32 sums)" if int8 else "f64", "data": "synthetic",
        "config": {"workload": f"{spec.name}: W {spec.d_row}x{spec.d_col} fp32, X {spec.d_col}x{spec.n} fp32, "
                               f"{spec.bits}-bit, group {spec.group}, damp {spec.damp}, sensitivity order",
                   "block": args.block or 64, "accumulate_calls_per_step": launches_per_step,
                   "hessian_input": "feature maps (implicit unfold)" if args.from_maps else "unfolded X",
                   "hessian_arithmetic": ("int8 slices (5 digits, 19 products) of two block rows, the other blocks by tap offsets"
                                          if offsets else "int8 slices (5 digits, 19 products), fp64 fold") if int8 else "fp64 MFMA"},
        "stages_ms": stage_ms,
        "roofline": roofline,
        "roofline_secondary": secondary,
        "workspace_bytes": workspace,
        "same_layer_from_feature_maps": from_maps,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))
    ctx.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
