#!/usr/bin/env python3
"""Benchmark of the batched INR decode hot path on one MI355X.

A "step" is one rinr_decode_batch_ex call over the whole batch of the chosen workload
(gather -> expand/dequant -> coordinates -> first / hidden / output layers -> NCHW store)
with the packed store, the image ids and the output tensors already resident in HBM.
Default workload: 256 images of 224x224, MLP 2->64 (x6 sine layers)->3, 8-bit hidden
layers, 70 % pruned, uint8 + fp32 NCHW outputs.  Data is synthetic (seeded).

Prints ONE JSON line: metric, value, unit, steps, ms_per_step, config, roofline and cpu_baseline objects.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3     # MI355X dense fp32 matrix peak (256 CUs x 256 FLOP/clk x 2.4 GHz)
PEAK_FP16_MFMA_TFLOPS = 2500.0    # MI355X dense fp16 matrix peak
# The method's own vector work is one sine per sine-layer output.  v_sin_f32 issues one wavefront instruction per
# 8 clocks per SIMD (half the plain vector rate; measured): 256 CUs x 4 SIMDs x 64 lanes / 8 clocks x 2.4 GHz.
PEAK_SINES_T = 256 * 4 * 64 / 8 * 2.4e9 / 1e12


def sines_per_pixel(model) -> int:
    """Sine evaluations per pixel: one per output of every sine layer (all linear layers but the last)."""
    return sum(ly.n_out for ly in model.layers[:-1])


def nonzero_flop_per_pixel(model) -> int:
    """2 x the number of kept (non-pruned) weights: what a decoder that skipped zeros would execute."""
    return 2 * sum(int(ly.n_in * ly.n_out if ly.keep is None else np.count_nonzero(ly.keep)) for ly in model.layers)


def host_threads() -> int:
    n = os.cpu_count() or 1
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit() and int(env) > 0:
        n = min(n, int(env))
    return n


# encode-side shapes: the three model shapes of Sec. VI-A at image sizes of their kind, and the headline decode model
FIT_SHAPES = {
    "cifar": ("3 linear layers, 15 hidden units, 32x32 images", [2, 15, 15, 3], 2048, 32, 32),
    "flowers": ("10 linear layers, 32 hidden units, 224x224 images", [2] + [32] * 9 + [3], 512, 224, 224),   # two images per CU
    "imagenet": ("10 linear layers, 40 hidden units, 224x224 images", [2] + [40] * 9 + [3], 256, 224, 224),
    "w64": ("7 linear layers, 64 hidden units (the cfg4 decode model), 224x224 images", [2] + [64] * 6 + [3], 256, 224, 224),
}



def time_fit_step(shape: str, fp32: bool, steps: int = 10, warm: int = 5):
    """Mean duration of one Adam step (HIP events) of an encode-side shape, for the extra figures of the default line."""
    import torch
    from paper_2306_16699_amd import rinr_fit, synth
    what, widths, n, H, W = FIT_SHAPES[shape]
    base = torch.from_numpy(synth.images(1, 8, H, W)).cuda()
    tgt = base.repeat((n + 7) // 8, 1, 1, 1)[:n].contiguous()
    f = rinr_fit.Fit(widths, n, H, W, fp32=fp32)
    f.set_params(np.tile(synth.init_params(2, widths, 8), ((n + 7) // 8, 1))[:n])
    f.steps(tgt, warm, 5e-4)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    f.steps(tgt, steps, 5e-4, t0=0, T=steps)
    ev1.record()
    torch.cuda.synchronize()
    ms = ev0.elapsed_time(ev1) / steps
    fam = "split16" if f.kernel_family == rinr_fit.KERNEL_SPLIT16 else "fp32"
    f.close()
    return {"shape": what, "images": n, "kernels": fam, "ms_per_step": ms, "pixel_steps_per_s": n * H * W / (ms * 1e-3)}


def bench_fit(args) -> int:
    """One step = one full-batch Adam step (every pixel) of every image's MLP.  The split-precision kernels are the default
    where they are built for the shape (--fp32-mfma takes the fp32 ones); the roofline is the matrix peak of the dtype the
    contractions run in."""
    import torch
    from paper_2306_16699_amd import rinr_fit, synth
    what, widths, n, H, W = FIT_SHAPES[args.fit]
    n = args.batch or n
    base = torch.from_numpy(synth.images(1, 8, H, W)).cuda()
    tgt = base.repeat((n + 7) // 8, 1, 1, 1)[:n].contiguous()
    f = rinr_fit.Fit(widths, n, H, W, fp32=args.fp32_mfma)
    split = f.kernel_family == rinr_fit.KERNEL_SPLIT16
    peak = PEAK_FP16_MFMA_TFLOPS if split else PEAK_FP32_MFMA_TFLOPS
    f.set_params(np.tile(synth.init_params(2, widths, 8), ((n + 7) // 8, 1))[:n])
    steps = max(1, min(args.steps, 50))
    tw, done = time.perf_counter(), 0
    while done < min(args.warmup, 5) or (time.perf_counter() - tw) * 1e3 < args.min_warmup_ms:
        f.steps(tgt, 1, 5e-4)
        torch.cuda.synchronize()
        done += 1
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    f.steps(tgt, steps, 5e-4, t0=0, T=steps)
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    kern_ms = ev0.elapsed_time(ev1) / steps
    flops = 6.0 * sum(widths[l] * widths[l + 1] for l in range(len(widths) - 1)) * H * W * n   # forward + two backward contractions
    ach = flops / (kern_ms * 1e-3) / 1e12
    res = {"metric": "fitted pixel-steps/sec on 1 MI355X (per-image MLP fit, Eq. 1): pixels x Adam steps",
           "value": n * H * W / (wall_ms * 1e-3), "unit": "pixel-steps/s", "image_steps_per_s": n / (wall_ms * 1e-3),
           "n_gpus": 1, "steps": steps, "warmup": done, "ms_per_step": wall_ms, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f16x2-split operands, f32 accumulate" if split else "f32", "data": "synthetic",
           "config": {"workload": f"fit {args.fit}: {what}", "images": n, "H": H, "W": W, "widths": widths},
           "roofline": {"bound": "mfma", "achieved": ach, "peak": peak, "unit": "TFLOP/s",
                        "frac": ach / peak, "traffic": None, "kernel_ms": kern_ms,
                        "flop_per_launch": flops, "executed_over_algorithmic_flop": 3.0 if split else 1.0,
                        "kernel": ("fit16_step_kernel (fp16 hi+lo operand pairs on MFMA 16x16x16, three terms per product, fp32 accumulate)"
                                   if split else "fit_step_kernel (fp32 MFMA 16x16x4 from LDS)")}}
    if not args.no_cpu_baseline:
        from oracle import fit_oracle
        p0 = synth.init_params(2, widths, 1)[0].astype(np.float64)
        sh, sw = min(H, 32), min(W, 32)                     # one image cropped to 32x32: the oracle is a scalar loop
        tc = time.perf_counter()
        reps = 0
        while time.perf_counter() - tc < 10.0:
            fit_oracle.loss_grad(widths, p0, synth.images(1, 1, H, W)[0][:, :sh, :sw].astype(np.float64))
            reps += 1
        dt = time.perf_counter() - tc
        res["cpu_baseline"] = {"value": reps * sh * sw / dt, "unit": "pixel-steps/s", "cores": 1, "kind": "oracle",
                               "sample": f"{reps} loss+gradient evaluations of one {sh}x{sw} crop, fp64 C oracle, one thread, {dt:.1f} s"}
    f.close()
    print(json.dumps(res))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--min-warmup-ms", type=float, default=400.0,
                    help="keep running untimed warm-up steps until this much wall time has passed (the GPU's clock "
                         "ramps up from idle over a few hundred ms; a handful of steps is timed on the ramp)")
    ap.add_argument("--config", type=int, default=4, help="workload 1..5 (default 4, the headline one)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-encode-side", action="store_true", help="skip the short fit-step timings appended to the default line")
    ap.add_argument("--tile", type=int, default=0, help="experiment: MFMA tile rows for widths 32/64 (16 or 32)")
    ap.add_argument("--blocks-per-cu", type=int, default=0)
    ap.add_argument("--threads", type=int, default=0)
    ap.add_argument("--fp32-mfma", action="store_true", help="time the fp32 MFMA kernels instead of the default split-precision path")
    ap.add_argument("--fp16-act", action="store_true",
                    help="time the opt-in mode that keeps one fp16 value per hidden activation (RINR_FLAG_FP16_ACT)")
    ap.add_argument("--fp16-all", action="store_true",
                    help="time the opt-in mode with fp16 weights and activations in the hidden layers (RINR_FLAG_FP16_ALL)")
    ap.add_argument("--augment", action="store_true",
                    help="time the decode with a per-slot affine map of the sampling grid and per-channel "
                         "normalisation fused in (fp32 output only)")
    ap.add_argument("--paper", choices=["cifar", "flowers", "imagenet"], default=None,
                    help="decode a batch of models of one of the paper's own shapes (Sec. VI-A) instead of --config")
    ap.add_argument("--batch", type=int, default=0, help="batch size for --paper (default: the paper's backbone batch size) or number of images for --fit")
    ap.add_argument("--fit", choices=sorted(FIT_SHAPES), default=None,
                    help="time the encode side instead: full-batch Adam steps of the per-image fit (one JSON line of its own)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="run only a plain device-to-device copy of MIB MiB per step (counter calibration) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build decodes on one GPU only (images are independent: with more GPUs every rank "
              "would decode its own slice of the batch's ids). Run with --gpus 1.", file=sys.stderr)
        return 2

    import torch
    from paper_2306_16699_amd import rinr, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    if args.copy_calibration:
        nbytes = args.copy_calibration << 20
        src = torch.full((nbytes // 4,), 1.0, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(args.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": nbytes, "bytes_written": nbytes, "steps": args.steps}))
        return 0
    rinr.lib()
    if args.fit:
        return bench_fit(args)

    w = synth.paper_workload(args.paper, args.batch or None) if args.paper else synth.workload(args.config)
    args.config = args.paper or args.config
    blob = rinr.pack(w.models, w.w0, w.coord_lo, w.coord_hi)
    st = rinr.Store(blob, fp32_tile_rows=args.tile)
    ids = torch.from_numpy(w.image_ids).cuda()
    n, H, W = w.n, w.H, w.W
    out = torch.empty((n, 3, H, W), dtype=torch.float32, device="cuda")
    out8 = torch.empty((n, 3, H, W), dtype=torch.uint8, device="cuda") if w.out_u8 else None
    dtype = rinr.OUT_F32_AND_U8 if w.out_u8 else rinr.OUT_F32
    affine, norm = None, None
    if args.augment:                    # flips, small rotations, zoom and shifts; ImageNet-style normalisation
        rng = np.random.default_rng(0)
        th, z = rng.uniform(-0.5, 0.5, n), rng.uniform(0.6, 1.2, n)
        fx = np.where(rng.uniform(size=n) < 0.5, -1.0, 1.0)
        aff = np.stack([fx * z * np.cos(th), -z * np.sin(th), rng.uniform(-.25, .25, n),
                        fx * z * np.sin(th), z * np.cos(th), rng.uniform(-.25, .25, n)], axis=1).astype(np.float32)
        affine = torch.from_numpy(aff).cuda()
        norm = ((1 / 0.229, 1 / 0.224, 1 / 0.225), (-0.485 / 0.229, -0.456 / 0.224, -0.406 / 0.225))
        dtype, out8 = rinr.OUT_F32, None

    # scratch for the heaviest-first slot order (used by stores that mix model widths: workload 5)
    workspace = torch.empty(rinr.workspace_bytes(n), dtype=torch.uint8, device="cuda")

    def timed(flags):
        """(wall ms per step, kernel ms per step over exactly args.steps launches, per-launch min / median ms, launch info)."""
        def step():
            st.decode_batch_ex(ids, H, W, dtype, flags, out=out, out_u8=out8, affine=affine, norm=norm, workspace=workspace,
                               threads=args.threads, blocks_per_cu=args.blocks_per_cu)
        tw, done = time.perf_counter(), 0
        while done < args.warmup or (time.perf_counter() - tw) * 1e3 < args.min_warmup_ms:
            step()
            done += 1
            if done % 16 == 0:
                torch.cuda.synchronize()
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        ev0.record()                      # same stream the library launches on (torch's current stream)
        for _ in range(args.steps):
            step()
        ev1.record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        # a second pass with an event between every two launches: the spread of single launches (not part of `value`)
        k = min(args.steps, 200)
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(k + 1)]
        evs[0].record()
        for i in range(k):
            step()
            evs[i + 1].record()
        torch.cuda.synchronize()
        per = np.array([evs[i].elapsed_time(evs[i + 1]) for i in range(k)])
        return (t1 - t0) * 1e3 / args.steps, ev0.elapsed_time(ev1) / args.steps, float(per.min()), float(np.median(per)), st.last_launch_info()

    pixels = n * H * W
    used = [w.models[int(i)] for i in w.image_ids]
    flop_px = np.array([synth.dense_flop_per_pixel(m) for m in used], dtype=np.float64)
    flops = float(flop_px.sum()) * H * W                         # algorithmic: 2 x sum(in x out) per pixel with the true widths
    nz_flops = float(sum(nonzero_flop_per_pixel(m) for m in used)) * H * W
    sines = float(sum(sines_per_pixel(m) for m in used)) * H * W
    out_bytes = pixels * (12 + (3 if out8 is not None else 0))

    def stored_traffic(tag):
        tpath = os.path.join(ROOT, "profiles", f"decode_{tag}_cfg{args.config}_traffic.json")
        if os.path.exists(tpath):
            try:
                return json.load(open(tpath)).get("hbm_bytes_per_launch"), os.path.relpath(tpath, ROOT)
            except Exception:
                return None, None
        return None, None

    def roofline(t, peak, tag, kernel, executed_factor):
        """The contraction's roofline: algorithmic FLOP per launch / mean launch duration against the dense matrix peak
        of the dtype the contraction runs in."""
        wall_ms, kern_ms, kmin, kmed, info = t
        ach = flops / (kern_ms * 1e-3) / 1e12
        traffic, src = stored_traffic(tag)
        return {"bound": "mfma", "achieved": ach, "peak": peak, "unit": "TFLOP/s", "frac": ach / peak,
                "traffic": traffic,
                "traffic_source": (f"stored figure from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE), {src}; not measured in this run"
                                   if traffic is not None else None),
                "kernel_ms": kern_ms, "kernel_ms_min": kmin, "kernel_ms_median": kmed,
                "flop_per_launch": flops, "flop_per_pixel_mean": float(flop_px.mean()),
                "executed_over_algorithmic_flop": executed_factor, "kernel": kernel,
                "nonzero_mac_tflops": nz_flops / (kern_ms * 1e-3) / 1e12,
                "output_write_GBps": out_bytes / (kern_ms * 1e-3) / 1e9,
                "vector_alu": {"bound": "alu", "work": "sine evaluations (one per sine-layer output per pixel)",
                               "achieved": sines / (kern_ms * 1e-3) / 1e12, "peak": PEAK_SINES_T, "unit": "T sines/s",
                               "frac": sines / (kern_ms * 1e-3) / 1e12 / PEAK_SINES_T, "sines_per_launch": sines}}

    def mode_entry(name, t, roof):
        return {"mode": name, "value": pixels / (t[0] * 1e-3), "unit": "pixels/s", "ms_per_step": t[0], "roofline": roof, "launch": t[4]}

    k32 = "decode_kernel (fp32 MFMA)"
    kx = "decode_xdl_kernel (fp16 hi+lo operand pairs on the fp16 matrix cores, fp32 accumulate)"
    k16 = "decode_xdl_kernel, one fp16 value per activation (fp16 MFMA, fp32 accumulate)"
    k16a = "decode_xdl_kernel, fp16 weights and activations in the hidden layers (fp16 MFMA, fp32 accumulate)"
    F16A = rinr.FLAG_FP16_ACT | rinr.FLAG_FP16_UNCHECKED
    F16W = rinr.FLAG_FP16_ALL | rinr.FLAG_FP16_UNCHECKED
    coded = all(2 <= ly.bits <= 8 for m in used[:64] for ly in m.layers[1:-1])
    fx = 2.0 if coded else 3.0            # MFMA terms per algorithmic product: Q*hi + Q*lo, or Wh*hh + Wh*hl + Wl*hh
    alt, alt16, alt16a = None, None, None
    if args.fp32_mfma:
        t = timed(rinr.FLAG_FP32_MFMA)
        roof, dtype_name = roofline(t, PEAK_FP32_MFMA_TFLOPS, "fp32mfma", k32, 1.0), "f32"
    elif args.fp16_act:
        t = timed(F16A)
        roof, dtype_name = roofline(t, PEAK_FP16_MFMA_TFLOPS, "xdl16", k16, fx / 2), "f16 activations, f32 accumulate"
    elif args.fp16_all:
        t = timed(F16W)
        roof, dtype_name = roofline(t, PEAK_FP16_MFMA_TFLOPS, "xdl16all", k16a, 1.0), "f16 weights and activations, f32 accumulate"
    else:
        t = timed(0)
        roof = roofline(t, PEAK_FP16_MFMA_TFLOPS, "xdl", kx, fx)
        dtype_name = "f16x2-split operands, f32 accumulate"
        t2 = timed(rinr.FLAG_FP32_MFMA)
        alt = mode_entry("RINR_FLAG_FP32_MFMA", t2, roofline(t2, PEAK_FP32_MFMA_TFLOPS, "fp32mfma", k32, 1.0))
        t3 = timed(F16A)
        alt16 = mode_entry("RINR_FLAG_FP16_ACT | RINR_FLAG_FP16_UNCHECKED (reduced precision, forced past its worst-case bound: "
                           "one fp16 value per hidden activation)", t3, roofline(t3, PEAK_FP16_MFMA_TFLOPS, "xdl16", k16, fx / 2))
        t4 = timed(F16W)
        alt16a = mode_entry("RINR_FLAG_FP16_ALL | RINR_FLAG_FP16_UNCHECKED (reduced precision, forced past its worst-case bound: "
                            "fp16 weights and activations in the hidden layers)", t4, roofline(t4, PEAK_FP16_MFMA_TFLOPS, "xdl16all", k16a, 1.0))
    wall_ms, kern_ms, info = t[0], t[1], t[4]
    assert st.status() == 0
    bounds = st.error_bounds()

    res = {
        "metric": "decoded pixels/sec (and images/sec) on 1 MI355X; % of MFMA/VALU FLOP peak",
        "value": pixels / (wall_ms * 1e-3),
        "unit": "pixels/s",
        "images_per_s": n / (wall_ms * 1e-3),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype_name, "data": "synthetic",
        "config": {"workload": w.name, "images": n, "H": H, "W": W,
                   "outputs": "fp32+uint8 NCHW" if (w.out_u8 and not args.augment) else "fp32 NCHW",
                   "augmentation": "per-slot affine grid map + per-channel normalisation" if args.augment else "none",
                   "flop_per_pixel_mean": float(flop_px.mean()), "sines_per_pixel_mean": sines / pixels,
                   "kept_weight_fraction": nz_flops / flops,
                   "reduced_precision_error_bounds": {"fp16_act": bounds[0], "fp16_all": bounds[1], "granted_below": 9.5e-4},
                   "launch": info},
        "roofline": roof,
    }
    if alt is not None:
        res["fp32_mfma_mode"] = alt
    if alt16 is not None:
        res["fp16_act_mode"] = alt16
    if alt16a is not None:
        res["fp16_all_mode"] = alt16a
    if args.config == 4 and not args.paper and not args.no_encode_side and not args.no_cpu_baseline:      # the full default run only
        # the encode side (one Adam step of every image's fit, Eq. 1) on two of the paper's shapes, both kernel families:
        # not part of `value`; `python bench.py --fit <shape>` is the full measurement
        res["encode_side"] = [time_fit_step(sh, fp32) for sh in ("imagenet", "cifar") for fp32 in (False, True)]

    if not args.no_cpu_baseline:
        from oracle import oracle
        cores = host_threads()
        per_img_s = float(flop_px.mean()) * H * W / 2.0e9        # the scalar fp64 oracle runs near 2 GFLOP/s per core
        n_s = int(max(1, min(n, round(12.0 * cores / max(per_img_s, 1e-4)))))   # about 12 s of wall time
        sample = w.image_ids[:n_s]
        tc = time.perf_counter()
        oracle.decode(w.models, sample, H, W, w.w0, w.coord_lo, w.coord_hi, want_u8=w.out_u8, n_threads=cores)
        dt = time.perf_counter() - tc
        n_1 = int(max(1, min(n, round(5.0 / max(per_img_s, 1e-4)))))             # about 5 s on one core
        tc = time.perf_counter()
        oracle.decode(w.models, w.image_ids[:n_1], H, W, w.w0, w.coord_lo, w.coord_hi, want_u8=w.out_u8, n_threads=1)
        dt1 = time.perf_counter() - tc
        res["cpu_baseline"] = {"value": n_s * H * W / dt, "unit": "pixels/s", "cores": cores, "kind": "oracle",
                               "sample": f"first {n_s} of {n} slots, all pixels, fp64 C oracle with OpenMP over images, {dt:.1f} s",
                               "single_core": {"value": n_1 * H * W / dt1, "unit": "pixels/s", "cores": 1,
                                               "sample": f"first {n_1} of {n} slots, all pixels, one thread, {dt1:.1f} s"}}
    st.close()
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
