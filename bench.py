"""Benchmark of the integer-only ViT encoder forward on one MI355X.

A step is one pass of the whole hot path (ivit_forward: 12 encoder blocks, every step integer-only) over one
batch of synthetic int8 tokens of the DeiT-S shape, already resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2_deit_s]

`value` comes from K un-instrumented steps bracketed by device synchronisation.  The per-kernel figures of the
`roofline` object come from further steps of the same workload in the same process with the library's event
trace switched on (two HIP events around every launch, on the launch stream).  `cpu_baseline` times the CPU
oracle (single thread) on a few images of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0      # MI355X dense int8 MFMA peak, TOP/s
PEAK_HBM_GBS = 8000.0


def measured_traffic(workload):
    """HBM bytes per GEMM launch from the committed hardware-counter summary of this workload (None if there is none).

    Byte counters cannot be read inside this process; the figure is the one the counter runs of this same command gave.
    """
    path = os.path.join(ROOT, "profiles", "forward_%s_hbm_traffic.txt" % workload)
    try:
        for line in open(path):
            if "traffic_bytes_per_launch:" in line:
                return int(line.rsplit(":", 1)[1])
    except OSError:
        pass
    return None


def time_swin(binding, synth, torch, name, steps, stream):
    """The hierarchical windowed model (Swin-T shape), patches in, logits out, with its per-kind kernel time."""
    scfg = synth.SWIN[name]
    sm = binding.swin_to_device(synth.make_swin_model(scfg))
    sp, keep = binding.swin_params(sm)
    SB = scfg["B"]
    sp_patches = torch.from_numpy(synth.make_swin_patches(scfg)).cuda()
    sp_logits = torch.empty((SB, scfg["n_classes"]), dtype=torch.int8, device="cuda")
    wss = torch.empty(binding.ivit_swin_workspace_bytes(sp, SB), dtype=torch.uint8, device="cuda")
    for _ in range(3):
        binding.ivit_forward_swin(sp_patches, sp_logits, sp, SB, wss, stream=stream)
    torch.cuda.synchronize()
    n = max(10, steps // 2)
    ts = time.perf_counter()
    for _ in range(n):
        binding.ivit_forward_swin(sp_patches, sp_logits, sp, SB, wss, stream=stream)
    torch.cuda.synchronize()
    el = (time.perf_counter() - ts) / n
    n_launch = 7 * sum(scfg["depths"]) + 3 * (len(scfg["depths"]) - 1) + 5
    binding.ivit_trace_begin(3 * n_launch + 16)
    for _ in range(3):
        binding.ivit_forward_swin(sp_patches, sp_logits, sp, SB, wss, stream=stream)
    srec = binding.ivit_trace_end(3 * n_launch + 16)
    by_kind = {}
    s_ops = 0
    for ms, kind, ops, nbytes in srec:
        by_kind[binding.KIND_NAMES[kind]] = by_kind.get(binding.KIND_NAMES[kind], 0.0) + ms / 3
        s_ops += ops
    return dict(workload=name, batch=SB, ms_per_step=round(el * 1e3, 4), images_per_s=round(SB / el, 1),
                launches_per_step=len(srec) // 3, int8_gops_per_image=round(s_ops / 3 / SB / 1e9, 3),
                kernel_ms_per_step={k: round(v, 4) for k, v in sorted(by_kind.items())})


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2_deit_s")
    ap.add_argument("--trace-steps", type=int, default=10)
    ap.add_argument("--cpu-images", type=int, default=2, help="images the CPU oracle runs for cpu_baseline (0 = skip)")
    ap.add_argument("--rowwise-gib", type=float, default=1.0,
                    help="input + output bytes of the stand-alone I-LayerNorm / Shiftmax bandwidth runs (0 = skip)")
    ap.add_argument("--batch-sweep", default="", help="comma-separated batch sizes to time as well (same weights), e.g. 1,8,16,32,64,128")
    ap.add_argument("--no-image-path", action="store_true", help="skip the patches-to-logits timing (embedding + blocks + head)")
    ap.add_argument("--swin", default="swin_t", help="windowed model to time as well, patches to logits ('' = skip)")
    ap.add_argument("--swin-only", action="store_true", help="time only the windowed model and print its figures (for profiling runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device copy a few times (reference for hardware byte counters) and exit")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only; --gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2207_01405_amd import binding, synth
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.calibrate_copy:
        src = torch.ones(1 << 30, dtype=torch.int8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": 1 << 30, "calibrate_copy_bytes_written": 1 << 30, "launches": 4}))
        return
    binding.load()
    if args.swin_only:
        print(json.dumps({"swin": time_swin(binding, synth, torch, args.swin or "swin_t", args.steps,
                                            torch.cuda.current_stream().cuda_stream)}))
        return

    cfg = synth.CONFIGS[args.workload]
    d = synth.dims_of(cfg)
    B, T, C, H, F, L = cfg["B"], cfg["T"], cfg["C"], cfg["H"], cfg["F"], cfg["L"]
    blocks_np = synth.make_model(cfg)
    x_np = synth.make_input(cfg)
    blocks = [binding.to_device(p) for p in blocks_np]
    x = torch.from_numpy(x_np).cuda()
    y = torch.empty_like(x)
    ws = torch.empty(binding.ivit_workspace_bytes(d), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    blk_structs = [binding.block_params(p) for p in blocks]          # marshal once, outside the timed region

    def step():
        binding.ivit_forward(x, y, blk_structs, d, ws, stream=stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    images_per_s = B * args.steps / dt

    # ---- optional: the same model at other batch sizes (Fig. 5 of the paper sweeps the batch)
    sweep = None
    if args.batch_sweep:
        sweep = []
        for bs in [int(v) for v in args.batch_sweep.split(",")]:
            ds = synth.dims_of(cfg, bs)
            xs = x[: bs * T] if bs <= B else x.repeat((bs + B - 1) // B, 1)[: bs * T].contiguous()
            ys = torch.empty_like(xs)
            wss = torch.empty(binding.ivit_workspace_bytes(ds), dtype=torch.uint8, device="cuda")
            for _ in range(3):
                binding.ivit_forward(xs, ys, blk_structs, ds, wss, stream=stream)
            torch.cuda.synchronize()
            n = max(10, args.steps // 2)
            ts = time.perf_counter()
            for _ in range(n):
                binding.ivit_forward(xs, ys, blk_structs, ds, wss, stream=stream)
            torch.cuda.synchronize()
            el = (time.perf_counter() - ts) / n
            sweep.append(dict(batch=bs, ms_per_step=round(el * 1e3, 4), images_per_s=round(bs / el, 1)))

    # ---- patches in, logits out (embedding layer + block stack + final I-LayerNorm + head): the end-to-end figure
    image_path = None
    if not args.no_image_path and cfg["name"] in synth.PATCH_DIM:
        img = binding.to_device(synth.make_image_params(cfg)); fl = binding.to_device(synth.make_final_ln(cfg))
        patches = torch.from_numpy(synth.make_patches(cfg)).cuda()
        logits = torch.empty((B, synth.N_CLASSES[cfg["name"]]), dtype=torch.int8, device="cuda")
        wsi = torch.empty(binding.ivit_image_workspace_bytes(d), dtype=torch.uint8, device="cuda")
        ip = binding.image_params(img)
        for _ in range(3):
            binding.ivit_forward_image(patches, logits, ip, blk_structs, d, wsi, fl, stream=stream)
        torch.cuda.synchronize()
        n = max(10, args.steps // 2)
        ts = time.perf_counter()
        for _ in range(n):
            binding.ivit_forward_image(patches, logits, ip, blk_structs, d, wsi, fl, stream=stream)
        torch.cuda.synchronize()
        el = (time.perf_counter() - ts) / n
        image_path = dict(ms_per_step=round(el * 1e3, 4), images_per_s=round(B / el, 1), patch_dim=synth.PATCH_DIM[cfg["name"]],
                          n_classes=synth.N_CLASSES[cfg["name"]])
        del patches, logits, wsi

    swin = time_swin(binding, synth, torch, args.swin, args.steps, stream) if args.swin else None

    # ---- per-kernel durations with HIP events, same workload, same process
    launches_per_step = 7 * L
    cap = launches_per_step * args.trace_steps + 16
    binding.ivit_trace_begin(cap)
    t1 = time.perf_counter()
    for _ in range(args.trace_steps):
        step()
    rec = binding.ivit_trace_end(cap)
    traced_ms_per_step = (time.perf_counter() - t1) / max(1, args.trace_steps) * 1e3
    kinds = {}
    for ms, kind, ops, nbytes in rec:
        k = kinds.setdefault(binding.KIND_NAMES.get(kind, str(kind)), dict(n=0, ms=0.0, ops=0, bytes=0))
        k["n"] += 1; k["ms"] += ms; k["ops"] += ops; k["bytes"] += nbytes
    kernels = {}
    for name, k in kinds.items():
        kernels[name] = dict(launches_per_step=k["n"] // max(1, args.trace_steps), avg_us=round(k["ms"] / k["n"] * 1e3, 2),
                             ms_per_step=round(k["ms"] / max(1, args.trace_steps), 4),
                             tops=round(k["ops"] / (k["ms"] * 1e-3) / 1e12, 1) if k["ops"] else None,
                             gbs=round(k["bytes"] / (k["ms"] * 1e-3) / 1e9, 1))
    gemm = [k for n, k in kinds.items() if n.startswith("gemm")]
    g_ms = sum(k["ms"] for k in gemm); g_ops = sum(k["ops"] for k in gemm); g_n = sum(k["n"] for k in gemm)
    achieved = g_ops / (g_ms * 1e-3) / 1e12 if g_ms > 0 else 0.0
    roofline = dict(bound="mfma", kernel="gemm_ws_kernel (weight-stationary Dense + requant epilogues: QKV, proj, fc1, fc2)",
                    achieved=round(achieved, 1), peak=PEAK_INT8_TOPS, unit="TOP/s",
                    frac=round(achieved / PEAK_INT8_TOPS, 4), traffic=measured_traffic(args.workload),
                    avg_launch_us=round(g_ms / max(1, g_n) * 1e3, 2), launches_per_step=g_n // max(1, args.trace_steps),
                    ops_per_launch=g_ops // max(1, g_n))

    # ---- stand-alone row-wise kernels on buffers far larger than the caches: the HBM figure of I-LN and Shiftmax
    rowwise = None
    if args.rowwise_gib > 0:
        rowwise = {}
        half = int(args.rowwise_gib * (1 << 30) / 2)
        sp = synth.shift_params(32)
        ln_p = blocks[0]

        def hbm_run(name, cols, launch):
            rows = half // cols
            small = torch.from_numpy(synth.make_rows(11, 4096, cols)).cuda()
            xin = small.repeat((rows + 4095) // 4096, 1)[:rows].contiguous()
            out = torch.empty_like(xin)
            for _ in range(2):
                launch(xin, out)
            torch.cuda.synchronize()
            binding.ivit_trace_begin(16)
            for _ in range(5):
                launch(xin, out)
            r = binding.ivit_trace_end(16)
            avg_ms = sum(t[0] for t in r) / len(r)
            nbytes = 2 * rows * cols
            gbs = nbytes / (avg_ms * 1e-3) / 1e9
            rowwise[name] = dict(rows=rows, cols=cols, algorithmic_bytes=nbytes, avg_us=round(avg_ms * 1e3, 1),
                                 gbs=round(gbs, 1), frac_of_hbm_peak=round(gbs / PEAK_HBM_GBS, 4))
            del xin, out

        hbm_run("ilayernorm", C, lambda a, o: binding.ivit_ilayernorm(a, ln_p["ln1_gamma"], ln_p["ln1_beta"], o,
                                                                       ln_p["ln1_f_bits"], ln_p["ln1_c_shift"], stream=stream))
        hbm_run("shiftmax", T, lambda a, o: binding.ivit_shiftmax(a, o, sp, stream=stream))
        wide = dict(i0=32, n_shift=24, m_bits=46, k_out=8)       # the row-maximum variant of ShiftGELU on MLP-hidden rows
        hbm_run("shiftgelu_rowmax", F, lambda a, o: binding.ivit_shiftgelu_rowmax(a, o, wide, (24171, 21), stream=stream))
        src = torch.ones(half, dtype=torch.int8, device="cuda"); dst = torch.empty_like(src)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        dst.copy_(src); torch.cuda.synchronize()
        e0.record()
        for _ in range(5):
            dst.copy_(src)
        e1.record(); torch.cuda.synchronize()
        cgbs = 2 * half / (e0.elapsed_time(e1) / 5 * 1e-3) / 1e9
        rowwise["plain_copy"] = dict(bytes=2 * half, gbs=round(cgbs, 1), frac_of_hbm_peak=round(cgbs / PEAK_HBM_GBS, 4))
        del src, dst

    # ---- the oracle on the host cores, a bounded sample of the same workload
    cpu = None
    if args.cpu_images > 0:
        import oracle
        n_img = min(args.cpu_images, B)
        xs = x_np[: n_img * T]
        t2 = time.perf_counter()
        y_ref = oracle.forward(xs, blocks_np, synth.dims_of(cfg, n_img))
        cdt = time.perf_counter() - t2
        same = bool(np.array_equal(y[: n_img * T].cpu().numpy(), y_ref))
        cpu = dict(value=round(n_img / cdt, 4), unit="images/s", cores=1, kind="oracle",
                   sample="%d of the %d images of the workload, full %d-block forward, single thread (gcc -O2)" % (n_img, B, L),
                   matches_gpu=same)

    # the headline metric is quoted on the DeiT-S shape; other workloads are labelled as what they are (the windowed
    # stage counts windows, not images)
    shape_name = {"c0_tiny": "tiny-block", "c1_deit_t": "DeiT-T", "c2_deit_s": "DeiT-S", "c3_vit_b": "ViT-B",
                  "c4_swin_t": "Swin-T-stage"}.get(args.workload, args.workload)
    unit_name = "windows" if args.workload == "c4_swin_t" else "images"
    out = {
        "metric": "%s/sec integer-only %s-shaped fwd" % (unit_name, shape_name), "value": round(images_per_s, 1), "unit": unit_name + "/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "%s: %d blocks, dim %d, %d heads, %d tokens, MLP %d, batch %d" % (args.workload, L, C, H, T, F, B)},
        "roofline": roofline, "cpu_baseline": cpu, "rowwise_hbm": rowwise, "batch_sweep": sweep, "image_path": image_path, "swin": swin,
        "ms_per_step_traced": round(traced_ms_per_step, 4), "kernels": kernels,
        "int8_tops_whole_step": round((24.0 * B * T * C * C + 4.0 * B * H * T * T * (C // H)) * L / (ms_per_step * 1e-3) / 1e12, 1),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
