"""Benchmark of the integer-only ViT encoder forward on one MI355X.

A step is one pass of the whole hot path (ivit_forward: 12 encoder blocks, every step integer-only) over one
batch of synthetic int8 tokens of the DeiT-S shape, already resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2_deit_s]

`value` comes from K un-instrumented steps bracketed by device synchronisation.  The per-kernel figures of the
`roofline` object come from further steps of the same workload in the same process with the library's event
trace switched on (two HIP events around every launch, on the launch stream).  `cpu_baseline` times the CPU
oracle (single thread) on a few images of the same workload.  Beside the headline the line carries: the other
four configurations (`configs`), the stand-alone row-wise operators on buffers far larger than the caches and at
their native size (`rowwise_hbm`), and the rate of an MFMA-only loop on this part (`mfma_issue_rate`).
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

SHAPE_NAMES = {"c0_tiny": "tiny-block", "c1_deit_t": "DeiT-T", "c2_deit_s": "DeiT-S", "c3_vit_b": "ViT-B",
               "c4_swin_t": "Swin-T-stage"}


def measured_traffic(workload, build_id=None):
    """HBM bytes per GEMM launch from the committed hardware-counter summary of this workload.

    Byte counters cannot be read inside this process; the figure is the one the counter runs of this same command
    gave.  The summary names the build of the library it was taken with: given `build_id`, a summary of another
    build (the kernels have changed since) is not used.  Returns None if there is no usable summary.
    """
    path = os.path.join(ROOT, "profiles", "forward_%s_hbm_traffic.txt" % workload)
    traffic = have_id = None
    try:
        for line in open(path):
            if "traffic_bytes_per_launch:" in line:
                traffic = int(line.rsplit(":", 1)[1])
            if line.startswith("build_id:"):
                have_id = line.split(":", 1)[1].strip()
    except OSError:
        return None
    if build_id is not None and have_id != build_id:
        return None
    return traffic


def ops_of(cfg):
    """Integer operations (2 per multiply-accumulate) of one forward of a configuration."""
    B, T, C, H, L = cfg["B"], cfg["T"], cfg["C"], cfg["H"], cfg["L"]
    return (24.0 * B * T * C * C + 4.0 * B * H * T * T * (C // H)) * L


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


class Forward:
    """One configuration resident on the GPU: parameters, input, output, workspace."""

    def __init__(self, binding, synth, torch, name):
        self.binding, self.torch, self.name = binding, torch, name
        self.cfg = cfg = synth.CONFIGS[name]
        self.d = synth.dims_of(cfg)
        self.blocks_np = synth.make_model(cfg)
        self.x_np = synth.make_input(cfg)
        self.blocks = [binding.to_device(p) for p in self.blocks_np]
        self.x = torch.from_numpy(self.x_np).cuda()
        self.y = torch.empty_like(self.x)
        self.ws = torch.empty(binding.ivit_workspace_bytes(self.d), dtype=torch.uint8, device="cuda")
        self.stream = torch.cuda.current_stream().cuda_stream
        # marshalled once, outside the timed region: the host array of block structs the C entry point takes
        self.structs = (binding.BlockParams * len(self.blocks))(*[binding.block_params(p) for p in self.blocks])

    def step(self):
        self.binding.ivit_forward(self.x, self.y, self.structs, self.d, self.ws, stream=self.stream)

    def timed(self, steps, warmup):
        for _ in range(warmup):
            self.step()
        self.torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        self.torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    def traced(self, steps):
        """Per-kind kernel figures from `steps` further forwards with an event pair around every launch."""
        cap = 7 * self.cfg["L"] * steps + 16
        self.binding.ivit_trace_begin(cap)
        t1 = time.perf_counter()
        for _ in range(steps):
            self.step()
        rec = self.binding.ivit_trace_end(cap)
        wall = (time.perf_counter() - t1) / max(1, steps)
        kinds = {}
        roof_s = 0.0
        for ms, kind, ops, nbytes in rec:
            k = kinds.setdefault(self.binding.KIND_NAMES.get(kind, str(kind)), dict(n=0, ms=0.0, ops=0, bytes=0))
            k["n"] += 1; k["ms"] += ms; k["ops"] += ops; k["bytes"] += nbytes
            roof_s += max(ops / (PEAK_INT8_TOPS * 1e12), nbytes / (PEAK_HBM_GBS * 1e9))
        return kinds, wall, roof_s / max(1, steps)


def gemm_family(kinds):
    gemm = [k for n, k in kinds.items() if n.startswith("gemm")]
    g_ms = sum(k["ms"] for k in gemm); g_ops = sum(k["ops"] for k in gemm); g_n = sum(k["n"] for k in gemm)
    achieved = g_ops / (g_ms * 1e-3) / 1e12 if g_ms > 0 else 0.0
    return achieved, g_ms, g_ops, g_n


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2_deit_s")
    ap.add_argument("--trace-steps", type=int, default=10)
    ap.add_argument("--cpu-images", type=int, default=4, help="images the CPU oracle runs for cpu_baseline (0 = skip)")
    ap.add_argument("--rowwise-gib", type=float, default=1.0,
                    help="input + output bytes of the stand-alone I-LayerNorm / Shiftmax bandwidth runs (0 = skip)")
    ap.add_argument("--batch-sweep", default="", help="comma-separated batch sizes to time as well (same weights), e.g. 1,8,16,32,64,128")
    ap.add_argument("--no-image-path", action="store_true", help="skip the patches-to-logits timing (embedding + blocks + head)")
    ap.add_argument("--swin", default="swin_t", help="windowed model to time as well, patches to logits ('' = skip)")
    ap.add_argument("--swin-only", action="store_true", help="time only the windowed model and print its figures (for profiling runs)")
    ap.add_argument("--other-configs", default="c0_tiny,c1_deit_t,c3_vit_b,c4_swin_t",
                    help="configurations reported in `configs` beside the headline workload ('' = skip)")
    ap.add_argument("--no-mfma-probe", action="store_true", help="skip the MFMA-only issue-rate loop")
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
    lib = binding.load()
    build_id = lib.ivit_build_id().decode()
    stream = torch.cuda.current_stream().cuda_stream
    if args.swin_only:
        print(json.dumps({"swin": time_swin(binding, synth, torch, args.swin or "swin_t", args.steps, stream)}))
        return

    fw = Forward(binding, synth, torch, args.workload)
    cfg, d = fw.cfg, fw.d
    B, T, C, H, F, L = cfg["B"], cfg["T"], cfg["C"], cfg["H"], cfg["F"], cfg["L"]
    x, y, blocks = fw.x, fw.y, fw.blocks
    el = fw.timed(args.steps, args.warmup)
    ms_per_step = el * 1e3
    images_per_s = B / el

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
                binding.ivit_forward(xs, ys, fw.structs, ds, wss, stream=stream)
            torch.cuda.synchronize()
            n = max(10, args.steps // 2)
            ts = time.perf_counter()
            for _ in range(n):
                binding.ivit_forward(xs, ys, fw.structs, ds, wss, stream=stream)
            torch.cuda.synchronize()
            e = (time.perf_counter() - ts) / n
            sweep.append(dict(batch=bs, ms_per_step=round(e * 1e3, 4), images_per_s=round(bs / e, 1)))

    # ---- patches in, logits out (embedding layer + block stack + final I-LayerNorm + head): the end-to-end figure
    image_path = None
    if not args.no_image_path and cfg["name"] in synth.PATCH_DIM:
        img = binding.to_device(synth.make_image_params(cfg)); fl = binding.to_device(synth.make_final_ln(cfg))
        patches = torch.from_numpy(synth.make_patches(cfg)).cuda()
        logits = torch.empty((B, synth.N_CLASSES[cfg["name"]]), dtype=torch.int8, device="cuda")
        wsi = torch.empty(binding.ivit_image_workspace_bytes(d), dtype=torch.uint8, device="cuda")
        ip = binding.image_params(img)
        for _ in range(3):
            binding.ivit_forward_image(patches, logits, ip, fw.structs, d, wsi, fl, stream=stream)
        torch.cuda.synchronize()
        n = max(10, args.steps // 2)
        ts = time.perf_counter()
        for _ in range(n):
            binding.ivit_forward_image(patches, logits, ip, fw.structs, d, wsi, fl, stream=stream)
        torch.cuda.synchronize()
        e = (time.perf_counter() - ts) / n
        image_path = dict(ms_per_step=round(e * 1e3, 4), images_per_s=round(B / e, 1), patch_dim=synth.PATCH_DIM[cfg["name"]],
                          n_classes=synth.N_CLASSES[cfg["name"]])
        del patches, logits, wsi

    swin = time_swin(binding, synth, torch, args.swin, args.steps, stream) if args.swin else None

    # ---- per-kernel durations with HIP events, same workload, same process
    kinds, traced_wall, roof_s = fw.traced(args.trace_steps)
    kernels = {}
    for name, k in kinds.items():
        kernels[name] = dict(launches_per_step=k["n"] // max(1, args.trace_steps), avg_us=round(k["ms"] / k["n"] * 1e3, 2),
                             ms_per_step=round(k["ms"] / max(1, args.trace_steps), 4),
                             tops=round(k["ops"] / (k["ms"] * 1e-3) / 1e12, 1) if k["ops"] else None,
                             gbs=round(k["bytes"] / (k["ms"] * 1e-3) / 1e9, 1))
    achieved, g_ms, g_ops, g_n = gemm_family(kinds)
    traffic = measured_traffic(args.workload, build_id)
    roofline = dict(bound="mfma", kernel="Dense kernels with requantisation epilogues (gemm_rs_kernel: QKV, fc1; gemm_ks_kernel: fc2; gemm_ws_kernel: proj)",
                    achieved=round(achieved, 1), peak=PEAK_INT8_TOPS, unit="TOP/s",
                    frac=round(achieved / PEAK_INT8_TOPS, 4), traffic=traffic,
                    traffic_note=None if traffic is not None else "no hardware-counter summary of this build of the library under profiles/",
                    avg_launch_us=round(g_ms / max(1, g_n) * 1e3, 2), launches_per_step=g_n // max(1, args.trace_steps),
                    ops_per_launch=g_ops // max(1, g_n),
                    # the whole step against the sum over its launches of max(ops / int8 peak, bytes / HBM peak)
                    step_roofline_ms=round(roof_s * 1e3, 4), step_frac=round(roof_s * 1e3 / ms_per_step, 4))

    # ---- the other configurations: forward time, Dense family rate (fewer steps; they are context for the headline)
    configs = None
    if args.other_configs:
        configs = {}
        del fw.ws
        for name in args.other_configs.split(","):
            if name == args.workload:
                continue
            o = Forward(binding, synth, torch, name)
            oc = o.cfg
            n = max(5, min(args.steps, int(0.6 / max(1e-4, o.timed(2, 2)))))
            e = o.timed(n, 2)
            if n * e < 0.05:                                    # a timed region of a few milliseconds: the best of three
                e = min(e, o.timed(n, 2), o.timed(n, 2))        # (one wake-up of the idle part would otherwise be most of it)
            ok, _, orf = o.traced(3)
            oa, og_ms, og_ops, og_n = gemm_family(ok)
            unit = "windows/s" if name == "c4_swin_t" else "images/s"
            configs[name] = {"shape": SHAPE_NAMES.get(name, name), "blocks": oc["L"], "batch": oc["B"], "steps": n,
                             "ms_per_step": round(e * 1e3, 4), unit: round(oc["B"] / e, 1),
                             "gemm_tops": round(oa, 1), "gemm_frac": round(oa / PEAK_INT8_TOPS, 4),
                             "int8_tops_whole_step": round(ops_of(oc) / e / 1e12, 1), "step_frac": round(orf / e, 4)}
            del o
            torch.cuda.empty_cache()

    # ---- stand-alone row-wise kernels: on buffers far larger than the caches (the HBM figure), and at the size they
    # have inside the forward (cache-resident).  The first and the last 4096 rows of every large run are compared with
    # the oracle in this same run (the input is a 4096-row tile repeated).
    rowwise = None
    if args.rowwise_gib > 0:
        import oracle
        rowwise = {}
        half = int(args.rowwise_gib * (1 << 30) / 2)
        sp = synth.shift_params(32)
        rng = np.random.default_rng(5)

        def run(name, rows, cols, launch, ref, reps=5):
            small_np = synth.make_rows(11 + cols, 4096, cols)
            small = torch.from_numpy(small_np).cuda()
            xin = small.repeat((rows + 4095) // 4096, 1)[:rows].contiguous()
            out = torch.empty_like(xin)
            for _ in range(2):
                launch(xin, out)
            torch.cuda.synchronize()
            binding.ivit_trace_begin(reps + 4)
            for _ in range(reps):
                launch(xin, out)
            r = binding.ivit_trace_end(reps + 4)
            avg_ms = sum(t[0] for t in r) / len(r)
            nbytes = 2 * rows * cols
            gbs = nbytes / (avg_ms * 1e-3) / 1e9
            want = ref(small_np)
            n_chk = min(4096, rows)
            tail0 = rows - n_chk
            want_tail = np.roll(want, -(tail0 % 4096), axis=0)[:n_chk] if rows >= 4096 else want[:n_chk]
            same = bool(np.array_equal(out[:n_chk].cpu().numpy(), want[:n_chk]) and
                        np.array_equal(out[tail0:].cpu().numpy(), want_tail))
            rowwise[name] = dict(rows=rows, cols=cols, algorithmic_bytes=nbytes, avg_us=round(avg_ms * 1e3, 1),
                                 gbs=round(gbs, 1), frac_of_hbm_peak=round(gbs / PEAK_HBM_GBS, 4), matches_oracle=same)
            del xin, out

        def ln_case(cols):
            g = np.rint((1.0 + 0.1 * rng.standard_normal(cols)) * 256).astype(np.int32)
            b = np.rint(0.1 * rng.standard_normal(cols) * 2 ** 24).astype(np.int32)
            gd, bd = torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda()
            return (lambda a, o: binding.ivit_ilayernorm(a, gd, bd, o, 16, 19, stream=stream)), (lambda s: oracle.ilayernorm(s, g, b, 16, 19))

        for cols in (64, 96, 192, 384, 768):
            launch, ref = ln_case(cols)
            run("ilayernorm_C%d" % cols, half // cols, cols, launch, ref)
        for cols in (49, 65, 197):
            run("shiftmax_cols%d" % cols, half // cols, cols, lambda a, o: binding.ivit_shiftmax(a, o, sp, stream=stream),
                lambda s: oracle.shiftmax(s, sp))
        wide = dict(i0=32, n_shift=24, m_bits=46, k_out=8)       # the row-maximum variant of ShiftGELU on MLP-hidden rows
        run("shiftgelu_rowmax_cols%d" % F, half // F, F, lambda a, o: binding.ivit_shiftgelu_rowmax(a, o, wide, (24171, 21), stream=stream),
            lambda s: oracle.shiftgelu_rowmax(s, wide, (24171, 21)))
        # native sizes (what one launch inside the forward handles; resident in the caches)
        launch, ref = ln_case(C)
        run("ilayernorm_native_%dx%d" % (B * T, C), B * T, C, launch, ref, reps=10)
        run("shiftmax_native_%dx%d" % (B * H * T, T), B * H * T, T, lambda a, o: binding.ivit_shiftmax(a, o, sp, stream=stream),
            lambda s: oracle.shiftmax(s, sp), reps=10)
        rowwise["ilayernorm"] = rowwise["ilayernorm_C%d" % C] if "ilayernorm_C%d" % C in rowwise else None
        rowwise["shiftmax"] = rowwise["shiftmax_cols%d" % T] if "shiftmax_cols%d" % T in rowwise else None
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

    # ---- what the matrix cores sustain on this part when they do nothing else (the practical ceiling of the Dense kernels)
    mfma = None
    if not args.no_mfma_probe:
        mfma = {}
        scratch = torch.zeros(256 + 1024 * 1024, dtype=torch.uint8, device="cuda")
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for label, rnd in (("constant_operands", 0), ("random_operands", 1)):
            binding.ivit_probe_mfma_rate(rnd, 2000, scratch, stream=stream)
            torch.cuda.synchronize()
            e0.record()
            ops = binding.ivit_probe_mfma_rate(rnd, 20000, scratch, stream=stream)
            e1.record(); torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            cycles = int(scratch[:8].view(torch.int64).item())
            mfma[label] = dict(tops=round(ops / (ms * 1e-3) / 1e12, 1), frac_of_peak=round(ops / (ms * 1e-3) / 1e12 / PEAK_INT8_TOPS, 4),
                               ms=round(ms, 3), shader_mhz=round(cycles / (ms * 1e3), 0),
                               cycles_per_mfma=round(cycles / (20000 * 16.0), 2))
        mfma["note"] = "v_mfma_i32_32x32x32_i8 only, one wavefront per SIMD, four independent accumulators, no memory traffic"

    # ---- the oracle on the host cores, a bounded sample of the same workload
    cpu = None
    if args.cpu_images > 0:
        import oracle
        n_img = min(args.cpu_images, B)
        xs = fw.x_np[: n_img * T]
        t2 = time.perf_counter()
        y_ref = oracle.forward(xs, fw.blocks_np, synth.dims_of(cfg, n_img))
        cdt = time.perf_counter() - t2
        same = bool(np.array_equal(y[: n_img * T].cpu().numpy(), y_ref))
        cpu = dict(value=round(n_img / cdt, 4), unit="images/s", cores=1, kind="oracle",
                   sample="%d of the %d images of the workload, full %d-block forward, single thread (gcc -O2)" % (n_img, B, L),
                   matches_gpu=same)

    # the headline metric is quoted on the DeiT-S shape; other workloads are labelled as what they are (the windowed
    # stage counts windows, not images)
    shape_name = SHAPE_NAMES.get(args.workload, args.workload)
    unit_name = "windows" if args.workload == "c4_swin_t" else "images"
    out = {
        "metric": "%s/sec integer-only %s-shaped fwd" % (unit_name, shape_name), "value": round(images_per_s, 1), "unit": unit_name + "/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "%s: %d blocks, dim %d, %d heads, %d tokens, MLP %d, batch %d" % (args.workload, L, C, H, T, F, B)},
        "roofline": roofline, "cpu_baseline": cpu, "configs": configs, "rowwise_hbm": rowwise, "mfma_issue_rate": mfma,
        "batch_sweep": sweep, "image_path": image_path, "swin": swin,
        "ms_per_step_traced": round(traced_wall * 1e3, 4), "kernels": kernels,
        "int8_tops_whole_step": round(ops_of(cfg) / (ms_per_step * 1e-3) / 1e12, 1), "library_build_id": build_id,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
