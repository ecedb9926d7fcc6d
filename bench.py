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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2_deit_s")
    ap.add_argument("--trace-steps", type=int, default=10)
    ap.add_argument("--cpu-images", type=int, default=2, help="images the CPU oracle runs for cpu_baseline (0 = skip)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only; --gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2207_01405_amd import binding, synth
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    binding.load()

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
    roofline = dict(bound="mfma", kernel="gemm_i8_kernel (Dense + requant epilogues: QKV, proj, fc1, fc2)",
                    achieved=round(achieved, 1), peak=PEAK_INT8_TOPS, unit="TOP/s",
                    frac=round(achieved / PEAK_INT8_TOPS, 4), traffic=None,
                    avg_launch_us=round(g_ms / max(1, g_n) * 1e3, 2), launches_per_step=g_n // max(1, args.trace_steps),
                    ops_per_launch=g_ops // max(1, g_n))

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

    out = {
        "metric": "images/sec integer-only DeiT-S-shaped fwd", "value": round(images_per_s, 1), "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "%s: %d blocks, dim %d, %d heads, %d tokens, MLP %d, batch %d" % (args.workload, L, C, H, T, F, B)},
        "roofline": roofline, "cpu_baseline": cpu,
        "ms_per_step_traced": round(traced_ms_per_step, 4), "kernels": kernels,
        "int8_tops_whole_step": round((24.0 * B * T * C * C + 4.0 * B * H * T * T * (C // H)) * L / (ms_per_step * 1e-3) / 1e12, 1),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
