#!/usr/bin/env python3
"""Benchmark of the Parle hot path on one MI355X.

Headline workload (`config.workload = "flat_update_n8_36.5M"`): n = 8 replicas of a flat fp32
parameter vector of 36.5M elements; a step is one fused inner update (8a)+(8b) on all replicas,
and after every 25th step the outer step (replica mean (8d) + fused outer update (8c) + reset).
Inputs are synthetic (params ~ N(0, 0.05^2), gradients ~ N(0, 1e-4)), resident in HBM before the
timed region.  `value` is algorithmic bytes of the timed steps divided by elapsed time.

Prints ONE JSON line.  `--gpus N` with N > 1 is refused: this build runs on one GPU.
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

HBM_PEAK_GBPS = 8000.0
N_REPLICAS, N_PARAMS, L = 8, 36_500_000, 25
# algorithmic bytes per element-replica: inner reads grad,y,x,vy,z and writes y,vy,z
INNER_B = 32
# replica mean reads n rows and writes one: (4n + 4) bytes per column
# outer update reads x,z,vx (+ x_ref once per column) and writes x,vx,y,z,vy
OUTER_B = 32


def algorithmic_bytes(n, n_elem, inner_steps, outer_steps, fused):
    inner = inner_steps * n * n_elem * INNER_B
    mean = 0 if fused else outer_steps * n_elem * (4 * n + 4)
    outer = outer_steps * (n * n_elem * OUTER_B + n_elem * (4 if not fused else 4))
    return inner + mean + outer


def cpu_baseline(sample_elems=N_PARAMS, inner=12):
    """The oracle as it stands (float32 mode), on a column sample of the same workload."""
    from oracle import parle as oparle
    from paper_1707_00424_amd import synth
    n = N_REPLICAS
    cfg = oparle.ParleConfig(n_replicas=n, gamma0=0.03, rho0=1.0)
    x0 = synth.flat_params(0, n, sample_elems)
    G = synth.flat_grads(0, 0, n, sample_elems)
    st = oparle.init_state(x0, cfg, dtype=np.float32)
    oparle.inner_update(st, G, cfg)            # warm-up (page faults, allocator)
    t0 = time.perf_counter()
    for _ in range(inner):
        oparle.inner_update(st, G, cfg)
    oparle.outer_step(st, cfg)
    dt = time.perf_counter() - t0
    byt = algorithmic_bytes(n, sample_elems, inner, 1, fused=False)
    return {"value": round(byt / dt / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"n={n}, {sample_elems} of {N_PARAMS} columns, {inner} inner updates + 1 outer step, "
                      f"float32 numpy, {dt:.1f} s", "host_cpus": os.cpu_count()}


def read_traffic():
    """HBM bytes per inner-update launch from the committed rocprofv3 counter summary, if present."""
    p = os.path.join(ROOT, "profiles", "inner_update_flat_n8_36p5M_pmc.txt")
    try:
        for line in open(p):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def profile_roofline(name):
    """Dominant contraction kernel of a model workload from the committed rocprofv3 summaries: its share of
    the kernel time and average duration (profiles/<name>_kernel_stats.txt) and the fraction of cycles its
    matrix units were busy (profiles/<name>_pmc_mfma.txt).  These are figures of the profiled runs recorded
    there, not of this run."""
    stats = os.path.join(ROOT, "profiles", f"{name}_kernel_stats.txt")
    pmc = os.path.join(ROOT, "profiles", f"{name}_pmc_mfma.txt")
    try:
        util = {}
        for line in open(pmc):
            f = line.split()
            if len(f) >= 6 and f[-1].endswith("%") and f[-4].endswith("%"):
                util[" ".join(f[:-5])] = (float(f[-4].rstrip("%")) / 100, float(f[-1].rstrip("%")) / 100)
        for line in open(stats):
            f = line.split()
            if len(f) >= 7 and f[-1].endswith("%") and f[0].startswith("k_"):
                kern = " ".join(f[:-6])
                if kern in util and util[kern][0] > 0:
                    return {"kernel": kern, "avg_launch_us": float(f[-5]), "share_of_kernel_time": round(float(f[-1].rstrip("%")) / 100, 4),
                            "mfma_util": round(util[kern][0], 4), "lds_bank_conflict": round(util[kern][1], 4),
                            "source": f"profiles/{name}_kernel_stats.txt, profiles/{name}_pmc_mfma.txt"}
    except (OSError, ValueError):
        pass
    return None


MODEL_WORKLOADS = {
    # name: (library model, arch[], n, compute_bf16, weight init, step size, oracle architecture)
    # Step sizes: 0.1 is what the MLP workload states.  The other workloads name none: the networks without
    # batch-norm overflow (All-CNN-C, within three steps) or jump (LeNet) at 0.1 on these inputs, and 0.01 is
    # what Section 4.4 starts WRN-16-4 with, so all of them run at 0.01: timing does not depend on it, but a
    # run that ends in NaN is no sanity signal.
    "mlp_n3_fp32": (1, (128,), 3, 0, "uniform", 0.1, ("mlp", {})),
    "lenet_n6_fp32": (2, (20, 50, 5, 500), 6, 0, "uniform", 0.01, ("lenet", {})),
    "allcnn_c_n3_bf16": (3, (96, 192), 3, 1, "he_normal", 0.01, ("allcnn", {})),
    "wrn16_4_n3_bf16": (4, (16, 4, 2), 3, 1, "he_normal", 0.01, ("wrn", {})),
    # the network of the paper's own timing figure (Section 4.1: 528 ms per mini-batch of 128 on one of its GPUs)
    "wrn28_10_n3_bf16": (4, (16, 10, 4), 3, 1, "he_normal", 0.01, ("wrn", dict(widen=10, nb=4))),
}
MFMA_PEAK_TFLOPS = {0: 157.3, 1: 2500.0}
# forward flops of the first layer per image: its input gradient is never computed, so a step has
# 3 x forward - first layer contraction flops
FIRST_LAYER_FLOPS = {1: 2 * 784 * 128, 2: 2 * 24 * 24 * 20 * 25, 3: 2 * 32 * 32 * 96 * 27, 4: 2 * 32 * 32 * 16 * 27}
PAPER_CONTEXT = "Section 4.1: 528 ms per mini-batch of 128 (WRN-28-10, one replica on one GPU of a 2017 three-GPU " \
                "desktop, precision not stated) = 242 images/s per replica"


def blas_threads():
    """Threads the BLAS behind numpy's matrix products uses (the oracle's convolutions are such products)."""
    try:
        from threadpoolctl import threadpool_info
        return max([int(i.get("num_threads", 1)) for i in threadpool_info() if i.get("user_api") == "blas"] or [1])
    except Exception:
        return int(os.environ.get("OMP_NUM_THREADS", "1"))


def model_cpu_baseline(name):
    """The oracle as it stands (float32 mode, numpy with its BLAS threads) on ONE inner step of the workload:
    all replicas at the full shape for the two small networks; one replica (of n) for the three large ones,
    WRN-28-10 at a quarter of the batch -- marked as extrapolated."""
    from oracle import nets as onets, parle as oparle, trainer as otrainer
    from paper_1707_00424_amd import synth
    model, arch, n, bf16, wi, eta, (oname, okw) = MODEL_WORKLOADS[name]
    a = onets.arch(oname, **okw)
    small = model in (1, 2)
    reps = n if small else 1
    B = 32 if name.startswith("wrn28") else 128
    x0 = np.tile(synth.init_params(onets.layout(a), 0, wi), (reps, 1))
    cfg = oparle.ParleConfig(n_replicas=reps, gamma0=0.03, rho0=1.0, eta_inner=eta, eta_outer=eta)
    O = otrainer.ParleNet(a, cfg, x0, dtype=np.float32)
    X, Y = synth.image_batches(0, 2, reps, B, a["H"], a["W"], a["C"], a["classes"])
    if small:
        O.inner_step(X[0], Y[0])                # warm-up; the large networks' single step is long enough as it is
    t0 = time.perf_counter()
    O.inner_step(X[1], Y[1])
    dt = time.perf_counter() - t0
    out = {"value": round(reps * B / dt, 1), "unit": "replica-images/s", "cores": blas_threads(), "kind": "oracle",
           "sample": f"one inner step (forward, loss, backward, (8a)-(8b)) of {reps} of {n} replicas at batch {B}, "
                     f"float32 numpy, {dt:.2f} s", "extrapolated": not small}
    if name.startswith("wrn28"):
        out["paper_context"] = PAPER_CONTEXT
    return out


def bench_model(name, torch, pb, blocks=2, graph=True, progress=False, cpu=False):
    """Replica-images/s of the whole step (forward, loss, backward, fused update; outer step every
    L = 25) on synthetic class-conditional Gaussian images, batch 128 per replica."""
    from paper_1707_00424_amd import synth
    model, arch, n, bf16, wi, eta = MODEL_WORKLOADS[name][:6]
    B, Lm = 128, 25
    a = dict(H=28, W=28, C=1, classes=10) if model in (1, 2) else dict(H=32, W=32, C=3, classes=10)
    cfg = pb.make_config(model=model, n_replicas=n, batch=B, L=Lm, compute_bf16=bf16, in_h=a["H"], in_w=a["W"],
                         in_c=a["C"], n_classes=a["classes"], arch=arch, eta_inner=eta, eta_outer=eta,
                         gamma0=0.03, rho0=1.0, fuse_outer=1, scoping_B=390 if model == 4 else 0,
                         graph_block=1 if graph else 0)
    lay = pb.parle_query_layout(cfg)
    x0 = np.tile(synth.init_params(lay, 0, wi), (n, 1))
    P = pb.Parle(cfg, x0)
    # L distinct mini-batches per replica, resident on the device; every block of L steps walks them once
    X, Y = synth.image_batches(0, Lm, n, B, a["H"], a["W"], a["C"], a["classes"])
    dX, dY = torch.as_tensor(X).cuda(), torch.as_tensor(Y).cuda()
    loss = torch.zeros((Lm, n), dtype=torch.float32, device="cuda")
    # warm-up: the first block call runs step by step, the second records the HIP graph and replays it
    def say(what):                      # profiler runs with counters are slow: show that blocks complete
        if progress:
            torch.cuda.synchronize()
            print(f"bench.py: {name}: {what}", file=sys.stderr, flush=True)

    for w in range(2):
        P.parle_inner_block(dX, dY, loss)
        P.parle_outer_step()
        say(f"warm-up block {w + 1} of 2 done")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for blk in range(blocks):
        P.parle_inner_block(dX, dY, loss)
        P.parle_outer_step()
        say(f"timed block {blk + 1} of {blocks} done")
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    steps = blocks * Lm
    loss = loss[-1]
    # forward + backward-data + backward-weight, minus the first layer's input gradient, which nothing needs
    flops_step = (3 * P.sizes.forward_flops_per_image - FIRST_LAYER_FLOPS[model]) * n * B
    ips = steps * n * B / dt
    tflops = flops_step * steps / dt / 1e12
    out = {"replica_images_per_sec": round(ips, 1), "ms_per_inner_step": round(dt / steps * 1e3, 4),
           "n_replicas": n, "batch_per_replica": B, "dtype": "bf16" if bf16 else "f32",
           "launch": "HIP graph of 25 inner steps" if graph else "step by step",
           "step_size": eta,
           "roofline": {"bound": "mfma", "achieved": round(tflops, 2), "peak": MFMA_PEAK_TFLOPS[bf16],
                        "unit": "TFLOP/s", "frac": round(tflops / MFMA_PEAK_TFLOPS[bf16], 4),
                        "what": "contraction flops of the whole step (forward, backward-data, backward-weight) / step time",
                        "dominant_kernel": profile_roofline(name)},
           "final_loss": [round(float(v), 4) for v in loss.cpu().numpy()]}
    if cpu:
        out["cpu_baseline"] = model_cpu_baseline(name)
    P.close()
    del P
    torch.cuda.empty_cache()
    return out


def outer_kernel_rates(torch, pb, P, n, n_pad, reps=5):
    """The outer step's kernels one by one on the workload's own state tensors (HIP events around `reps` launches
    each): replica mean (8d), (8c) + reset with the mean taken from memory, and both in one kernel."""
    out = {"unit": "GB/s", "peak": HBM_PEAK_GBPS}
    cases = {
        "k_replica_mean": ((4 * n + 4) * n_pad, lambda: pb.parle_k_replica_mean(P.x, P.x_ref)),
        "k_outer_update": (n * n_pad * OUTER_B + 4 * n_pad,
                           lambda: pb.parle_k_outer_update(P.x, P.z, P.vx, P.y, P.vy, P.x_ref, None, 0.1, 0.9, 0.03, 1.0, 3, 0, 0)),
        "k_outer_fused": (n * n_pad * OUTER_B + 4 * n_pad,
                          lambda: pb.parle_k_outer_update(P.x, P.z, P.vx, P.y, P.vy, P.x_ref, None, 0.1, 0.9, 0.03, 1.0, 3, 1, 0)),
    }
    for name, (byt, fn) in cases.items():
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        out[name] = {"achieved": round(byt / (ms * 1e-3) / 1e9, 1), "frac": round(byt / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                     "avg_launch_ms": round(ms, 4), "algorithmic_bytes_per_launch": byt}
    # the fused kernel does the work of the two others in one pass: the same time set against their bytes
    both = cases["k_replica_mean"][0] + cases["k_outer_update"][0]
    out["k_outer_fused"]["frac_of_the_two_kernels_it_replaces"] = round(
        both / (out["k_outer_fused"]["avg_launch_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)
    return out


def stream_reference(torch, pb, count, reps=10):
    """What the memory system of this GPU gives plain streams of the update kernels' access shape
    (GB/s, bytes moved / HIP-event time): one array read, one written, a copy, and the fused inner
    update's mix of five arrays read and three written.  `count` floats per array."""
    src = torch.zeros(5 * count, dtype=torch.float32, device="cuda")
    dst = torch.zeros(3 * count, dtype=torch.float32, device="cuda")
    out = {"unit": "GB/s", "floats_per_array": count}
    for name, (r, w) in {"read": (1, 0), "write": (0, 1), "copy": (1, 1), "read5_write3": (5, 3)}.items():
        for _ in range(2):
            pb.parle_k_stream_reference(r, w, count, src, dst)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            pb.parle_k_stream_reference(r, w, count, src, dst)
        e1.record()
        torch.cuda.synchronize()
        out[name] = round((r + w) * count * 4 * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
    del src, dst
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=25)
    ap.add_argument("--fuse-outer", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--models", default="all", help="comma list of model workloads to time as well, or none")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="profiling aid: also run 3 plain device copies of one [n, n_pad] fp32 tensor, "
                         "the known-size kernel the HBM counters are scaled by")
    ap.add_argument("--no-graph", action="store_true", help="model workloads: enqueue every step instead of replaying "
                                                            "a HIP graph of L inner steps")
    ap.add_argument("--no-stream-reference", action="store_true",
                    help="skip the plain-stream kernels that show what HBM gives the update's access mix")
    ap.add_argument("--progress", action="store_true",
                    help="model workloads: report every finished block of 25 steps on stderr (synchronises: "
                         "for profiler runs, not for timing)")
    ap.add_argument("--counters", action="store_true",
                    help="for runs under `rocprofv3 --pmc`: the backward pass on ONE stream (sets PARLE_OVERLAP_WGRAD=0 "
                         "before the library is loaded).  Counter collection serialises dispatches across hardware "
                         "queues, and queues that wait on each other's events have gone silent under it")
    ap.add_argument("--blocks", type=int, default=2, help="model workloads: timed blocks of 25 inner steps (counter runs of the "
                                                           "largest network use 1: fewer dispatches for the profiler to hold)")
    ap.add_argument("--only-models", action="store_true",
                    help="profiling aid: skip the headline workload and print only the model timings")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs the Parle step on ONE GPU (all replicas stacked on it); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    if args.counters:
        os.environ["PARLE_OVERLAP_WGRAD"] = "0"
    import torch
    from paper_1707_00424_amd import binding as pb
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    pb.lib()
    torch.cuda.set_device(0)
    names = list(MODEL_WORKLOADS) if args.models == "all" else [m for m in args.models.split(",") if m and m != "none"]
    if args.only_models:
        print(json.dumps({"models": {nm: bench_model(nm, torch, pb, blocks=args.blocks, graph=not args.no_graph and not args.counters,
                                                      progress=args.progress) for nm in names}}))
        return
    n, N = N_REPLICAS, N_PARAMS
    cfg = pb.make_config(model=pb.MODEL_FLAT, n_replicas=n, n_params=N, L=L, eta_inner=0.1, eta_outer=0.1,
                         momentum=0.9, alpha=0.75, gamma0=0.03, rho0=1.0, fuse_outer=args.fuse_outer)
    # seeded synthetic inputs, generated on the device (host generation of 292M normals is slow)
    gen = torch.Generator(device="cuda").manual_seed(0)
    x0 = torch.empty((n, N), dtype=torch.float32, device="cuda").normal_(0.0, 0.05, generator=gen)
    P = pb.Parle(cfg, x0)
    del x0
    P.grad[:, :N].normal_(0.0, 1e-2, generator=gen)
    n_pad = P.sizes.n_pad

    def step(i):
        P.parle_inner_step()
        if (i + 1) % L == 0:
            P.parle_outer_step()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    outer_steps = 0
    t0 = time.perf_counter()
    for i in range(args.steps):
        ev[i][0].record()
        P.parle_inner_step()
        ev[i][1].record()
        if (args.warmup + i + 1) % L == 0:
            P.parle_outer_step()
            outer_steps += 1
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    inner_ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))
    total_bytes = algorithmic_bytes(n, n_pad, args.steps, outer_steps, bool(args.fuse_outer))
    value = total_bytes / elapsed / 1e9
    inner_bytes = n * n_pad * INNER_B
    achieved = inner_bytes / (inner_ms * 1e-3) / 1e9
    out = {
        "metric": "fused update HBM GB/s (algorithmic bytes / elapsed), Parle update-only workload",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(elapsed / args.steps * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "flat_update_n8_36.5M", "n_replicas": n, "n_params": N, "L": L,
                   "outer_steps_timed": outer_steps, "fuse_outer": args.fuse_outer,
                   "inner_updates_per_sec": round(args.steps / elapsed, 2)},
        "roofline": {"bound": "hbm", "kernel": "k_inner_update", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "avg_launch_ms": round(inner_ms, 4), "algorithmic_bytes_per_launch": inner_bytes,
                     "traffic": read_traffic(),
                     "traffic_source": "profiles/inner_update_flat_n8_36p5M_pmc.txt (rocprofv3 FETCH_SIZE / WRITE_SIZE of an "
                                       "earlier run of this command, scaled by plain copies; not a counter of this run)"},
    }
    out["outer_step_kernels"] = outer_kernel_rates(torch, pb, P, n, n_pad)
    if args.copy_calibration:
        scratch = torch.empty_like(P.grad)
        for _ in range(3):
            scratch.copy_(P.grad)
        torch.cuda.synchronize()
        out["config"]["copy_calibration_bytes_read"] = P.grad.numel() * 4
        del scratch
    P.close()
    del P
    torch.cuda.empty_cache()
    if not args.no_stream_reference:
        ref = stream_reference(torch, pb, n * n_pad)
        ref["inner_update_vs_read5_write3"] = round(achieved / ref["read5_write3"], 4)
        out["stream_reference"] = ref
    if names:
        out["models"] = {nm: bench_model(nm, torch, pb, blocks=args.blocks, graph=not args.no_graph and not args.counters,
                                         progress=args.progress, cpu=not args.no_cpu_baseline) for nm in names}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
