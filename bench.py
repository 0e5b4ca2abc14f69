#!/usr/bin/env python3
"""Benchmark of the LLVQ hot path on one MI355X: fused dequant-GEMV at batch 1 (paper App. C) over the seven linear
layers of a Llama-3-8B-shaped transformer block.

A step = one pass of the whole hot path (index fetch, class lookup, unflatten, placement, signs, shape-gain scale,
24-wide dot products, row reduction) over the block's layers at ~2 bits/weight (48-bit index + fp16 gain per block of
24 weights): q/k/v in one llvq_matmul_multi launch, o, gate/up in one llvq_matmul_multi launch, down -- four launches,
9,103,360 blocks, 72.8 MB of packed weights, inputs resident in HBM.  Steps cycle through a ring of distinct
transformer blocks larger than the last-level cache, so the packed weights really stream from HBM.

Prints ONE JSON line: whole-job packed-weight GB/s, the HBM roofline of the matmul kernel (algorithmic bytes: 8 per
block, against its HIP-event time), the vector-ALU view of the same launches, the single 4096 x 4104 layer of the
paper's own timing table, and the oracle timed on the host CPU on a sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, vendor figure
BYTES_PER_BLOCK = 8            # 6-byte index + 2-byte gain
ALU_PEAK_TLOPS = 39.3          # 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz, one vector instruction per lane and cycle
COUNTER_SUMMARY = os.path.join(ROOT, "profiles", "matmul_llama3_8b_layer_set_counters.txt")
GROUPS = (("q", "k", "v"), ("o",), ("gate", "up"), ("down",))      # launches of a step: matrices that share their input


def read_counter_summary(path=COUNTER_SUMMARY):
    """`key = number` lines of the machine-written counter summary (paper_2603_11021_amd/profile_summary.py)."""
    vals = {}
    try:
        for line in open(path):
            if "=" in line and not line.lstrip().startswith("#"):
                k, v = line.split("=", 1)
                try:
                    vals[k.strip()] = float(v.split()[0])
                except (ValueError, IndexError):
                    pass
    except OSError:
        pass
    return vals


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--ring", type=int, default=4, help="distinct transformer blocks in the ring (4 x 72.8 MB = 291 MB)")
    ap.add_argument("--single-layers", type=int, default=48, help="distinct layers in the ring of the single-layer figure (48 x 5.6 MB = 269 MB)")
    ap.add_argument("--rows", type=int, default=4096,
                    help="output rows N of the single-layer figure; larger values amortise the per-launch fixed cost")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-single", action="store_true", help="skip the figures that ride along: single 4096 x 4104 layer, batch 16, 70B-shaped set")
    ap.add_argument("--only-single", action="store_true",
                    help="run ONLY the single rows x 4104 layer loop and print its figures (for rocprofv3 runs of that launch)")
    ap.add_argument("--extra", action="store_true", help="also time the layer sets launch by launch, batch 16, prefill and bulk decode (stderr)")
    ap.add_argument("--sweep", action="store_true",
                    help="also run the batch-1 product over a range of sizes, 320 launches each (stderr); under "
                         "rocprofv3 --kernel-trace the dispatches appear in this order")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain 256 MiB device copy, so that a rocprofv3 --pmc run has a kernel of known HBM traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus %d is not supported (sharding is design-only)" % args.gpus)

    import numpy as np
    import torch
    from paper_2603_11021_amd import LLVQ, synth

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the library has no CPU path")
    dev = torch.device("cuda:0")
    q = LLVQ(13, 0)
    M = 1
    if args.only_single:
        from oracle.llvq_oracle import Oracle
        print(json.dumps(single_layer(q, synth, torch, dev, args, Oracle(13))))
        return

    # ring of distinct Llama-3-8B-shaped transformer blocks: uniform indices over the union of shells 2..13, log-normal gains
    shapes = synth.LLAMA3_8B
    host0 = {}                                   # block 0 stays on the host for the parity check and the CPU baseline
    ring = []
    nblk = 0
    for b in range(args.ring):
        mats = {}
        for i, (name, (N, K)) in enumerate(shapes.items()):
            KB = synth.blocks_per_row(K)
            r = synth.rng_for(3, 10 * b + i)
            idx, gain = synth.indices(r, (N, KB)), synth.gains(r, (N, KB))
            if b == 0:
                host0[name] = (idx, gain)
                nblk += N * KB
            mats[name] = (torch.from_numpy(synth.pack_u48(idx).reshape(-1)).to(dev), torch.from_numpy(gain.reshape(-1)).to(dev), N, KB)
        launches = []
        for group in GROUPS:
            ms = [mats[g] for g in group]
            launches.append((group, [m[0] for m in ms], [m[1] for m in ms], [m[2] for m in ms], ms[0][3],
                             [torch.empty((M, m[2]), dtype=torch.float32, device=dev) for m in ms]))
        ring.append(launches)
    x_host = {}
    for K in sorted({K for (_, K) in shapes.values()}):
        x_host[synth.blocks_per_row(K)] = synth.activations(synth.rng_for(3, 900 + K % 997), M, K)
    d_x = {KB: torch.from_numpy(x.astype(np.float16)).to(dev) for KB, x in x_host.items()}
    n_launch = len(GROUPS)

    def step(i):
        for (_, idxs, gains, Ns, KB, ys) in ring[i % args.ring]:
            q.llvq_matmul_multi(d_x[KB], idxs, gains, Ns, KB, outs=ys)

    # What a plain device copy reaches on this machine: 1 GiB read + 1 GiB written, HIP events, best of five.  Measured first,
    # well before the timed region: it is not part of a step.
    csrc = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    cdst = torch.empty_like(csrc)
    cdst.copy_(csrc)
    copy_gbs = 0.0
    for _ in range(5):
        c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        c0.record()
        cdst.copy_(csrc)
        c1.record()
        torch.cuda.synchronize()
        copy_gbs = max(copy_gbs, 2.0 * (1 << 30) / (c0.elapsed_time(c1) * 1e-3) / 1e9)
    del csrc, cdst

    # The figures that ride along are taken next (they are separate measurements, not steps; taking them before the
    # timed region also means that it does not start on a GPU that has idled through the host-side input generation):
    # the fused prefill product at M = 1024, the Llama-3-70B-shaped layer set at batch 1 (one transformer block, 285.6 MB
    # packed, same four launches per step), the single layer of the paper's own timing table (App. C: 4096 x 4104, ring of
    # distinct layers, one launch per step), and the same ring of transformer blocks at batch 16 (the batched-decode kernel).
    from oracle.llvq_oracle import Oracle
    oracle = Oracle(13)
    single = None
    batch16 = None
    set70b = None
    prefill = None
    if not args.no_single:
        prefill = prefill_layer(q, synth, torch, dev, ring)
        set70b = llama70b_set(q, synth, torch, dev, max(args.steps // 10, 5), max(args.warmup // 10, 2))
        single = single_layer(q, synth, torch, dev, args, oracle)
        batch16 = layer_set_pass(q, synth, torch, dev, ring, {KB: synth.activations(synth.rng_for(3, 950 + KB), 16, 24 * KB) for KB in x_host},
                                 nblk, args.steps, args.warmup)       # the headline's own protocol, so that the ratio compares like with like

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(args.steps):
        step(args.warmup + i)
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ev_ms = e0.elapsed_time(e1) / args.steps            # HIP events on the launch stream: all launches of a step
    ms_per_step = wall * 1e3 / args.steps
    gbs = BYTES_PER_BLOCK * nblk / (ms_per_step * 1e-3) / 1e9
    ach = BYTES_PER_BLOCK * nblk / (ev_ms * 1e-3) / 1e9

    if batch16 is not None:
        batch16["ms_per_step_batch1_events"] = ev_ms
        batch16["ratio_to_batch1"] = batch16["ms_per_step_events"] / ev_ms

    # parity of the timed configuration against the oracle on sampled rows of every layer of block 0
    step(0)
    torch.cuda.synchronize()
    err = 0.0
    for (group, _, _, Ns, KB, ys) in ring[0]:
        for name, N, y in zip(group, Ns, ys):
            rows = np.arange(0, N, 64)
            idx, gain = host0[name]
            ref = oracle.matmul(x_host[KB], idx[rows], gain[rows])
            err = max(err, float(np.abs(y.cpu().numpy().astype(np.float64)[:, rows] - ref).max() / np.abs(ref).max()))

    cpu = None
    if not args.no_cpu_baseline:
        # the oracle on one layer of the step (q of block 0: 4096 x 4104, 700,416 blocks), one thread, then all cores
        idx0, gain0 = host0["q"]
        x0 = x_host[idx0.shape[1]]
        nq = idx0.size
        t = time.perf_counter()
        reps = 0
        while time.perf_counter() - t < 10.0:
            oracle.matmul(x0, idx0, gain0)
            reps += 1
        dt = (time.perf_counter() - t) / reps
        # rows split among threads (the C routine holds no lock and writes only its own output slice; ctypes releases
        # the interpreter lock during the call)
        from concurrent.futures import ThreadPoolExecutor
        ncores = max(1, min(16, os.cpu_count() or 1))
        bounds = np.linspace(0, idx0.shape[0], ncores + 1).astype(int)
        with ThreadPoolExecutor(ncores) as pool:
            t = time.perf_counter()
            reps_all = 0
            while time.perf_counter() - t < 5.0:
                list(pool.map(lambda i: oracle.matmul(x0, idx0[bounds[i]:bounds[i + 1]], gain0[bounds[i]:bounds[i + 1]]), range(ncores)))
                reps_all += 1
            dt_all = (time.perf_counter() - t) / reps_all
        cpu = {"value": BYTES_PER_BLOCK * nq / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
               "all_cores": {"value": BYTES_PER_BLOCK * nq / dt_all / 1e9, "unit": "GB/s", "cores": ncores,
                             "blocks_per_s": nq / dt_all},
               "sample": "the q layer of the step (4096x4104, %d of the step's %d blocks), batch 1, %d repetitions, single thread" % (nq, nblk, reps),
               "blocks_per_s": nq / dt}

    if args.extra:
        extra_layer_set(q, synth, torch, dev)
        extra_shapes(q, synth, torch, dev)
    if args.sweep:
        extra_sweep(q, synth, torch, dev)
    if args.calib_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)                       # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()

    # instruction and traffic counts of these launches come from the tracked counter summary (rocprofv3 --pmc runs of
    # this script, condensed by paper_2603_11021_amd/profile_summary.py); absent file: the fields are null
    cs = read_counter_summary()
    valu_per_block = cs.get("valu_instructions_per_block")
    traffic = cs.get("hbm_traffic_bytes_per_step")
    alu = None
    if valu_per_block:
        lane_ops = valu_per_block * nblk / (ev_ms * 1e-3) / 1e12
        alu = {"valu_instructions_per_block": valu_per_block, "lds_instructions_per_block": cs.get("lds_instructions_per_block"),
               "achieved": lane_ops, "peak": ALU_PEAK_TLOPS, "unit": "T lane-ops/s", "valu_issue_frac": lane_ops / ALU_PEAK_TLOPS,
               "source": os.path.relpath(COUNTER_SUMMARY, ROOT)}
    out = {
        "metric": "LLVQ dequant-GEMV GB/s (packed weights)", "value": gbs, "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": "Llama-3-8B-shaped layer set, dequant-GEMV batch 1: q/o 4096x4096, k/v 1024x4096, gate/up 14336x4096, "
                               "down 4096x14336 (K padded to a multiple of 24), 48-bit indices uniform over Lambda24(13) + fp16 gain per "
                               "block, x fp16, y fp32; q/k/v and gate/up through llvq_matmul_multi (4 launches per step); ring of %d "
                               "distinct transformer blocks (%.0f MB)" % (args.ring, args.ring * nblk * 8 / 1e6),
                   "M": M, "blocks_per_step": nblk, "launches_per_step": n_launch, "packed_bytes_per_step": BYTES_PER_BLOCK * nblk},
        "pct_hbm_peak": 100.0 * gbs / HBM_PEAK_GBS,
        "hbm_copy_measured_GBs": copy_gbs, "pct_of_measured_copy": 100.0 * gbs / copy_gbs,
        "decoded_weights_per_s": 24.0 * nblk / (ms_per_step * 1e-3),
        "blocks_per_s": nblk / (ev_ms * 1e-3),
        "max_rel_err_vs_oracle": err,
        # HBM roofline of the matmul kernel: algorithmic bytes (8 per block) of the launches of a step against their
        # HIP-event time, per launch.  The kernel is in fact bound by the vector-ALU and LDS-gather work of the index
        # decode, far below this roof: that view of the same launches is under "alu".
        "roofline": {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                     "traffic": (traffic / n_launch) if traffic else None,
                     "kernel": "matmul_kernel<U48,f16> (the four launches of a step: q/k/v, o, gate/up, down)",
                     "kernel_ms": ev_ms / n_launch,
                     "algorithmic_bytes_per_launch": BYTES_PER_BLOCK * nblk / n_launch,
                     "launches_timed": args.steps * n_launch,
                     "alu": alu},
        "single_layer_4096x4104": single,
        "layer_set_batch16": batch16,
        "llama3_70b_layer_set": set70b,
        "prefill_14336x4104_m1024": prefill,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


MFMA_PEAK_TFLOPS = 2500.0      # dense fp16 / bf16 matrix-core peak of MI355X


def prefill_layer(q, synth, torch, dev, ring):
    """the fused dequant-GEMM (llvq_matmul, no workspace, no library GEMM) on the gate layer of block 0 at M = 1024, fp16
    activations: HIP-event time per call and the share of the matrix cores' dense fp16 peak"""
    import numpy as np
    for (group, idxs, gains, Ns, KB, _) in ring[0]:
        if "gate" in group:
            i = list(group).index("gate")
            idx, gain, N = idxs[i], gains[i], Ns[i]
            break
    M = 1024
    x = torch.from_numpy(synth.activations(synth.rng_for(3, 990), M, 24 * KB).astype(np.float16)).to(dev)
    y = torch.empty((M, N), dtype=torch.float32, device=dev)
    for _ in range(3):
        q.llvq_matmul(x, idx, gain, N, KB, out=y)
    torch.cuda.synchronize()
    reps = 10
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        q.llvq_matmul(x, idx, gain, N, KB, out=y)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    tf = 2.0 * M * N * KB * 24 / (ms * 1e-3) / 1e12
    return {"workload": "%d x %d, M = %d, x fp16, y fp32, fused (weights decoded inside the kernel, once per 512 tokens)" % (N, 24 * KB, M),
            "ms_per_call_events": ms, "TFLOPs": tf, "roofline": {"bound": "mfma", "achieved": tf, "peak": MFMA_PEAK_TFLOPS,
                                                                  "unit": "TFLOP/s", "frac": tf / MFMA_PEAK_TFLOPS}}


def layer_set_pass(q, synth, torch, dev, ring, x_host, nblk, steps, warmup):
    """the ring of transformer blocks with other activations (M rows): HIP-event time per step"""
    import numpy as np
    d_x = {KB: torch.from_numpy(x.astype(np.float16)).to(dev) for KB, x in x_host.items()}
    M = next(iter(x_host.values())).shape[0]
    outs = [[[torch.empty((M, N), dtype=torch.float32, device=dev) for N in Ns] for (_, _, _, Ns, _, _) in blk] for blk in ring]

    def step(i):
        b = i % len(ring)
        for (launch, ys) in zip(ring[b], outs[b]):
            _, idxs, gains, Ns, KB, _ = launch
            q.llvq_matmul_multi(d_x[KB], idxs, gains, Ns, KB, outs=ys)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        step(warmup + i)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    return {"workload": "the same ring of transformer blocks at batch %d (llvq_matmul_multi, 4 launches per step)" % M, "M": M, "steps": steps,
            "warmup": warmup, "ms_per_step_events": ms, "packed_GBs_events": BYTES_PER_BLOCK * nblk / ms / 1e6,
            "blocks_per_s": nblk / (ms * 1e-3)}


def llama70b_set(q, synth, torch, dev, steps, warmup):
    import numpy as np
    shapes = synth.LLAMA3_70B
    mats = {}
    nblk = 0
    for i, (name, (N, K)) in enumerate(shapes.items()):
        KB = synth.blocks_per_row(K)
        r = synth.rng_for(5, i)
        mats[name] = (torch.from_numpy(synth.pack_u48(synth.indices(r, (N, KB))).reshape(-1)).to(dev),
                      torch.from_numpy(synth.gains(r, (N, KB)).reshape(-1)).to(dev), N, KB)
        nblk += N * KB
    launches = []
    for group in GROUPS:
        ms_ = [mats[g] for g in group]
        KB = ms_[0][3]
        x = torch.from_numpy(synth.activations(synth.rng_for(5, 900 + KB % 997), 1, 24 * KB).astype(np.float16)).to(dev)
        launches.append((x, [m[0] for m in ms_], [m[1] for m in ms_], [m[2] for m in ms_], KB,
                         [torch.empty((1, m[2]), dtype=torch.float32, device=dev) for m in ms_]))

    def step():
        for (x, idxs, gains, Ns, KB, ys) in launches:
            q.llvq_matmul_multi(x, idxs, gains, Ns, KB, outs=ys)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    return {"workload": "Llama-3-70B-shaped layer set, batch 1: q/o 8192x8192, k/v 1024x8192, gate/up 28672x8192, down 8192x28672; one transformer "
                        "block (%.1f MB packed, larger than the last-level cache), 4 launches per step" % (nblk * 8 / 1e6),
            "blocks_per_step": nblk, "steps": steps, "warmup": warmup, "ms_per_step_events": ms,
            "packed_GBs_events": BYTES_PER_BLOCK * nblk / ms / 1e6, "hbm_frac_events": BYTES_PER_BLOCK * nblk / ms / 1e6 / HBM_PEAK_GBS,
            "blocks_per_s": nblk / (ms * 1e-3)}


def single_layer(q, synth, torch, dev, args, oracle):
    """llvq_matmul at batch 1 on one rows x 4104 layer (the shape of the paper's App. C table), ring of distinct layers."""
    import numpy as np
    N, K = args.rows, 4096
    KB = synth.blocks_per_row(K)
    nblk = N * KB
    rng = synth.rng_for(2, 0)
    idx0 = synth.indices(rng, (N, KB))
    gain0 = synth.gains(rng, (N, KB))
    x0 = synth.activations(rng, 1, K)
    ring_idx, ring_gain = [], []
    for l in range(args.single_layers):
        if l == 0:
            idx, gain = idx0, gain0
        else:
            r = synth.rng_for(2, l)
            idx, gain = synth.indices(r, (N, KB)), synth.gains(r, (N, KB))
        ring_idx.append(torch.from_numpy(synth.pack_u48(idx).reshape(-1)).to(dev))
        ring_gain.append(torch.from_numpy(gain.reshape(-1)).to(dev))
    d_x = torch.from_numpy(x0.astype(np.float16)).to(dev)
    y = torch.empty((1, N), dtype=torch.float32, device=dev)
    steps, warmup = max(args.steps, 20), max(args.warmup, 5)

    def step(i):
        l = i % args.single_layers
        q.llvq_matmul(d_x, ring_idx[l], ring_gain[l], N, KB, out=y)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(steps):
        step(warmup + i)
    e1.record()
    torch.cuda.synchronize()
    wall_us = (time.perf_counter() - t0) * 1e6 / steps
    ev_us = e0.elapsed_time(e1) * 1e3 / steps
    step(0)
    rows = np.arange(0, N, 64)
    ref = oracle.matmul(x0, idx0[rows], gain0[rows])
    err = float(np.abs(y.cpu().numpy().astype(np.float64)[:, rows] - ref).max() / np.abs(ref).max())
    return {"workload": "dequant-GEMV batch 1, W %dx4104, ring of %d distinct layers, one llvq_matmul launch per step" % (N, args.single_layers),
            "steps": steps, "warmup": warmup, "us_per_launch_wall": wall_us, "us_per_launch_events": ev_us,
            "packed_GBs_events": BYTES_PER_BLOCK * nblk / ev_us / 1e3, "hbm_frac_events": BYTES_PER_BLOCK * nblk / ev_us / 1e3 / HBM_PEAK_GBS,
            "blocks": nblk, "max_rel_err_vs_oracle": err,
            "paper_context": "the paper's App. C prints 11.94 us for a single-shell 24-bit code of this shape on an unnamed NVIDIA GPU"}


def extra_layer_set(q, synth, torch, dev):
    """One pass over the seven linear layers of a Llama-3-8B-shaped block (four distinct copies) and of a
    Llama-3-70B-shaped block, distinct buffers, batch 1; then the bulk decode of the 70B-shaped block to bf16 (stderr)."""
    import numpy as np
    for label, shapes, copies in (("llama3-8b", synth.LLAMA3_8B, 4), ("llama3-70b", synth.LLAMA3_70B, 1)):
        layers = []
        tot = 0
        for rep in range(copies):
            for i, (name, (N, K)) in enumerate(shapes.items()):
                KB = synth.blocks_per_row(K)
                r = synth.rng_for(3 if copies > 1 else 5, 10 * rep + i)
                idx = torch.from_numpy(synth.pack_u48(synth.indices(r, (N, KB))).reshape(-1)).to(dev)
                gain = torch.from_numpy(synth.gains(r, (N, KB)).reshape(-1)).to(dev)
                x = torch.from_numpy(synth.activations(r, 1, K).astype(np.float16)).to(dev)
                y = torch.empty((1, N), dtype=torch.float32, device=dev)
                layers.append((name, x, idx, gain, N, KB, y))
                tot += N * KB
        for _ in range(2):
            for (_, x, idx, gain, N, KB, y) in layers:
                q.llvq_matmul(x, idx, gain, N, KB, out=y)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 5
        e0.record()
        for _ in range(reps):
            for (_, x, idx, gain, N, KB, y) in layers:
                q.llvq_matmul(x, idx, gain, N, KB, out=y)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        print("%s layer set x%d (%.1f MB packed): %.3f ms per pass, %.1f GB/s packed, %.2f G blocks/s" %
              (label, copies, tot * 8 / 1e6, ms, tot * 8 / ms / 1e6, tot / ms / 1e6), file=sys.stderr)
        if copies > 1:
            # the same layer set at batch 16 (the batched-decode kernel on the matrix cores)
            x16 = {}
            for (name, x, idx, gain, N, KB, y) in layers:
                if KB not in x16:
                    r = synth.rng_for(3, 900 + KB)
                    x16[KB] = torch.from_numpy(synth.activations(r, 16, x.shape[1]).astype(np.float16)).to(dev)
            y16 = [torch.empty((16, l[4]), dtype=torch.float32, device=dev) for l in layers]
            for (l, yy) in zip(layers, y16):
                q.llvq_matmul(x16[l[5]], l[2], l[3], l[4], l[5], out=yy)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                for (l, yy) in zip(layers, y16):
                    q.llvq_matmul(x16[l[5]], l[2], l[3], l[4], l[5], out=yy)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps
            print("%s layer set x%d at batch 16: %.3f ms per pass, %.1f GB/s packed, %.2f G blocks/s" %
                  (label, copies, ms, tot * 8 / ms / 1e6, tot / ms / 1e6), file=sys.stderr)
            # and with q/k/v and gate/up going through llvq_matmul_multi (one batched-decode launch each)
            per16 = len(shapes)
            multi16 = []
            for rep in range(copies):
                ls_all = layers[rep * per16:(rep + 1) * per16]
                ys_all = y16[rep * per16:(rep + 1) * per16]
                blk = {l[0]: (l, yy) for l, yy in zip(ls_all, ys_all)}
                for group in (("q", "k", "v"), ("o",), ("gate", "up"), ("down",)):
                    ls = [blk[g][0] for g in group]
                    multi16.append((x16[ls[0][5]], [l[2] for l in ls], [l[3] for l in ls], [l[4] for l in ls], ls[0][5],
                                    [blk[g][1] for g in group]))
            for (xx, idxs, gains, Ns, KB, ys) in multi16:
                q.llvq_matmul_multi(xx, idxs, gains, Ns, KB, outs=ys)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                for (xx, idxs, gains, Ns, KB, ys) in multi16:
                    q.llvq_matmul_multi(xx, idxs, gains, Ns, KB, outs=ys)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps
            print("%s layer set x%d at batch 16, llvq_matmul_multi for q/k/v and for gate/up: %.3f ms per pass, %.2f G blocks/s" %
                  (label, copies, ms, tot / ms / 1e6), file=sys.stderr)
            del x16, y16, multi16
        # the same weights with the layers that share their input stored as one matrix (q, k, v rows concatenated;
        # gate, up likewise): four launches per block instead of seven, same bytes
        fused = []
        per = len(shapes)
        for rep in range(copies):
            blk = {l[0]: l for l in layers[rep * per:(rep + 1) * per]}
            for group in (("q", "k", "v"), ("o",), ("gate", "up"), ("down",)):
                ls = [blk[g] for g in group]
                Nt = sum(l[4] for l in ls)
                fused.append((ls[0][1], torch.cat([l[2] for l in ls]), torch.cat([l[3] for l in ls]), Nt, ls[0][5],
                              torch.empty((1, Nt), dtype=torch.float32, device=dev)))
        for (x, idx, gain, N, KB, y) in fused:
            q.llvq_matmul(x, idx, gain, N, KB, out=y)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            for (x, idx, gain, N, KB, y) in fused:
                q.llvq_matmul(x, idx, gain, N, KB, out=y)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        print("%s layer set x%d, q/k/v and gate/up stored as one matrix each (4 launches per block): %.3f ms per pass, "
              "%.2f G blocks/s" % (label, copies, ms, tot / ms / 1e6), file=sys.stderr)
        del fused
        # the same with the separate matrices left as they are and llvq_matmul_multi running q/k/v and gate/up in one launch each
        multi = []
        for rep in range(copies):
            blk = {l[0]: l for l in layers[rep * per:(rep + 1) * per]}
            for group in (("q", "k", "v"), ("o",), ("gate", "up"), ("down",)):
                ls = [blk[g] for g in group]
                multi.append((ls[0][1], [l[2] for l in ls], [l[3] for l in ls], [l[4] for l in ls], ls[0][5], [l[6] for l in ls]))
        for (x, idxs, gains, Ns, KB, ys) in multi:
            q.llvq_matmul_multi(x, idxs, gains, Ns, KB, outs=ys)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            for (x, idxs, gains, Ns, KB, ys) in multi:
                q.llvq_matmul_multi(x, idxs, gains, Ns, KB, outs=ys)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        print("%s layer set x%d, llvq_matmul_multi for q/k/v and for gate/up (4 launches per block, matrices stored separately): "
              "%.3f ms per pass, %.2f G blocks/s" % (label, copies, ms, tot / ms / 1e6), file=sys.stderr)
        del multi
        if copies == 1:
            outs = [torch.empty((N * KB, 24), dtype=torch.bfloat16, device=dev) for (_, _, _, _, N, KB, _) in layers]
            for (_, _, idx, gain, N, KB, _), o in zip(layers, outs):
                q.llvq_decode(idx, gain, out_dtype=torch.bfloat16, out=o)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                for (_, _, idx, gain, N, KB, _), o in zip(layers, outs):
                    q.llvq_decode(idx, gain, out_dtype=torch.bfloat16, out=o)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps
            print("%s bulk decode of the block to bf16 (%d blocks): %.3f ms, %.2f G blocks/s, read+write %.1f GB/s" %
                  (label, tot, ms, tot / ms / 1e6, tot * 56 / ms / 1e6), file=sys.stderr)
            del outs
            # decode-only throughput on more than 2^26 blocks in one call: the block's indices twice (union of shells), and
            # as many indices uniform over the first shell (the distribution of the decode-unit configuration)
            big = torch.cat([l[2] for l in layers] * 2)
            nbig = big.numel() // 6
            out8 = torch.empty((nbig, 24), dtype=torch.int8, device=dev)
            first = synth.pack_u48(synth.rng_for(1, 7).integers(0, 196560, size=1 << 22, dtype=np.uint64)).reshape(-1)
            first = torch.from_numpy(first).to(dev).repeat(nbig // (1 << 22) + 1)[:nbig * 6].contiguous()
            for what, src in (("union of shells 2..13", big), ("first shell", first)):
                q.llvq_decode_i8(src, out=out8)
                torch.cuda.synchronize()
                e0.record()
                for _ in range(reps):
                    q.llvq_decode_i8(src, out=out8)
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1) / reps
                print("decode to int8, %d blocks (%s) in one call: %.3f ms, %.2f G blocks/s, read+write %.1f GB/s" %
                      (nbig, what, ms, nbig / ms / 1e6, nbig * 30 / ms / 1e6), file=sys.stderr)
            del big, first, out8
        del layers


SWEEP_SHAPES = ((1, 1), (256, 1), (256, 64), (256, 171), (512, 171), (1024, 171), (2048, 171), (4096, 171), (8192, 171),
                (4096, 342), (4096, 683))


def extra_sweep(q, synth, torch, dev):
    """Batch-1 product on N x 24*KB layers from one block to 2.8 M blocks, same buffers every launch (hot cache): shows
    the fixed cost of a launch and the slope per block.  HIP-event times of launches this short include the host's
    launch rate; kernel durations come from a kernel trace of the same run."""
    import numpy as np
    rng = synth.rng_for(7, 1)
    for (N, KB) in SWEEP_SHAPES:
        idx = torch.from_numpy(synth.pack_u48(synth.indices(rng, (N, KB))).reshape(-1)).to(dev)
        gain = torch.from_numpy(synth.gains(rng, (N, KB)).reshape(-1)).to(dev)
        x = torch.from_numpy(synth.activations(rng, 1, 24 * KB).astype(np.float16)).to(dev)
        y = torch.empty((1, N), dtype=torch.float32, device=dev)
        for _ in range(20):
            q.llvq_matmul(x, idx, gain, N, KB, out=y)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(300):
            q.llvq_matmul(x, idx, gain, N, KB, out=y)
        e1.record()
        torch.cuda.synchronize()
        print("sweep N=%5d KB=%4d (%8d blocks): %7.2f us per launch" % (N, KB, N * KB, e0.elapsed_time(e1) / 300 * 1e3), file=sys.stderr)


def extra_shapes(q, synth, torch, dev):
    """Batch 16, prefill and bulk-decode timings on one gate/up-shaped layer (14336 x 4104), to stderr."""
    import numpy as np
    N, K = synth.LLAMA3_8B["gate"]
    KB = synth.blocks_per_row(K)
    r = synth.rng_for(3, 77)
    idx = torch.from_numpy(synth.pack_u48(synth.indices(r, (N, KB))).reshape(-1)).to(dev)
    gain = torch.from_numpy(synth.gains(r, (N, KB)).reshape(-1)).to(dev)

    def timeit(f, reps=20):
        for _ in range(3):
            f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            f()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3

    for M, dt in ((1, torch.float16), (16, torch.float16), (64, torch.bfloat16), (256, torch.bfloat16), (1024, torch.bfloat16)):
        x = torch.from_numpy(synth.activations(r, M, K)).to(dev).to(dt)
        y = torch.empty((M, N), dtype=torch.float32, device=dev)
        us = timeit(lambda: q.llvq_matmul(x, idx, gain, N, KB, out=y))
        print("matmul %dx%d M=%-4d %s: %9.2f us  %.1f GB/s packed  %.1f TFLOP/s" %
              (N, 24 * KB, M, str(dt).split(".")[-1], us, N * KB * 8 / us / 1e3, 2.0 * M * N * KB * 24 / us / 1e6), file=sys.stderr)
    n = N * KB
    for name, dt in (("int8", None), ("float16", torch.float16), ("bfloat16", torch.bfloat16), ("float32", torch.float32)):
        if dt is None:
            out = torch.empty((n, 24), dtype=torch.int8, device=dev)
            us = timeit(lambda: q.llvq_decode_i8(idx, out=out))
        else:
            out = torch.empty((n, 24), dtype=dt, device=dev)
            us = timeit(lambda: q.llvq_decode(idx, gain, out_dtype=dt, out=out))
        ob = 24 * out.element_size()
        print("bulk decode -> %-8s %d blocks: %9.2f us  %.2f G blocks/s  read+write %.1f GB/s" %
              (name, n, us, n / us / 1e3, n * (8 + ob) / us / 1e3), file=sys.stderr)
    # encoder side of the index map on the decoded points, then the coded-word layouts (6 B and 3 B per block)
    pts = q.llvq_decode_i8(idx)
    back = torch.empty((n, 6), dtype=torch.uint8, device=dev)
    us = timeit(lambda: q.llvq_encode(pts, out=back))
    same = bool(torch.equal(back.reshape(-1), idx))
    print("encode int8 points -> index %d blocks: %9.2f us  %.2f G blocks/s  read+write %.1f GB/s  round trip %s" %
          (n, us, n / us / 1e3, n * 30 / us / 1e3, "exact" if same else "MISMATCH"), file=sys.stderr)
    # the same product with a caller workspace: dequantise once, then the library GEMM (after the bulk-decode timings:
    # kernels timed right after a long library GEMM run several microseconds slower, presumably at a lower clock)
    ws = torch.empty(N * KB * 24, dtype=torch.bfloat16, device=dev)
    for M in (256, 1024):
        x = torch.from_numpy(synth.activations(r, M, K)).to(dev).to(torch.bfloat16)
        y = torch.empty((M, N), dtype=torch.float32, device=dev)
        us = timeit(lambda: q.llvq_matmul(x, idx, gain, N, KB, out=y, workspace=ws))
        print("matmul_ws %dx%d M=%-4d bfloat16: %9.2f us  %.1f TFLOP/s (dequantise once + library GEMM)" %
              (N, 24 * KB, M, us, 2.0 * M * N * KB * 24 / us / 1e6), file=sys.stderr)
    del ws
    # quantiser: nearest direction of Lambda_24(13) for Gaussian blocks (one 4096 x 384 slice of a layer)
    from paper_2603_11021_amd import LLVQ_ANGULAR
    nq = 4096 * 16
    wq = torch.from_numpy(r.standard_normal((nq, 24)).astype(np.float32)).to(dev)
    res = []
    us = timeit(lambda: res.append(q.llvq_quantize(wq, LLVQ_ANGULAR)) or res.clear(), reps=3)
    qp, qi, qs = q.llvq_quantize(wq, LLVQ_ANGULAR)
    cosm = float((qs / wq.norm(dim=1)).mean())
    print("quantize (angular search + encode) %d blocks: %9.1f us  %.3f M blocks/s  mean cosine %.4f" %
          (nq, us, nq / us, cosm), file=sys.stderr)
    # the same 65,536 blocks as a 4096 x 384 layer through the block-wise loop with Hessian corrections
    Kq = 384
    Xc = r.standard_normal((4 * Kq, Kq)) * np.linspace(1.0, 6.0, Kq)[None, :]
    Hq = Xc.T @ Xc / Xc.shape[0] + 0.01 * np.eye(Kq)
    Gq = np.linalg.inv(Hq)
    Uq = torch.from_numpy(np.linalg.cholesky((Gq + Gq.T) / 2).T.astype(np.float32).copy()).to(dev)
    W0 = wq.reshape(4096, Kq).clone()
    Wg = W0.clone()
    def gptq_once():
        Wg.copy_(W0)
        q.llvq_gptq_quantize(Wg, Uq)
    us = timeit(gptq_once, reps=3)
    print("gptq loop 4096 x %d (16 block columns, search + encode + gain reset + BLAS propagation): %9.1f us  %.3f M blocks/s" %
          (Kq, us, nq / us), file=sys.stderr)
    x = torch.from_numpy(synth.activations(r, 1, K)).to(dev).to(torch.float16)
    y = torch.empty((1, N), dtype=torch.float32, device=dev)
    lut = torch.from_numpy(synth.chi_gain_levels(1, scale=0.02)).to(dev)
    w47 = torch.from_numpy(synth.pack_u48(r.integers(0, 1 << 48, size=n, dtype=np.uint64) % np.uint64(1 << 47) |
                                          (r.integers(0, 2, size=n, dtype=np.uint64) << np.uint64(47))).reshape(-1)).to(dev)
    us = timeit(lambda: q.llvq_matmul_coded(x, w47, N, KB, 47, gain_lut=lut, out=y))
    print("matmul %dx%d M=1 coded 47+1 bits (6 B/block): %9.2f us  %.1f GB/s packed  %.2f G blocks/s" %
          (N, 24 * KB, us, n * 6 / us / 1e3, n / us / 1e3), file=sys.stderr)
    packed = q.llvq_repack(idx, gain)
    us = timeit(lambda: q.llvq_matmul_coded(x, packed, N, KB, 48, out=y))
    print("matmul %dx%d M=1 packed words, index + fp16 gain in one aligned 64-bit word (8 B/block): %9.2f us  %.1f GB/s packed  "
          "%.2f G blocks/s" % (N, 24 * KB, us, n * 8 / us / 1e3, n / us / 1e3), file=sys.stderr)
    del packed
    from paper_2603_11021_amd import LLVQ_IDX_U24
    base = q.llvq_shell_offset(3)
    w24 = torch.from_numpy(synth.pack_u24(r.integers(0, q.llvq_shell_offset(4) - base, size=n, dtype=np.uint64)).reshape(-1)).to(dev)
    us = timeit(lambda: q.llvq_matmul_coded(x, w24, N, KB, 24, base, gain=gain, fmt=LLVQ_IDX_U24, out=y))
    print("matmul %dx%d M=1 single shell 3, 24-bit words + fp16 gain (5 B/block): %9.2f us  %.1f GB/s packed  %.2f G blocks/s" %
          (N, 24 * KB, us, n * 5 / us / 1e3, n / us / 1e3), file=sys.stderr)
    # a context for the union up to shell 19 (55-bit indices): the generic decoder with tables in global memory
    q19 = type(q)(19, 0)
    i19 = torch.from_numpy(r.integers(0, q19.num_points, size=n, dtype=np.uint64).view(np.int64)).to(dev)
    out8 = torch.empty((n, 24), dtype=torch.int8, device=dev)
    us = timeit(lambda: q19.llvq_decode_i8(i19, out=out8), reps=5)
    print("m_max = 19 (1,457 classes, 55-bit indices): decode to int8 %d blocks: %9.2f us  %.2f G blocks/s" % (n, us, n / us / 1e3), file=sys.stderr)
    us = timeit(lambda: q19.llvq_matmul(x, i19, gain, N, KB, out=y), reps=5)
    print("m_max = 19: matmul %dx%d M=1: %9.2f us  %.2f G blocks/s" % (N, 24 * KB, us, n / us / 1e3), file=sys.stderr)
    del q19, i19, out8
    # the configuration of the paper's own timing table (App. C): 4096 x 4104, single shell, 24-bit words, constant norm
    Np, KBp = 4096, 171
    one = torch.ones(1, dtype=torch.float16, device=dev)
    ring = [torch.from_numpy(synth.pack_u24(r.integers(0, q.llvq_shell_offset(4) - base, size=Np * KBp, dtype=np.uint64)).reshape(-1)).to(dev)
            for _ in range(64)]
    xp = torch.from_numpy(synth.activations(r, 1, 4096)).to(dev).to(torch.float16)
    yp = torch.empty((1, Np), dtype=torch.float32, device=dev)
    turn = [0]
    def paper_cfg():
        turn[0] += 1
        q.llvq_matmul_coded(xp, ring[turn[0] % 64], Np, KBp, 24, base, gain_lut=one, fmt=LLVQ_IDX_U24, out=yp)
    us = timeit(paper_cfg, reps=256)
    print("matmul 4096x4104 M=1 single shell 3, 24-bit words, one gain level (3 B/block, ring of 64 layers): %9.2f us "
          "(the paper's App. C prints 11.94 us for this configuration on an unnamed NVIDIA GPU)" % us, file=sys.stderr)


if __name__ == "__main__":
    main()
