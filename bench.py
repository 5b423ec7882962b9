#!/usr/bin/env python3
"""Throughput of the DES sparse forward+backward step on one MI355X.

A step is one pass of the whole hot path over one synthetic batch that is already resident in
HBM: des_table_find (inserting unseen IDs where the workload grows) -> des_partial_forward
(LR, FM, pooled partials of all K shards) -> des_aggregate_forward (the three aggregations + fm2) ->
des_backward_update_{adagrad,sgd} (sort by row, duplicate merge, fused row update).  Upstream
gradients are seeded random tensors of the real shapes (the loss head is outside the path).

Prints ONE JSON line.  `value` = lookups (CSR entries) per second; samples/s is alongside.
The roofline object is for the kernel with the largest share of the step, timed with HIP
events on the launch stream in a second pass over the same steps; the CPU baseline is the
oracle, single-threaded, on a bounded sample of the same workload.
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

HBM_PEAK_GBS = 8000.0


def batch_stats(keys: np.ndarray, short_max: int = 32, chunk: int = 512):
    """Input statistics the byte model needs: distinct keys and how the entries split into short
    (<= short_max occurrences) and long merge segments (cut into chunks of `chunk` entries)."""
    _, counts = np.unique(keys, return_counts=True)
    long_ = counts > short_max
    return {
        "U": int(counts.size), "U_long": int(long_.sum()), "U_short": int((~long_).sum()),
        "n_long": int(counts[long_].sum()), "n_short": int(counts[~long_].sum()),
        "n_chunks": int(((counts[long_] + chunk - 1) // chunk).sum()),
    }


def algorithmic_bytes(w, nnz, st, sort_passes, state_mult):
    """Compulsory bytes per step of each kernel (what the method itself has to move)."""
    B, F, D, K = w.B, w.F, w.D, w.K
    R = D + 1
    n, U = nnz, st["U"]
    gp = 4.0 * B * F * D                      # g_pool, each bag row once
    return {
        "table_probe": 8 * n + 4 * n + 16 * U,
        "forward_gather_pool": 8 * n + 4 * n + 4 * (B * F + 1) + 4 * R * U + 4 * K * B * (D + 2) + 4 * B * F * D,
        "aggregate_partials": 4 * (K + 1) * B * (D + 2),
        "fm_finalize": 4 * B * (D + 2),
        "backward_expand": 4 * n + 4 * (B * F + 1) + 8 * n,
        "sort_histogram": sort_passes * 4 * n,
        "sort_scatter": sort_passes * 16 * n,
        "backward_segment_heads": 8 * n + 8 * U,
        "backward_short_update": 4 * st["n_short"] + 8 * U + gp * st["n_short"] / max(n, 1) + 4 * B * (D + 2) * st["n_short"] / max(n, 1)
                                 + 2 * state_mult * 4 * R * st["U_short"],
        "backward_long_partial": 4 * st["n_long"] + gp * st["n_long"] / max(n, 1) + 4 * B * (D + 2) * st["n_long"] / max(n, 1)
                                 + 8 * (D + 4) * st["n_chunks"],
        "backward_long_final": 8 * (D + 4) * st["n_chunks"] + 2 * state_mult * 4 * R * st["U_long"],
    }


PROFILE_TAG = {0: "tiny_lr_fm", 1: "dlrm_pooled", 2: "deepfm", 3: "streaming", 4: "large_table"}


def measured_traffic(index: int, label: str):
    """(HBM bytes per launch of kernel `label`, commit the counters were collected at) from the committed
    rocprofv3 counter summary of this workload (profiles/<tag>_hbm_traffic.md: columns fetch MB / write MB, and a
    line "Measured at commit: <id>"), or (None, None)."""
    path = os.path.join(ROOT, "profiles", f"{PROFILE_TAG[index]}_hbm_traffic.md")
    if not os.path.exists(path):
        return None, None
    total, seen, commit = 0.0, False, None
    for line in open(path):
        if line.lower().startswith("measured at commit:"):
            commit = line.split(":", 1)[1].strip().strip("`")
        cells = [c.strip() for c in line.split("|")]
        if len(cells) >= 6 and cells[2] == label:
            try:
                total += (float(cells[3]) + float(cells[4])) * 1e6
                seen = True
            except ValueError:
                pass
    return (int(total), commit) if seen else (None, commit)


def cpu_baseline(w, batch, sample_B, opt_code):
    """The oracle, as it stands, on the first `sample_B` samples of batch 0 with a table that
    holds exactly the IDs those samples touch (pre-inserted head with initialiser weights; the
    rest is inserted by the timed lookup, as on the GPU).  Two legs: the plain single-threaded
    build on half of the sample, then the OpenMP build of the same source (lookups split over entries,
    forward over samples, merge + update over distinct rows) on the whole sample with the threads
    the box gives this process."""
    import oracle
    F, D = w.F, w.D
    rng = np.random.default_rng(1)
    host_cores = os.cpu_count() or 1
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = host_cores

    def leg(openmp, nb):
        threads = oracle.use_openmp(openmp)
        end = int(batch.offsets[nb * F])
        keys, offsets = batch.keys[:end].copy(), batch.offsets[:nb * F + 1].copy()
        if batch.ranks is not None:
            head = np.unique(keys[batch.ranks[:end] <= w.preinsert])
        else:
            head = np.unique(keys)
        t = oracle.Table(D, head.size + np.unique(keys).size + 16, seed=w.seed, init_scale=w.init_std)
        t.insert(head)
        g_lr = (rng.standard_normal(nb) / w.B).astype(np.float32)
        g_fm = (rng.standard_normal(nb) / w.B).astype(np.float32)
        g_pool = (rng.standard_normal((nb, F, D)) / w.B).astype(np.float32)
        t0 = time.perf_counter()
        rows = t.find(keys, insert_missing=True)
        P = t.partial_forward(nb, F, keys, offsets, rows, w.K, 0, None, pool=False)
        pool = t.partial_forward(nb, F, keys, offsets, rows, 1, 0, None, lr=False, fm=False, pool=True)["P_pool"]
        A_sum = oracle.aggregate(P["P_sum"]); A_sq = oracle.aggregate(P["P_sq"]); oracle.aggregate(P["P_lr"])
        oracle.aggregate(pool)
        oracle.fm_finalize(A_sum, A_sq)
        t.backward_update(nb, F, offsets, rows, g_lr, g_fm, A_sum.astype(np.float32), g_pool, opt_code, w.lr,
                          w.eps if w.eps else 1e-8)
        dt = time.perf_counter() - t0
        t.close()
        return {"value": end / dt, "unit": "lookups/s", "cores": threads, "samples_per_s": nb / dt,
                "sample": f"first {nb} of {w.B} samples of batch 0 ({end} lookups, {dt:.2f} s); table holds only the "
                          f"{head.size} pre-inserted IDs these samples touch, initialiser weights"}

    nb = min(sample_B, w.B)
    single = leg(False, max(1, nb // 2))
    try:
        multi = leg(True, nb)
    finally:
        oracle.use_openmp(False)
    out = dict(multi)
    out.update({"kind": "oracle", "host_cores": host_cores, "usable_cores": usable,
                "build": "oracle/des_oracle.c, gcc -O2 -fopenmp", "single_thread": single})
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=4, help="index into the benchmark configurations (0-4)")
    ap.add_argument("--also", type=str, default=None,
                    help="comma-separated further configurations measured after the main one and reported under "
                         "\"also\" (default: 0,1,2,3 when the main one is 4, so that one line carries all five; "
                         "\"none\" to skip)")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (debugging only)")
    ap.add_argument("--batches", type=int, default=0, help="distinct pre-generated batches (default 8, fewer for huge ones)")
    ap.add_argument("--cpu-lookups", type=float, default=1e7,
                    help="size of the oracle's timed sample, in lookups (all-cores leg; the single-thread leg takes "
                         "half of it: about 7 s of CPU work each)")
    ap.add_argument("--dnn-hidden", type=int, default=256,
                    help="width H of the first fully-connected layer measured after the sparse step and reported "
                         "under \"dnn_layer\" (0 to skip)")
    ap.add_argument("--model", type=str, default="deepfm", choices=["none", "lr", "fm", "wd", "deepfm", "dcn"],
                    help="after the sparse steps, also time whole training steps of this model (tower widths "
                         "--dnn-hidden and half of it) on the main workload; reported under \"model_step\"")
    ap.add_argument("--policy", type=str, default="key", choices=["key", "field"],
                    help="shard rule of the K logical shards: hash of the ID (default) or field index mod K "
                         "(the placement of the paper's Section 5)")
    ap.add_argument("--step-series", action="store_true",
                    help="also report every timed step's duration (events on the main stream) under \"series_ms\"")
    ap.add_argument("--graph", action="store_true",
                    help="record the step of every distinct batch into a HIP graph and time replays (not for the "
                         "streaming workload, whose every step has a new batch)")
    ap.add_argument("--no-overlap", action="store_true",
                    help="run the whole step on one stream (default: the backward pass's sort runs on a second "
                         "stream beside the forward pass)")
    ap.add_argument("--tower", type=str, default=None,
                    help="comma-separated hidden widths of the model step's tower (default: dnn-hidden, dnn-hidden/2)")
    ap.add_argument("--cross-layers", type=int, default=2, help="cross layers of --model dcn")
    ap.add_argument("--no-cross", action="store_true",
                    help="skip the DCN cross layer timed at the main workload's shape (reported under \"cross_layer\")")
    ap.add_argument("--no-compact", action="store_true",
                    help="skip the in-place eviction of half of the main workload's rows, timed last (\"table_compact\")")
    ap.add_argument("--only", type=str, default=None, choices=["cross", "dnn"],
                    help="time only the cross network or only the first fully-connected layer at the workload's shape "
                         "(no table is built; for profiling runs of those kernels)")
    ap.add_argument("--no-ceiling", action="store_true",
                    help="skip the access-pattern ceilings (row gather and row read-modify-write alone on the workload's "
                         "index streams), reported under \"ceilings\"")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-kernel-pass", action="store_true", help="skip the per-kernel timing pass (profiling runs)")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (reference reading for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (K logical shards on one device); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    if args.only:
        if args.calib_copy_mib > 0:
            n = args.calib_copy_mib << 20
            a, b = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1), torch.empty(n, dtype=torch.uint8, device="cuda")
            b.copy_(a)
            torch.cuda.synchronize()
            del a, b
        key = "cross_layer" if args.only == "cross" else "dnn_layer"
        print(json.dumps({key: (run_cross_layer if args.only == "cross" else run_dnn_layer)(args, args.config)}))
        return
    out = run_workload(args, args.config, cpu=not args.no_cpu)
    also = args.also if args.also is not None else ("0,1,2,3" if args.config == 4 and args.scale == 1.0 else "none")
    if also != "none":
        out["also"] = []
        for idx in [int(x) for x in also.split(",") if x.strip()]:
            torch.cuda.empty_cache()
            r = run_workload(args, idx, cpu=False)
            out["also"].append({k: r[k] for k in ("value", "unit", "samples_per_s", "ms_per_step", "steps", "warmup",
                                                  "config", "roofline", "kernels", "table_migrate", "insert_heavy_step", "ceilings")
                                if k in r})
    if args.dnn_hidden > 0:
        torch.cuda.empty_cache()
        out["dnn_layer"] = run_dnn_layer(args, args.config)
    if not args.no_cross:
        torch.cuda.empty_cache()
        out["cross_layer"] = run_cross_layer(args, args.config)
    print(json.dumps(out))


FP32_MFMA_PEAK_TFLOPS = 157.3


def run_dnn_layer(args, index):
    """The first fully-connected layer under DES at the workload's shape (outside `value`: it is the
    dense step that follows the sparse path): K per-shard partials + their aggregation, then the
    backward products g_pool = dY W^T and dW = V dY.  Timed per kernel with HIP events on the launch
    stream; flops = 2*B*F*D*H per product, against the dense fp32 matrix-core peak."""
    import torch
    from paper_1909_04823_amd import des, synth
    w = synth.workload(index, scale=args.scale)
    B, F, D, K, H = w.B, w.F, w.D, w.K, args.dnn_hidden
    gen = torch.Generator(device="cuda"); gen.manual_seed(7)
    pool = torch.randn((B, F, D), device="cuda", generator=gen) * 0.05
    W = torch.randn((F * D, H), device="cuda", generator=gen) / float(np.sqrt(F * D))
    dY = torch.randn((B, H), device="cuda", generator=gen) * 0.01
    Yp = torch.empty((K, B, H), device="cuda"); Y = torch.empty((B, H), device="cuda")
    g_pool = torch.empty((B, F, D), device="cuda"); dW = torch.empty((F * D, H), device="cuda")
    ws = torch.empty(des.dnn_backward_bytes(B, F, D, H), dtype=torch.uint8, device="cuda")

    def layer():
        des.dnn_partial_forward(pool, W, K, out=Yp)
        des.aggregate_partials(Yp, Y)
        des.dnn_backward(pool, W, dY, g_pool, dW, ws)

    reps = max(3, min(args.steps, 10))
    for _ in range(2):
        layer()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        layer()
    torch.cuda.synchronize()
    ms = 1e3 * (time.perf_counter() - t0) / reps
    des.profile_enable(True)
    for _ in range(reps):
        layer()
    prof = des.profile_read()
    des.profile_enable(False)
    flops = 2.0 * B * F * D * H
    kernels = {}
    for name, (launches, total_ms) in prof.items():
        per = total_ms / reps
        e = {"launches_per_pass": launches / reps, "ms_per_pass": round(per, 4)}
        if name.startswith("dnn_") and per > 0:
            e["TFLOPs"] = round(flops / (per * 1e-3) / 1e12, 2)
            e["frac_of_fp32_mfma_peak"] = round(e["TFLOPs"] / FP32_MFMA_PEAK_TFLOPS, 4)
        kernels[name] = e
    assert bool(torch.isfinite(Y).all()) and bool(torch.isfinite(dW).all())
    return {"workload": f"configs[{w.index}] {w.name}", "B": B, "F": F, "D": D, "H": H, "K": K, "dtype": "f32",
            "ms_per_pass": round(ms, 4), "flops_per_product": flops, "peak_TFLOPs": FP32_MFMA_PEAK_TFLOPS,
            "kernels": kernels}


def run_cross_layer(args, index):
    """One DCN cross layer under DES at the workload's shape (outside `value`): per-shard dot products, their
    aggregation, y = x0*s + b + xl, and the backward pass with accumulation into the gradient of x0.
    Streaming work: algorithmic bytes = every [B,d] array once per kernel that needs it, against the HBM peak."""
    import torch
    from paper_1909_04823_amd import des, synth
    w = synth.workload(index, scale=args.scale)
    B, F, D, K = w.B, w.F, w.D, w.K
    d = F * D
    gen = torch.Generator(device="cuda"); gen.manual_seed(9)
    x0 = torch.randn((B, F, D), device="cuda", generator=gen) * 0.3
    xl = torch.randn((B, F, D), device="cuda", generator=gen) * 0.3
    g_y = torch.randn((B, F, D), device="cuda", generator=gen) * 0.01
    wl = torch.randn(d, device="cuda", generator=gen) / float(np.sqrt(d))
    bias = torch.randn(d, device="cuda", generator=gen) * 0.1
    P, s = torch.empty((K, B), device="cuda"), torch.empty(B, device="cuda")
    y, g_xl, g_x0 = torch.empty_like(x0), torch.empty_like(x0), torch.zeros_like(x0)
    dw, db = torch.empty(d, device="cuda"), torch.empty(d, device="cuda")
    ws = torch.empty(des.cross_backward_bytes(B, d), dtype=torch.uint8, device="cuda")

    def layer():
        des.cross_partial(xl, wl, K, out=P)
        des.aggregate_partials(P, s)
        des.cross_apply(x0, xl, s, bias, out=y)
        des.cross_backward(x0, xl, wl, s, g_y, g_xl, g_x0, True, dw, db, ws)

    # the whole network (n layers and the output unit's dot product) in its two-pass form
    n = args.cross_layers
    m = n + 1
    U = torch.randn((m, d), device="cuda", generator=gen) / float(np.sqrt(d))
    nb = torch.randn((n, d), device="cuda", generator=gen) * 0.1 if n else None
    g = torch.randn(B, device="cuda", generator=gen) * 0.01
    nP, nt, ngam, nc = torch.empty((K, B, m), device="cuda"), torch.empty((B, m), device="cuda"), \
        torch.empty((B, m), device="cuda"), torch.empty(B, device="cuda")
    dU, dB = torch.empty_like(U), (torch.empty_like(nb) if n else None)
    nws = torch.empty(des.cross_net_bytes(B, d, n), dtype=torch.uint8, device="cuda")

    def network():
        des.cross_net_partial(x0, U, K, out=nP)
        des.aggregate_partials(nP.view(K, -1), nt.view(-1))
        des.cross_net_forward(nt, U, nb, ngam, nc, nws)
        des.cross_net_backward(x0, U, nb, nt, ngam, g, g_x0, True, dU, dB, nws)

    reps = max(3, min(args.steps, 10))
    for _ in range(2):
        layer()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        layer()
    torch.cuda.synchronize()
    ms = 1e3 * (time.perf_counter() - t0) / reps
    des.profile_enable(True)
    for _ in range(reps):
        layer()
    prof = des.profile_read()
    des.profile_enable(False)
    arr = 4.0 * B * d
    algo = {"cross_partial": arr + 4.0 * d + 4.0 * K * B, "cross_apply": 3 * arr + 4.0 * d + 4.0 * B,
            "cross_backward": 7 * arr + 12.0 * d + 12.0 * B}
    kernels = {}
    for name, (launches, total_ms) in prof.items():
        per = total_ms / reps
        e = {"launches_per_pass": launches / reps, "ms_per_pass": round(per, 4)}
        if name in algo and per > 0:
            e["algorithmic_GB"] = round(algo[name] / 1e9, 3)
            e["GBps"] = round(algo[name] / (per * 1e-3) / 1e9, 1)
            e["frac_of_hbm_peak"] = round(e["GBps"] / HBM_PEAK_GBS, 4)
        kernels[name] = e
    assert bool(torch.isfinite(y).all()) and bool(torch.isfinite(dw).all())
    for _ in range(2):
        network()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        network()
    torch.cuda.synchronize()
    net_ms = 1e3 * (time.perf_counter() - t0) / reps
    des.profile_enable(True)
    for _ in range(reps):
        network()
    prof = des.profile_read()
    des.profile_enable(False)
    net_algo = {"cross_partial": arr + 4.0 * m * d + 4.0 * K * B * m, "cross_backward": 3 * arr + 8.0 * m * d + 8.0 * B * m}
    net_kernels = {}
    for name, (launches, total_ms) in prof.items():
        per = total_ms / reps
        e = {"launches_per_pass": launches / reps, "ms_per_pass": round(per, 4)}
        if name in net_algo and per > 0:
            e["algorithmic_GB"] = round(net_algo[name] / 1e9, 3)
            e["GBps"] = round(net_algo[name] / (per * 1e-3) / 1e9, 1)
            e["frac_of_hbm_peak"] = round(e["GBps"] / HBM_PEAK_GBS, 4)
        net_kernels[name] = e
    assert bool(torch.isfinite(nc).all()) and bool(torch.isfinite(dU).all())
    return {"workload": f"configs[{w.index}] {w.name}", "B": B, "F": F, "D": D, "d": d, "K": K, "dtype": "f32",
            "peak_GBps": HBM_PEAK_GBS,
            "one_layer": {"ms_per_pass": round(ms, 4), "kernels": kernels},
            "whole_network": {"layers": n, "ms_per_pass": round(net_ms, 4), "kernels": net_kernels}}


def run_workload(args, index, cpu):
    import torch
    from paper_1909_04823_amd import des, synth

    w = synth.workload(index, scale=args.scale)
    streaming = bool(w.p_new)
    opt = des.OPT_SGD if w.opt == "sgd" else des.OPT_ADAGRAD
    state_mult = 1 if w.opt == "sgd" else 2
    total_steps = args.warmup + args.steps
    # streaming: every step needs its own batch (the table grows), and the per-kernel pass runs on
    # the batches after the timed ones
    n_batches = args.batches or (2 if w.index == 4 and args.scale == 1.0 else 8)
    n_batches = min(n_batches, total_steps)
    if streaming:
        n_batches = total_steps + (0 if args.no_kernel_pass else args.steps)

    # ---- inputs (host generation, then resident in HBM) --------------------------------------
    t_setup = time.perf_counter()
    if streaming:
        gen = synth.StreamingGenerator(w)
        first_keys = gen.initial_keys()
        host_batches = []
        for i in range(n_batches):
            host_batches.append(gen.next_batch())
            if i % 10 == 9:                       # long set-ups stay visibly alive
                print(f"bench.py: generated {i + 1} of {n_batches} streaming batches", file=sys.stderr, flush=True)
        # one more step in which 30 % of the entries are brand-new IDs (the literal reading of the workload's
        # description; it cannot be sustained inside the stated final size, one step of it can), timed on its own
        heavy_batch = None
        if gen.row_keys.shape[0] + int(0.33 * host_batches[-1].nnz) <= w.capacity:
            heavy_batch = gen.next_batch(p_new=0.30)
    else:
        host_batches = [synth.gen_batch(w, i) for i in range(n_batches)]
    max_nnz = max(b.nnz for b in host_batches)
    if streaming and heavy_batch is not None:
        max_nnz = max(max_nnz, heavy_batch.nnz)
    chunk = 1 << 22
    policy = des.SHARD_KEY_HASH if args.policy == "key" else des.SHARD_FIELD_MOD
    table = des.Table(w.D, w.capacity, w.K, policy, opt, init_seed=w.seed, init_scale=w.init_std,
                      max_n=max(max_nnz, min(chunk, w.preinsert)))
    if streaming:
        for lo in range(0, first_keys.size, chunk):
            table.insert(torch.from_numpy(first_keys[lo:lo + chunk].view(np.int64)).cuda())
    else:
        for lo in range(0, w.preinsert, chunk):
            k = synth.preinsert_keys(w, lo, min(w.preinsert, lo + chunk))
            vals = None
            if w.host_values:
                vals = torch.from_numpy(synth.host_values(w, w.preinsert)[lo:lo + chunk]).cuda()
            table.insert(torch.from_numpy(k.view(np.int64)).cuda(), vals)
    assert table.status() == 0
    rows_before = table.size()
    batches = [des.Batch.from_numpy(b) for b in host_batches]
    g_lr, g_fm, g_pool = synth.upstream_gradients(w, 0)
    g_lr, g_fm, g_pool = (torch.from_numpy(a).cuda() for a in (g_lr, g_fm, g_pool))
    B, F, D, K = w.B, w.F, w.D, w.K
    dev = torch.device("cuda")
    rows = torch.empty(max_nnz, dtype=torch.int32, device=dev)
    P_lr = torch.empty((K, B), dtype=torch.float32, device=dev)
    P_sum = torch.empty((K, B, D), dtype=torch.float32, device=dev)
    P_sq = torch.empty((K, B), dtype=torch.float32, device=dev)
    pool = torch.empty((B, F, D), dtype=torch.float32, device=dev)
    A_lr = torch.empty(B, dtype=torch.float32, device=dev)
    A_sum = torch.empty((B, D), dtype=torch.float32, device=dev)
    A_sq = torch.empty(B, dtype=torch.float32, device=dev)
    fm2 = torch.empty(B, dtype=torch.float32, device=dev)
    n_uniq = torch.zeros(1, dtype=torch.int64, device=dev)
    miss = des.MISS_INSERT if (w.preinsert < w.key_space or streaming) else des.MISS_ZERO
    eps = w.eps if w.eps else 1e-8
    setup_s = time.perf_counter() - t_setup

    # the row-sorting half of the backward pass needs only the rows, so it runs on a second stream
    # (default priority) beside the forward pass; events order find -> sort -> update
    main, aux = torch.cuda.current_stream(), torch.cuda.Stream()
    overlap = [not args.no_overlap]      # the per-kernel pass below switches it off: concurrent kernels stretch each other

    def step(i):
        b = batches[i % len(batches)]
        r = rows[:b.nnz]
        main = torch.cuda.current_stream()               # the capture stream while a graph is being recorded
        ev_found, ev_sorted = torch.cuda.Event(), torch.cuda.Event()
        table.find(b.keys, miss, r)
        if overlap[0]:
            ev_found.record(main)
            aux.wait_event(ev_found)
            with torch.cuda.stream(aux):
                table.backward_prepare(b, r)
                ev_sorted.record(aux)
        table.partial_forward(b, r, P_lr, P_sum, P_sq, pool)
        des.aggregate_forward(P_lr, P_sum, P_sq, A_lr, A_sum, A_sq, fm2)     # the three aggregations and F in one launch
        dbg = {"n_uniq": n_uniq}
        if overlap[0]:
            main.wait_event(ev_sorted)
        if opt == des.OPT_SGD:
            table.backward_update_sgd(b, r, w.lr, g_lr, g_fm, A_sum, g_pool, dbg=dbg)
        else:
            table.backward_update_adagrad(b, r, w.lr, eps, g_lr, g_fm, A_sum, g_pool, dbg=dbg)
        return b.nnz

    if args.calib_copy_mib:
        src = torch.empty(args.calib_copy_mib << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                    # the plain copy kernel of known size: reads and writes calib_copy_mib MiB
        torch.cuda.synchronize()
        del src, dst

    # ---- timed region ---------------------------------------------------------------------------
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    graphs = None
    if args.graph and not streaming:
        # one HIP graph per distinct batch: the whole step (both streams) is recorded once and replayed, which
        # takes the ~30 launches and the Python calls off the critical path of the small workloads
        graphs = []
        for bi in range(len(batches)):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                step(bi)
            graphs.append(g)
        torch.cuda.synchronize()

    def run(i):
        if graphs is None:
            return step(i)
        graphs[i % len(batches)].replay()
        return batches[i % len(batches)].nnz

    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)] if args.step_series else None
    t0 = time.perf_counter()
    lookups = 0
    for i in range(args.warmup, total_steps):
        if marks:
            marks[i - args.warmup].record(main)
        lookups += run(i)
    if marks:
        marks[-1].record(main)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    series = [round(marks[i].elapsed_time(marks[i + 1]), 4) for i in range(args.steps)] if marks else None
    assert table.status() == 0, "device-side error during the timed steps"
    assert bool(torch.isfinite(fm2).all()) and bool(torch.isfinite(pool).all())
    ms_per_step = 1e3 * dt / args.steps

    # ---- per-kernel pass: same steps again, HIP events on the launch stream around every launch --
    kernels, roof = {}, None
    if not args.no_kernel_pass:
        first = total_steps if streaming else args.warmup
        des.profile_enable(True)
        overlap[0] = False
        for i in range(first, first + args.steps):
            step(i)
        prof = des.profile_read()
        des.profile_enable(False)
        overlap[0] = not args.no_overlap
        used = sorted({i % len(batches) for i in range(first, first + args.steps)})
        stats = [batch_stats(host_batches[i].keys) for i in used[:2]]
        st = {k: float(np.mean([s[k] for s in stats])) for k in stats[0]}
        cap_bits = max(1, int(w.capacity).bit_length())
        sort_passes = (cap_bits + 8) // 9
        nnz_mean = lookups / args.steps
        model = algorithmic_bytes(w, nnz_mean, st, sort_passes, state_mult)
        for name, (launches, total_ms) in prof.items():
            per_step_ms = total_ms / args.steps
            entry = {"launches_per_step": launches / args.steps, "ms_per_step": round(per_step_ms, 4)}
            if name in model and per_step_ms > 0:
                entry["algorithmic_GBps"] = round(model[name] / (per_step_ms * 1e-3) / 1e9, 1)
            kernels[name] = entry
        dom = max((k for k in kernels if k in model), key=lambda k: kernels[k]["ms_per_step"])
        lps = kernels[dom]["launches_per_step"]
        per_launch_bytes = model[dom] / lps
        per_launch_s = kernels[dom]["ms_per_step"] * 1e-3 / lps
        achieved = per_launch_bytes / per_launch_s / 1e9
        traffic, traffic_commit = measured_traffic(w.index, dom) if args.scale == 1.0 else (None, None)
        roof = {"kernel": dom, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": traffic,
                "algorithmic_bytes_per_launch": int(per_launch_bytes), "avg_launch_ms": round(per_launch_s * 1e3, 4),
                "distinct_rows_per_step": st["U"], "kernel_ms_sum_per_step": round(sum(v["ms_per_step"] for v in kernels.values()), 4)}

        if roof["traffic"]:          # counted bytes (committed counter summary of a separate run) over the live launch time
            roof["traffic_GBps"] = round(roof["traffic"] / per_launch_s / 1e9, 1)
            roof["traffic_source"] = {"file": f"profiles/{PROFILE_TAG[w.index]}_hbm_traffic.md", "measured_at_commit": traffic_commit}

    # ---- access-pattern ceilings: the forward gather's row reads and the update's row read-modify-writes alone,
    # on this workload's own index streams (des_ceiling_*), beside the real kernels' times of the pass above
    ceil_res = None
    if not args.no_kernel_pass and not args.no_ceiling and w.opt != "sgd":
        b = batches[(total_steps if streaming else args.warmup) % len(batches)]
        r = rows[:b.nnz]
        table.find(b.keys, des.MISS_ZERO, r)
        uniq = torch.empty(b.nnz, dtype=torch.int32, device=dev)
        n_u = torch.zeros(1, dtype=torch.int64, device=dev)
        table.backward_merge(b, r, g_lr=g_lr, dbg={"uniq_rows": uniq, "n_uniq": n_u})      # merged order only, no update
        U = int(n_u.item())
        sink = des.ceiling_gather(table.emb, r)
        des.ceiling_update(table.emb, table.acc_emb, uniq[:U])
        torch.cuda.synchronize()
        reps = 5
        des.profile_enable(True)
        for _ in range(reps):
            des.ceiling_gather(table.emb, r, sink)
            des.ceiling_update(table.emb, table.acc_emb, uniq[:U])
        prof = des.profile_read()
        des.profile_enable(False)
        g_ms, u_ms = prof["ceiling_gather"][1] / reps, prof["ceiling_update"][1] / reps
        present = int((r >= 0).sum().item())
        ceil_res = {
            "batch_entries": b.nnz, "distinct_rows": U,
            "gather": {"ms": round(g_ms, 4), "logical_GB": round(present * D * 4 / 1e9, 3),
                       "logical_GBps": round(present * D * 4 / (g_ms * 1e-3) / 1e9, 1)},
            "update": {"ms": round(u_ms, 4), "logical_GB": round(U * D * 16 / 1e9, 3),
                       "logical_GBps": round(U * D * 16 / (u_ms * 1e-3) / 1e9, 1)},
        }
        if "forward_gather_pool" in kernels:
            ceil_res["forward_gather_pool_ms"] = kernels["forward_gather_pool"]["ms_per_step"]
            ceil_res["gather_ceiling_over_forward"] = round(g_ms / kernels["forward_gather_pool"]["ms_per_step"], 3)
        upd = sum(kernels[k]["ms_per_step"] for k in ("backward_short_update", "backward_long_partial", "backward_long_final") if k in kernels)
        if upd > 0:
            ceil_res["merge_and_update_ms"] = round(upd, 4)
            ceil_res["update_ceiling_over_merge_and_update"] = round(u_ms / upd, 3)
        del uniq, sink

    heavy_res = None
    if streaming and heavy_batch is not None and not args.no_kernel_pass:
        # the table is exactly in the state the generator's mirror expects: every generated batch has been run once
        batches.append(des.Batch.from_numpy(heavy_batch))
        rows_was = table.size()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(main)
        step(len(batches) - 1)
        e1.record(main)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        assert table.status() == 0
        heavy_res = {"p_new": 0.30, "ms": round(ms, 4), "nnz": heavy_batch.nnz, "new_rows": table.size() - rows_was,
                     "lookups_per_s": heavy_batch.nnz / (ms * 1e-3), "table_rows_before": rows_was}

    cpu_res = None
    if cpu:
        n_cpu = max(1, min(B, int(np.ceil(args.cpu_lookups / max(1.0, host_batches[0].nnz / B)))))
        cpu_res = cpu_baseline(w, host_batches[0], n_cpu, 1 if w.opt == "sgd" else 2)

    model_res = None
    if args.model != "none" and index == args.config and not streaming and args.dnn_hidden >= 8:
        del pool, g_pool, P_sum, P_lr, P_sq
        torch.cuda.empty_cache()
        model_res = run_model_step(args, w, table, batches, opt, eps)

    migrate_res = None
    state_bytes_per_row = (w.D + 1) * 4 * state_mult + 8
    if 2.5 * w.capacity * state_bytes_per_row < 100e9:          # a second table of the same size must fit beside it
        migrate_res = run_migrate(w, table, opt, state_bytes_per_row)

    out = {
        "metric": "sparse lookups/sec, DES fwd+bwd step (samples/sec alongside)",
        "value": lookups / dt, "unit": "lookups/s", "samples_per_s": args.steps * B / dt,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 (f64 accumulation)", "data": "synthetic",
        "config": {"workload": f"configs[{w.index}] {w.name}" + ("" if args.scale == 1.0 else f" scaled x{args.scale}"),
                   "B": B, "F": F, "D": D, "K": K, "optimizer": w.opt, "nnz_per_step": lookups / args.steps,
                   "table_rows": rows_before, "table_rows_after": table.size(), "distinct_batches": len(batches),
                   "find_policy": "insert" if miss == des.MISS_INSERT else "lookup", "setup_s": round(setup_s, 1),
                   "streams": 1 if args.no_overlap else 2, "shard_policy": args.policy,
                   "hip_graph": bool(graphs)},
        "roofline": roof, "cpu_baseline": cpu_res, "kernels": kernels,
    }
    if ceil_res is not None:
        out["ceilings"] = ceil_res
    if heavy_res is not None:
        out["insert_heavy_step"] = heavy_res
    if series is not None:
        out["series_ms"] = series
    if model_res is not None:
        out["model_step"] = model_res
    if migrate_res is not None:
        out["table_migrate"] = migrate_res
    if index == args.config and not args.no_compact:
        out["table_compact"] = run_compact(w, table, state_bytes_per_row)     # last: it drops half of the rows
    table.close()
    del table, batches
    return out


def run_migrate(w, table, opt, state_bytes_per_row):
    """Eviction of a seeded random half of the rows into a second table of the same capacity
    (des_table_migrate: flags, prefix sum, row copy, re-insert), timed on the host around the call,
    which synchronises.  Bytes: every kept row's key, weights and state read and written once, plus one
    flag byte per source row and one 16-byte slot per kept row."""
    import torch
    from paper_1909_04823_amd import des
    n = table.size()
    dst = des.Table(w.D, w.capacity, w.K, des.SHARD_KEY_HASH, opt, init_seed=w.seed, init_scale=w.init_std,
                    max_n=max(n, 1 << 16))
    gen = torch.Generator(device="cuda"); gen.manual_seed(13)
    keep = (torch.rand(n, device="cuda", generator=gen) < 0.5).to(torch.uint8)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    kept = table.migrate_into(dst, keep)
    dt = time.perf_counter() - t0
    ok = dst.status() == 0 and dst.size() == kept == int(keep.sum().item())
    dst.close()
    del dst, keep
    torch.cuda.empty_cache()
    assert ok
    nbytes = n * 1 + kept * (2 * state_bytes_per_row + 16)
    return {"rows": n, "kept": kept, "ms": round(1e3 * dt, 3), "algorithmic_GBps": round(nbytes / dt / 1e9, 1)}


def run_compact(w, table, state_bytes_per_row):
    """Eviction of a seeded random half of the rows inside the table (des_table_compact, 1 GiB staging buffer),
    timed on the host around the call, which synchronises.  Bytes: every kept row read and written twice (through
    the staging buffer), one flag byte per row, the slot array cleared and one slot written per kept row."""
    import torch
    n = table.size()
    gen = torch.Generator(device="cuda"); gen.manual_seed(17)
    keep = (torch.rand(n, device="cuda", generator=gen) < 0.5).to(torch.uint8)
    staging = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    want = int(keep.sum().item())
    # a sample of kept rows to follow through the move: their keys and first weights, and where they must land
    # (new row = number of kept rows below; counted with torch on the device, which is not the code under test)
    sample = torch.nonzero(keep, as_tuple=False).flatten()
    picks = min(2048, sample.numel())                 # evenly spaced, in integer arithmetic (indices beyond 2^24 are not exact in fp32)
    sample = sample[(torch.arange(picks, dtype=torch.int64, device="cuda") * (sample.numel() - 1)) // max(picks - 1, 1)]
    new_row = torch.stack([keep[:int(r)].sum(dtype=torch.int64) for r in sample[:64].tolist()]) if sample.numel() else sample
    old_keys, old_emb = table.row_keys[sample].clone(), table.emb[sample, 0].clone()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    kept = table.compact(keep, staging)
    dt = time.perf_counter() - t0
    assert table.status() == 0 and table.size() == kept == want
    if sample.numel():
        found = table.find(old_keys, 0)                                  # DES_MISS_ZERO
        assert bool((found[:64].long() == new_row).all()) and bool((found >= 0).all())
        assert torch.equal(table.row_keys[found.long()], old_keys) and torch.equal(table.emb[found.long(), 0], old_emb)
    del staging, keep
    torch.cuda.empty_cache()
    nbytes = n * 1 + kept * (4 * state_bytes_per_row + 16) + table.slots.numel()
    return {"rows": n, "kept": kept, "ms": round(1e3 * dt, 3), "algorithmic_GBps": round(nbytes / dt / 1e9, 1)}


def run_model_step(args, w, table, batches, opt, eps):
    """Whole training steps of `--model` on the workload's table and batches: the sparse path as above
    plus the first layer under DES, the tower (H, H/2), the output unit with log-loss on random
    Bernoulli(0.2) labels, all backward passes and both optimizers.  Outside `value`."""
    import torch
    from paper_1909_04823_amd import des, synth
    from paper_1909_04823_amd.model import Model
    H = args.dnn_hidden
    hidden = tuple(int(x) for x in args.tower.split(",")) if args.tower else (H, max(4, H // 2 // 4 * 4))
    tower = synth.tower_init(w.seed, w.F, w.D, hidden=hidden)
    if args.model == "dcn":
        tower.update(synth.cross_init(w.seed, w.F, w.D, n_cross=args.cross_layers))
    # throughput only: the table has just been through the sparse steps above, whose upstream gradients
    # are random, so the loss value of these steps means nothing (it is only checked to be finite)
    m = Model(table, w.F, args.model, tower, w.B, dict(opt_emb=opt, opt_w=opt, lr=1e-5, eps=eps),
              dict(opt_emb=des.OPT_ADAGRAD, lr=1e-3, eps=1e-8))
    gen = torch.Generator(device="cuda"); gen.manual_seed(11)
    labels = (torch.rand(w.B, device="cuda", generator=gen) < 0.2).float()
    insert = w.preinsert < w.key_space
    reps = max(3, min(args.steps, 5))
    for i in range(2):
        m.train_step(batches[i % len(batches)], labels, insert=insert, overlap=not args.no_overlap)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    lookups = 0
    for i in range(reps):
        b = batches[i % len(batches)]
        m.train_step(b, labels, insert=insert, overlap=not args.no_overlap)
        lookups += b.nnz
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    des.profile_enable(True)
    for i in range(reps):
        m.train_step(batches[i % len(batches)], labels, insert=insert, overlap=False)    # per-kernel times: one stream
    prof = des.profile_read()
    des.profile_enable(False)
    assert table.status() == 0 and bool(torch.isfinite(m.loss).all())
    flops = 2.0 * w.B * w.F * w.D * hidden[0]
    kernels = {}
    for name, (launches, total_ms) in prof.items():
        e = {"launches_per_step": launches / reps, "ms_per_step": round(total_ms / reps, 4)}
        kernels[name] = e
    return {"model": args.model, "hidden": list(hidden), "steps": reps,
            "ms_per_step": round(1e3 * dt / reps, 4), "lookups_per_s": lookups / dt, "samples_per_s": reps * w.B / dt,
            "first_layer_flops_per_product": flops,
            "kernel_ms_sum_per_step": round(sum(v["ms_per_step"] for v in kernels.values()), 4), "kernels": kernels}


if __name__ == "__main__":
    main()
