#!/usr/bin/env python3
"""Benchmark of the CO3 codec hot path on one MI355X.

A step is one whole iteration of Algorithm 1's uplink for all clients of the workload: the user
side (anchor + error correction + fp conversion + histogram, code build, compression: one
co3_user_encode call, or co3_convert_ef -> co3_build_code -> co3_encode with --separate-calls)
and the server side co3_ps_aggregate (decode + average), on synthetic GenNorm gradients that
are resident in HBM before the timed region starts.

Prints ONE JSON line: elements/s of the whole path with its fraction of the HBM roofline
(path_roofline; the target of 0.60 on C3 is stated beside it), the roofline of the dominant
kernel (the conversion kernel, timed live with HIP events on the launch stream), the first
iteration's time, the measured device copy bandwidth, and the CPU oracle timed on a bounded
sample of the device batches on this host (one core, and one thread per client).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
K_CONVERT = 2                  # kernel ids of the library's timing facility: k_convert_ef ...
K_COOP = 12                    # ... and k_coop_convert, the resident-grid form of the conversion
PATH_TARGET_FRAC = 0.60        # end-to-end target on C3: fraction of the HBM roofline


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def make_workload(name):
    """(workload, per-user betas, scale, description) of one of the five benchmark configurations."""
    import co3_inputs as inp
    if name == "C3":
        w = inp.c3()
        betas = [float(b) for b in inp.c3_client_betas(w.U)]
        return w, betas, 1e-3, ("C3: 10 clients x 11,173,962 fp32, GenNorm beta~U(0.5,1.5) per client, scale 1e-3, "
                                "E3M0, per-client empirical Huffman, PS decode+average")
    if name == "C1":
        w = inp.c1()
        return w, [1.0], 1e-3, "C1: 1 client x 65,536 fp32, GenNorm beta=1 scale 1e-3, E3M1"
    if name == "C2":
        w = inp.c2()
        return w, [0.8], None, ("C2: 1 client x 11,173,962 fp32 in 62 tensors (per-tensor anchors), GenNorm beta=0.8, "
                                "per-tensor scale 10^U(-5,-2), E4M3")
    if name == "C4":
        w = inp.c4()
        return w, [1.0], 1e-4, "C4: 1 client x 100,000,000 fp32, GenNorm beta=1 scale 1e-4 (1e-4 of the samples at 100x), E5M2"
    if name.startswith("C5"):
        point = int(name[3:]) if len(name) > 3 else 4
        w = inp.c5(point)
        beta = inp.C5_BETAS[point % 3]
        return w, [beta], 1e-3, f"C5[{point}]: 16 clients x 25,000,000 fp32, E{w.E}M{w.M}, GenNorm beta={beta} scale 1e-3"
    raise SystemExit(f"unknown workload {name} (C1, C2, C3, C4, C5.<point 0..11>)")


def device_batches(w, betas, alpha, pool, pipe):
    """`pool` gradient batches [U][stride] drawn on the device (seeded), one per iteration slot, by the
    recipe of the workload: C2 one scale per tensor, C4 1e-4 of the samples at 100 times the scale."""
    import torch
    import co3_inputs as inp
    out = []
    for t in range(pool):
        g = pipe.new_gradient_buffer()
        for u in range(w.U):
            seed = inp.BASE_SEED * 1000003 + w.cfg * 10007 + u * 101 + t
            beta = betas[u % len(betas)]
            if w.cfg == 2:
                scales = inp.c2_tensor_scales()
                g[u, :w.n] = torch.cat([inp.device_gennorm(sz, beta, float(a), seed + 7919 * (k + 1))
                                        for k, (sz, a) in enumerate(zip(w.sizes, scales))])
            elif w.cfg == 4:
                g[u, :w.n] = inp.device_gennorm_outliers(w.n, beta, alpha, 1e-4, 100.0, seed)
            else:
                g[u, :w.n] = inp.device_gennorm(w.n, beta, alpha, seed)
        out.append(g)
    torch.cuda.synchronize()
    return out


def cpu_baseline(w, batches, chunk_syms, n_sample, reps):
    """The oracle as it stands on the bytes the GPU leg consumed (copied back from the device batches): the
    same call sequence per iteration, on the first `n_sample` elements of every client.  Two figures: one
    thread over 2 clients, then threads over all clients of the workload (each oracle call stays
    single-threaded) on up to all host cores."""
    from concurrent.futures import ThreadPoolExecutor
    import numpy as np
    import oracle
    fmt = oracle.Fmt(w.E, w.M)
    seg_off = None
    if w.sizes is not None and n_sample == w.n:
        seg_off = w.seg_off
    host = [[b[u, :n_sample].cpu().numpy() for u in range(w.U)] for b in batches]
    oracle.lib()

    def client_iteration(g, err):
        A = oracle.anchor(g, fmt, seg_off)
        s, e_new = oracle.convert_ef(g, err, A, 1.0, fmt, seg_off)
        cnt = oracle.histogram(s, fmt)
        l = oracle.huffman_lengths(cnt)
        c = oracle.canonical_codes(l)
        words, off, total = oracle.encode(s, l, c, chunk_syms)
        d = oracle.decode(words, total, l, c, n_sample)
        return d, A, e_new

    def run(users, threads, reps):
        errs = {u: np.zeros(n_sample, np.float32) for u in users}
        with ThreadPoolExecutor(max_workers=threads) as tp:
            t0 = time.perf_counter()
            for t in range(reps):
                res = list(tp.map(lambda u: client_iteration(host[t % len(host)][u], errs[u]), users))
                for u, r in zip(users, res):
                    errs[u] = r[2]
                syms, anchors = np.stack([r[0] for r in res]), np.stack([r[1] for r in res])
                if seg_off is None:          # the average: element ranges over the threads
                    cuts = np.linspace(0, n_sample, threads + 1).astype(np.int64)
                    list(tp.map(lambda k: oracle.aggregate(np.ascontiguousarray(syms[:, cuts[k]:cuts[k + 1]]), anchors, fmt),
                                range(threads)))
                else:
                    oracle.aggregate(syms, anchors, fmt, seg_off)
            return time.perf_counter() - t0

    U1 = list(range(min(w.U, 2)))
    dt1 = run(U1, 1, reps)
    nproc = os.cpu_count() or 1
    UN = list(range(w.U))
    threads = max(1, min(nproc, len(UN)))
    repsN = max(2, reps // 2)
    dtN = run(UN, threads, repsN)
    return {"value": len(U1) * n_sample * reps / dt1, "unit": "elements/s", "cores": 1, "kind": "oracle",
            "sample": f"{len(U1)} clients x {n_sample} elements x {reps} iterations, the device batches' own bytes "
                      f"({dt1:.1f} s, single thread)",
            "all_cores": {"value": len(UN) * n_sample * repsN / dtN, "unit": "elements/s", "cores": threads,
                          "nproc": nproc, "sample": f"{len(UN)} clients x {n_sample} elements x {repsN} iterations, "
                                                    f"one thread per client ({dtN:.1f} s)"}}


def measured_copy_bandwidth():
    """GB/s (read + written bytes) of a plain device-to-device copy of 1 GiB on this machine."""
    import torch
    a = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    b = torch.empty_like(a)
    for _ in range(3):
        b.copy_(a)
    torch.cuda.synchronize()
    reps = 10
    t0 = time.perf_counter()
    for _ in range(reps):
        b.copy_(a)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    del a, b
    torch.cuda.empty_cache()
    return 2.0 * (1 << 30) * reps / dt / 1e9


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C3", help="C3 (default, the headline configuration), C1, C2, C4, C5.<point>")
    ap.add_argument("--chunk", type=int, default=256)
    ap.add_argument("--bias", default="absmax", choices=("absmax", "moments"),
                    help="absmax: integer anchor from max|g| (the headline configuration); moments: the paper's bias "
                         "rule (moment sums, GenNorm fit, multiplier) on the fixed grid of anchor 2^(E-1)")
    ap.add_argument("--codes", default="user", choices=("user", "user-model", "user-lagged", "layer", "layer-model", "layer-lagged"),
                    help="user: one empirical code per client, rebuilt every step (the headline configuration); "
                         "layer: one code per tensor shared by the clients, rebuilt every step from the pooled "
                         "per-tensor counts; user-model: one fixed code per client designed once from the GenNorm law "
                         "of the workload (C4's model table; no histogram, no code build inside the step); "
                         "user-lagged: one empirical code per client built from the counts of the previous step, "
                         "gathered by the one-pass user side (conversion + compression in one pass every step); "
                         "layer-lagged: the same for one code per tensor shared by the clients (pooled counts); "
                         "layer-model: one fixed code per tensor designed once from the GenNorm "
                         "law of the tensor (no histogram, no code build inside the step)")
    ap.add_argument("--single-pass", action="store_true",
                    help="with --codes user-model or layer-model: conversion and compression in one pass "
                         "(co3_convert_encode, co3_convert_encode_layers), no symbol array")
    ap.add_argument("--gamma", type=float, default=1.0, help="memory decay coefficient (1.0 in all five configurations)")
    ap.add_argument("--format", default=None, help="override the workload's format, e.g. E1M2")
    ap.add_argument("--pool", type=int, default=3, help="distinct gradient batches cycled through")
    ap.add_argument("--graph", action="store_true",
                    help="capture one iteration per batch buffer in a HIP graph and time replays (launch-bound workloads)")
    ap.add_argument("--sweep-c5", action="store_true",
                    help="run the 12 points of C5 (4 formats x 3 shapes) one after the other, each in a child process, "
                         "and print one line with elements/s and bits/element per point")
    ap.add_argument("--separate-calls", action="store_true",
                    help="the user's steps through co3_convert_ef, co3_build_code and co3_encode instead of one "
                         "co3_user_encode call (which, where a user's gradient fits the register files, reads every "
                         "gradient once in a resident grid)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--breakdown", action="store_true", help="extra untimed pass timing every kernel (stderr)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a plain elementwise copy of 1 GiB (reads 2^30 B, writes 2^30 B) three times: "
                         "the known-size kernel that scales the rocprofv3 FETCH_SIZE / WRITE_SIZE readings")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1")

    if args.sweep_c5:
        import subprocess
        points, total_elems, total_s = [], 0.0, 0.0
        for pt in range(12):
            out = subprocess.run([sys.executable, os.path.abspath(__file__), "--workload", f"C5.{pt}", "--no-cpu",
                                  "--steps", str(min(args.steps, 10)), "--warmup", "2", "--chunk", str(args.chunk)],
                                 capture_output=True, text=True, check=True).stdout
            r = json.loads([l for l in out.splitlines() if l.startswith("{")][-1])
            points.append({"point": pt, "format": r["config"]["format"], "workload": r["config"]["workload"],
                           "elements_per_s": r["value"], "ms_per_step": r["ms_per_step"],
                           "bits_per_element": sum(r["bits_per_element"].values()),
                           "path_roofline_frac": r["path_roofline"]["frac"]})
            total_elems += r["config"]["U"] * r["config"]["n"] * r["steps"]
            total_s += r["ms_per_step"] * 1e-3 * r["steps"]
            log(f"[bench] C5.{pt} {r['config']['format']}: {r['value'] / 1e9:.1f} G elements/s, "
                f"{points[-1]['bits_per_element']:.3f} bit/element")
        print(json.dumps({"metric": "gradient elements/s (encode+decode, 1 GPU)", "value": total_elems / total_s,
                          "unit": "elements/s", "n_gpus": 1, "higher_is_better": True, "data": "synthetic",
                          "dtype": "f32", "config": {"workload": "C5 sweep: 16 clients x 25,000,000, 12 points"},
                          "points": points}), flush=True)
        return

    import torch
    assert torch.cuda.is_available(), "bench.py needs an MI355X"
    if args.calibrate_copy:
        a = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        b = torch.empty_like(a)
        for _ in range(3):
            torch.add(a, 1.0, out=b)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": 1 << 30, "calibrate_copy_bytes_written": 1 << 30}))
        return
    from paper_2203_09044_amd import Co3Pipeline, Fmt, binding as B

    w, betas, alpha, desc = make_workload(args.workload)
    if args.format:
        import dataclasses
        w = dataclasses.replace(w, E=int(args.format[1]), M=int(args.format[3]))
        desc += f", format overridden to {args.format}"
    if args.bias == "moments":
        desc += ", bias rule from moments"
    fmt = Fmt(w.E, w.M)
    code_seg_off = None
    if args.codes in ("layer", "layer-model", "layer-lagged") and w.sizes is not None:
        import co3_inputs as inp
        groups = inp.group_small_tensors(w.sizes)
        code_seg_off = inp.seg_offsets(groups)
        desc += f", {len(groups)} code groups (tensors under 16,384 elements share the code of the large tensor before them)"
    fixed_user_tables = args.codes == "user-model"
    lagged = args.codes in ("user-lagged", "layer-lagged")
    if args.codes == "user-lagged" and args.bias != "absmax":
        raise SystemExit("--codes user-lagged goes with the integer anchor")
    if args.single_pass and args.codes not in ("user-model", "layer-model"):
        raise SystemExit("--single-pass needs --codes user-model or layer-model (the codes must be known before the step)")
    if args.single_pass and fixed_user_tables and args.bias != "absmax":
        raise SystemExit("--single-pass with --bias moments needs --codes layer-model")
    one_call = (not args.separate_calls and args.bias == "absmax" and args.codes == "user")
    pipe = Co3Pipeline(w.U, w.n, fmt, chunk_syms=args.chunk, seg_off=w.seg_off if w.sizes is not None else None,
                       bias=args.bias, gamma=args.gamma, codes="user" if args.codes.startswith("user") else "layer",
                       code_seg_off=code_seg_off, statistics=not fixed_user_tables,
                       single_pass=args.single_pass or lagged, lagged_codes=lagged,
                       one_call=one_call, keep_symbols=not one_call,
                       cap_words=2 * B.cap_words_empirical(w.n, fmt) if fixed_user_tables or lagged else None)
    import co3_inputs as inp
    # scale of the law of every tensor (C2 draws one per tensor)
    tensor_alpha = [float(a) for a in inp.c2_tensor_scales()] if w.cfg == 2 else [alpha] * pipe.nseg
    log(f"[bench] {desc}; generating {args.pool} device batches")
    batches = device_batches(w, betas, alpha, args.pool, pipe)

    rebuild = args.codes in ("user", "layer", "user-lagged", "layer-lagged")   # lagged: the step builds the next step's codes
    if fixed_user_tables:
        # one table per client from the law the client's gradients are drawn from, on the grid of the client's
        # anchor of the first batch (every emit-able symbol has a codeword, so the table serves every step)
        import numpy as np
        pipe.convert(batches[0])
        j = int(np.argmax(w.sizes)) if w.sizes is not None else 0      # several tensors: the law of the largest one
        A0 = pipe.anchor[:, j].cpu().numpy()
        pipe.err.zero_()
        wts = np.stack([B.model_weights(int(A0[u]), fmt, float(betas[u % len(betas)]), float(tensor_alpha[j])).numpy().view(np.uint32)
                        for u in range(w.U)])
        pipe.build(torch.from_numpy(wts.view(np.int32)).cuda())
        desc += ", fixed per-client model tables" + (", single pass" if args.single_pass else "")
    elif not rebuild:
        # fixed tables: the GenNorm law of each tensor (workload parameters) on the grid of client 0's anchors
        # of the first batch; every emit-able symbol has a codeword, so the tables serve all clients and steps
        import numpy as np
        if args.bias == "moments":       # the multiplier c of the first batch: c * x follows GenNorm(beta, c * alpha)
            pipe.fit_bias(batches[0])
            c0 = pipe.scale[0].cpu().numpy()
        else:
            c0 = np.ones(pipe.nseg, np.float32)
        pipe.convert(batches[0])
        A0 = pipe.anchor[0].cpu().numpy()
        pipe.err.zero_()
        model_beta = sum(betas) / len(betas)
        # anchor of the first tensor of each code group
        cso = pipe.code_seg_off.cpu().numpy()
        aso = [0, w.n] if pipe.seg_off is None else pipe.seg_off.cpu().numpy()
        first_tensor = [int(np.searchsorted(aso, cso[k], side="right") - 1) for k in range(pipe.ncodes)]
        wts = np.zeros((pipe.ncodes, fmt.K), np.uint32)
        for k in range(pipe.ncodes):
            wts[k] = B.model_weights(int(A0[first_tensor[k]]), fmt, float(model_beta),
                                     float(tensor_alpha[first_tensor[k]]) * float(c0[first_tensor[k]])).numpy().view(np.uint32)
        pipe.build(torch.from_numpy(wts.view(np.int32)).cuda())
        desc += ", fixed per-tensor model tables" + (", single pass" if args.single_pass else "")
    elif args.codes == "layer":
        desc += ", per-tensor codes shared by the clients"
    elif lagged:
        desc += ", codes from the counts of the previous step (one-pass user side)"
    copy_gbs = measured_copy_bandwidth()
    # the first iteration on its own (cold caches, first launches of every kernel)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pipe.step(batches[0], rebuild=rebuild)
    torch.cuda.synchronize()
    first_step_ms = (time.perf_counter() - t0) * 1e3
    pipe.err.zero_()
    for i in range(args.warmup):
        pipe.step(batches[i % args.pool], rebuild=rebuild)
    torch.cuda.synchronize()
    assert pipe.poll() == 0, "device status after warmup"
    graphs = None
    if args.graph:
        graphs = []
        for b in batches:
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr):
                pipe.step(b, rebuild=rebuild)
            graphs.append(gr)
        torch.cuda.synchronize()
        desc += ", HIP graph replay"

    B.timing_reset()
    if graphs is None:
        B.timing_enable((1 << K_CONVERT) | (1 << K_COOP))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    if graphs is None:
        for i in range(args.steps):
            pipe.step(batches[i % args.pool], rebuild=rebuild)
    else:
        for i in range(args.steps):
            graphs[i % args.pool].replay()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    if graphs is not None:
        # the event timing of the dominant kernel cannot be recorded inside a graph: a separate eager pass
        B.timing_enable((1 << K_CONVERT) | (1 << K_COOP))
        for i in range(min(args.steps, 10)):
            pipe.step(batches[i % args.pool], rebuild=rebuild)
        torch.cuda.synchronize()
    # the conversion ran as one of two kernels: the resident grid where the batch fits it, else k_convert_ef
    dominant = K_COOP if B.timing_read(K_COOP)[1] else K_CONVERT
    conv_ms, conv_launches = B.timing_read(dominant)
    B.timing_enable(0)
    assert pipe.poll() == 0, "device status after the timed region"

    elems_step = w.U * w.n
    value = elems_step * args.steps / dt
    total_bits = pipe.total_bits.cpu().numpy().astype("float64")
    payload_bpe = float(total_bits.sum()) / elems_step
    index_bpe = 64.0 * (pipe.nchunks + 1) / w.n
    header_bpe = (8.0 * fmt.K + 32 + 64) / w.n
    b = payload_bpe + index_bpe + header_bpe
    b_alg = 12.0 + b / 4.0 + 4.0 / w.U                 # algorithmic bytes per client-element, whole path
    conv_avg_ms = conv_ms / max(conv_launches, 1)
    conv_bytes = 12.0 * elems_step                     # the conversion kernel: read g, read m, write m
    achieved = conv_bytes / (conv_avg_ms * 1e-3) / 1e9 if conv_avg_ms > 0 else 0.0

    # HBM traffic of the dominant kernel: not measured in this run; read from the stored rocprofv3 counter
    # summary of the same command (fetched + written MB per launch)
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_C3.txt")
    if args.workload == "C3" and args.bias == "absmax" and args.codes == "user" and os.path.exists(tpath):
        for line in open(tpath):
            if line.startswith(B.kernel_name(dominant)):
                try:
                    traffic = float(line.split()[-1]) * 1e6
                    traffic_source = "profiles/hbm_traffic_C3.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, stored summary)"
                except ValueError:
                    traffic = None
                break

    if args.breakdown:
        B.timing_reset()
        B.timing_enable((1 << B.KERNEL_COUNT) - 1)
        reps = 5
        for i in range(reps):
            pipe.step(batches[i % args.pool], rebuild=rebuild)
        torch.cuda.synchronize()
        tot = 0.0
        for k in range(B.KERNEL_COUNT):
            ms, cnt = B.timing_read(k)
            if cnt:
                log(f"[bench] {B.kernel_name(k):14s} {ms / reps:8.4f} ms/step  ({cnt // reps} launches/step)")
                tot += ms / reps
        log(f"[bench] sum of kernels {tot:.4f} ms/step")
        B.timing_enable(0)

    res = {
        "metric": "gradient elements/s (encode+decode, 1 GPU)",
        "value": value,
        "unit": "elements/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": desc, "U": w.U, "n": w.n, "format": f"E{w.E}M{w.M}", "chunk_syms": args.chunk,
                   "table": {"user": "empirical per client, rebuilt every step",
                             "user-model": "fixed per client, designed from the GenNorm law of the workload",
                             "user-lagged": "empirical per client from the previous step's counts (+1), rebuilt every step",
                             "layer-lagged": "empirical per tensor from the previous step's pooled counts (+1), rebuilt every step",
                             "layer": "empirical per tensor, pooled over the clients, rebuilt every step",
                             "layer-model": "fixed per tensor, designed from the GenNorm law of the workload"}[args.codes],
                   "gamma": args.gamma, "bias": args.bias, "codes": args.codes,
                   "user_side": "co3_user_encode" if one_call else "separate calls"},
        "bits_per_element": {"payload": payload_bpe, "index": index_bpe, "header": header_bpe},
        "first_step_ms": first_step_ms,
        "path_roofline": {"bound": "hbm", "scope": "whole path (encode + decode), all kernels of a step",
                          "algorithmic_bytes_per_element": b_alg,
                          "achieved": b_alg * value / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                          "frac": b_alg * value / 1e9 / HBM_PEAK_GBS,
                          "target_frac": PATH_TARGET_FRAC if args.workload == "C3" else None,
                          "target_met": (b_alg * value / 1e9 / HBM_PEAK_GBS >= PATH_TARGET_FRAC) if args.workload == "C3" else None,
                          "measured_copy_GBs": copy_gbs,
                          "frac_of_measured_copy": b_alg * value / 1e9 / copy_gbs},
        "roofline": {"bound": "hbm", "scope": "dominant kernel only", "kernel": B.kernel_name(dominant),
                     "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "avg_launch_ms": conv_avg_ms, "launches": conv_launches,
                     "algorithmic_bytes_per_launch": conv_bytes},
    }
    if not args.no_cpu:
        log("[bench] timing the CPU oracle on a bounded sample")
        if args.bias != "absmax" or args.gamma != 1.0 or args.codes != "user":
            raise SystemExit("bench.py: the CPU leg times the headline path; use --no-cpu with --bias moments / --gamma")
        # about 6 s of oracle time per leg at its usual 15-20 M elements/s per thread
        n_sample = w.n if w.sizes is not None else min(w.n, 1 << 24)
        reps = max(2, min(200, -(-110_000_000 // (min(w.U, 2) * n_sample))))
        res["cpu_baseline"] = cpu_baseline(w, batches, args.chunk, n_sample=n_sample, reps=reps)
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
