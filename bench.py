#!/usr/bin/env python3
"""Benchmark of the LSH-MoE compression path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload t5]

One step = one pass of the whole path over one batch of synthetic tokens that
are already resident in HBM: lshmoe_hash -> lshmoe_compress (group + centroid)
-> lshmoe_decompress.  The expert stand-in that sits between compress and
decompress is evaluated once, before timing, on the centroids of the same
inputs; its output buffer is what every timed decompress reads.

Prints ONE JSON line: tokens/s for the step, the roofline figures of the
dominant kernel (the restore kernel) measured with events on the launch
stream inside the timed loop, per-stage times, and the CPU oracle timed on a
bounded sample of the same workload as a reported baseline.
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

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
# HBM bytes per restore_kernel launch from rocprofv3 --pmc (FETCH_SIZE x 2.00 + WRITE_SIZE x 1.00, factors from
# a 1 GiB calibration copy); figures and commands are kept in profiles/path_t5_hbm_traffic.txt
MEASURED_TRAFFIC_BYTES = {("t5", "topk_logits"): 633.3e6}
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}


def _fail(msg: str, code: int = 2):
    sys.stderr.write(msg + "\n")
    sys.exit(code)


def cpu_baseline(w, sample_tokens: int):
    """Time the CPU oracle, as it stands, on the arrays of the benched workload (all of them when sample_tokens is 0,
    else the first sample_tokens tokens).  The oracle is numpy: its rotation step is a BLAS matmul and is timed
    twice, on one thread and on every core the process may use; its other steps are single-threaded numpy and
    are timed once."""
    import oracle
    cfg = w.cfg
    Ts = cfg.T if sample_tokens <= 0 else min(sample_tokens, cfg.T)
    tokens, expert = w.tokens[:Ts], w.expert[:Ts]
    try:
        import threadpoolctl
        threads = max([p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()] or [1])
    except Exception:
        threadpoolctl, threads = None, 1
    hash_1 = None
    if threadpoolctl is not None and threads > 1:
        with threadpoolctl.threadpool_limits(limits=1):
            t0 = time.perf_counter()
            oracle.hash_ref(tokens, w.rot, cfg.dtype)
            hash_1 = time.perf_counter() - t0
    t0 = time.perf_counter()
    bucket, _, _, _ = oracle.hash_ref(tokens, w.rot, cfg.dtype)
    t1 = time.perf_counter()
    g = oracle.group_ref(expert, bucket, cfg.E)
    t2 = time.perf_counter()
    c = oracle.centroid_ref(tokens, g["perm"], g["seg_offsets"], cfg.k, cfg.dtype)
    t3 = time.perf_counter()
    # expert output stand-in: any [S, d] array serves for timing the restore
    y = oracle.restore_ref(tokens, c, c, g["seg_of"], cfg.k, cfg.dtype)
    t4 = time.perf_counter()
    del y
    rest = t4 - t1
    total = t4 - t0
    total_1 = (hash_1 if hash_1 is not None else t1 - t0) + rest
    what = "all %d tokens" % cfg.T if Ts == cfg.T else "first %d of %d tokens" % (Ts, cfg.T)
    return {
        "value": Ts / total, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
        "sample": "%s of the benched workload (the same arrays); numpy float64 oracle; rotation matmul on %d BLAS "
                  "threads, grouping / centroid / restore steps single-threaded numpy" % (what, threads),
        "value_single_thread": Ts / total_1,
        "seconds": {"hash": t1 - t0, "hash_single_thread": hash_1 if hash_1 is not None else t1 - t0,
                    "group": t2 - t1, "centroid": t3 - t2, "restore": t4 - t3},
    }


def event_window(steps: int):
    """(first, count): the run of consecutive steps of the timed region whose stages are timed with events.  An event
    record costs 3 to 5 us of stream time, so the records are kept few: the steps of the window follow one another, so
    that the event after a step's decompress call is also the one before the next step's hash call (3 records per
    step and one more, instead of 4 per step), and the window holds 8 steps (16 from 100 steps on), in the middle of
    the run: any run of 8 steps or more yields 8 or more intervals per stage."""
    count = min(steps, 8 if steps < 100 else 16)
    return (steps - count) // 2, count


def measured_peaks():
    """What this GPU sustains, from the small probe library built beside the main one: a streaming read and a
    streaming copy of 2 GiB (far beyond the 256 MB last-level cache) and a loop of independent bf16 MFMAs.
    Best of 5 runs each, timed with events on the current stream."""
    import ctypes
    import torch
    from paper_2411_08446_amd import build as lsh_build
    lib = ctypes.CDLL(lsh_build.PEAKS_LIB_PATH)
    lib.peaks_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
    lib.peaks_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p]
    lib.peaks_mfma_bf16.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    lib.peaks_mfma_bf16_random.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    stream = torch.cuda.current_stream().cuda_stream
    nbytes = 2 << 30
    src = torch.ones(nbytes // 4, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    blocks, iters = 4096, 1000
    mout = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")

    def best(fn):
        times = []
        for _ in range(6):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            rc = fn()
            e1.record()
            torch.cuda.synchronize()
            if rc != 0:
                raise RuntimeError("peak probe failed with HIP error %d" % rc)
            times.append(e0.elapsed_time(e1))
        return min(times[1:])

    t_read = best(lambda: lib.peaks_read(src.data_ptr(), nbytes, sink.data_ptr(), 8192, stream))
    t_copy = best(lambda: lib.peaks_copy(src.data_ptr(), dst.data_ptr(), nbytes, 8192, stream))
    t_mfma = best(lambda: lib.peaks_mfma_bf16(blocks, iters, mout.data_ptr(), stream))
    gen = torch.Generator(device="cuda").manual_seed(7)
    operands = torch.randn(16 * 64 * 8, generator=gen, device="cuda").to(torch.bfloat16)
    t_mfma_r = best(lambda: lib.peaks_mfma_bf16_random(operands.data_ptr(), blocks, iters, mout.data_ptr(), stream))
    return {"hbm_read_gbs": nbytes / (t_read * 1e-3) / 1e9,
            "hbm_copy_gbs": 2 * nbytes / (t_copy * 1e-3) / 1e9,      # bytes read plus bytes written
            "mfma_bf16_tflops": blocks * 4 * iters * 4 * 32768 / (t_mfma * 1e-3) / 1e12,
            "mfma_bf16_random_operands_tflops": blocks * 4 * iters * 4 * 32768 / (t_mfma_r * 1e-3) / 1e12,
            "note": "2 GiB streaming read / copy (read + written bytes) by 8192 workgroups, %d x 4 waves x %d x 4 MFMA "
                    "32x32x16 bf16, once on constant operands and once on eight changing pairs of Gaussian ones (the "
                    "matrix cores clock lower on those)" % (blocks, iters)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="t5", choices=["tiny", "swin", "roberta", "gpt", "t5"])
    ap.add_argument("--gate", default=None, help="override the gate kind (e.g. 'content' for the supplementary run)")
    ap.add_argument("--centers", type=int, default=None, help="override the number of mixture centers (supplementary runs)")
    ap.add_argument("--sigma", type=float, default=None, help="override the within-cluster noise (supplementary runs)")
    ap.add_argument("--paper-regime-steps", type=int, default=50,
                    help="steps of the supplementary run at the paper's compression rates (0 = skip)")
    ap.add_argument("--sweep-hashes", default="",
                    help="comma-separated numbers of hash functions, e.g. 2,4,6,8,10: adds supplementary_hash_count_sweep "
                         "(compression rate and step time per count, content gate, sigma 0.02)")
    ap.add_argument("--sweep-r", type=int, default=16, help="rotated dimensions per hash function in --sweep-hashes")
    ap.add_argument("--no-peaks", dest="peaks", action="store_false",
                    help="skip measuring what this GPU sustains (streaming read, streaming copy, bf16 MFMA loop: "
                         "measured_peaks and the fractions against them)")
    ap.add_argument("--copies", type=int, default=2, help="independent input copies rotated between steps")
    ap.add_argument("--cpu-sample", type=int, default=0,
                    help="tokens in the CPU-oracle baseline (0 = all tokens of the workload, the default; -1 = skip)")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="before the loop, run one plain device-to-device copy of this many MiB (a kernel of known "
                         "traffic against which rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        _fail("bench.py: this path is single-GPU by construction (no collectives are built); run with --gpus 1")

    import numpy as np
    import torch
    if not torch.cuda.is_available():
        _fail("bench.py: no GPU visible; the HIP path has no CPU fallback")
    import paper_2411_08446_amd as lsh
    from workloads import synth

    lsh.load_library()
    over = {key: val for key, val in (("gate", args.gate), ("centers", args.centers), ("sigma", args.sigma)) if val is not None}
    cfg = synth.config(args.workload, **over)
    w = synth.generate(cfg)
    T, d, k, E, L, r, N = cfg.T, cfg.d, cfg.k, cfg.E, cfg.L, cfg.r, cfg.N
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    item = cfg.itemsize

    def dev(arr):
        if cfg.dtype == "f32":
            return torch.from_numpy(np.ascontiguousarray(arr)).cuda()
        return torch.from_numpy(np.ascontiguousarray(arr).view(np.int16)).cuda().view(torch.bfloat16)

    copies = max(1, args.copies)
    xs = [dev(w.tokens) for _ in range(copies)]
    rot = dev(w.rot)
    expert = torch.from_numpy(w.expert).cuda()
    bucket = torch.empty(T, dtype=torch.int64, device="cuda")
    outs = [lsh.CompressOutputs.allocate(T, d, k, E, L, r, tdt) for _ in range(copies)]
    ys = [torch.empty((T, k, d), dtype=tdt, device="cuda") for _ in range(copies)]

    # untimed: centroids of these inputs -> expert stand-in output
    lsh.lshmoe_hash(xs[0], rot, bucket)
    lsh.lshmoe_compress(xs[0], expert, bucket, E, L, r, outs[0])
    torch.cuda.synchronize()
    S = int(outs[0].num_segments.item())
    ecs = []
    for i in range(copies):
        ec = torch.empty((N, d), dtype=tdt, device="cuda")
        ec[:S] = synth.expert_standin(outs[0].centroids[:S], cfg, w.seed)
        ecs.append(ec)
    seg_len = np.diff(outs[0].seg_offsets[:S + 1].cpu().numpy())
    n_single = int((seg_len == 1).sum())

    def step(i, ev=None, first_of_window=True):
        c = i % copies
        x, o = xs[c], outs[c]
        if ev and first_of_window: ev[0].record()   # otherwise ev[0] is the previous step's ev[3], already recorded
        lsh.lshmoe_hash(x, rot, bucket)
        if ev: ev[1].record()
        lsh.lshmoe_compress(x, expert, bucket, E, L, r, o)
        if ev: ev[2].record()
        lsh.lshmoe_decompress(x, o.centroids, ecs[c], o.seg_of, o.seg_offsets, k, ys[c], perm=o.perm,
                              num_segments=o.num_segments)
        if ev: ev[3].record()

    if args.calibration_copy_mib > 0:
        n_el = args.calibration_copy_mib * (1 << 20) // 4
        src_buf = torch.ones(n_el, dtype=torch.float32, device="cuda")
        dst_buf = torch.empty_like(src_buf)
        torch.cuda.synchronize()
        dst_buf.copy_(src_buf)          # reads and writes calibration_copy_mib MiB each
        torch.cuda.synchronize()
        del src_buf, dst_buf

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    K = args.steps
    # Per-stage durations come from events on the launch stream inside the timed region, on a window of consecutive
    # steps that share their boundary events (see event_window).
    win_first, win_count = event_window(K)
    sampled = list(range(win_first, win_first + win_count))
    chain = [torch.cuda.Event(enable_timing=True) for _ in range(3 * win_count + 1)]
    events = {win_first + j: chain[3 * j:3 * j + 4] for j in range(win_count)}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        step(i, events.get(i), i == win_first)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K
    stage_ms = np.array([[events[i][j].elapsed_time(events[i][j + 1]) for j in range(3)] for i in sampled])
    hash_ms, comp_ms, dec_ms = np.median(stage_ms, axis=0)      # medians: a sample that caught a stall does not move them

    # algorithmic bytes of the restore kernel for this workload: expert-output row read and output row
    # written for every assignment; token row and centroid row read only by members of multi-member clusters
    row = d * item
    n_multi_assign = N - n_single
    n_multi_seg = S - n_single
    restore_bytes = (S + N + n_multi_assign + n_multi_seg) * row + 4 * N + 4 * (S + 1)
    restore_bytes_noskip = (T + 2 * S + N) * row + 4 * N
    achieved = restore_bytes / (dec_ms * 1e-3) / 1e9
    hash_flops = 2.0 * T * d * L * r
    result = {
        "metric": "tokens/sec hash+compress+decompress per GPU",
        "value": T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": "%s: T=%d d=%d k=%d E=%d L=%d r=%d, Gaussian mixture of %d centers, gate=%s" %
                               (cfg.name, T, d, k, E, L, r, cfg.centers, cfg.gate),
                   "tokens": T, "assignments": N, "segments": S, "compression_rate": S / N,
                   "single_member_segments": n_single, "input_copies_rotated": copies, "stage_event_samples": len(sampled),
                   "stage_event_steps": "%d consecutive steps from step %d; %d event records" % (win_count, win_first, len(chain))},
        "roofline": {"kernel": "restore_kernel (lshmoe_decompress)", "bound": "hbm", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get((cfg.name, cfg.gate)),
                     "traffic_source": "profiles/path_t5_hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an "
                                       "earlier run of this kernel on this workload; not measured by this run)"
                                       if MEASURED_TRAFFIC_BYTES.get((cfg.name, cfg.gate)) else None,
                     "algorithmic_bytes": restore_bytes,
                     "algorithmic_bytes_without_singleton_skip": restore_bytes_noskip,
                     "avg_launch_ms": float(dec_ms)},
        "stages_ms": {"hash": float(hash_ms), "compress": float(comp_ms), "decompress": float(dec_ms)},
        "stages_note": "medians of the sampled steps; compress = the grouping launches + the centroid kernel. The "
                       "centroid kernel's token rows are partly still in the 256 MB last-level cache behind the hash, "
                       "so its bytes per second can exceed what a streaming read from HBM sustains",
        "stages_p50_ms": {n: float(np.median(stage_ms[:, j])) for j, n in enumerate(("hash", "compress", "decompress"))},
        "stages_p10_ms": {n: float(np.percentile(stage_ms[:, j], 10)) for j, n in enumerate(("hash", "compress", "decompress"))},
        "stages_p90_ms": {n: float(np.percentile(stage_ms[:, j], 90)) for j, n in enumerate(("hash", "compress", "decompress"))},
        "hash_mfma": {"tflops": hash_flops / (hash_ms * 1e-3) / 1e12, "peak": MFMA_PEAK_TFLOPS[cfg.dtype],
                      "frac": hash_flops / (hash_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS[cfg.dtype],
                      "token_read_gbs": T * row / (hash_ms * 1e-3) / 1e9},
    }
    # supplementary (not part of `value`): the restore fused with the gate-weighted top-k combine, which
    # writes one row per token instead of k
    gw = torch.from_numpy(np.ascontiguousarray(w.gate_weight, dtype=np.float32)).cuda()
    yc = torch.empty((T, d), dtype=tdt, device="cuda")
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(min(K, 50))]
    for i, (e0, e1) in enumerate(ev):
        c = i % copies
        e0.record()
        lsh.lshmoe_decompress_combine(xs[c], outs[c].centroids, ecs[c], outs[c].seg_of, outs[c].seg_offsets, gw, yc)
        e1.record()
    torch.cuda.synchronize()
    comb_ms = float(np.mean([e0.elapsed_time(e1) for e0, e1 in ev[5:]])) if len(ev) > 5 else None
    comb_bytes = (S + T + n_multi_assign + n_multi_seg) * row + 8 * N + 4 * (S + 1)
    result["supplementary_fused_combine"] = {
        "decompress_combine_ms": comb_ms, "algorithmic_bytes": comb_bytes,
        "achieved_gbs": comb_bytes / (comb_ms * 1e-3) / 1e9 if comb_ms else None}
    # supplementary: the same shape at the paper's compression rates (gate correlated with the token, tighter
    # clusters: S/N ~ 0.15 instead of 0.9); same calls, fewer steps, not part of `value`
    if not over and args.paper_regime_steps > 0:
        pcfg = synth.config(args.workload, gate="content", sigma=0.02)
        pw = synth.generate(pcfg)
        px, pe = dev(pw.tokens), torch.from_numpy(pw.expert).cuda()
        lsh.lshmoe_hash(px, rot, bucket)
        lsh.lshmoe_compress(px, pe, bucket, E, L, r, outs[0])
        torch.cuda.synchronize()
        pS = int(outs[0].num_segments.item())
        plen = np.diff(outs[0].seg_offsets[:pS + 1].cpu().numpy())
        p_single = int((plen == 1).sum())

        def pstep(ev=None):
            if ev: ev[0].record()
            lsh.lshmoe_hash(px, rot, bucket)
            if ev: ev[1].record()
            lsh.lshmoe_compress(px, pe, bucket, E, L, r, outs[0])
            if ev: ev[2].record()
            lsh.lshmoe_decompress(px, outs[0].centroids, ecs[0], outs[0].seg_of, outs[0].seg_offsets, k, ys[0],
                                  perm=outs[0].perm, num_segments=outs[0].num_segments)
            if ev: ev[3].record()
        for _ in range(5):
            pstep()
        torch.cuda.synchronize()
        tp0 = time.perf_counter()
        for _ in range(args.paper_regime_steps):
            pstep()
        torch.cuda.synchronize()
        pms = (time.perf_counter() - tp0) * 1e3 / args.paper_regime_steps
        # per-stage times of the same steps, with events on every step (outside the figure above)
        pev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(min(args.paper_regime_steps, 30))]
        for e4 in pev:
            pstep(e4)
        torch.cuda.synchronize()
        pst = np.array([[e4[j].elapsed_time(e4[j + 1]) for j in range(3)] for e4 in pev])
        p_hash, p_comp, p_dec = (float(v) for v in np.median(pst, axis=0))
        p_restore_bytes = (pS + N + (N - p_single) + (pS - p_single)) * row + 4 * N + 4 * (pS + 1)
        p_centroid_bytes = (N + pS) * row + 4 * N + 4 * (pS + 1)
        result["supplementary_paper_regime"] = {
            "workload": "%s, gate=content, sigma=0.02" % cfg.name, "compression_rate": pS / N, "segments": pS,
            "single_member_segments": p_single, "largest_cluster": int(plen.max()),
            "ms_per_step": pms, "tokens_per_s": T / (pms * 1e-3), "steps": args.paper_regime_steps,
            "stages_ms": {"hash": p_hash, "compress": p_comp, "decompress": p_dec},
            "restore": {"algorithmic_bytes": p_restore_bytes, "achieved_gbs": p_restore_bytes / (p_dec * 1e-3) / 1e9,
                        "frac_of_hbm_peak": p_restore_bytes / (p_dec * 1e-3) / 1e9 / HBM_PEAK_GBS},
            "centroid": {"algorithmic_bytes": p_centroid_bytes,
                         "note": "the compress stage is the grouping launches plus the centroid kernel; the kernel "
                                 "trace under profiles/ splits them"}}
        del px, pe
    # supplementary: the hash fused with the gate's projection of the tokens (logits [T, E])
    if d * item % 512 == 0 and r % 8 == 0 and E <= 128:
        gate_w = (torch.randn((E, d), device="cuda") * 0.05).to(tdt)
        logits = torch.empty((T, E), dtype=torch.float32, device="cuda")
        evg = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(min(K, 50))]
        for i, (e0, e1) in enumerate(evg):
            e0.record()
            lsh.lshmoe_hash_gate(xs[i % copies], rot, gate_w, bucket, logits)
            e1.record()
        torch.cuda.synchronize()
        if len(evg) > 5:
            result["supplementary_hash_gate"] = {
                "hash_gate_ms": float(np.mean([e0.elapsed_time(e1) for e0, e1 in evg[5:]])), "hash_ms": float(hash_ms),
                "one_pass_over_tokens": bool(L * r + E <= 128 or (L * r <= 256 and E <= 64 and T >= 32768))}
    # context for the hash kernel: the vendor library's GEMM of the same shape (rotation only: [T, d] x [d, L*r],
    # the rotated coordinates written out, no arg-max), timed the same way on the same rotated token copies.
    # It is not part of the path and not part of `value`.
    if cfg.dtype == "bf16":
        rot2 = rot.reshape(L * r, d)
        yrot = torch.empty((L * r, T), dtype=tdt, device="cuda")
        evl = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(min(K, 50))]
        for i, (e0, e1) in enumerate(evl):
            e0.record()
            torch.matmul(rot2, xs[i % copies].t(), out=yrot)
            e1.record()
        torch.cuda.synchronize()
        if len(evl) > 5:
            lib_ms = float(np.mean([e0.elapsed_time(e1) for e0, e1 in evl[5:]]))
            result["hash_mfma"]["library_gemm_same_shape_ms"] = lib_ms
            result["hash_mfma"]["library_gemm_tflops"] = hash_flops / (lib_ms * 1e-3) / 1e12
        del yrot
    # supplementary: the paper's sweep of the number of hash functions (Section 4.3), on this workload's shape with
    # the content gate: hash lists are prefixes of one list, tokens and gate are the same for every count
    if args.sweep_hashes:
        counts = sorted(int(v) for v in args.sweep_hashes.split(","))
        sr = args.sweep_r
        scfg = synth.config(args.workload, L=counts[-1], r=sr, gate="content", sigma=0.02)
        sw = synth.generate(scfg)
        sx, se, srot = dev(sw.tokens), torch.from_numpy(sw.expert).cuda(), dev(sw.rot)
        sweep = []
        for Ls in counts:
            rot_l = srot[:Ls].contiguous()
            so = lsh.CompressOutputs.allocate(T, d, k, E, Ls, sr, tdt)

            def sstep():
                lsh.lshmoe_hash(sx, rot_l, bucket)
                lsh.lshmoe_compress(sx, se, bucket, E, Ls, sr, so)
                lsh.lshmoe_decompress(sx, so.centroids, ecs[0], so.seg_of, so.seg_offsets, k, ys[0], perm=so.perm,
                                      num_segments=so.num_segments)
            for _ in range(5):
                sstep()
            torch.cuda.synchronize()
            ts0 = time.perf_counter()
            for _ in range(30):
                sstep()
            torch.cuda.synchronize()
            sms = (time.perf_counter() - ts0) * 1e3 / 30
            sweep.append({"hash_functions": Ls, "compression_rate": int(so.num_segments.item()) / N, "ms_per_step": sms})
            del so
        result["supplementary_hash_count_sweep"] = {"workload": "%s, gate=content, sigma=0.02, r=%d" % (cfg.name, sr),
                                                    "points": sweep}
        del sx, se, srot
    # supplementary: backward of the path (segment sums of dL/dY, then dL/dx), on random gradients
    gy = torch.randn((T, k, d), device="cuda").to(tdt)
    hc = torch.randn((N, d), device="cuda").to(tdt)
    gec = torch.empty((N, d), dtype=tdt, device="cuda")
    gx = torch.empty((T, d), dtype=tdt, device="cuda")
    bws = torch.empty(lsh.lshmoe_backward_workspace_bytes(T, d, k, lsh.LSHMOE_F32 if cfg.dtype == "f32" else lsh.LSHMOE_BF16) + 256,
                      dtype=torch.uint8, device="cuda")
    evb = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(min(K, 50))]
    for i, (e0, e1, e2) in enumerate(evb):
        o = outs[i % copies]
        e0.record()
        lsh.lshmoe_decompress_backward(gy, o.perm, o.seg_offsets, o.seg_of, o.num_segments, gec, bws)
        e1.record()
        lsh.lshmoe_compress_backward(gy, hc, gec, o.seg_of, o.seg_offsets, k, gx)
        e2.record()
    torch.cuda.synchronize()
    if len(evb) > 5:
        seg_ms = float(np.mean([e0.elapsed_time(e1) for e0, e1, _ in evb[5:]]))
        gtok_ms = float(np.mean([e1.elapsed_time(e2) for _, e1, e2 in evb[5:]]))
        seg_bytes = (N + S) * row + 4 * N + 4 * (S + 1)                       # N gradient rows read, S sums written
        gtok_bytes = (S + T + n_multi_assign + n_multi_seg) * row + 4 * N + 4 * (S + 1)
        # the two calls run back to back as in a backward pass (the second finds part of the gradient rows the
        # first has just read in the last-level cache); the event between them splits the pair's time only
        # roughly - the kernel trace under profiles/ has the per-kernel durations
        result["supplementary_backward"] = {
            "pair_ms": float(np.mean([e0.elapsed_time(e2) for e0, _, e2 in evb[5:]])),
            "decompress_backward_ms": seg_ms, "decompress_backward_gbs": seg_bytes / (seg_ms * 1e-3) / 1e9,
            "compress_backward_ms": gtok_ms, "compress_backward_gbs": gtok_bytes / (gtok_ms * 1e-3) / 1e9}
    # supplementary: the spherical hash family (Section 4.5), 32 spheres with balanced radii, on the same tokens
    sb = 32
    piv = (torch.randn((sb, d), device="cuda")).to(tdt)
    rsq = torch.full((sb,), float(d * (2.0 + cfg.sigma ** 2)), dtype=torch.float32, device="cuda")
    sbucket = torch.empty(T, dtype=torch.int64, device="cuda")
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(min(K, 50))]
    for i, (e0, e1) in enumerate(evs):
        e0.record()
        lsh.lshmoe_hash_sphere(xs[i % copies], piv, rsq, sbucket)
        e1.record()
    torch.cuda.synchronize()
    if len(evs) > 5:
        sp_ms = float(np.median([e0.elapsed_time(e1) for e0, e1 in evs[5:]]))
        result["supplementary_sphere_hash"] = {"spheres": sb, "ms": sp_ms, "token_read_gbs": T * row / (sp_ms * 1e-3) / 1e9,
                                               "distinct_codes": int(torch.unique(sbucket).numel())}
    del piv, rsq, sbucket
    # supplementary: backward of the fused combine (gate-weight gradient and the row gradients w * dL/dout)
    go = torch.randn((T, d), device="cuda").to(tdt)
    gwo = torch.empty((T, k), dtype=torch.float32, device="cuda")
    gyo = torch.empty((T, k, d), dtype=tdt, device="cuda")
    evc = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(min(K, 50))]
    for i, (e0, e1) in enumerate(evc):
        c = i % copies
        e0.record()
        lsh.lshmoe_decompress_combine_backward(xs[c], outs[c].centroids, ecs[c], outs[c].seg_of, outs[c].seg_offsets, gw,
                                               go, gwo, gyo)
        e1.record()
    torch.cuda.synchronize()
    if len(evc) > 5:
        cb_ms = float(np.median([e0.elapsed_time(e1) for e0, e1 in evc[5:]]))
        # expert-output rows once per cluster, token and centroid rows where the residual can be non-zero, the output
        # gradient once per token, one row gradient written per assignment
        cb_bytes = (S + n_multi_assign + n_multi_seg + T + N) * row + 12 * N + 4 * (S + 1)
        result["supplementary_combine_backward"] = {"ms": cb_ms, "algorithmic_bytes": cb_bytes,
                                                    "achieved_gbs": cb_bytes / (cb_ms * 1e-3) / 1e9}
    del go, gwo, gyo
    if args.peaks:
        mp = measured_peaks()
        result["measured_peaks"] = mp
        traffic = MEASURED_TRAFFIC_BYTES.get((cfg.name, cfg.gate))
        result["roofline"]["frac_of_measured_read_rate"] = achieved / mp["hbm_read_gbs"]
        result["roofline"]["frac_of_measured_copy_rate"] = (traffic if traffic else restore_bytes) / (dec_ms * 1e-3) / 1e9 / mp["hbm_copy_gbs"]
        if cfg.dtype == "bf16":
            result["hash_mfma"]["frac_of_measured_mfma_rate"] = result["hash_mfma"]["tflops"] / mp["mfma_bf16_tflops"]
            result["hash_mfma"]["frac_of_measured_mfma_rate_random_operands"] = (
                result["hash_mfma"]["tflops"] / mp["mfma_bf16_random_operands_tflops"])
    result["cpu_baseline"] = cpu_baseline(w, args.cpu_sample) if args.cpu_sample >= 0 else None
    print(json.dumps(result))


if __name__ == "__main__":
    main()
