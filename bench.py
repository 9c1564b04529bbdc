#!/usr/bin/env python3
"""Benchmark of the IVF-PQ search hot path on one MI355X.

Default workload: C4 = IVF65536,PQ32x8 (L2) over 100M 96-d vectors, 10k queries, k = 100,
nprobe = 64 -- the largest configuration; its 3.2 GB code store exceeds every cache, so the
scan's bytes really come from HBM.  Data are drawn on the device and the index is built in
pieces (about 10 s, outside the timed region).

A "step" is one pass of the whole path -- coarse quantizer, look-up-table
construction, ADC scan, k-selection and merge -- over the full query batch of
the workload, through the C ABI (vs_ivfpq_search), with all inputs resident
in HBM.  Index construction is outside the timed region.

Prints ONE JSON line.  `value` is queries/s; `roofline` describes the
dominant kernel (the fused LUT + scan kernel), timed live with HIP events
that the library records on the same stream around that launch;
`cpu_baseline` is the CPU oracle timed on the host cores on a bounded sample
of the same queries.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
FP32_VECTOR_PEAK_TFLOPS = 157.3
BF16_MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 matrix cores, published
# ADC look-ups per second the vector ALUs can issue: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-operations
# (no packed fp32), 1.5 of them per look-up (its addition + half an address instruction), in units of 1e12
LOOKUP_PEAK_T = 256 * 4 * 16 * 2.4e9 / 1.5 / 1e12
# Next to the published peaks the JSON line carries what THIS GPU reached in THIS run on a
# read-only stream over 2 GiB and on a register-only loop of v_mfma_f32_32x32x16_bf16
# (libvs_calibrate.so; --no-calibrate-peaks leaves them null).
SCAN_SOURCES = ("kernels_ivfpq.hip", "common.hpp")   # what the scan kernels are compiled from


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def scan_kernel_name(cfg, search_type, list_major=False):
    """The scan kernel the library picks for this shape (same rule as its launcher).  list_major:
    the search ran list by list (the call's statistics say so): the dominant kernel is that scan."""
    code_size = cfg["M"] * cfg["nbits"] // 8
    if list_major:
        return "ivfpq_scan_listmajor_kernel"
    if cfg["nbits"] == 8 and (cfg["M"], cfg["d"] // cfg["M"]) in ((16, 8), (32, 3), (8, 4)):
        short = cfg["M"] in (8, 16) and cfg["nb"] <= cfg["nlist"] * 1024
        if short and (cfg["metric"] == 1 or search_type != "tables"):
            return "ivfpq_scan_wave_kernel"
        return "ivfpq_scan_bank_kernel"
    return "ivfpq_scan_pipe_kernel" if code_size in (16, 32, 64) else "ivfpq_scan_kernel"


def calibrate_lib():
    import ctypes
    from paper_2401_08281_amd import build
    path = build.calibrate_lib_path()
    if not os.path.exists(path):
        build.build_calibrate_lib()
    L = ctypes.CDLL(path)
    vp = ctypes.c_void_p
    L.vsc_copy.restype = ctypes.c_int
    L.vsc_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    L.vsc_read_stream.restype = ctypes.c_int
    L.vsc_read_stream.argtypes = [vp, ctypes.c_size_t, ctypes.c_int, vp, ctypes.POINTER(ctypes.c_double), vp]
    L.vsc_mfma_loop.restype = ctypes.c_int
    L.vsc_mfma_loop.argtypes = [ctypes.c_int, vp, ctypes.POINTER(ctypes.c_double), vp]
    return L


def calibrate_peaks(torch):
    """{"read_stream_GBps", "mfma_loop_TFLOPs"} measured now on this GPU, on torch's current stream."""
    import ctypes
    L = calibrate_lib()
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    buf = torch.empty(1 << 29, dtype=torch.float32, device="cuda").normal_()      # 2 GiB: beyond every cache
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    gbs = ctypes.c_double(0.0)
    rc = L.vsc_read_stream(ctypes.c_void_p(buf.data_ptr()), buf.numel() * 4, 5, ctypes.c_void_p(sink.data_ptr()),
                           ctypes.byref(gbs), st)
    assert rc == 0, "vsc_read_stream failed: %d" % rc
    del buf
    out = torch.empty(256 * 2 * 256, dtype=torch.float32, device="cuda")
    tf = ctypes.c_double(0.0)
    rc = L.vsc_mfma_loop(20000, ctypes.c_void_p(out.data_ptr()), ctypes.byref(tf), st)
    assert rc == 0, "vsc_mfma_loop failed: %d" % rc
    torch.cuda.synchronize()
    return {"read_stream_GBps": round(gbs.value, 1), "mfma_loop_TFLOPs": round(tf.value, 1)}


def calibrate_copy(torch):
    """Three 1 GiB device-to-device copies by vs_calibrate_copy_kernel: the known-size reference
    for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE."""
    import ctypes
    L = calibrate_lib()
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    for _ in range(3):
        assert L.vsc_copy(ctypes.c_void_p(src.data_ptr()), ctypes.c_void_p(dst.data_ptr()), src.numel() * 4, st) == 0
    torch.cuda.synchronize()
    del src, dst


def source_stamp():
    """Identifies the scan kernels' source text: traffic figures measured on another text are not
    this build's."""
    import hashlib
    h = hashlib.sha256()
    for name in SCAN_SOURCES:
        with open(os.path.join(ROOT, "paper_2401_08281_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def traffic_key(args, nprobe):
    return "ivfpq_scan_%s_nprobe%d%s" % (args.workload, nprobe,
                                         "" if args.search_type == "tables" else "_" + args.search_type)


def record_traffic(args):
    """--record-traffic FETCH_DIR WRITE_DIR: reads the counter_collection.csv files that two
    `rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE ... -- python3 bench.py --calibrate-copy ...` runs of the
    same workload left in the two folders, scales the scan kernel's counters by what the same
    counters show for the 1 GiB copies of vs_calibrate_copy_kernel, and stores the result, stamped
    with the scan kernels' source text and the commit, in profiles/traffic.json.  No GPU needed."""
    import csv
    import glob
    import subprocess
    import synth_inputs as S
    cfg = S.config(args.workload)
    nprobe = args.nprobe or cfg["nprobe"]
    # (which kernel is the dominant one: the same rule as the library's, search_layout in csrc/api.hip)
    nq_, npr_ = cfg["nq"], min(nprobe, cfg["nlist"])
    list_major = (args.search_type == "tables" and cfg["metric"] == 0 and cfg["nbits"] == 8 and
                  (cfg["M"], cfg["d"] // cfg["M"]) in ((16, 8), (32, 3), (8, 4)) and nq_ >= 4096 and npr_ >= 16 and
                  nq_ * (npr_ - 4) >= 3 * cfg["nlist"] and cfg["nb"] * cfg["M"] >= (512 << 20) and
                  cfg["nb"] >= 1024 * cfg["nlist"])
    kernel = scan_kernel_name(cfg, args.search_type, list_major)
    GIB_KIB = float(1 << 20)
    got = {}
    for counter, folder in zip(("FETCH_SIZE", "WRITE_SIZE"), args.record_traffic):
        vals = {"scan": [], "copy": []}
        files = glob.glob(os.path.join(folder, "**", "*counter_collection.csv"), recursive=True)
        assert files, "no counter_collection.csv under " + folder
        for path in files:
            with open(path) as f:
                for r in csv.DictReader(f):
                    if r["Counter_Name"] != counter:
                        continue
                    if kernel in r["Kernel_Name"]:
                        vals["scan"].append(float(r["Counter_Value"]))
                    elif "vs_calibrate_copy_kernel" in r["Kernel_Name"]:
                        vals["copy"].append(float(r["Counter_Value"]))
        assert vals["scan"] and vals["copy"], "%s: %d scan and %d copy dispatches in %s" % (
            counter, len(vals["scan"]), len(vals["copy"]), folder)
        scan = sum(vals["scan"]) / len(vals["scan"])
        copy = sum(vals["copy"]) / len(vals["copy"])
        scale = GIB_KIB / copy                       # actual KiB per counted KiB
        got[counter] = (scan, copy, scale, len(vals["scan"]))
        print("%s %s: n=%d avg=%.1f KiB per dispatch; 1 GiB copy reads as %.1f KiB -> scale %.3f -> %.3f GB" % (
            kernel, counter, len(vals["scan"]), scan, copy, scale, scan * 1024 * scale / 1e9))
    try:
        commit = subprocess.run(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], capture_output=True,
                                text=True).stdout.strip() or "unknown"
    except OSError:
        commit = "unknown"
    fetch = got["FETCH_SIZE"][0] * 1024 * got["FETCH_SIZE"][2]
    write = got["WRITE_SIZE"][0] * 1024 * got["WRITE_SIZE"][2]
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            table = json.load(f)
    except (OSError, ValueError):
        table = {}
    table[traffic_key(args, nprobe)] = {
        "hbm_bytes_per_launch": int(fetch + write), "fetch_bytes": int(fetch), "write_bytes": int(write),
        "fetch_scale": round(got["FETCH_SIZE"][2], 3), "write_scale": round(got["WRITE_SIZE"][2], 3),
        "kernel": kernel, "scan_source_sha256_16": source_stamp(), "measured_after_commit": commit,
    }
    with open(path, "w") as f:
        json.dump(table, f, indent=1, sort_keys=True)
        f.write("\n")
    print("wrote %s [%s]" % (path, traffic_key(args, nprobe)))
    return 0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C4", choices=["C1", "C3", "C2", "C4", "C5"],
                    help="C4 (default): IVF65536,PQ32x8 on 100M x 96-d vectors, the largest configuration "
                         "and the one whose code store (3.2 GB) exceeds every cache; C3: IVF4096,PQ16x8 on "
                         "1M x 128-d; C5: IVF16384,PQ64x4 inner product on 10M x 768-d; C2: flat search")
    ap.add_argument("--nprobe", type=int, default=None)
    ap.add_argument("--nb", type=int, default=None, help="override database size (debug)")
    ap.add_argument("--refine", type=int, default=0, metavar="K2",
                    help="after the timed search, also time the second stage vs_refine(search's k results "
                         "-> K2 best by exact distance) and report it under config.refine (the headline "
                         "value stays the search alone)")
    ap.add_argument("--train", type=int, default=0, metavar="NITER",
                    help="train the coarse centroids and the PQ codebooks with NITER rounds of k-means "
                         "(vs_ivfpq_train, from the sampled parameters, on the first min(nb, 256 * nlist) "
                         "vectors) before building the index; reported under config.train")
    ap.add_argument("--search-type", default="tables", choices=["tables", "norms", "precomputed"],
                    help="tables (default, the headline form): one look-up table per (query, list) on the "
                         "residual; norms: |q|^2 + |x'|^2 - 2<q,x'> with the norm stored next to every code "
                         "(4 more bytes per vector, one table per query); precomputed: the table of a "
                         "(query, list) pair as a per-query term plus a per-list term computed at set-up "
                         "(nlist * M * 2^nbits floats), one addition per entry instead of d / M multiply-adds")
    ap.add_argument("--index", default="ivfpq", choices=["ivfpq", "ivfflat", "ivfsq8"],
                    help="ivfflat: the same workload's vectors and centroids in an IVF-Flat index "
                         "(secondary line; the default ivfpq is the headline metric)")
    ap.add_argument("--flat-stateless", action="store_true",
                    help="workload C2: time vs_flat_search (database prepared in every call) instead of a "
                         "flat index (prepared once, at add)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three 1 GiB device-to-device copies by vs_calibrate_copy_kernel "
                         "(the known-size reference for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs)")
    ap.add_argument("--calibrate-peaks", dest="calibrate_peaks", action="store_true", default=True,
                    help="measure this GPU's read-stream rate and bf16 matrix-core loop rate in this run and "
                         "report them next to the published peaks (default)")
    ap.add_argument("--no-calibrate-peaks", dest="calibrate_peaks", action="store_false")
    ap.add_argument("--record-traffic", nargs=2, metavar=("FETCH_DIR", "WRITE_DIR"),
                    help="no benchmark: turn the output folders of two rocprofv3 --pmc runs of this workload "
                         "(FETCH_SIZE, then WRITE_SIZE, both with --calibrate-copy) into the workload's entry "
                         "of profiles/traffic.json")
    args = ap.parse_args()
    if args.record_traffic:
        return record_traffic(args)
    if args.gpus != 1:
        print("bench.py: this library runs on ONE GPU; --gpus %d is not supported (to use several, "
              "shard the stored vectors by id over one process per GPU and merge the k best of each)."
              % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2401_08281_amd as vs
    import synth_inputs as S

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    vs.lib()

    if args.calibrate_copy:
        calibrate_copy(torch)
    args.peaks = calibrate_peaks(torch) if args.calibrate_peaks else None
    if args.peaks:
        log("this GPU now: read stream %.0f GB/s, bf16 matrix-core loop %.0f TFLOP/s" % (
            args.peaks["read_stream_GBps"], args.peaks["mfma_loop_TFLOPs"]))

    over = {}
    if args.nb:
        over["nb"] = args.nb
    cfg = S.config(args.workload, **over)
    if args.nprobe and "nprobe" in cfg:
        cfg["nprobe"] = args.nprobe
    t0 = time.time()
    big = cfg["nb"] * cfg["d"] * 4 > (8 << 30)       # generated on the device, added in pieces
    if big:
        xd, qd = S.make_data_device(cfg)
        torch.cuda.synchronize()
        x, q = None, qd.cpu().numpy()
    else:
        x, q = S.make_data(cfg)
        xd, qd = torch.from_numpy(x).cuda(), torch.from_numpy(q).cuda()
    log("data %s: x %s q %s in %.1fs" % (args.workload, tuple(xd.shape), q.shape, time.time() - t0))
    nq, k, metric = cfg["nq"], cfg["k"], cfg["metric"]

    if args.workload == "C2":
        return bench_flat(args, cfg, x, q, xd, qd)

    cent, cb = S.make_index_params_device(cfg, xd) if big else S.make_index_params(cfg, x)
    if args.index in ("ivfflat", "ivfsq8"):
        return bench_ivfflat(args, cfg, x, q, xd, qd, cent)
    train = None
    if args.train > 0:
        n_train = min(cfg["nb"], 256 * cfg["nlist"])
        cent_d, cb_d = torch.from_numpy(cent).cuda(), torch.from_numpy(cb).cuda()
        torch.cuda.synchronize()
        t0 = time.time()
        objs = vs.vs_ivfpq_train(xd[:n_train], metric, cent_d, cb_d, cfg["nbits"], args.train)
        torch.cuda.synchronize()
        t_train = time.time() - t0
        cent, cb = cent_d.cpu().numpy(), cb_d.cpu().numpy()
        train = {"niter": args.train, "n_train": int(n_train), "seconds": round(t_train, 2),
                 "coarse_mse_first_last": [objs[0][0], objs[0][-1]],
                 "pq_mse_first_last": [float(sum(o[0] for o in objs[1:])), float(sum(o[-1] for o in objs[1:]))]}
        log("trained in %.2fs: coarse MSE %.4g -> %.4g, PQ residual MSE %.4g -> %.4g" % (
            t_train, objs[0][0], objs[0][-1], train["pq_mse_first_last"][0], train["pq_mse_first_last"][1]))
    ix = vs.IVFPQ(cfg["d"], metric, torch.from_numpy(cent).cuda(), torch.from_numpy(cb).cuda(),
                  cfg["nbits"])
    if args.search_type == "norms":
        ix.set_search_type(vs.ST_STORED_NORMS)
    if args.search_type == "precomputed":
        ix.set_search_type(vs.ST_PRECOMPUTED_TABLES)
    torch.cuda.synchronize()
    t0 = time.time()
    piece = 10_000_000
    for s0 in range(0, cfg["nb"], piece):
        ix.add(xd[s0:s0 + piece])
        if big:
            torch.cuda.synchronize()
            log("  added %d / %d (%.1fs)" % (min(s0 + piece, cfg["nb"]), cfg["nb"], time.time() - t0))
    torch.cuda.synchronize()
    t_add = time.time() - t0
    log("index built: ntotal=%d in %.2fs" % (ix.ntotal, t_add))
    nprobe = cfg["nprobe"]
    code_size = cfg["M"] * cfg["nbits"] // 8 + (4 if args.search_type == "norms" else 0)

    # algorithmic work of the scan: codes visited by the batch, counted by the library in the
    # same call that searches (vs_ivfpq_search_stats)
    sizes = ix.list_sizes()
    _, _, stats = ix.search_stats(qd, k, nprobe)
    scanned = stats["scanned_codes"]
    pairs = nq * min(nprobe, cfg["nlist"])
    imbalance = float((sizes.double() ** 2).sum().item() * cfg["nlist"] / float(cfg["nb"]) ** 2)

    D = torch.empty((nq, k), dtype=torch.float32, device="cuda")
    I = torch.empty((nq, k), dtype=torch.int64, device="cuda")
    for _ in range(args.warmup):
        ix.search(qd, k, nprobe, D, I)
    torch.cuda.synchronize()
    vs.vs_profile_enable(True)
    vs.vs_profile_read()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ix.search(qd, k, nprobe, D, I)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = vs.vs_profile_read()
    vs.vs_profile_enable(False)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    qps = nq / (ms_per_step * 1e-3)
    stage_ms = {s: v[0] / args.steps for s, v in prof.items()}        # per step, all launches
    log("per-step ms: " + ", ".join("%s=%.3f" % (s, v) for s, v in stage_ms.items() if v))

    scan_ms = prof["scan"][0] / max(prof["scan"][1], 1)               # per launch (one per step)
    # a list-major search: stage "scan" is the list-major kernel alone, which visits the codes of
    # all probes but the first few of every query (those are stage "scan_first", query-major)
    list_major = stats["list_major_first_probes"] > 0
    scanned_dominant = scanned - stats["list_major_first_codes"]
    algo_bytes = scanned_dominant * code_size
    if list_major:
        pairs = nq * (min(nprobe, cfg["nlist"]) - stats["list_major_first_probes"])
    achieved = algo_bytes / (scan_ms * 1e-3) / 1e9 if scan_ms > 0 else 0.0

    # accuracy against exact search (GPU flat search, itself checked against the oracle by the tests)
    nrec = nq if not big else 1000                    # exact search over 1e8 rows: first 1000 queries
    Dg, Ig = vs.vs_flat_search(xd, qd[:nrec].contiguous(), k, metric)
    torch.cuda.synchronize()
    I_h, Ig_h = I.cpu().numpy(), Ig.cpu().numpy()
    hit_k = np.mean([len(set(I_h[a].tolist()) & set(Ig_h[a].tolist())) / float(k) for a in range(nrec)])
    hit_1 = np.mean([Ig_h[a, 0] in I_h[a] for a in range(nrec)])
    k10 = min(10, k)   # 10-recall@10 from the first 10 ranks of both result lists
    hit_10 = np.mean([len(set(I_h[a, :k10].tolist()) & set(Ig_h[a, :k10].tolist())) / float(k10)
                      for a in range(nrec)])

    refine = None
    if args.refine > 0:
        # second stage (Sec. 3.5): exact distances for the k results of the first stage
        k2 = min(args.refine, k)
        D2 = torch.empty((nq, k2), dtype=torch.float32, device="cuda")
        I2 = torch.empty((nq, k2), dtype=torch.int64, device="cuda")
        for _ in range(args.warmup):
            vs.vs_refine(xd, qd, I, k2, metric, D2, I2)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            vs.vs_refine(xd, qd, I, k2, metric, D2, I2)
        torch.cuda.synchronize()
        r_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        I2_h = I2.cpu().numpy()
        hit_r = np.mean([len(set(I2_h[a].tolist()) & set(Ig_h[a, :k2].tolist())) / float(k2)
                         for a in range(nrec)])
        hit_f = np.mean([len(set(I_h[a, :k2].tolist()) & set(Ig_h[a, :k2].tolist())) / float(k2)
                         for a in range(nrec)])
        gathered = float((I >= 0).sum().item()) * cfg["d"] * 4
        refine = {"k_in": k, "k_out": k2, "ms_per_step": round(r_ms, 4),
                  "gather_GBps": round(gathered / (r_ms * 1e-3) / 1e9, 1),
                  "recall_%d_at_%d_first_stage" % (k2, k2): round(float(hit_f), 4),
                  "recall_%d_at_%d_refined" % (k2, k2): round(float(hit_r), 4),
                  "queries_per_s_search_plus_refine": nq / ((ms_per_step + r_ms) * 1e-3)}
        log("refine %d -> %d: %.3f ms, recall %.4f -> %.4f" % (k, k2, r_ms, hit_f, hit_r))

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline_ivfpq(cfg, cent, cb, ix, q, k, nprobe)

    # rows of the coarse quantizer that the last timed call redid exactly (the first call of an
    # index may redo many while the sweeps learn which operand precision this data needs)
    _, _, stats_after = ix.search_stats(qd, k, nprobe)
    traffic = load_traffic(traffic_key(args, nprobe))
    peaks = args.peaks or {}
    read_now = peaks.get("read_stream_GBps")
    # the coarse quantizer's distance stage: algorithmic flop of one nq x nlist x d contraction
    # over the stage's time (operand preparation and every sweep and pass included)
    coarse_ms = stage_ms.get("coarse_dist", 0.0)
    coarse_flop = 2.0 * nq * cfg["nlist"] * cfg["d"]
    on_mfma = stats["coarse_rows_matrix_core"] > 0
    coarse_tf = coarse_flop / (coarse_ms * 1e-3) / 1e12 if coarse_ms > 0 else 0.0
    coarse_peak = BF16_MFMA_PEAK_TFLOPS if on_mfma else FP32_VECTOR_PEAK_TFLOPS
    roofline_coarse = {
        "bound": "mfma" if on_mfma else "alu",
        "kernel": ("%s (stage: operand preparation + minima sweep + collect sweep)" % (
            "mfma_sweep_kernel" if cfg["d"] in (32, 64, 96, 128) else "mfma_sweep_kc_kernel")) if on_mfma
                  else "canon_matrix_kernel",
        "achieved": coarse_tf, "peak": coarse_peak, "unit": "TFLOP/s", "frac": coarse_tf / coarse_peak,
        "algorithmic_flop_per_step": coarse_flop, "stage_ms": coarse_ms,
        "peak_measured_mfma_loop": peaks.get("mfma_loop_TFLOPs") if on_mfma else None,
        "rows_matrix_core": stats["coarse_rows_matrix_core"],
        "rows_exact_fallback": stats_after["coarse_rows_fallback"],
        "rows_exact_fallback_first_call": stats["coarse_rows_fallback"], "traffic": None}
    roofline = {"bound": "hbm", "kernel": scan_kernel_name(cfg, args.search_type, list_major), "achieved": achieved,
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                "peak_measured_read_stream": read_now,
                "frac_of_measured": achieved / read_now if read_now else None,
                "traffic": traffic, "algorithmic_bytes_per_launch": algo_bytes,
                "kernel_ms": scan_ms, "pairs_per_launch": pairs,
                "probed_nonempty_lists_per_launch": stats["probed_lists"]}
    if list_major:
        # The list-major scan reads every probed list from HBM about once per batch, so HBM no
        # longer bounds it: its limit is the issue rate of the vector ALUs.  Algorithmic work: one
        # fp32 addition per table entry looked up (M per code).  Peak: 256 CUs x 4 SIMDs x 16
        # lanes x 2.4 GHz = 39.3e12 vector lane-operations/s without packed fp32; a look-up takes
        # at least its addition and half an address instruction (one address serves the tables
        # of two queries): 39.3e12 / 1.5 = 26.2e12 look-ups/s.
        lookups = float(scanned_dominant) * cfg["M"]
        alu_peak = LOOKUP_PEAK_T
        alu = lookups / (scan_ms * 1e-3) / 1e12 if scan_ms > 0 else 0.0
        roofline = {"bound": "alu", "kernel": roofline["kernel"], "achieved": alu, "peak": alu_peak,
                    "unit": "TFLOP/s", "frac": alu / alu_peak,
                    "peak_derivation": "256 CU x 4 SIMD x 16 lanes x 2.4 GHz / 1.5 vector instructions per "
                                       "look-up (one fp32 addition + half an address instruction); no packed fp32",
                    "algorithmic_flop_per_launch": lookups, "traffic": traffic, "kernel_ms": scan_ms,
                    "pairs_per_launch": pairs, "probed_nonempty_lists_per_launch": stats["probed_lists"],
                    "hbm_equivalent": {"algorithmic_bytes_per_launch": algo_bytes, "achieved_GBps": achieved,
                                       "frac_of_peak": achieved / HBM_PEAK_GBS,
                                       "peak_measured_read_stream": read_now,
                                       "note": "codes visited x code size over the kernel's time; every probed "
                                               "list comes from HBM about once per batch (see traffic), so this "
                                               "rate is not an HBM rate and may exceed the HBM peak"},
                    "list_major": {"first_probes_per_query": stats["list_major_first_probes"],
                                   "codes_scanned_query_major_first": stats["list_major_first_codes"],
                                   "queries_rescanned": stats_after["list_major_rescanned"]}}
    out = {
        "metric": "IVF-PQ queries/sec at fixed nprobe & recall@10; ADC-scan HBM GB/s vs peak",
        "value": qps, "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: IVF%d,PQ%dx%d %s, nb=%d d=%d nq=%d k=%d nprobe=%d" % (
            args.workload, cfg["nlist"], cfg["M"], cfg["nbits"], "IP" if metric else "L2", cfg["nb"],
            cfg["d"], nq, k, nprobe),
            "search_type": args.search_type, "scan_bytes_per_code": code_size,
            "nprobe": nprobe, "k": k, "recall_k_at_k": round(float(hit_k), 4),
            "recall_1_at_k": round(float(hit_1), 4), "recall_10_at_10": round(float(hit_10), 4),
            "recall_queries": int(nrec), "scanned_codes_per_query": scanned / nq,
            "imbalance_factor": round(imbalance, 3), "index_build_s": round(t_add, 2),
            "stage_ms_per_step": {s: round(v, 4) for s, v in stage_ms.items() if v},
            **({"refine": refine} if refine else {}), **({"train": train} if train else {})},
        "roofline": roofline,
        "roofline_coarse": roofline_coarse,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    return 0


def cpu_baseline_ivfpq(cfg, cent, cb, ix, q, k, nprobe):
    """The oracle's IVF-PQ search on the GPU-built store, bounded sample of queries."""
    import numpy as np
    import oracle
    ids, _ = ix.assignments()
    sizes = ix.list_sizes().cpu().numpy()
    off = np.zeros(cfg["nlist"] + 1, dtype=np.int64)
    np.cumsum(sizes, out=off[1:])
    orc = oracle.OracleIVFPQ.from_storage(cfg["d"], cfg["metric"], cent, cb, cfg["nbits"], off,
                                          ix.codes().cpu().numpy(), ids.cpu().numpy())
    n = min(cfg["nq"], 200)
    t0 = time.perf_counter(); orc.search(q[:n], k, nprobe); dt = time.perf_counter() - t0
    # size the timed sample for ~10 s of CPU work: more queries, then whole-batch repeats
    want = n * 10.0 / max(dt, 1e-3)
    n2 = int(min(cfg["nq"], max(n, want)))
    reps = int(max(1, min(50, round(want / n2))))
    t0 = time.perf_counter()
    for _ in range(reps):
        orc.search(q[:n2], k, nprobe)
    dt = time.perf_counter() - t0
    log("oracle: %d queries x %d passes in %.2fs on %d threads" % (n2, reps, dt, oracle.num_threads()))
    return {"value": n2 * reps / dt, "unit": "queries/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": "first %d of %d queries x %d passes, same index and nprobe, %.1f s" % (
                n2, cfg["nq"], reps, dt)}


def bench_flat(args, cfg, x, q, xd, qd):
    """Secondary workload: flat exact search (C2).  Same JSON shape, its own metric name."""
    import torch
    import oracle
    import paper_2401_08281_amd as vs
    nq, k, metric, d, nb = cfg["nq"], cfg["k"], cfg["metric"], cfg["d"], cfg["nb"]
    D = torch.empty((nq, k), dtype=torch.float32, device="cuda")
    I = torch.empty((nq, k), dtype=torch.int64, device="cuda")
    vs.vs_counters_read()
    if args.flat_stateless:      # the stateless entry point: prepares the database in every call
        search = lambda: vs.vs_flat_search(xd, qd, k, metric, D, I)
    else:                        # a flat index: the database is prepared when it is added
        ix = vs.Flat(d, metric)
        ix.add(xd)
        search = lambda: ix.search(qd, k, D, I)
    for _ in range(args.warmup):
        search()
    torch.cuda.synchronize()
    vs.vs_profile_enable(True); vs.vs_profile_read()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        search()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = vs.vs_profile_read(); vs.vs_profile_enable(False)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    dist_ms_total = prof["flat_dist"][0] / args.steps
    mfma_rows, fallback_rows = vs.vs_counters_read()
    if mfma_rows > 0:
        # matrix-core route: the distance stage is operand preparation + the sampled minima sweep +
        # the collect sweep (the dominant kernel).  Algorithmic work = one nq x nb x d contraction;
        # the whole stage's time is charged to it, so the fraction is a lower bound for the kernel.
        flops = 2.0 * nq * nb * d
        achieved = flops / (dist_ms_total * 1e-3) / 1e12
        roof = {"bound": "mfma", "kernel": "mfma_sweep_kernel (stage: operand preparation + minima sweep + collect sweep)",
                "achieved": achieved, "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / BF16_MFMA_PEAK_TFLOPS,
                "peak_measured_mfma_loop": (args.peaks or {}).get("mfma_loop_TFLOPs"),
                "frac_of_measured": achieved / args.peaks["mfma_loop_TFLOPs"] if args.peaks else None,
                "algorithmic_flop_per_step": flops, "traffic": None,
                "exact_fallback_rows_per_step": fallback_rows / (args.warmup + args.steps)}
    else:
        flops = 3.0 * nq * nb * d      # sub + fma per pair and dimension
        achieved = flops / (dist_ms_total * 1e-3) / 1e12
        roof = {"bound": "alu", "kernel": "canon_matrix_kernel", "achieved": achieved,
                "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / FP32_VECTOR_PEAK_TFLOPS, "traffic": None}
    cpu = None
    if not args.no_cpu_baseline:
        n = 16
        t0 = time.perf_counter(); oracle.flat_search(x, q[:n], k, metric); dt = time.perf_counter() - t0
        cpu = {"value": n / dt, "unit": "queries/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": "first %d of %d queries, %.1f s" % (n, nq, dt)}
    out = {
        "metric": "flat exact k-NN queries/sec", "value": nq / (ms_per_step * 1e-3),
        "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "C2: flat L2, nb=%d d=%d nq=%d k=%d" % (nb, d, nq, k),
                   "entry_point": "vs_flat_search" if args.flat_stateless else "vs_flat_index_search",
                   "stage_ms_per_step": {s: round(v[0] / args.steps, 3) for s, v in prof.items() if v[1]}},
        "roofline": roof,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    return 0


def bench_ivfflat(args, cfg, x, q, xd, qd, cent):
    """Secondary workload: IVF-Flat on the vectors and centroids of an IVF-PQ configuration."""
    import numpy as np
    import torch
    import oracle
    import paper_2401_08281_amd as vs
    nq, k, metric, d, nb, nprobe = cfg["nq"], cfg["k"], cfg["metric"], cfg["d"], cfg["nb"], cfg["nprobe"]
    sq8 = args.index == "ivfsq8"
    if sq8:   # ranges of the scalar quantizer from the first 1M vectors (min / max per component)
        head = xd[: min(nb, 1_000_000)]
        vmin = head.min(dim=0).values.contiguous()
        step = ((head.max(dim=0).values - vmin) / 256.0).clamp_min(1e-30).contiguous()
        ix = vs.IVFSQ8(d, metric, torch.from_numpy(cent).cuda(), vmin, step)
    else:
        ix = vs.IVFFlat(d, metric, torch.from_numpy(cent).cuda())
    t0 = time.time()
    for s0 in range(0, nb, 10_000_000):
        ix.add(xd[s0:s0 + 10_000_000])
    torch.cuda.synchronize()
    t_add = time.time() - t0
    sizes = ix.list_sizes()
    D = torch.empty((nq, k), dtype=torch.float32, device="cuda")
    I = torch.empty((nq, k), dtype=torch.int64, device="cuda")
    for _ in range(args.warmup):
        ix.search(qd, k, nprobe, D, I)
    torch.cuda.synchronize()
    vs.vs_profile_enable(True); vs.vs_profile_read()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ix.search(qd, k, nprobe, D, I)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = vs.vs_profile_read(); vs.vs_profile_enable(False)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    scan_ms = prof["scan"][0] / max(prof["scan"][1], 1)
    # algorithmic bytes of the scan: rows visited x d x 4 (probes from the same coarse quantizer)
    ixq = vs.IVFPQ(d, metric, torch.from_numpy(cent).cuda(),
                   torch.zeros((1, 256, d), dtype=torch.float32, device="cuda"), 8)
    probes, _ = ixq.coarse(qd, nprobe)
    ixq.close()
    scanned = int(sizes[probes.long()].sum().item())
    algo = scanned * d * (1 if sq8 else 4)
    achieved = algo / (scan_ms * 1e-3) / 1e9
    nrec = min(nq, 1000)
    Dg, Ig = vs.vs_flat_search(xd, qd[:nrec].contiguous(), k, metric)
    I_h, Ig_h = I.cpu().numpy(), Ig.cpu().numpy()
    hit_k = np.mean([len(set(I_h[a].tolist()) & set(Ig_h[a].tolist())) / float(k) for a in range(nrec)])
    cpu = None
    if not args.no_cpu_baseline and x is not None:
        orc = oracle.OracleIVFSQ8(d, metric, cent, vmin.cpu().numpy(), step.cpu().numpy()) if sq8 \
            else oracle.OracleIVFFlat(d, metric, cent)
        orc.add(x)
        n = min(nq, 500)
        t0 = time.perf_counter(); orc.search(q[:n], k, nprobe); dt = time.perf_counter() - t0
        cpu = {"value": n / dt, "unit": "queries/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": "first %d of %d queries, %.1f s" % (n, nq, dt)}
    out = {
        "metric": "%s queries/sec at fixed nprobe" % ("IVF-SQ8" if sq8 else "IVF-Flat"),
        "value": nq / (ms_per_step * 1e-3),
        "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s vectors in IVF%d,%s %s, nb=%d d=%d nq=%d k=%d nprobe=%d" % (
            args.workload, cfg["nlist"], "SQ8" if sq8 else "Flat", "IP" if metric else "L2", nb, d, nq, k,
            nprobe),
            "recall_k_at_k": round(float(hit_k), 4), "recall_queries": int(nrec),
            "scanned_vectors_per_query": scanned / nq, "index_build_s": round(t_add, 2),
            "stage_ms_per_step": {s: round(v[0] / args.steps, 4) for s, v in prof.items() if v[1]}},
        "roofline": {"bound": "hbm", "kernel": ("ivfsq8_scan" if sq8 else "ivfflat_scan") + ("_tiled_kernel" if d % 32 == 0 else "_kernel"), "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "peak_measured_read_stream": (args.peaks or {}).get("read_stream_GBps"),
                     "frac_of_measured": achieved / args.peaks["read_stream_GBps"] if args.peaks else None,
                     "traffic": None, "algorithmic_bytes_per_launch": algo, "kernel_ms": scan_ms},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    return 0


def load_traffic(key):
    """HBM bytes per launch measured with rocprofv3 --pmc in separate runs (--record-traffic), if
    recorded for the scan kernels' present source text; None otherwise."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            rec = json.load(f).get(key)
        if not rec or rec.get("scan_source_sha256_16") != source_stamp():
            return None
        return rec["hbm_bytes_per_launch"]
    except (OSError, ValueError, KeyError):
        return None


if __name__ == "__main__":
    sys.exit(main())
