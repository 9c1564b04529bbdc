"""Host-side checks that need no GPU: the C-ABI library loads, exports every
symbol the header declares, and rejects bad arguments before touching the
device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "vs.h")


@pytest.fixture(scope="module")
def L():
    import paper_2401_08281_amd as vs
    return vs.lib()


def declared_symbols():
    text = open(HEADER).read()
    return re.findall(r"VS_API\s+[\w\s\*]+?\b(vs_\w+)\s*\(", text)


# The boundary, name by name.  The paper's interface (App. A.1 "add / search", Sec. 5.1 inverted
# lists, Sec. 4.1 / 4.3 training, Sec. 3.2 refinement) as this library exports it.
BOUNDARY = """
vs_flat_search vs_flat_create vs_flat_destroy vs_flat_ntotal vs_flat_add vs_flat_index_search
vs_trim vs_refine vs_kmeans vs_ivfpq_train
vs_ivfpq_create vs_ivfpq_add vs_ivfpq_search vs_ivfpq_search_stats vs_ivfpq_search_static vs_ivfpq_destroy
vs_ivfpq_ntotal vs_ivfpq_code_size vs_ivfpq_get_list_sizes vs_ivfpq_get_assignments vs_ivfpq_get_codes
vs_ivfpq_coarse vs_ivfpq_set_search_type vs_ivfpq_set_coarse_metric vs_ivfpq_get_norms
vs_ivfflat_create vs_ivfflat_destroy vs_ivfflat_ntotal vs_ivfflat_add vs_ivfflat_search
vs_ivfflat_get_list_sizes vs_ivfflat_get_storage
vs_ivfsq8_create vs_ivfsq8_destroy vs_ivfsq8_ntotal vs_ivfsq8_add vs_ivfsq8_search
vs_ivfsq8_get_list_sizes vs_ivfsq8_get_storage
vs_profile_enable vs_profile_read vs_set_option vs_counters_read vs_knn_workspace_bytes
vs_last_error vs_version
""".split()


def test_header_declares_the_boundary():
    """The header declares exactly the boundary: nothing missing, nothing extra, nothing twice."""
    names = declared_symbols()
    assert len(names) == len(set(names))
    assert sorted(names) == sorted(BOUNDARY)


def test_binding_has_a_function_of_the_same_name_for_every_entry_point():
    import paper_2401_08281_amd as vs
    for name in BOUNDARY:
        assert callable(getattr(vs, name, None)), name


def test_library_exports_every_declared_symbol(L):
    for name in declared_symbols():
        assert hasattr(L, name), name
    assert L.vs_version().decode().startswith("vs ")


def test_no_internal_symbols_leak(L):
    import subprocess
    import paper_2401_08281_amd.build as b
    out = subprocess.run(["nm", "-D", "--defined-only", b.lib_path()], capture_output=True, text=True).stdout
    exported = [l.split()[-1] for l in out.splitlines() if " T " in l]
    assert sorted(exported) == sorted(declared_symbols())


def test_argument_errors_are_reported_without_a_device(L):
    nul = ctypes.c_void_p(0)
    one = ctypes.c_void_p(16)   # never dereferenced: validation fails first
    INVALID, UNSUPPORTED = -1, -2
    assert L.vs_flat_search(one, 10, one, 1, 0, 0, 1, one, one, nul) == INVALID      # d < 1
    assert b"d = 0" in L.vs_last_error()
    assert L.vs_flat_search(one, 10, one, 1, 4, 0, 0, one, one, nul) == INVALID      # k < 1
    assert L.vs_flat_search(one, 10, one, 1, 4, 0, 1025, one, one, nul) == INVALID   # k > VS_MAX_K
    assert L.vs_flat_search(one, 10, one, 1, 4, 7, 1, one, one, nul) == INVALID      # metric
    assert L.vs_flat_search(one, 10, nul, 1, 4, 0, 1, one, one, nul) == INVALID      # null q
    assert L.vs_flat_search(one, -1, one, 1, 4, 0, 1, one, one, nul) == INVALID
    assert L.vs_flat_search(nul, 10, nul, 0, 4, 0, 1, nul, nul, nul) == 0            # nq == 0: no-op
    # flat index: vs_flat_create(out, d, metric), vs_flat_add(ix, x, n, stream),
    # vs_flat_index_search(ix, q, nq, k, out_dist, out_ids, stream)
    h = ctypes.c_void_p()
    assert L.vs_flat_create(None, 4, 0) == INVALID
    assert L.vs_flat_create(ctypes.byref(h), 0, 0) == INVALID and not h.value       # d < 1
    assert L.vs_flat_create(ctypes.byref(h), 4, 5) == INVALID and not h.value       # metric
    assert L.vs_flat_add(nul, one, 3, nul) == INVALID                                # null index
    assert L.vs_flat_index_search(nul, one, 1, 1, one, one, nul) == INVALID
    assert L.vs_flat_ntotal(nul) == -1
    L.vs_flat_destroy(nul)                                                           # no-op
    assert L.vs_refine(one, 10, one, 1, 0, 0, one, 5, 1, one, one, nul) == INVALID       # d < 1
    assert L.vs_refine(one, 10, one, 1, 4, 0, one, 0, 1, one, one, nul) == INVALID       # kc < 1
    assert b"kc = 0" in L.vs_last_error()
    assert L.vs_refine(one, 10, one, 1, 4, 0, one, 5, 0, one, one, nul) == INVALID       # k < 1
    assert L.vs_refine(one, 10, one, 1, 4, 0, one, 5, 1025, one, one, nul) == INVALID    # k > VS_MAX_K
    assert L.vs_refine(one, 10, one, 1, 4, 3, one, 5, 1, one, one, nul) == INVALID       # metric
    assert L.vs_refine(one, 10, one, 1, 4, 0, nul, 5, 1, one, one, nul) == INVALID       # null shortlist
    assert L.vs_refine(one, 1 << 32, one, 1, 4, 0, one, 5, 1, one, one, nul) == INVALID  # ids must fit 32 bits
    assert L.vs_refine(one, 10, one, 1, 20000, 0, one, 5, 1024, one, one, nul) == UNSUPPORTED   # LDS
    assert L.vs_refine(nul, 10, nul, 0, 4, 0, nul, 5, 1, nul, nul, nul) == 0             # nq == 0: no-op
    # vs_kmeans(x, n, d, K, niter, centroids, objective, assign, stream)
    assert L.vs_kmeans(one, 10, 0, 4, 1, one, nul, nul, nul) == INVALID                       # d < 1
    assert L.vs_kmeans(one, 10, 4, 0, 1, one, nul, nul, nul) == INVALID                       # K < 1
    assert L.vs_kmeans(one, 10, 4, 4, -1, one, nul, nul, nul) == INVALID                      # niter < 0
    assert L.vs_kmeans(one, 1 << 31, 4, 4, 1, one, nul, nul, nul) == INVALID                  # n
    assert L.vs_kmeans(one, 10, 4, 4, 1, nul, nul, nul, nul) == INVALID                       # null centroids
    assert L.vs_kmeans(one, 10, 4, 4, 0, one, nul, nul, nul) == 0                             # no round: no-op
    # vs_ivfpq_train(x, n, d, metric, nlist, M, nbits, niter, centroids, codebooks, objective, stream)
    assert L.vs_ivfpq_train(one, 10, 32, 0, 4, 5, 8, 1, one, one, nul, nul) == INVALID   # d % M
    assert L.vs_ivfpq_train(one, 10, 32, 0, 4, 8, 5, 1, one, one, nul, nul) == UNSUPPORTED  # nbits
    assert L.vs_ivfpq_train(one, 0, 32, 0, 4, 8, 8, 1, one, one, nul, nul) == INVALID    # n < 1
    assert L.vs_ivfpq_train(one, 10, 32, 2, 4, 8, 8, 1, one, one, nul, nul) == INVALID   # metric
    assert L.vs_ivfpq_train(one, 10, 32, 0, 4, 8, 8, 1, one, nul, nul, nul) == INVALID   # null codebooks
    hf = ctypes.c_void_p(0)
    reff = ctypes.byref(hf)
    assert L.vs_ivfflat_create(reff, 0, 0, 16, one, nul) == INVALID                      # d < 1
    assert L.vs_ivfflat_create(reff, 32, 0, 0, one, nul) == INVALID                      # nlist < 1
    assert L.vs_ivfflat_create(reff, 32, 5, 16, one, nul) == INVALID                     # metric
    assert L.vs_ivfflat_create(reff, 32, 0, 16, nul, nul) == INVALID                     # null centroids
    assert L.vs_ivfflat_create(None, 32, 0, 16, one, nul) == INVALID
    assert hf.value is None
    assert L.vs_ivfflat_add(nul, one, 5, nul, nul) == INVALID
    assert L.vs_ivfflat_search(nul, one, 5, 10, 4, one, one, nul) == INVALID
    assert L.vs_ivfflat_ntotal(nul) == -1
    L.vs_ivfflat_destroy(nul)                                                             # allowed
    hs = ctypes.c_void_p(0)
    refs = ctypes.byref(hs)
    assert L.vs_ivfsq8_create(refs, 0, 0, 16, one, one, one, nul) == INVALID              # d < 1
    assert L.vs_ivfsq8_create(refs, 32, 0, 16, one, nul, one, nul) == INVALID             # null vmin
    assert L.vs_ivfsq8_create(refs, 32, 9, 16, one, one, one, nul) == INVALID             # metric
    assert hs.value is None
    assert L.vs_ivfsq8_add(nul, one, 5, nul, nul) == INVALID
    assert L.vs_ivfsq8_search(nul, one, 5, 10, 4, one, one, nul) == INVALID
    assert L.vs_ivfsq8_ntotal(nul) == -1
    L.vs_ivfsq8_destroy(nul)
    h = ctypes.c_void_p(0)
    ref = ctypes.byref(h)
    assert L.vs_ivfpq_create(ref, 32, 0, 16, 5, 8, one, one, nul) == INVALID         # d % M
    assert b"multiple" in L.vs_last_error()
    assert L.vs_ivfpq_create(ref, 32, 0, 16, 8, 6, one, one, nul) == UNSUPPORTED     # nbits
    assert L.vs_ivfpq_create(ref, 30, 0, 16, 5, 4, one, one, nul) == INVALID         # odd M, 4 bit
    assert L.vs_ivfpq_create(ref, 32, 0, 0, 8, 8, one, one, nul) == INVALID          # nlist
    assert L.vs_ivfpq_create(ref, 32, 0, 16, 8, 8, nul, one, nul) == INVALID         # null centroids
    assert L.vs_ivfpq_create(None, 32, 0, 16, 8, 8, one, one, nul) == INVALID
    assert h.value is None
    assert L.vs_ivfpq_add(nul, one, 5, nul, nul) == INVALID
    assert L.vs_ivfpq_search(nul, one, 5, 10, 4, one, one, nul) == INVALID
    assert L.vs_ivfpq_search_stats(nul, one, 5, 10, 4, one, one, one, nul) == INVALID
    assert L.vs_ivfpq_search_static(nul, one, 5, 10, 4, one, one, nul) == INVALID
    assert L.vs_ivfpq_set_coarse_metric(nul, 0) == INVALID
    assert L.vs_ivfpq_ntotal(nul) == -1 and L.vs_ivfpq_code_size(nul) == -1
    L.vs_ivfpq_destroy(nul)                                                           # allowed


def test_binding_rejects_host_tensors():
    import torch
    import paper_2401_08281_amd as vs
    with pytest.raises(TypeError):
        vs.vs_flat_search(torch.zeros(4, 2), torch.zeros(1, 2), 1)


def test_knn_workspace_covers_every_piece_size():
    """The scratch planned for n rows in pieces must hold every piece that will run -- the full
    ones and the shorter last one, which may be laid out with more splits than a full piece
    (host arithmetic only: no GPU).  Checked over seeded random shapes and on the shape that
    once wrote past a buffer planned from the full piece alone."""
    import numpy as np
    import paper_2401_08281_amd as vs
    rng = np.random.default_rng(5)
    cases = [((1 << 20) + 931_328, 1 << 20, 1024, 96, 1, True)]
    for _ in range(300):
        piece = int(rng.choice([1 << 10, 1 << 14, 1 << 17, 1 << 20]))
        n = int(rng.integers(1, 5 * piece))
        nb = int(rng.choice([1, 7, 256, 1024, 4096, 65536, 1_000_000]))
        d = int(rng.choice([4, 30, 32, 64, 96, 128, 160, 768]))
        k = int(rng.choice([1, 10, 64, 100, 150, 151, 1024]))
        cases.append((n, piece, nb, d, k, bool(rng.integers(0, 2))))
    for n, piece, nb, d, k, prepared in cases:
        planned = vs.vs_knn_workspace_bytes(n, nb, d, k, piece, prepared)
        sizes = {min(n, piece)}
        if n > piece and n % piece:
            sizes.add(n % piece)
        for m in sizes:
            need = vs.vs_knn_workspace_bytes(m, nb, d, k, 0, prepared)
            assert planned >= need, (n, piece, nb, d, k, prepared, m, planned, need)
    assert vs.vs_knn_workspace_bytes(0, 10, 8, 1) == 0
    with pytest.raises(vs.VSError):
        vs.vs_knn_workspace_bytes(10, 10, 0, 1)


def test_bench_traffic_record_is_stamped_and_ignored_when_the_kernels_change(tmp_path, monkeypatch):
    """bench.py --record-traffic (host only): two counter files of a profiler run become one entry
    of profiles/traffic.json, scaled by the named 1 GiB copy kernel and stamped with the scan
    kernels' source text; load_traffic returns it for that text only."""
    import csv
    import importlib
    import json
    import sys
    sys.path.insert(0, ROOT)
    bench = importlib.import_module("bench")
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    (tmp_path / "profiles").mkdir()
    src = tmp_path / "paper_2401_08281_amd" / "csrc"
    src.mkdir(parents=True)
    for name in bench.SCAN_SOURCES:
        (src / name).write_text("// " + name)
    def counters(folder, counter, scan_kib, copy_kib):
        d = tmp_path / folder
        d.mkdir()
        with open(d / "x_counter_collection.csv", "w", newline="") as f:
            w = csv.DictWriter(f, fieldnames=["Kernel_Name", "Counter_Name", "Counter_Value"])
            w.writeheader()
            for v in (scan_kib, scan_kib + 2.0):
                # (C4 is searched list by list: that scan is the dominant kernel; the query-major kernel
                # runs in the same search, for every query's first probes, and is not counted)
                w.writerow({"Kernel_Name": "void ivfpq_scan_listmajor_kernel<32, 3, 256>(float const*)",
                            "Counter_Name": counter, "Counter_Value": v})
                w.writerow({"Kernel_Name": "void ivfpq_scan_bank_kernel<32, 3, 0, 4, 256>(float const*)",
                            "Counter_Name": counter, "Counter_Value": 7e8})
            w.writerow({"Kernel_Name": "vs_calibrate_copy_kernel(uint4 const*, uint4*, unsigned long)",
                        "Counter_Name": counter, "Counter_Value": copy_kib})
            w.writerow({"Kernel_Name": "other_kernel", "Counter_Name": counter, "Counter_Value": 1e9})
        return str(d)
    class Args:
        workload, nprobe, search_type = "C4", None, "tables"
    Args.record_traffic = [counters("f", "FETCH_SIZE", 1000.0, 524288.0), counters("w", "WRITE_SIZE", 10.0, 1048576.0)]
    assert bench.record_traffic(Args) == 0
    rec = json.load(open(tmp_path / "profiles" / "traffic.json"))["ivfpq_scan_C4_nprobe64"]
    assert rec["kernel"] == "ivfpq_scan_listmajor_kernel"
    assert rec["fetch_scale"] == 2.0 and rec["write_scale"] == 1.0
    assert rec["fetch_bytes"] == int(1001.0 * 1024 * 2.0) and rec["write_bytes"] == int(11.0 * 1024)
    assert bench.load_traffic("ivfpq_scan_C4_nprobe64") == rec["hbm_bytes_per_launch"]
    (src / bench.SCAN_SOURCES[0]).write_text("// changed")
    assert bench.load_traffic("ivfpq_scan_C4_nprobe64") is None
    assert bench.load_traffic("no_such_key") is None
