"""ctypes binding of libvs.so: same names as the C ABI in include/vs.h.

Argument marshalling only.  Tensors must be CUDA/HIP tensors, contiguous, of
the dtype the ABI states; the current torch stream is handed over as the HIP
stream.  There is no CPU fallback: if the library is missing, loading fails.
"""
import ctypes
import os

import torch

METRIC_L2 = 0
METRIC_IP = 1
VS_MAX_K = 1024

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libvs.so")
_lib = None


class VSError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("vs error %d: %s" % (code, msg))
        self.code = code


def lib():
    """Loads libvs.so, building it first if it is missing or older than one of its sources
    (VS_NO_REBUILD=1 in the environment loads a stale library as it is)."""
    global _lib
    if _lib is not None:
        return _lib
    from . import build
    if not os.path.exists(_LIB_PATH) or (build.is_stale() and os.environ.get("VS_NO_REBUILD") != "1"):
        build.build_lib()
    L = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    L.vs_flat_search.restype = ctypes.c_int
    L.vs_flat_search.argtypes = [vp, i64, vp, i64, i32, i32, i32, vp, vp, vp]
    L.vs_trim.restype = ctypes.c_int
    L.vs_trim.argtypes = []
    L.vs_flat_create.restype = ctypes.c_int
    L.vs_flat_create.argtypes = [ctypes.POINTER(vp), i32, i32]
    L.vs_flat_destroy.restype = None
    L.vs_flat_destroy.argtypes = [vp]
    L.vs_flat_ntotal.restype = i64
    L.vs_flat_ntotal.argtypes = [vp]
    L.vs_flat_add.restype = ctypes.c_int
    L.vs_flat_add.argtypes = [vp, vp, i64, vp]
    L.vs_flat_index_search.restype = ctypes.c_int
    L.vs_flat_index_search.argtypes = [vp, vp, i64, i32, vp, vp, vp]
    L.vs_knn_workspace_bytes.restype = i64
    L.vs_knn_workspace_bytes.argtypes = [i64, i64, i32, i32, i64, i32]
    L.vs_ivfpq_set_search_type.restype = ctypes.c_int
    L.vs_ivfpq_set_search_type.argtypes = [vp, i32]
    L.vs_ivfpq_get_norms.restype = ctypes.c_int
    L.vs_ivfpq_get_norms.argtypes = [vp, vp, vp]
    L.vs_ivfflat_create.restype = ctypes.c_int
    L.vs_ivfflat_create.argtypes = [ctypes.POINTER(vp), i32, i32, i32, vp, vp]
    L.vs_ivfflat_destroy.restype = None
    L.vs_ivfflat_destroy.argtypes = [vp]
    L.vs_ivfflat_ntotal.restype = i64
    L.vs_ivfflat_ntotal.argtypes = [vp]
    L.vs_ivfflat_add.restype = ctypes.c_int
    L.vs_ivfflat_add.argtypes = [vp, vp, i64, vp, vp]
    L.vs_ivfflat_search.restype = ctypes.c_int
    L.vs_ivfflat_search.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp]
    L.vs_ivfflat_get_list_sizes.restype = ctypes.c_int
    L.vs_ivfflat_get_list_sizes.argtypes = [vp, vp, vp]
    L.vs_ivfflat_get_storage.restype = ctypes.c_int
    L.vs_ivfflat_get_storage.argtypes = [vp, vp, vp, vp, vp]
    L.vs_ivfsq8_create.restype = ctypes.c_int
    L.vs_ivfsq8_create.argtypes = [ctypes.POINTER(vp), i32, i32, i32, vp, vp, vp, vp]
    L.vs_ivfsq8_destroy.restype = None
    L.vs_ivfsq8_destroy.argtypes = [vp]
    L.vs_ivfsq8_ntotal.restype = i64
    L.vs_ivfsq8_ntotal.argtypes = [vp]
    L.vs_ivfsq8_add.restype = ctypes.c_int
    L.vs_ivfsq8_add.argtypes = [vp, vp, i64, vp, vp]
    L.vs_ivfsq8_search.restype = ctypes.c_int
    L.vs_ivfsq8_search.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp]
    L.vs_ivfsq8_get_list_sizes.restype = ctypes.c_int
    L.vs_ivfsq8_get_list_sizes.argtypes = [vp, vp, vp]
    L.vs_ivfsq8_get_storage.restype = ctypes.c_int
    L.vs_ivfsq8_get_storage.argtypes = [vp, vp, vp, vp, vp]
    L.vs_kmeans.restype = ctypes.c_int
    L.vs_kmeans.argtypes = [vp, i64, i32, i32, i32, vp, vp, vp, vp]
    L.vs_ivfpq_train.restype = ctypes.c_int
    L.vs_ivfpq_train.argtypes = [vp, i64, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp]
    L.vs_refine.restype = ctypes.c_int
    L.vs_refine.argtypes = [vp, i64, vp, i64, i32, i32, vp, i32, i32, vp, vp, vp]
    L.vs_ivfpq_create.restype = ctypes.c_int
    L.vs_ivfpq_create.argtypes = [ctypes.POINTER(vp), i32, i32, i32, i32, i32, vp, vp, vp]
    L.vs_ivfpq_add.restype = ctypes.c_int
    L.vs_ivfpq_add.argtypes = [vp, vp, i64, vp, vp]
    L.vs_ivfpq_search.restype = ctypes.c_int
    L.vs_ivfpq_search.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp]
    L.vs_ivfpq_search_stats.restype = ctypes.c_int
    L.vs_ivfpq_search_stats.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp, vp]
    L.vs_ivfpq_search_static.restype = ctypes.c_int
    L.vs_ivfpq_search_static.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp]
    L.vs_ivfpq_destroy.restype = None
    L.vs_ivfpq_destroy.argtypes = [vp]
    L.vs_ivfpq_ntotal.restype = i64
    L.vs_ivfpq_ntotal.argtypes = [vp]
    L.vs_ivfpq_code_size.restype = i32
    L.vs_ivfpq_code_size.argtypes = [vp]
    L.vs_ivfpq_get_list_sizes.restype = ctypes.c_int
    L.vs_ivfpq_get_list_sizes.argtypes = [vp, vp, vp]
    L.vs_ivfpq_get_assignments.restype = ctypes.c_int
    L.vs_ivfpq_get_assignments.argtypes = [vp, vp, vp, vp]
    L.vs_ivfpq_get_codes.restype = ctypes.c_int
    L.vs_ivfpq_get_codes.argtypes = [vp, vp, vp]
    L.vs_ivfpq_coarse.restype = ctypes.c_int
    L.vs_ivfpq_coarse.argtypes = [vp, vp, i64, i32, vp, vp, vp]
    L.vs_profile_enable.restype = ctypes.c_int
    L.vs_profile_enable.argtypes = [ctypes.c_int]
    L.vs_profile_read.restype = ctypes.c_int
    L.vs_profile_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
    L.vs_set_option.restype = ctypes.c_int
    L.vs_set_option.argtypes = [ctypes.c_char_p, ctypes.c_double]
    L.vs_counters_read.restype = ctypes.c_int
    L.vs_counters_read.argtypes = [ctypes.POINTER(i64)]
    L.vs_last_error.restype = ctypes.c_char_p
    L.vs_version.restype = ctypes.c_char_p
    _lib = L
    return L


def _check(rc):
    if rc != 0:
        raise VSError(rc, lib().vs_last_error().decode())


def _dev(t, dtype, name):
    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda):
        raise TypeError("%s must be a device tensor" % name)
    if t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (name, dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    return t


def _p(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None and t.numel() > 0 else ctypes.c_void_p(0)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def vs_last_error():
    return lib().vs_last_error().decode()


def vs_version():
    return lib().vs_version().decode()


STAGES = ("coarse_dist", "coarse_select", "scan", "merge", "flat_dist", "flat_select", "refine", "scan_first")


def vs_profile_enable(on):
    _check(lib().vs_profile_enable(1 if on else 0))


def vs_profile_read():
    """Returns {stage: (total_ms, launches)} for the calls made since the last read."""
    ms = (ctypes.c_double * len(STAGES))()
    n = (ctypes.c_int64 * len(STAGES))()
    _check(lib().vs_profile_read(ms, n))
    return {s: (float(ms[i]), int(n[i])) for i, s in enumerate(STAGES)}


def vs_trim():
    _check(lib().vs_trim())


def vs_set_option(name, value):
    _check(lib().vs_set_option(name.encode(), float(value)))


def vs_knn_workspace_bytes(na, nb, d, k, piece=0, b_prepared=False):
    """Device scratch of one k-nearest-rows problem, in bytes (host arithmetic only)."""
    r = int(lib().vs_knn_workspace_bytes(int(na), int(nb), int(d), int(k), int(piece), int(bool(b_prepared))))
    if r < 0:
        raise VSError(-1, lib().vs_last_error().decode())
    return r


def vs_counters_read():
    """Returns (rows through the matrix-core route, rows that needed the exact fallback)."""
    c = (ctypes.c_int64 * 2)()
    _check(lib().vs_counters_read(c))
    return int(c[0]), int(c[1])


def vs_flat_search(x, q, k, metric=METRIC_L2, out_dist=None, out_ids=None):
    x = _dev(x, torch.float32, "x")
    q = _dev(q, torch.float32, "q")
    nb, d = x.shape
    nq = q.shape[0]
    if q.shape[1] != d:
        raise ValueError("x and q differ in dimension")
    if out_dist is None:
        out_dist = torch.empty((nq, max(k, 0)), dtype=torch.float32, device=q.device)
    if out_ids is None:
        out_ids = torch.empty((nq, max(k, 0)), dtype=torch.int64, device=q.device)
    _dev(out_dist, torch.float32, "out_dist")
    _dev(out_ids, torch.int64, "out_ids")
    _check(lib().vs_flat_search(_p(x), nb, _p(q), nq, d, metric, k, _p(out_dist), _p(out_ids), _stream()))
    return out_dist, out_ids


def vs_flat_create(d, metric=METRIC_L2):
    h = ctypes.c_void_p()
    _check(lib().vs_flat_create(ctypes.byref(h), int(d), int(metric)))
    return h


def vs_flat_destroy(h):
    lib().vs_flat_destroy(h)


def vs_flat_ntotal(h):
    return int(lib().vs_flat_ntotal(h))


def vs_flat_add(h, x):
    x = _dev(x, torch.float32, "x")
    _check(lib().vs_flat_add(h, _p(x), x.shape[0], _stream()))


def vs_flat_index_search(h, q, k, out_dist=None, out_ids=None):
    q = _dev(q, torch.float32, "q")
    nq = q.shape[0]
    if out_dist is None:
        out_dist = torch.empty((nq, max(k, 0)), dtype=torch.float32, device=q.device)
    if out_ids is None:
        out_ids = torch.empty((nq, max(k, 0)), dtype=torch.int64, device=q.device)
    _dev(out_dist, torch.float32, "out_dist")
    _dev(out_ids, torch.int64, "out_ids")
    _check(lib().vs_flat_index_search(h, _p(q), nq, k, _p(out_dist), _p(out_ids), _stream()))
    return out_dist, out_ids


def vs_refine(x, q, cand_ids, k, metric=METRIC_L2, out_dist=None, out_ids=None):
    x = _dev(x, torch.float32, "x")
    q = _dev(q, torch.float32, "q")
    cand_ids = _dev(cand_ids, torch.int64, "cand_ids")
    nb, d = x.shape
    nq = q.shape[0]
    if q.shape[1] != d:
        raise ValueError("x and q differ in dimension")
    if cand_ids.dim() != 2 or cand_ids.shape[0] != nq:
        raise ValueError("cand_ids must be [nq, kc]")
    kc = cand_ids.shape[1]
    if out_dist is None:
        out_dist = torch.empty((nq, max(k, 0)), dtype=torch.float32, device=q.device)
    if out_ids is None:
        out_ids = torch.empty((nq, max(k, 0)), dtype=torch.int64, device=q.device)
    _dev(out_dist, torch.float32, "out_dist")
    _dev(out_ids, torch.int64, "out_ids")
    _check(lib().vs_refine(_p(x), nb, _p(q), nq, d, metric, _p(cand_ids), kc, k, _p(out_dist),
                           _p(out_ids), _stream()))
    return out_dist, out_ids


def vs_kmeans(x, centroids, niter, return_assign=False):
    """Trains `centroids` [K, d] (device tensor, updated in place) on x [n, d]; returns the
    objective of every round as a list of floats and, with return_assign, the last round's
    assignment as an int32 device tensor [n]."""
    x = _dev(x, torch.float32, "x")
    centroids = _dev(centroids, torch.float32, "centroids")
    n, d = x.shape
    K = centroids.shape[0]
    if centroids.dim() != 2 or centroids.shape[1] != d:
        raise ValueError("centroids must be [K, d]")
    obj = (ctypes.c_double * max(niter, 1))()
    assign = torch.empty(n, dtype=torch.int32, device=x.device) if return_assign else None
    _check(lib().vs_kmeans(_p(x), n, d, K, niter, _p(centroids), obj,
                           _p(assign) if return_assign else None, _stream()))
    objs = [float(obj[r]) for r in range(max(niter, 0))]
    return (objs, assign) if return_assign else objs


def vs_ivfpq_train(x, metric, centroids, codebooks, nbits, niter):
    """Trains centroids [nlist, d] and codebooks [M, 2^nbits, d / M] (device tensors, updated
    in place) on x [n, d]; returns the objectives as a list of 1 + M lists."""
    x = _dev(x, torch.float32, "x")
    centroids = _dev(centroids, torch.float32, "centroids")
    codebooks = _dev(codebooks, torch.float32, "codebooks")
    n, d = x.shape
    nlist = centroids.shape[0]
    if codebooks.dim() != 3 or centroids.dim() != 2 or centroids.shape[1] != d:
        raise ValueError("centroids must be [nlist, d] and codebooks [M, K, dsub]")
    M = codebooks.shape[0]
    if codebooks.shape[1] != 1 << nbits or M * codebooks.shape[2] != d:
        raise ValueError("codebooks must be [M, 2^nbits, d / M]")
    obj = (ctypes.c_double * ((1 + M) * max(niter, 1)))()
    _check(lib().vs_ivfpq_train(_p(x), n, d, metric, nlist, M, nbits, niter, _p(centroids),
                                _p(codebooks), obj, _stream()))
    return [[float(obj[r * niter + t]) for t in range(niter)] for r in range(1 + M)]


def vs_ivfpq_create(d, metric, nlist, M, nbits, centroids, codebooks):
    centroids = _dev(centroids, torch.float32, "centroids")
    codebooks = _dev(codebooks, torch.float32, "codebooks")
    if centroids is not None and centroids.numel() != nlist * d:
        raise ValueError("centroids must hold nlist * d floats")
    if codebooks is not None and M > 0 and d % M == 0 and 0 < nbits <= 16 and \
            codebooks.numel() != (1 << nbits) * d:
        raise ValueError("codebooks must hold M * 2^nbits * (d / M) floats")
    h = ctypes.c_void_p(0)
    _check(lib().vs_ivfpq_create(ctypes.byref(h), d, metric, nlist, M, nbits, _p(centroids),
                                 _p(codebooks), _stream()))
    return h


def vs_ivfpq_destroy(h):
    lib().vs_ivfpq_destroy(h)


def vs_ivfpq_add(h, x, ids=None):
    x = _dev(x, torch.float32, "x")
    ids = _dev(ids, torch.int64, "ids")
    if ids is not None and ids.numel() != x.shape[0]:
        raise ValueError("ids must hold one id per row of x")
    _check(lib().vs_ivfpq_add(h, _p(x), x.shape[0], _p(ids), _stream()))


def vs_ivfpq_search(h, q, k, nprobe, out_dist=None, out_ids=None):
    q = _dev(q, torch.float32, "q")
    nq = q.shape[0]
    if out_dist is None:
        out_dist = torch.empty((nq, max(k, 0)), dtype=torch.float32, device=q.device)
    if out_ids is None:
        out_ids = torch.empty((nq, max(k, 0)), dtype=torch.int64, device=q.device)
    _dev(out_dist, torch.float32, "out_dist")
    _dev(out_ids, torch.int64, "out_ids")
    _check(lib().vs_ivfpq_search(h, _p(q), nq, k, nprobe, _p(out_dist), _p(out_ids), _stream()))
    return out_dist, out_ids


SEARCH_STATS_FIELDS = ("scanned_codes", "probed_lists", "coarse_rows_matrix_core", "coarse_rows_fallback",
                       "list_major_first_probes", "list_major_first_codes", "list_major_rescanned")


def vs_ivfpq_search_stats(h, q, k, nprobe):
    """vs_ivfpq_search plus the call's vs_search_stats block: (dist, ids, stats) with stats an
    int64 device tensor of the struct's fields in SEARCH_STATS_FIELDS order, written in stream
    order (reading it on the host synchronises)."""
    q = _dev(q, torch.float32, "q")
    nq = q.shape[0]
    out_dist = torch.empty((nq, k), dtype=torch.float32, device=q.device)
    out_ids = torch.empty((nq, k), dtype=torch.int64, device=q.device)
    stats = torch.empty(len(SEARCH_STATS_FIELDS), dtype=torch.int64, device=q.device)
    _check(lib().vs_ivfpq_search_stats(h, _p(q), nq, k, nprobe, _p(out_dist), _p(out_ids), _p(stats), _stream()))
    return out_dist, out_ids, stats


def vs_ivfpq_search_static(h, q, k, nprobe, out_dist, out_ids):
    """vs_ivfpq_search on the library's static work space: no device allocation inside the
    call, so the outputs are the caller's (tensors [nq, k], fp32 and int64)."""
    q = _dev(q, torch.float32, "q")
    _dev(out_dist, torch.float32, "out_dist")
    _dev(out_ids, torch.int64, "out_ids")
    nq = q.shape[0]
    if tuple(out_dist.shape) != (nq, k) or tuple(out_ids.shape) != (nq, k):
        raise ValueError("out_dist and out_ids must be [nq, k]")
    _check(lib().vs_ivfpq_search_static(h, _p(q), nq, k, nprobe, _p(out_dist), _p(out_ids), _stream()))
    return out_dist, out_ids


def vs_ivfpq_ntotal(h):
    return int(lib().vs_ivfpq_ntotal(h))


def vs_ivfpq_code_size(h):
    return int(lib().vs_ivfpq_code_size(h))


def vs_ivfpq_get_list_sizes(h, nlist, device):
    sizes = torch.empty(nlist, dtype=torch.int64, device=device)
    _check(lib().vs_ivfpq_get_list_sizes(h, _p(sizes), _stream()))
    return sizes


def vs_ivfpq_get_assignments(h, device):
    n = vs_ivfpq_ntotal(h)
    ids = torch.empty(n, dtype=torch.int64, device=device)
    list_of = torch.empty(n, dtype=torch.int32, device=device)
    _check(lib().vs_ivfpq_get_assignments(h, _p(ids), _p(list_of), _stream()))
    return ids, list_of


def vs_ivfpq_get_codes(h, device):
    n = vs_ivfpq_ntotal(h)
    codes = torch.empty((n, vs_ivfpq_code_size(h)), dtype=torch.uint8, device=device)
    if n > 0:
        _check(lib().vs_ivfpq_get_codes(h, _p(codes), _stream()))
    return codes


def vs_ivfpq_coarse(h, q, nprobe, nlist):
    q = _dev(q, torch.float32, "q")
    nq = q.shape[0]
    npr = max(min(nprobe, nlist), 0)
    probes = torch.empty((nq, npr), dtype=torch.int32, device=q.device)
    cdist = torch.empty((nq, npr), dtype=torch.float32, device=q.device)
    _check(lib().vs_ivfpq_coarse(h, _p(q), nq, nprobe, _p(probes), _p(cdist), _stream()))
    return probes, cdist


ST_RESIDUAL_TABLES, ST_STORED_NORMS, ST_PRECOMPUTED_TABLES = 0, 1, 2


def vs_ivfpq_set_search_type(h, search_type):
    _check(lib().vs_ivfpq_set_search_type(h, int(search_type)))


def vs_ivfpq_set_coarse_metric(h, metric):
    _check(lib().vs_ivfpq_set_coarse_metric(h, int(metric)))


def vs_ivfpq_get_norms(h, device):
    norms = torch.empty(vs_ivfpq_ntotal(h), dtype=torch.float32, device=device)
    _check(lib().vs_ivfpq_get_norms(h, _p(norms), _stream()))
    return norms


def vs_ivfflat_create(d, metric, nlist, centroids):
    centroids = _dev(centroids, torch.float32, "centroids")
    if centroids is not None and centroids.numel() != nlist * d:
        raise ValueError("centroids must hold nlist * d floats")
    h = ctypes.c_void_p(0)
    _check(lib().vs_ivfflat_create(ctypes.byref(h), d, metric, nlist, _p(centroids), _stream()))
    return h


def vs_ivfflat_destroy(h):
    lib().vs_ivfflat_destroy(h)


def vs_ivfflat_ntotal(h):
    return int(lib().vs_ivfflat_ntotal(h))


def vs_ivfflat_add(h, x, ids=None):
    x = _dev(x, torch.float32, "x")
    ids = _dev(ids, torch.int64, "ids")
    if ids is not None and ids.numel() != x.shape[0]:
        raise ValueError("ids must hold one id per row of x")
    _check(lib().vs_ivfflat_add(h, _p(x), x.shape[0], _p(ids), _stream()))


def vs_ivfflat_search(h, q, k, nprobe, out_dist=None, out_ids=None):
    q = _dev(q, torch.float32, "q")
    nq = q.shape[0]
    if out_dist is None:
        out_dist = torch.empty((nq, max(k, 0)), dtype=torch.float32, device=q.device)
    if out_ids is None:
        out_ids = torch.empty((nq, max(k, 0)), dtype=torch.int64, device=q.device)
    _dev(out_dist, torch.float32, "out_dist")
    _dev(out_ids, torch.int64, "out_ids")
    _check(lib().vs_ivfflat_search(h, _p(q), nq, k, nprobe, _p(out_dist), _p(out_ids), _stream()))
    return out_dist, out_ids


def vs_ivfflat_get_list_sizes(h, nlist, device):
    sizes = torch.empty(nlist, dtype=torch.int64, device=device)
    _check(lib().vs_ivfflat_get_list_sizes(h, _p(sizes), _stream()))
    return sizes


def vs_ivfflat_get_storage(h, d, device):
    """(ids [ntotal], list of every entry [ntotal], stored rows [ntotal, d]) in storage order."""
    n = vs_ivfflat_ntotal(h)
    ids = torch.empty(n, dtype=torch.int64, device=device)
    list_of = torch.empty(n, dtype=torch.int32, device=device)
    rows = torch.empty((n, d), dtype=torch.float32, device=device)
    _check(lib().vs_ivfflat_get_storage(h, _p(ids), _p(list_of), _p(rows), _stream()))
    return ids, list_of, rows


def vs_ivfsq8_create(d, metric, nlist, centroids, vmin, step):
    centroids = _dev(centroids, torch.float32, "centroids")
    vmin = _dev(vmin, torch.float32, "vmin")
    step = _dev(step, torch.float32, "step")
    if vmin.numel() != d or step.numel() != d or centroids.numel() != nlist * d:
        raise ValueError("centroids must be [nlist, d], vmin and step [d]")
    h = ctypes.c_void_p(0)
    _check(lib().vs_ivfsq8_create(ctypes.byref(h), d, metric, nlist, _p(centroids), _p(vmin), _p(step), _stream()))
    return h


def vs_ivfsq8_destroy(h):
    lib().vs_ivfsq8_destroy(h)


def vs_ivfsq8_ntotal(h):
    return int(lib().vs_ivfsq8_ntotal(h))


def vs_ivfsq8_add(h, x, ids=None):
    x = _dev(x, torch.float32, "x")
    ids = _dev(ids, torch.int64, "ids")
    if ids is not None and ids.numel() != x.shape[0]:
        raise ValueError("ids must hold one id per row of x")
    _check(lib().vs_ivfsq8_add(h, _p(x), x.shape[0], _p(ids), _stream()))


def vs_ivfsq8_search(h, q, k, nprobe, out_dist=None, out_ids=None):
    q = _dev(q, torch.float32, "q")
    nq = q.shape[0]
    if out_dist is None:
        out_dist = torch.empty((nq, max(k, 0)), dtype=torch.float32, device=q.device)
    if out_ids is None:
        out_ids = torch.empty((nq, max(k, 0)), dtype=torch.int64, device=q.device)
    _dev(out_dist, torch.float32, "out_dist")
    _dev(out_ids, torch.int64, "out_ids")
    _check(lib().vs_ivfsq8_search(h, _p(q), nq, k, nprobe, _p(out_dist), _p(out_ids), _stream()))
    return out_dist, out_ids


def vs_ivfsq8_get_list_sizes(h, nlist, device):
    sizes = torch.empty(nlist, dtype=torch.int64, device=device)
    _check(lib().vs_ivfsq8_get_list_sizes(h, _p(sizes), _stream()))
    return sizes


def vs_ivfsq8_get_storage(h, n, d, device):
    ids = torch.empty(n, dtype=torch.int64, device=device)
    list_of = torch.empty(n, dtype=torch.int32, device=device)
    codes = torch.empty((n, d), dtype=torch.uint8, device=device)
    _check(lib().vs_ivfsq8_get_storage(h, _p(ids), _p(list_of), _p(codes), _stream()))
    return ids, list_of, codes


class IVFSQ8:
    """Owner of one vs_ivfsq8 handle (thin convenience over the functions above)."""

    def __init__(self, d, metric, centroids, vmin, step):
        self.d, self.metric = int(d), int(metric)
        self.nlist = int(centroids.shape[0])
        self.device = centroids.device
        self.h = vs_ivfsq8_create(self.d, self.metric, self.nlist, centroids, vmin, step)

    def close(self):
        if getattr(self, "h", None) is not None:
            vs_ivfsq8_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def ntotal(self):
        return vs_ivfsq8_ntotal(self.h)

    def add(self, x, ids=None):
        vs_ivfsq8_add(self.h, x, ids)

    def search(self, q, k, nprobe, out_dist=None, out_ids=None):
        return vs_ivfsq8_search(self.h, q, k, nprobe, out_dist, out_ids)

    def list_sizes(self):
        return vs_ivfsq8_get_list_sizes(self.h, self.nlist, self.device)

    def storage(self):
        return vs_ivfsq8_get_storage(self.h, self.ntotal, self.d, self.device)


class Flat:
    """Owner of one vs_flat handle (thin convenience over the functions above)."""

    def __init__(self, d, metric=METRIC_L2):
        self.d, self.metric = int(d), int(metric)
        self.h = vs_flat_create(self.d, self.metric)

    def close(self):
        if getattr(self, "h", None) is not None:
            vs_flat_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def ntotal(self):
        return vs_flat_ntotal(self.h)

    def add(self, x):
        if x.shape[1] != self.d:
            raise ValueError("x has dimension %d, the index %d" % (x.shape[1], self.d))
        vs_flat_add(self.h, x)

    def search(self, q, k, out_dist=None, out_ids=None):
        if q.shape[1] != self.d:
            raise ValueError("q has dimension %d, the index %d" % (q.shape[1], self.d))
        return vs_flat_index_search(self.h, q, k, out_dist, out_ids)


class IVFFlat:
    """Owner of one vs_ivfflat handle (thin convenience over the functions above)."""

    def __init__(self, d, metric, centroids):
        self.d, self.metric = int(d), int(metric)
        self.nlist = int(centroids.shape[0])
        self.device = centroids.device
        self.h = vs_ivfflat_create(self.d, self.metric, self.nlist, centroids)

    def close(self):
        if getattr(self, "h", None) is not None:
            vs_ivfflat_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def ntotal(self):
        return vs_ivfflat_ntotal(self.h)

    def add(self, x, ids=None):
        vs_ivfflat_add(self.h, x, ids)

    def search(self, q, k, nprobe, out_dist=None, out_ids=None):
        return vs_ivfflat_search(self.h, q, k, nprobe, out_dist, out_ids)

    def list_sizes(self):
        return vs_ivfflat_get_list_sizes(self.h, self.nlist, self.device)

    def storage(self):
        return vs_ivfflat_get_storage(self.h, self.d, self.device)


class IVFPQ:
    """Owner of one vs_ivfpq handle (thin convenience over the functions above)."""

    def __init__(self, d, metric, centroids, codebooks, nbits):
        self.d, self.metric, self.nbits = int(d), int(metric), int(nbits)
        self.nlist = int(centroids.shape[0])
        self.M = int(codebooks.shape[0])
        self.device = centroids.device
        self.h = vs_ivfpq_create(self.d, self.metric, self.nlist, self.M, self.nbits, centroids,
                                 codebooks)

    def close(self):
        if getattr(self, "h", None) is not None:
            vs_ivfpq_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def ntotal(self):
        return vs_ivfpq_ntotal(self.h)

    def add(self, x, ids=None):
        vs_ivfpq_add(self.h, x, ids)

    def search(self, q, k, nprobe, out_dist=None, out_ids=None):
        return vs_ivfpq_search(self.h, q, k, nprobe, out_dist, out_ids)

    def search_stats(self, q, k, nprobe):
        """(dist, ids, stats): stats is a dict of the call's vs_search_stats (synchronises)."""
        D, I, st = vs_ivfpq_search_stats(self.h, q, k, nprobe)
        return D, I, dict(zip(SEARCH_STATS_FIELDS, (int(v) for v in st.tolist())))

    def search_static(self, q, k, nprobe, out_dist, out_ids):
        return vs_ivfpq_search_static(self.h, q, k, nprobe, out_dist, out_ids)

    def coarse(self, q, nprobe):
        return vs_ivfpq_coarse(self.h, q, nprobe, self.nlist)

    def list_sizes(self):
        return vs_ivfpq_get_list_sizes(self.h, self.nlist, self.device)

    def assignments(self):
        return vs_ivfpq_get_assignments(self.h, self.device)

    def codes(self):
        return vs_ivfpq_get_codes(self.h, self.device)

    def set_search_type(self, search_type):
        vs_ivfpq_set_search_type(self.h, search_type)

    def set_coarse_metric(self, metric):
        vs_ivfpq_set_coarse_metric(self.h, metric)

    def norms(self):
        return vs_ivfpq_get_norms(self.h, self.device)
