"""ctypes front end of the CPU oracle (oracle.c) plus the index bookkeeping.

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
bench's cpu_baseline leg; never by the product package.  The arithmetic lives
in oracle.c; this file only marshals numpy arrays and keeps the inverted lists
(stable append per list, Sec. 5.1 "Inverted files": the vectors of a cluster
are stored contiguously).
"""
import ctypes
import os
import subprocess

import numpy as np

METRIC_L2 = 0
METRIC_IP = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_SO = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force=False):
    """Compile oracle.c with gcc.  Contraction is off and fmaf is explicit, so
    the canon arithmetic is the IEEE one on any x86-64 with FMA."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-mfma", "-fopenmp", "-shared", "-fPIC",
               "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    if force:   # the sanitizer driver too (plain build: "does it compile"; the test builds it with sanitizers)
        chk = os.path.join(_HERE, "sanitize_check.c")
        subprocess.run(["gcc", "-O1", "-ffp-contract=off", "-mfma", "-fsyntax-only", chk], check=True)
    return _SO


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_SO)
    f32p = ctypes.POINTER(ctypes.c_float)
    lib.or_canon_l2.restype = ctypes.c_float
    lib.or_canon_l2.argtypes = [f32p, f32p, ctypes.c_int]
    lib.or_canon_ip.restype = ctypes.c_float
    lib.or_canon_ip.argtypes = [f32p, f32p, ctypes.c_int]
    lib.or_num_threads.restype = ctypes.c_int
    _lib = lib
    return lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data) if a is not None else ctypes.c_void_p(0)


def num_threads():
    return int(_load().or_num_threads())


def canon_l2(a, b):
    a, pa = _f32(a)
    b, pb = _f32(b)
    assert a.shape == b.shape and a.ndim == 1
    return np.float32(_load().or_canon_l2(pa, pb, a.shape[0]))


def canon_ip(a, b):
    a, pa = _f32(a)
    b, pb = _f32(b)
    assert a.shape == b.shape and a.ndim == 1
    return np.float32(_load().or_canon_ip(pa, pb, a.shape[0]))


def flat_search(x, q, k, metric=METRIC_L2):
    """Eq. 2: the k best database rows for every query row, best first."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    q = np.ascontiguousarray(q, dtype=np.float32)
    nb, d = x.shape
    nq = q.shape[0]
    assert q.shape[1] == d
    D = np.empty((nq, k), dtype=np.float32)
    I = np.empty((nq, k), dtype=np.int64)
    _load().or_flat_search(_ptr(x), ctypes.c_int64(nb), _ptr(q), ctypes.c_int64(nq),
                           ctypes.c_int(d), ctypes.c_int(metric), ctypes.c_int(k), _ptr(D), _ptr(I))
    return D, I


def refine(x, q, cand, k, metric=METRIC_L2):
    """Sec. 3.5 "Refining": exact distances between each query and the vectors of its
    shortlist `cand` [nq, kc] (row numbers of x; entries outside [0, nb) are skipped), then
    the k best, best first."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    q = np.ascontiguousarray(q, dtype=np.float32)
    cand = np.ascontiguousarray(cand, dtype=np.int64)
    nb, d = x.shape
    nq, kc = cand.shape
    assert q.shape == (nq, d)
    D = np.empty((nq, k), dtype=np.float32)
    I = np.empty((nq, k), dtype=np.int64)
    _load().or_refine(_ptr(x), ctypes.c_int64(nb), _ptr(q), ctypes.c_int64(nq), ctypes.c_int(d),
                      ctypes.c_int(metric), _ptr(cand), ctypes.c_int(kc), ctypes.c_int(k),
                      _ptr(D), _ptr(I))
    return D, I


def kmeans(x, init, niter, return_assign=False):
    """Sec. 4.1: niter rounds of Lloyd's iteration from the centroids `init` [K, d].
    Returns (centroids [K, d] fp32, objective [niter] float64: the mean squared distance to
    the assigned centroid at each round's assignment step) and, with return_assign, the
    assignment [n] int32 of the last round's assignment step."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    c = np.array(init, dtype=np.float32, order="C", copy=True)
    n, d = x.shape
    K = c.shape[0]
    assert c.shape[1] == d
    obj = np.zeros(max(niter, 0), dtype=np.float64)
    a = np.full(n, -1, dtype=np.int32)
    _load().or_kmeans(_ptr(x), ctypes.c_int64(n), ctypes.c_int(d), ctypes.c_int(K),
                      ctypes.c_int(niter), _ptr(c), _ptr(obj), _ptr(a))
    if return_assign:
        return c, obj, a
    return c, obj


def train_ivfpq(x, metric, init_centroids, init_codebooks, nbits, niter):
    """Training of an IVF-PQ index's parameters (Sec. 5.1: the coarse quantizer is a k-means;
    Sec. 4.1: each sub-quantizer of the product quantizer is a k-means on its sub-vectors, here
    of the residuals, Sec. 5.1 "Encoding residuals"):
      1. coarse centroids = k-means on x from init_centroids;
      2. every training vector goes to its best centroid under the index metric (or_assign);
      3. residual = x - centroid, one fp32 subtraction per component;
      4. sub-codebook m = k-means on the m-th slices of the residuals from init_codebooks[m].
    Returns (centroids, codebooks [M, K, dsub], objectives [1 + M, niter])."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    M, K, dsub = init_codebooks.shape
    assert K == 1 << nbits and M * dsub == x.shape[1]
    objs = np.zeros((1 + M, niter), dtype=np.float64)
    cent, objs[0] = kmeans(x, init_centroids, niter)
    a = assign(x, cent, metric)
    res = x - cent[a]
    cbs = np.empty_like(np.asarray(init_codebooks, dtype=np.float32))
    for m in range(M):
        cbs[m], objs[1 + m] = kmeans(res[:, m * dsub:(m + 1) * dsub], init_codebooks[m], niter)
    return cent, cbs, objs


def assign(x, centroids, metric=METRIC_L2):
    x = np.ascontiguousarray(x, dtype=np.float32)
    centroids = np.ascontiguousarray(centroids, dtype=np.float32)
    n, d = x.shape
    nlist = centroids.shape[0]
    out = np.empty(n, dtype=np.int32)
    _load().or_assign(_ptr(x), ctypes.c_int64(n), _ptr(centroids), ctypes.c_int(nlist),
                      ctypes.c_int(d), ctypes.c_int(metric), _ptr(out))
    return out


def coarse_probe(q, centroids, nprobe, metric=METRIC_L2):
    q = np.ascontiguousarray(q, dtype=np.float32)
    centroids = np.ascontiguousarray(centroids, dtype=np.float32)
    nq, d = q.shape
    nlist = centroids.shape[0]
    nprobe = min(nprobe, nlist)
    probes = np.empty((nq, nprobe), dtype=np.int32)
    cdist = np.empty((nq, nprobe), dtype=np.float32)
    _load().or_coarse_probe(_ptr(q), ctypes.c_int64(nq), _ptr(centroids), ctypes.c_int(nlist),
                            ctypes.c_int(d), ctypes.c_int(metric), ctypes.c_int(nprobe),
                            _ptr(probes), _ptr(cdist))
    return probes, cdist


def pq_encode(x, list_of, centroids, codebooks, nbits):
    """codebooks: [M, 2**nbits, dsub].  Returns uint8 [n, M*nbits/8]."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    centroids = np.ascontiguousarray(centroids, dtype=np.float32)
    codebooks = np.ascontiguousarray(codebooks, dtype=np.float32)
    list_of = np.ascontiguousarray(list_of, dtype=np.int32)
    n, d = x.shape
    M, K, dsub = codebooks.shape
    assert K == 1 << nbits and M * dsub == d and (M * nbits) % 8 == 0
    codes = np.empty((n, M * nbits // 8), dtype=np.uint8)
    _load().or_pq_encode(_ptr(x), ctypes.c_int64(n), ctypes.c_int(d), _ptr(list_of),
                         _ptr(centroids), ctypes.c_int(M), ctypes.c_int(nbits), _ptr(codebooks),
                         _ptr(codes))
    return codes


def pq_decode(codes, list_of, centroids, codebooks, nbits):
    """D(C(x)) in float64: centroid + concatenated sub-codewords."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    centroids = np.ascontiguousarray(centroids, dtype=np.float32)
    codebooks = np.ascontiguousarray(codebooks, dtype=np.float32)
    list_of = np.ascontiguousarray(list_of, dtype=np.int32)
    n = codes.shape[0]
    M, K, dsub = codebooks.shape
    d = M * dsub
    out = np.empty((n, d), dtype=np.float64)
    _load().or_pq_decode(_ptr(codes), ctypes.c_int64(n), ctypes.c_int(d), _ptr(list_of),
                         _ptr(centroids), ctypes.c_int(M), ctypes.c_int(nbits), _ptr(codebooks),
                         _ptr(out))
    return out


def pq_norms(codes, list_of, centroids, codebooks, nbits):
    """fp32 squared norm of every decoded vector (Sec. 4.3: the norm stored next to the code),
    by the fixed chain of or_pq_norms."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    centroids = np.ascontiguousarray(centroids, dtype=np.float32)
    codebooks = np.ascontiguousarray(codebooks, dtype=np.float32)
    list_of = np.ascontiguousarray(list_of, dtype=np.int32)
    n = codes.shape[0]
    M, K, dsub = codebooks.shape
    out = np.empty(n, dtype=np.float32)
    _load().or_pq_norms(_ptr(codes), ctypes.c_int64(n), ctypes.c_int(M * dsub), _ptr(list_of),
                        _ptr(centroids), ctypes.c_int(M), ctypes.c_int(nbits), _ptr(codebooks),
                        _ptr(out))
    return out


def recall(I_found, I_true, n=None):
    """n-recall@k (Sec. 3.2 "Metrics for approximate nearest neighbor search"): fraction of the n ground-truth
    nearest neighbours found among the k returned ids.  n = None means n = k
    (the intersection measure)."""
    I_found = np.asarray(I_found)
    I_true = np.asarray(I_true)
    n = I_true.shape[1] if n is None else n
    hits = 0
    for a in range(I_found.shape[0]):
        hits += len(set(I_true[a, :n].tolist()) & set(I_found[a].tolist()) - {-1})
    return hits / float(I_found.shape[0] * n)


def sq8_params(x):
    """Range of every component over the training vectors x, as (vmin [d], step [d]) fp32 with
    256 cells of width step covering [min, max] (a constant component gets step 1)."""
    x = np.asarray(x, dtype=np.float32)
    lo, hi = x.min(axis=0), x.max(axis=0)
    step = ((hi.astype(np.float64) - lo) / 256.0).astype(np.float32)
    step[step <= 0] = 1.0
    return np.ascontiguousarray(lo), np.ascontiguousarray(step)


def sq8_encode(x, vmin, step):
    x = np.ascontiguousarray(x, dtype=np.float32)
    n, d = x.shape
    codes = np.empty((n, d), dtype=np.uint8)
    _load().or_sq8_encode(_ptr(x), ctypes.c_int64(n), ctypes.c_int(d),
                          _ptr(np.ascontiguousarray(vmin, dtype=np.float32)),
                          _ptr(np.ascontiguousarray(step, dtype=np.float32)), _ptr(codes))
    return codes


def sq8_decode(codes, vmin, step):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    n, d = codes.shape
    out = np.empty((n, d), dtype=np.float32)
    _load().or_sq8_decode(_ptr(codes), ctypes.c_int64(n), ctypes.c_int(d),
                          _ptr(np.ascontiguousarray(vmin, dtype=np.float32)),
                          _ptr(np.ascontiguousarray(step, dtype=np.float32)), _ptr(out))
    return out


class OracleIVFSQ8:
    """IVF index whose entries are 8-bit scalar-quantizer codes of the vectors (Sec. 4.1, 5.1)."""

    def __init__(self, d, metric, centroids, vmin, step):
        self.d, self.metric = int(d), int(metric)
        self.centroids = np.ascontiguousarray(centroids, dtype=np.float32)
        self.vmin = np.ascontiguousarray(vmin, dtype=np.float32)
        self.step = np.ascontiguousarray(step, dtype=np.float32)
        self.nlist = self.centroids.shape[0]
        self.add_ids = np.empty(0, dtype=np.int64)
        self.add_list_of = np.empty(0, dtype=np.int32)
        self.add_codes = np.empty((0, self.d), dtype=np.uint8)
        self._relayout()

    @property
    def ntotal(self):
        return self.add_ids.shape[0]

    def _relayout(self):
        order = np.argsort(self.add_list_of, kind="stable")
        self.ids = np.ascontiguousarray(self.add_ids[order])
        self.codes = np.ascontiguousarray(self.add_codes[order])
        sizes = np.bincount(self.add_list_of, minlength=self.nlist).astype(np.int64)
        self.list_offsets = np.zeros(self.nlist + 1, dtype=np.int64)
        np.cumsum(sizes, out=self.list_offsets[1:])

    def add(self, x, ids=None):
        x = np.ascontiguousarray(x, dtype=np.float32)
        n = x.shape[0]
        if ids is None:
            ids = np.arange(self.ntotal, self.ntotal + n, dtype=np.int64)
        list_of = assign(x, self.centroids, self.metric)
        self.add_ids = np.concatenate([self.add_ids, np.asarray(ids, dtype=np.int64)])
        self.add_list_of = np.concatenate([self.add_list_of, list_of])
        self.add_codes = np.concatenate([self.add_codes, sq8_encode(x, self.vmin, self.step)])
        self._relayout()

    def list_sizes(self):
        return np.diff(self.list_offsets)

    def search(self, q, k, nprobe, return_stats=False):
        q = np.ascontiguousarray(q, dtype=np.float32)
        nq = q.shape[0]
        D = np.empty((nq, k), dtype=np.float32)
        I = np.empty((nq, k), dtype=np.int64)
        nscanned = np.zeros(nq, dtype=np.int64)
        _load().or_ivfsq8_search(
            _ptr(q), ctypes.c_int64(nq), ctypes.c_int(self.d), ctypes.c_int(self.metric),
            ctypes.c_int(self.nlist), _ptr(self.centroids), _ptr(self.vmin), _ptr(self.step),
            _ptr(self.list_offsets), _ptr(self.codes), _ptr(self.ids), ctypes.c_int(k),
            ctypes.c_int(nprobe), _ptr(D), _ptr(I), _ptr(nscanned))
        if return_stats:
            return D, I, nscanned
        return D, I


class OracleIVFFlat:
    """IVF index that stores the vectors themselves (Sec. 5.1), as plain numpy arrays.
    add(): assignment as in OracleIVFPQ, stable append; search(): probes, exact distances to
    the vectors of the probed lists, selection."""

    def __init__(self, d, metric, centroids):
        self.d = int(d)
        self.metric = int(metric)
        self.centroids = np.ascontiguousarray(centroids, dtype=np.float32)
        self.nlist = self.centroids.shape[0]
        assert self.centroids.shape[1] == self.d
        self.add_ids = np.empty(0, dtype=np.int64)
        self.add_list_of = np.empty(0, dtype=np.int32)
        self.add_vecs = np.empty((0, self.d), dtype=np.float32)
        self._relayout()

    @property
    def ntotal(self):
        return self.add_ids.shape[0]

    def _relayout(self):
        order = np.argsort(self.add_list_of, kind="stable")
        self.ids = np.ascontiguousarray(self.add_ids[order])
        self.vecs = np.ascontiguousarray(self.add_vecs[order])
        sizes = np.bincount(self.add_list_of, minlength=self.nlist).astype(np.int64)
        self.list_offsets = np.zeros(self.nlist + 1, dtype=np.int64)
        np.cumsum(sizes, out=self.list_offsets[1:])

    def add(self, x, ids=None):
        x = np.ascontiguousarray(x, dtype=np.float32)
        n = x.shape[0]
        if ids is None:  # sequential ids continue from ntotal (Sec. 6.1)
            ids = np.arange(self.ntotal, self.ntotal + n, dtype=np.int64)
        list_of = assign(x, self.centroids, self.metric)
        self.add_ids = np.concatenate([self.add_ids, np.asarray(ids, dtype=np.int64)])
        self.add_list_of = np.concatenate([self.add_list_of, list_of])
        self.add_vecs = np.concatenate([self.add_vecs, x])
        self._relayout()
        return list_of

    def list_sizes(self):
        return np.diff(self.list_offsets)

    def search(self, q, k, nprobe, return_stats=False):
        q = np.ascontiguousarray(q, dtype=np.float32)
        nq = q.shape[0]
        npr = min(nprobe, self.nlist)
        D = np.empty((nq, k), dtype=np.float32)
        I = np.empty((nq, k), dtype=np.int64)
        nscanned = np.zeros(nq, dtype=np.int64)
        probes = np.empty((nq, npr), dtype=np.int32)
        _load().or_ivfflat_search(
            _ptr(q), ctypes.c_int64(nq), ctypes.c_int(self.d), ctypes.c_int(self.metric),
            ctypes.c_int(self.nlist), _ptr(self.centroids), _ptr(self.list_offsets),
            _ptr(self.vecs), _ptr(self.ids), ctypes.c_int(k), ctypes.c_int(nprobe), _ptr(D),
            _ptr(I), _ptr(nscanned), _ptr(probes))
        if return_stats:
            return D, I, nscanned, probes
        return D, I


class OracleIVFPQ:
    """IVF-PQ index held as plain numpy arrays (Sec. 5.1).

    add():    O2 assignment, O3/O4 residual encoding, O5 stable append.
    search(): O6 probes, O7 ADC on the decoded vector, O8 selection.
    coarse_metric: the metric of list assignment and probing; the index metric unless given
    (Sec. 5.1, maximum inner product search: an inner-product index may assign by L2).
    """

    def __init__(self, d, metric, centroids, codebooks, nbits, coarse_metric=None):
        self.d = int(d)
        self.metric = int(metric)
        self.coarse_metric = self.metric if coarse_metric is None else int(coarse_metric)
        self.centroids = np.ascontiguousarray(centroids, dtype=np.float32)
        self.codebooks = np.ascontiguousarray(codebooks, dtype=np.float32)
        self.nbits = int(nbits)
        self.nlist = self.centroids.shape[0]
        self.M = self.codebooks.shape[0]
        assert self.centroids.shape[1] == self.d
        assert self.codebooks.shape == (self.M, 1 << self.nbits, self.d // self.M)
        self.code_size = self.M * self.nbits // 8
        # in add order
        self.add_ids = np.empty(0, dtype=np.int64)
        self.add_list_of = np.empty(0, dtype=np.int32)
        self.add_codes = np.empty((0, self.code_size), dtype=np.uint8)
        self.add_norms = np.empty(0, dtype=np.float32)
        self._relayout()

    @classmethod
    def from_storage(cls, d, metric, centroids, codebooks, nbits, list_offsets, codes, ids, coarse_metric=None):
        """Wraps an already laid-out store (list l owns rows list_offsets[l] ..
        list_offsets[l+1] of codes / ids) so that search() can run on it."""
        ix = cls(d, metric, centroids, codebooks, nbits, coarse_metric)
        ix.list_offsets = np.ascontiguousarray(list_offsets, dtype=np.int64)
        ix.codes = np.ascontiguousarray(codes, dtype=np.uint8).reshape(-1, ix.code_size)
        ix.ids = np.ascontiguousarray(ids, dtype=np.int64)
        assert ix.list_offsets.shape[0] == ix.nlist + 1
        assert ix.list_offsets[-1] == ix.ids.shape[0] == ix.codes.shape[0]
        sizes = np.diff(ix.list_offsets)
        ix.add_ids = ix.ids
        ix.add_codes = ix.codes
        ix.add_list_of = np.repeat(np.arange(ix.nlist, dtype=np.int32), sizes)
        ix.add_norms = pq_norms(ix.codes, ix.add_list_of, ix.centroids, ix.codebooks, ix.nbits)
        ix.norms = ix.add_norms
        return ix

    @property
    def ntotal(self):
        return self.add_ids.shape[0]

    def _relayout(self):
        order = np.argsort(self.add_list_of, kind="stable")
        self.ids = np.ascontiguousarray(self.add_ids[order])
        self.codes = np.ascontiguousarray(self.add_codes[order])
        self.norms = np.ascontiguousarray(self.add_norms[order])
        sizes = np.bincount(self.add_list_of, minlength=self.nlist).astype(np.int64)
        self.list_offsets = np.zeros(self.nlist + 1, dtype=np.int64)
        np.cumsum(sizes, out=self.list_offsets[1:])

    def add(self, x, ids=None):
        x = np.ascontiguousarray(x, dtype=np.float32)
        n = x.shape[0]
        if ids is None:  # sequential ids continue from ntotal (Sec. 6.1)
            ids = np.arange(self.ntotal, self.ntotal + n, dtype=np.int64)
        list_of = assign(x, self.centroids, self.coarse_metric)
        codes = pq_encode(x, list_of, self.centroids, self.codebooks, self.nbits)
        self.add_ids = np.concatenate([self.add_ids, np.asarray(ids, dtype=np.int64)])
        self.add_list_of = np.concatenate([self.add_list_of, list_of])
        self.add_codes = np.concatenate([self.add_codes, codes])
        self.add_norms = np.concatenate(
            [self.add_norms, pq_norms(codes, list_of, self.centroids, self.codebooks, self.nbits)])
        self._relayout()
        return list_of, codes

    def list_sizes(self):
        return np.diff(self.list_offsets)

    def search(self, q, k, nprobe, form=0, return_stats=False):
        q = np.ascontiguousarray(q, dtype=np.float32)
        nq = q.shape[0]
        npr = min(nprobe, self.nlist)
        D = np.empty((nq, k), dtype=np.float32)
        I = np.empty((nq, k), dtype=np.int64)
        nscanned = np.zeros(nq, dtype=np.int64)
        probes = np.empty((nq, npr), dtype=np.int32)
        _load().or_ivfpq_search(
            _ptr(q), ctypes.c_int64(nq), ctypes.c_int(self.d), ctypes.c_int(self.metric),
            ctypes.c_int(self.coarse_metric), ctypes.c_int(self.nlist), _ptr(self.centroids), ctypes.c_int(self.M),
            ctypes.c_int(self.nbits), _ptr(self.codebooks), _ptr(self.list_offsets),
            _ptr(self.codes), _ptr(self.ids), _ptr(self.norms), ctypes.c_int(k),
            ctypes.c_int(nprobe), ctypes.c_int(form), _ptr(D), _ptr(I), _ptr(nscanned), _ptr(probes))
        if return_stats:
            return D, I, nscanned, probes
        return D, I
