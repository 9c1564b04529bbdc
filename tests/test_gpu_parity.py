"""Parity of the HIP path (through the C ABI) against the CPU oracle, on the
same seeded inputs.  Needs a real MI355X."""
import os
import sys
import zlib

import numpy as np
import pytest

import synth_inputs as S
from parity_util import EXTRA, check_search, l2_table_cancel, storage_map

pytestmark = pytest.mark.gpu

L2, IP = 0, 1


_PROGRESS = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out", "progress.log")


def say(msg):
    """Names the case before it runs: on stdout (shown for a failing test) and, because pytest holds
    stdout back while a test runs, also in a log file that grows with the work done."""
    print("[case] " + msg, flush=True)
    sys.stdout.flush()
    try:
        os.makedirs(os.path.dirname(_PROGRESS), exist_ok=True)
        with open(_PROGRESS, "a") as f:
            f.write(msg + "\n")
    except OSError:
        pass


@pytest.fixture(scope="module")
def vs():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2401_08281_amd as vs_
    vs_.lib()            # fails loudly when libvs.so is missing
    return vs_


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    import torch
    torch.cuda.synchronize()
    return t.cpu().numpy()


# ------------------------------------------------------------------ flat search

FLAT_CASES = [
    # name, nb, nq, d, k, metric, kind
    ("c1_l2", 10_000, 100, 32, 10, L2, "gauss"),
    ("c1_ip", 10_000, 100, 32, 10, IP, "gauss"),
    ("odd_d_ragged", 4_133, 67, 18, 7, L2, "gauss"),
    ("k1", 3_000, 50, 24, 1, L2, "gauss"),
    ("k100_two_chunks", 40_000, 70, 16, 100, L2, "gauss"),
    ("k1024", 5_000, 9, 8, 1024, L2, "gauss"),
    ("k1024_ip", 3_000, 5, 8, 1024, IP, "gauss"),
    ("nb_smaller_than_k", 37, 5, 12, 64, L2, "gauss"),
    ("single_query", 2_000, 1, 40, 10, IP, "gauss"),
]


@pytest.mark.parametrize("name,nb,nq,d,k,metric,kind", FLAT_CASES, ids=[c[0] for c in FLAT_CASES])
def test_flat_matches_oracle(vs, oracle, name, nb, nq, d, k, metric, kind):
    say("flat %s nb=%d nq=%d d=%d k=%d metric=%d" % (name, nb, nq, d, k, metric))
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    x = rng.standard_normal((nb, d), dtype=np.float32)
    q = rng.standard_normal((nq, d), dtype=np.float32)
    D, I = vs.vs_flat_search(dev(x), dev(q), k, metric)
    D, I = host(D), host(I)
    Do, Io = oracle.flat_search(x, q, min(k + EXTRA, max(nb, k)), metric)
    xn = np.sqrt((x.astype(np.float64) ** 2).sum(1).max())
    same = check_search(D, I, Do, Io, metric, q, xn)
    assert same > 0.999


def test_flat_sift_like_is_bit_exact(vs, oracle):
    # integer-valued data: every arithmetic gives the exact distance
    cfg = S.config("C2", nb=60_000, nq=128, ncomp=50)
    say("flat sift-like nb=%d nq=%d k=100" % (cfg["nb"], cfg["nq"]))
    x, q = S.make_data(cfg)
    D, I = vs.vs_flat_search(dev(x), dev(q), 100, L2)
    D, I = host(D), host(I)
    Do, Io = oracle.flat_search(x, q, 100, L2)
    np.testing.assert_array_equal(D, Do)
    # equal distances are ordered by id on both sides
    np.testing.assert_array_equal(I, Io)


def test_trim_releases_the_work_buffer_and_search_still_works(vs, oracle):
    import torch
    rng = np.random.default_rng(8)
    x = rng.standard_normal((4000, 64), dtype=np.float32)
    q = rng.standard_normal((30, 64), dtype=np.float32)
    D1, I1 = [host(t).copy() for t in vs.vs_flat_search(dev(x), dev(q), 7, L2)]
    vs.vs_trim()
    vs.vs_trim()                                             # nothing to free: still fine
    D2, I2 = [host(t) for t in vs.vs_flat_search(dev(x), dev(q), 7, L2)]
    np.testing.assert_array_equal(D1, D2)
    np.testing.assert_array_equal(I1, I2)


def test_flat_searches_on_two_streams_share_the_work_space_safely(vs):
    """vs_flat_search keeps one work buffer per device.  Calls issued on two streams without any
    synchronisation between them must not see each other's candidate lists: the later call waits
    on the device for the earlier one's kernels."""
    import torch
    g = torch.Generator(device="cuda"); g.manual_seed(5)
    xs = [torch.randn((40_000, 64), generator=g, device="cuda") for _ in range(2)]
    qs = [torch.randn((500, 64), generator=g, device="cuda") for _ in range(2)]
    ref = [[host(t).copy() for t in vs.vs_flat_search(xs[i], qs[i], 10, L2)] for i in range(2)]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rep in range(6):
        say("two streams, round %d" % rep)
        outs = []
        for i in (0, 1, 0, 1):
            with torch.cuda.stream(streams[i]):
                outs.append((i, vs.vs_flat_search(xs[i], qs[i], 10, L2)))
        torch.cuda.synchronize()
        for i, (D, I) in outs:
            np.testing.assert_array_equal(host(I), ref[i][1])
            np.testing.assert_array_equal(host(D), ref[i][0])


def test_index_searches_on_two_streams_share_the_work_space_safely(vs):
    """The same for the per-index work buffer of vs_ivfpq_search: two query batches searched on
    two streams, back to back without synchronisation, equal the searches done one at a time."""
    import torch
    cfg = S.config("C3", nb=60_000, nq=400, ncomp=100, nlist=256)
    x, q = S.make_data(cfg)
    cent, cb = S.make_index_params(cfg, x)
    ix = vs.IVFPQ(cfg["d"], L2, dev(cent), dev(cb), 8)
    ix.add(dev(x))
    qs = [dev(q[:200]), dev(q[200:])]
    ref = [[host(t).copy() for t in ix.search(qs[i], 10, 16)] for i in range(2)]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rep in range(6):
        say("index, two streams, round %d" % rep)
        outs = []
        for i in (0, 1, 0, 1):
            with torch.cuda.stream(streams[i]):
                outs.append((i, ix.search(qs[i], 10, 16)))
        torch.cuda.synchronize()
        for i, (D, I) in outs:
            np.testing.assert_array_equal(host(I), ref[i][1])
            np.testing.assert_array_equal(host(D), ref[i][0])
    ix.close()


def test_flat_empty_database_and_no_queries(vs):
    import torch
    say("flat nb=0 / nq=0")
    x = torch.empty((0, 8), dtype=torch.float32, device="cuda")
    q = torch.randn((3, 8), dtype=torch.float32, device="cuda")
    D, I = vs.vs_flat_search(x, q, 4, L2)
    assert (host(I) == -1).all() and np.isposinf(host(D)).all()
    D, I = vs.vs_flat_search(x, q, 4, IP)
    assert (host(I) == -1).all() and np.isneginf(host(D)).all()
    D, I = vs.vs_flat_search(q, x, 4, L2)
    assert D.shape == (0, 4)


# ------------------------------------------------------------------ IVF-PQ

def build_both(vs, oracle, cfg, x, pieces=1, custom_ids=False):
    cent, cb = S.make_index_params(cfg, x)
    ix = vs.IVFPQ(cfg["d"], cfg["metric"], dev(cent), dev(cb), cfg["nbits"])
    orc = oracle.OracleIVFPQ(cfg["d"], cfg["metric"], cent, cb, cfg["nbits"])
    ids = (np.arange(x.shape[0], dtype=np.int64) * 7 + 3) if custom_ids else None
    bounds = np.linspace(0, x.shape[0], pieces + 1).astype(int)
    for s, e in zip(bounds[:-1], bounds[1:]):
        ix.add(dev(x[s:e]), dev(ids[s:e]) if custom_ids else None)
        orc.add(x[s:e], ids[s:e] if custom_ids else None)
    return ix, orc


def check_storage(ix, orc):
    """assignments and codes bit-exact, as the map id -> (list, code)."""
    ids, list_of = ix.assignments()
    ids, list_of, codes = host(ids), host(list_of), host(ix.codes())
    assert ix.ntotal == orc.ntotal == ids.shape[0]
    g = storage_map(ids, list_of, codes)
    o = storage_map(orc.add_ids, orc.add_list_of, orc.add_codes)
    np.testing.assert_array_equal(g[0], o[0])
    np.testing.assert_array_equal(g[1], o[1])
    np.testing.assert_array_equal(g[2], o[2])
    np.testing.assert_array_equal(host(ix.list_sizes()), orc.list_sizes())
    # lists are contiguous and in list order; within a list, entries keep add order
    assert (np.diff(list_of) >= 0).all()
    np.testing.assert_array_equal(ids, orc.ids)
    np.testing.assert_array_equal(codes, orc.codes)


IVF_CASES = {
    "c1": (S.config("C1"), [(10, 4), (10, 1), (10, 16), (10, 99), (1, 4), (100, 8)]),
    "c3_small": (S.config("C3", nb=100_000, nq=200, ncomp=100, nlist=512), [(10, 1), (10, 16), (10, 64)]),
    "c4_small": (S.config("C4", nb=50_000, nq=100, ncomp=100, nlist=256), [(100, 64), (10, 3)]),
    "c5_small": (S.config("C5", nb=20_000, nq=100, ncomp=50, nlist=128), [(10, 32), (100, 128)]),
    "pq4_l2": (S.config("C1", nb=5_000, M=16, nbits=4), [(10, 4)]),
    "ip_8bit": (S.config("C4", nb=20_000, nq=64, ncomp=40, nlist=64, metric=1, M=8), [(10, 8)]),
    # inner product on the shapes whose codes are stored rotated: short lists (one wavefront per
    # (query, probe split)) and long ones (one workgroup)
    "c1_ip": (S.config("C1", metric=1), [(10, 4), (100, 8), (300, 99)]),
    "c3_small_ip": (S.config("C3", nb=60_000, nq=100, ncomp=100, nlist=256, metric=1), [(10, 16), (100, 64)]),
    "c3_long_lists_ip": (S.config("C3", nb=40_000, nq=100, ncomp=100, nlist=16, metric=1), [(10, 4)]),
    # long lists (>= 1024 codes per list on average): the single-table scan variant
    "c4_long_lists": (S.config("C4", nb=40_000, nq=100, ncomp=100, nlist=32), [(100, 8), (10, 32)]),
    "c3_long_lists": (S.config("C3", nb=40_000, nq=100, ncomp=100, nlist=16), [(10, 4)]),
    "c1_long_lists": (S.config("C1", nb=20_000, nlist=8), [(10, 3), (500, 8)]),
    "odd_shapes": (S.config("C1", nb=3_001, nq=33, d=30, M=5, nlist=7), [(10, 3), (300, 7)]),
    # generic shapes with 16-, 32- and 64-byte codes: the software-pipelined scan kernel
    "pq16x8_d64": (S.config("C1", nb=30_000, nq=64, d=64, M=16, nlist=64), [(10, 8), (100, 64)]),
    "pq32x4_d64": (S.config("C1", nb=30_000, nq=64, d=64, M=32, nbits=4, nlist=64), [(10, 8)]),
    "pq64x8_ip": (S.config("C4", nb=30_000, nq=64, ncomp=40, nlist=64, metric=1, d=128, M=64), [(10, 8), (100, 3)]),
    "pq64x4_l2_empty_lists": (S.config("C5", nb=3_000, nq=50, ncomp=10, nlist=256, metric=0), [(10, 32)]),
    # the largest k and nprobe the boundary accepts, every list probed
    "max_k_and_nprobe": (S.config("C1", nb=30_000, nq=40, nlist=1024), [(1024, 1024)]),
}


def test_search_can_be_captured_in_a_hip_graph(vs):
    """The search entry points only enqueue kernels on the caller's stream (after a warm-up has
    grown the scratch buffers): captured in a graph, every replay on new queries must return
    what the eager call returns, with eager work and synchronisations between the replays."""
    import torch
    cfg = S.config("C3", nb=100_000, nq=512, ncomp=100, nlist=512)
    x, q = S.make_data(cfg)
    cent, cb = S.make_index_params(cfg, x)
    ix = vs.IVFPQ(cfg["d"], L2, dev(cent), dev(cb), 8)
    ix.add(dev(x))
    qd = dev(q)
    for nq in (1, 128):
        say("graph capture of ivfpq search, nq=%d" % nq)
        qs = qd[:nq].contiguous().clone()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for _ in range(3):
                ix.search(qs, 10, 16)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            Dg, Ig = ix.search(qs, 10, 16)
        torch.cuda.synchronize()
        for rep in range(4):
            qs.copy_(qd[rep * nq:(rep + 1) * nq])
            g.replay()
            torch.cuda.synchronize()
            De, Ie = ix.search(qs, 10, 16)
            Df, If = vs.vs_flat_search(dev(x[:1000]), qs, 5, L2)     # unrelated eager work in between
            torch.cuda.synchronize()
            assert torch.equal(Dg, De) and torch.equal(Ig, Ie), "replay %d differs from the eager search" % rep
    # the same for a search that runs list-major (eight kernels in a row, counters and candidate
    # buffers reset by kernels of the search itself)
    vs.vs_set_option("list_major", 1)
    try:
        nq = 128
        say("graph capture of a list-major ivfpq search, nq=%d" % nq)
        qs = qd[:nq].contiguous().clone()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for _ in range(3):
                ix.search(qs, 10, 16)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            Dg, Ig = ix.search(qs, 10, 16)
        torch.cuda.synchronize()
        for rep in range(4):
            qs.copy_(qd[rep * nq:(rep + 1) * nq])
            g.replay()
            torch.cuda.synchronize()
            vs.vs_set_option("list_major", -1)
            De, Ie = ix.search(qs, 10, 16)                           # eager, query-major
            vs.vs_set_option("list_major", 1)
            torch.cuda.synchronize()
            assert torch.equal(Dg, De) and torch.equal(Ig, Ie), "list-major replay %d differs from the eager search" % rep
    finally:
        vs.vs_set_option("list_major", 0)
    ix.close()


def random_ivf_shapes(n_cases, seed):
    """Seeded draws of small valid index shapes: every combination the launcher tells apart
    (metric, code width, code size, sub-vector length, list length against the chunk size,
    k against the selection's register variants) turns up among them."""
    rng = np.random.default_rng(seed)
    out = []
    for c in range(n_cases):
        nbits = int(rng.choice([8, 8, 4]))
        M = int(rng.choice([1, 2, 4, 8, 16, 32, 64] if nbits == 8 else [2, 4, 8, 16, 32, 64, 128]))
        dsub = int(rng.choice([1, 2, 3, 4, 8, 12]))
        while M * dsub > 768:
            dsub = max(1, dsub // 2)
        kind = str(rng.choice(["C1", "C3", "C4"]))             # gaussian / integer / unit-norm data
        nlist = int(rng.choice([1, 3, 16, 50, 200]))
        nb = int(rng.choice([300, 2_000, 9_000]))
        cfg = S.config(kind, nb=nb, nq=int(rng.choice([1, 7, 40])), d=M * dsub, M=M, nbits=nbits, nlist=nlist,
                       metric=int(rng.choice([L2, L2, IP])), ncomp=min(20, nb), seed=1000 + c)
        k = int(rng.choice([1, 10, 100, 300]))
        nprobe = int(min(nlist, rng.choice([1, 2, 8, 64])))
        out.append((cfg, k, nprobe))
    return out


def test_random_shapes_match_oracle(vs, oracle):
    """Forty seeded small indexes of mixed shapes: storage bit-exact, coarse stage bit-exact,
    search results within the distance tolerance, for both L2 search types."""
    for n, (cfg, k, nprobe) in enumerate(random_ivf_shapes(40, 20240127)):
        say("random shape %d: %s nb=%d nq=%d d=%d M=%d nbits=%d nlist=%d metric=%d k=%d nprobe=%d" % (
            n, cfg["kind"], cfg["nb"], cfg["nq"], cfg["d"], cfg["M"], cfg["nbits"], cfg["nlist"], cfg["metric"],
            k, nprobe))
        x, q = S.make_data(cfg)
        cent, cb = S.make_index_params(cfg, x)
        ix = vs.IVFPQ(cfg["d"], cfg["metric"], dev(cent), dev(cb), cfg["nbits"])
        if cfg["metric"] == L2:
            ix.set_search_type(vs.ST_STORED_NORMS)             # norms are stored by every add
        orc = oracle.OracleIVFPQ(cfg["d"], cfg["metric"], cent, cb, cfg["nbits"])
        bounds = np.linspace(0, x.shape[0], 2 + n % 3).astype(int)
        for s0, e0 in zip(bounds[:-1], bounds[1:]):
            ix.add(dev(x[s0:e0]))
            orc.add(x[s0:e0])
        check_storage(ix, orc)
        xn = float(np.sqrt(orc.norms.max()))                   # largest decoded vector
        probes, cdist = ix.coarse(dev(q), nprobe)
        po, co = oracle.coarse_probe(q, orc.centroids, nprobe, cfg["metric"])
        np.testing.assert_array_equal(host(probes), po)
        np.testing.assert_array_equal(host(cdist), co)
        ix.set_search_type(vs.ST_RESIDUAL_TABLES)
        D, I = ix.search(dev(q), k, nprobe)
        Do, Io = orc.search(q, k + EXTRA, nprobe)
        tc, te = l2_table_cancel(co, cb) if cfg["metric"] == L2 else (None, 0.0)
        check_search(host(D), host(I), Do, Io, cfg["metric"], q, xn, cancel=tc, cancel_eps=te)
        if cfg["metric"] == L2:
            ix.set_search_type(vs.ST_STORED_NORMS)
            np.testing.assert_array_equal(host(ix.norms()), orc.norms)
            cancel = (q.astype(np.float64) ** 2).sum(1) + float(orc.norms.max())
            D, I = ix.search(dev(q), k, nprobe)
            check_search(host(D).copy(), host(I).copy(), Do, Io, L2, cancel=cancel)
        ix.close()


NEAR_ZERO_CASES = {
    # the three shapes whose tables are built from the expanded square, on non-integer data
    "pq8x8_d32": S.config("C1", nb=8_000),
    "pq16x8_d128": S.config("C4", nb=20_000, nq=8, ncomp=40, nlist=64, d=128, M=16),
    "pq32x8_d96": S.config("C4", nb=20_000, nq=8, ncomp=40, nlist=64),
    # and one that goes through the subtraction form
    "pq16x8_d64": S.config("C1", nb=8_000, d=64, M=16, nlist=32),
}


@pytest.mark.parametrize("name", list(NEAR_ZERO_CASES))
def test_queries_equal_or_close_to_decoded_vectors(vs, oracle, name):
    """L2 distances near zero: the query IS the reconstruction of a stored code (or within 1e-6 of
    it).  A table entry evaluated as |r_m|^2 + |t|^2 - 2 <r_m, t> then cancels almost completely;
    the result must stay non-negative and within the rounding that expansion can cost, relative
    to the cancelling terms (l2_table_cancel), of the oracle's value."""
    cfg = NEAR_ZERO_CASES[name]
    say("near-zero %s nb=%d d=%d M=%d nlist=%d" % (name, cfg["nb"], cfg["d"], cfg["M"], cfg["nlist"]))
    x, _ = S.make_data(cfg)
    ix, orc = build_both(vs, oracle, cfg, x)
    rng = np.random.default_rng(11)
    pick = rng.choice(cfg["nb"], 48, replace=False)
    dec = oracle.pq_decode(orc.add_codes[pick], orc.add_list_of[pick], orc.centroids, orc.codebooks, 8)
    q = np.concatenate([dec.astype(np.float32), (dec * (1.0 + 1e-6)).astype(np.float32),
                        (dec + 1e-3 * rng.standard_normal(dec.shape)).astype(np.float32)])
    for k, nprobe in ((10, 4), (3, cfg["nlist"])):
        D, I = ix.search(dev(q), k, nprobe)
        D, I = host(D), host(I)
        assert (D >= 0).all(), "negative squared distance %r" % float(D.min())
        # (this synthetic set holds runs of vectors with one and the same code: they tie exactly in
        # the oracle and within rounding on the GPU, whose summation order depends on the position
        # in the list -- enough oracle ranks are asked for to hold every such run)
        Do, Io = orc.search(q, k + 400, nprobe)
        _, co = oracle.coarse_probe(q, orc.centroids, nprobe, L2)
        tc, te = l2_table_cancel(co, orc.codebooks)
        check_search(D, I, Do, Io, L2, cancel=tc, cancel_eps=te)
        # the stored vector itself is found first (its reconstruction is the query, or next to it)
        found = (I[:48, 0] == orc.add_ids[pick]) | (Do[:48, 0] == Do[:48, 1])
        assert found.all()
    ix.close()


@pytest.mark.parametrize("name", list(IVF_CASES))
def test_ivfpq_matches_oracle(vs, oracle, name):
    cfg, searches = IVF_CASES[name]
    say("ivfpq %s nb=%d d=%d nlist=%d M=%d nbits=%d metric=%d" % (
        name, cfg["nb"], cfg["d"], cfg["nlist"], cfg["M"], cfg["nbits"], cfg["metric"]))
    x, q = S.make_data(cfg)
    ix, orc = build_both(vs, oracle, cfg, x)
    check_storage(ix, orc)
    xn = float(np.sqrt(orc.norms.max()))                       # largest decoded vector
    for k, nprobe in searches:
        say("  search k=%d nprobe=%d" % (k, nprobe))
        probes, cdist = ix.coarse(dev(q), nprobe)
        po, co = oracle.coarse_probe(q, orc.centroids, nprobe, cfg["metric"])
        np.testing.assert_array_equal(host(probes), po)       # probe order is bit-exact
        np.testing.assert_array_equal(host(cdist), co)
        D, I = ix.search(dev(q), k, nprobe)
        Do, Io = orc.search(q, k + EXTRA, nprobe)
        tc, te = l2_table_cancel(co, orc.codebooks) if cfg["metric"] == L2 else (None, 0.0)
        same = check_search(host(D), host(I), Do, Io, cfg["metric"], q, xn, cancel=tc, cancel_eps=te)
        assert same > 0.99, same
    ix.close()


@pytest.mark.parametrize("name", ["c1_ip", "c3_small_ip", "ip_8bit", "pq64x8_ip", "c5_small"])
def test_inner_product_index_with_l2_assignment_matches_oracle(vs, oracle, name):
    """Sec. 5.1, maximum inner product search: lists chosen by L2 at add and at search, scores by
    inner product.  The centroids are scaled to very different norms so that L2 and inner-product
    assignment disagree; storage is bit-exact, probes are the L2 probes, results match the oracle."""
    cfg, searches = IVF_CASES[name]
    assert cfg["metric"] == IP
    say("ip index, l2 assignment: %s nb=%d d=%d nlist=%d M=%d nbits=%d" % (
        name, cfg["nb"], cfg["d"], cfg["nlist"], cfg["M"], cfg["nbits"]))
    x, q = S.make_data(cfg)
    cent, cb = S.make_index_params(cfg, x)
    cent = (cent * np.linspace(0.5, 2.0, cfg["nlist"], dtype=np.float32)[:, None]).astype(np.float32)
    ix = vs.IVFPQ(cfg["d"], IP, dev(cent), dev(cb), cfg["nbits"])
    ix.set_coarse_metric(L2)
    orc = oracle.OracleIVFPQ(cfg["d"], IP, cent, cb, cfg["nbits"], coarse_metric=L2)
    half = cfg["nb"] // 2
    ix.add(dev(x[:half])); ix.add(dev(x[half:]))
    orc.add(x[:half]); orc.add(x[half:])
    check_storage(ix, orc)
    assert (orc.add_list_of != oracle.assign(x, cent, IP)).mean() > 0.05     # the option changes the index
    with pytest.raises(vs.VSError):
        ix.set_coarse_metric(IP)                                   # not once vectors are stored
    xn = float(np.sqrt(orc.norms.max()))
    for k, nprobe in searches:
        say("  search k=%d nprobe=%d" % (k, nprobe))
        probes, cdist = ix.coarse(dev(q), nprobe)
        po, co = oracle.coarse_probe(q, cent, nprobe, L2)
        np.testing.assert_array_equal(host(probes), po)
        np.testing.assert_array_equal(host(cdist), co)
        D, I = ix.search(dev(q), k, nprobe)
        Do, Io = orc.search(q, k + EXTRA, nprobe)
        same = check_search(host(D), host(I), Do, Io, IP, q, xn)
        assert same > 0.99, same
    ix.close()
    l2 = vs.IVFPQ(cfg["d"], L2, dev(cent), dev(cb), cfg["nbits"])
    with pytest.raises(vs.VSError):
        l2.set_coarse_metric(IP)
    l2.close()


def test_ivfpq_add_in_pieces_with_custom_ids(vs, oracle):
    cfg = S.config("C1", nb=6_000)
    say("ivfpq pieces + custom ids")
    x, q = S.make_data(cfg)
    ix, orc = build_both(vs, oracle, cfg, x, pieces=3, custom_ids=True)
    check_storage(ix, orc)
    D, I = ix.search(dev(q), 10, 4)
    Do, Io = orc.search(q, 10 + EXTRA, 4)
    check_search(host(D), host(I), Do, Io, L2)
    ix.close()


def test_ivfpq_empty_index_and_padding(vs, oracle):
    cfg = S.config("C1", nb=60, nq=7)
    say("ivfpq empty index, then fewer candidates than k")
    x, q = S.make_data(cfg)
    cent, cb = S.make_index_params(S.config("C1"), S.make_data(S.config("C1"))[0])
    ix = vs.IVFPQ(cfg["d"], L2, dev(cent), dev(cb), 8)
    D, I = ix.search(dev(q), 5, 4)
    assert (host(I) == -1).all() and np.isposinf(host(D)).all()
    orc = oracle.OracleIVFPQ(cfg["d"], L2, cent, cb, 8)
    ix.add(dev(x)); orc.add(x)
    D, I = ix.search(dev(q), 40, 2)
    Do, Io = orc.search(q, 40 + EXTRA, 2)
    check_search(host(D), host(I), Do, Io, L2)
    assert (host(I) == -1).any()
    ix.close()


def test_search_is_deterministic(vs):
    cfg = S.config("C1")
    say("determinism")
    x, q = S.make_data(cfg)
    cent, cb = S.make_index_params(cfg, x)
    ix = vs.IVFPQ(cfg["d"], L2, dev(cent), dev(cb), 8)
    ix.add(dev(x))
    r1 = [host(t).copy() for t in ix.search(dev(q), 10, 4)]
    r2 = [host(t).copy() for t in ix.search(dev(q), 10, 4)]
    np.testing.assert_array_equal(r1[0], r2[0])
    np.testing.assert_array_equal(r1[1], r2[1])
    ix.close()


# ------------------------------------------------- full-size configurations

def test_search_stats_count_what_the_search_read(vs):
    """vs_ivfpq_search_stats: same results as vs_ivfpq_search, and a block that adds up the sizes
    of the probed lists (from the library's own probes and list sizes)."""
    cfg = S.config("C3", nb=60_000, nq=333, ncomp=100, nlist=300)      # some lists stay empty
    say("ivfpq search stats nb=%d nlist=%d" % (cfg["nb"], cfg["nlist"]))
    x, q = S.make_data(cfg)
    cent, cb = S.make_index_params(cfg, x)
    ix = vs.IVFPQ(cfg["d"], L2, dev(cent), dev(cb), 8)
    ix.add(dev(x[:30_000]))
    sizes = host(ix.list_sizes())
    for k, nprobe in ((10, 1), (10, 17), (100, 300), (10, 1000)):
        D, I = ix.search(dev(q), k, nprobe)
        D2, I2, st = ix.search_stats(dev(q), k, nprobe)
        np.testing.assert_array_equal(host(D2), host(D)); np.testing.assert_array_equal(host(I2), host(I))
        probes, _ = ix.coarse(dev(q), nprobe)
        sz = sizes[host(probes)]
        assert st["scanned_codes"] == int(sz.sum()) and st["probed_lists"] == int((sz > 0).sum())
        assert st["coarse_rows_matrix_core"] in (0, cfg["nq"])
        assert 0 <= st["coarse_rows_fallback"] <= st["coarse_rows_matrix_core"]
    import torch
    empty = torch.empty((0, cfg["d"]), dtype=torch.float32, device="cuda")
    _, _, st = ix.search_stats(empty, 10, 4)
    assert all(v == 0 for v in st.values())
    ix.close()


LIST_MAJOR_CASES = {
    # name: (config, [(k, nprobe, first, candidates)]) -- L2, the three shapes of the list-major scan
    "c3_like": (S.config("C3", nb=150_000, nq=1500, ncomp=200, nlist=256), [(10, 16, 4, 1024), (100, 64, 2, 1024), (1, 8, 1, 256)]),
    "c4_like": (S.config("C4", nb=120_000, nq=900, ncomp=100, nlist=128), [(100, 32, 4, 1024), (10, 16, 3, 512)]),
    "c1_like": (S.config("C1", nb=60_000, nq=700, nlist=64), [(10, 8, 2, 1024), (40, 64, 4, 1024)]),
    # a candidate buffer far too small: most queries overflow and are scanned again query by query
    "c3_like_overflow": (S.config("C3", nb=150_000, nq=600, ncomp=200, nlist=256), [(10, 32, 1, 64)]),
    # first lists shorter than k: no bound from the first stage, every code of the other lists is a candidate
    "c4_like_short_lists": (S.config("C4", nb=6_000, nq=300, ncomp=100, nlist=256), [(100, 32, 1, 128), (100, 64, 4, 65536)]),
    # a handful of queries
    "c4_like_few_queries": (S.config("C4", nb=120_000, nq=5, ncomp=100, nlist=128), [(100, 64, 4, 1024)]),
}


@pytest.mark.parametrize("name", list(LIST_MAJOR_CASES))
def test_list_major_scan_equals_query_major_scan_and_oracle(vs, oracle, name):
    """The list-major scan (every list read once per batch; codes kept under the bound that the
    query's first lists give; queries whose candidate buffer overflows scanned again) returns,
    bit for bit, what the query-major scan returns -- the distances are formed by the same
    arithmetic -- also when the buffer overflows, when the first lists give no bound, and call
    after call; both agree with the oracle.  The statistics block says what was done."""
    cfg, searches = LIST_MAJOR_CASES[name]
    say("list-major %s nb=%d nq=%d nlist=%d M=%d" % (name, cfg["nb"], cfg["nq"], cfg["nlist"], cfg["M"]))
    x, q = S.make_data(cfg)
    ix, orc = build_both(vs, oracle, cfg, x)
    xn = float(np.sqrt(orc.norms.max()))
    try:
        for k, nprobe, first, cand in searches:
            say("  k=%d nprobe=%d first=%d candidates=%d" % (k, nprobe, first, cand))
            vs.vs_set_option("list_major", -1)
            D0, I0, st0 = ix.search_stats(dev(q), k, nprobe)
            D0, I0 = host(D0).copy(), host(I0).copy()
            assert st0["list_major_first_probes"] == 0 and st0["list_major_rescanned"] == 0
            vs.vs_set_option("list_major", 1)
            vs.vs_set_option("list_major_first", first)
            vs.vs_set_option("list_major_candidates", cand)
            for rep in range(2):
                D1, I1, st1 = ix.search_stats(dev(q), k, nprobe)
                np.testing.assert_array_equal(host(I1), I0)
                np.testing.assert_array_equal(host(D1), D0)
                npr = min(nprobe, cfg["nlist"])
                assert st1["list_major_first_probes"] == min(first, npr - 1)
                assert st1["scanned_codes"] == st0["scanned_codes"]
                assert 0 < st1["list_major_first_codes"] <= st1["scanned_codes"]
                assert 0 <= st1["list_major_rescanned"] <= cfg["nq"]
                if name == "c3_like_overflow":
                    assert st1["list_major_rescanned"] > 0
                if cand >= 65536:
                    assert st1["list_major_rescanned"] == 0
            po, co = oracle.coarse_probe(q, orc.centroids, nprobe, L2)
            Do, Io = orc.search(q, k + EXTRA, nprobe)
            tc, te = l2_table_cancel(co, orc.codebooks)
            same = check_search(host(D1), host(I1), Do, Io, L2, q, xn, cancel=tc, cancel_eps=te)
            assert same > 0.99, same
    finally:
        vs.vs_set_option("list_major", 0)
        vs.vs_set_option("list_major_first", 4)
        vs.vs_set_option("list_major_candidates", 1024)
        ix.close()


def test_list_major_random_shapes_equal_query_major(vs):
    """Seeded odd shapes (empty index, one list, half of the lists empty, k beyond the index,
    nprobe beyond nlist, first-stage probes and candidate buffers of every size): the list-major
    search returns the query-major search's bits, and says how many queries it scanned again."""
    import torch
    rng = np.random.default_rng(2024)
    shapes = [(128, 16), (96, 32), (32, 8)]
    try:
        for case in range(24):
            d, M = shapes[case % 3]
            nlist = int(rng.choice([1, 3, 17, 64, 300, 1000]))
            nb = int(rng.choice([0, 50, 3000, 40_000, 150_000]))
            nq = int(rng.choice([1, 7, 100, 1000, 5000]))
            k = int(rng.choice([1, 5, 10, 100, 300, 1000]))
            nprobe = int(rng.choice([1, 2, 5, 16, 64, 200]))
            first = int(rng.choice([1, 2, 4, 9]))
            cap = int(rng.choice([64, 100, 1024, 8192]))
            say("list-major random %d: d=%d M=%d nlist=%d nb=%d nq=%d k=%d nprobe=%d first=%d candidates=%d" % (
                case, d, M, nlist, nb, nq, k, nprobe, first, cap))
            g = torch.Generator(device="cuda"); g.manual_seed(case)
            cent = torch.randn((nlist, d), generator=g, device="cuda")
            sel = torch.randint(0, nlist // 2 + 1, (max(nb, 1),), generator=g, device="cuda")[:nb]
            x = cent[sel] + 0.4 * torch.randn((nb, d), generator=g, device="cuda")
            q = cent[torch.randint(0, nlist, (nq,), generator=g, device="cuda")] + \
                0.4 * torch.randn((nq, d), generator=g, device="cuda")
            cb = 0.4 * torch.randn((M, 256, d // M), generator=g, device="cuda")
            ix = vs.IVFPQ(d, L2, cent, cb, 8)
            if nb:
                ix.add(x)
            vs.vs_set_option("list_major", -1)
            D0, I0 = [host(t).copy() for t in ix.search(q, k, nprobe)]
            vs.vs_set_option("list_major", 1)
            vs.vs_set_option("list_major_first", first)
            vs.vs_set_option("list_major_candidates", cap)
            D1, I1, st = ix.search_stats(q, k, nprobe)
            np.testing.assert_array_equal(host(I1), I0)
            np.testing.assert_array_equal(host(D1), D0)
            assert 0 <= st["list_major_rescanned"] <= nq
            ix.close()
    finally:
        vs.vs_set_option("list_major", 0)
        vs.vs_set_option("list_major_first", 4)
        vs.vs_set_option("list_major_candidates", 1024)


def test_list_major_option_rules(vs):
    for name, bad in (("list_major", 2), ("list_major_first", 0), ("list_major_first", 65), ("list_major_candidates", 63)):
        with pytest.raises(Exception):
            vs.vs_set_option(name, bad)
    vs.vs_set_option("list_major", 0)


def test_c3_full_size_sampled(vs, oracle):
    """IVF4096,PQ16x8 on 1M vectors in the launch configuration the bench times.
    The oracle cannot add 1M vectors in seconds, so assignments and codes are checked
    bit-exactly on a seeded sample, and the oracle then searches the GPU-built
    store for a seeded subset of the queries."""
    cfg = S.config("C3")
    say("C3 full size: nb=%d nlist=%d" % (cfg["nb"], cfg["nlist"]))
    x, q = S.make_data(cfg)
    cent, cb = S.make_index_params(cfg, x)
    ix = vs.IVFPQ(cfg["d"], L2, dev(cent), dev(cb), 8)
    ix.add(dev(x))
    ids, list_of = ix.assignments()
    ids, list_of, codes = host(ids), host(list_of), host(ix.codes())
    sizes = host(ix.list_sizes())
    assert sizes.sum() == cfg["nb"] and (np.sort(ids) == np.arange(cfg["nb"])).all()
    rng = np.random.default_rng(5)
    sample = np.sort(rng.choice(cfg["nb"], 20_000, replace=False))
    say("  oracle assign + encode on %d sampled vectors" % sample.size)
    lo = oracle.assign(x[sample], cent, L2)
    co = oracle.pq_encode(x[sample], lo, cent, cb, 8)
    pos = np.empty(cfg["nb"], dtype=np.int64); pos[ids] = np.arange(cfg["nb"])
    np.testing.assert_array_equal(list_of[pos[sample]], lo)
    np.testing.assert_array_equal(codes[pos[sample]], co)
    offsets = np.zeros(cfg["nlist"] + 1, dtype=np.int64); np.cumsum(sizes, out=offsets[1:])
    orc = oracle.OracleIVFPQ.from_storage(cfg["d"], L2, cent, cb, 8, offsets, codes, ids)
    qs = np.sort(rng.choice(cfg["nq"], 200, replace=False))
    dq = dev(q)
    for k, nprobe in ((10, 1), (10, 16), (10, 64), (100, 64)):
        say("  search all %d queries, k=%d nprobe=%d; oracle on %d of them" % (cfg["nq"], k, nprobe, qs.size))
        D, I = ix.search(dq, k, nprobe)
        Do, Io = orc.search(q[qs], k + EXTRA, nprobe)
        _, co = oracle.coarse_probe(q[qs], cent, nprobe, L2)
        tc, te = l2_table_cancel(co, cb)
        check_search(host(D)[qs], host(I)[qs], Do, Io, L2, cancel=tc, cancel_eps=te)
    # the other two search types on the same store, at the widest setting (Sec. 4.3)
    cancel = (q[qs].astype(np.float64) ** 2).sum(1) + float((cent.astype(np.float64) ** 2).sum(1).max()) + \
        float((cb.astype(np.float64) ** 2).sum(2).max(1).sum())
    Do, Io = orc.search(q[qs], 100 + EXTRA, 64)
    for st in (vs.ST_STORED_NORMS, vs.ST_PRECOMPUTED_TABLES):
        say("  search type %d, k=100 nprobe=64" % st)
        ix.set_search_type(st)
        D, I = ix.search(dq, 100, 64)
        check_search(host(D)[qs], host(I)[qs], Do, Io, L2, cancel=cancel)
    ix.close()


def test_c2_full_size_sampled(vs, oracle):
    """Flat search, 1M x 128, k = 100: all 10k queries on the GPU, the oracle on a
    seeded sample of them (data are integer-valued, so distances are exact)."""
    cfg = S.config("C2")
    say("C2 full size: nb=%d nq=%d k=%d" % (cfg["nb"], cfg["nq"], cfg["k"]))
    x, q = S.make_data(cfg)
    D, I = vs.vs_flat_search(dev(x), dev(q), 100, L2)
    D, I = host(D), host(I)
    qs = np.sort(np.random.default_rng(6).choice(cfg["nq"], 48, replace=False))
    say("  oracle on %d sampled queries" % qs.size)
    Do, Io = oracle.flat_search(x, q[qs], 100, L2)
    np.testing.assert_array_equal(D[qs], Do)
    np.testing.assert_array_equal(I[qs], Io)
    assert (np.diff(D, axis=1) >= 0).all() and (I >= 0).all()


# ------------------------------------------------- the two k-nearest-row routes

ROUTE_CASES = [
    # name, nb, nq, d, k, metric, kind
    ("gauss_d32_k10", 20_000, 300, 32, 10, L2, "gauss"),
    ("gauss_d128_k100", 30_000, 150, 128, 100, L2, "gauss"),
    ("gauss_d96_k64_ip", 9_000, 77, 96, 64, IP, "gauss"),
    ("gauss_d64_k1", 5_000, 1000, 64, 1, L2, "gauss"),
    ("unit_d96_k20", 15_000, 100, 96, 20, L2, "unit"),
    ("sift_d128_k100", 50_000, 100, 128, 100, L2, "sift"),
    ("tiny_nb_d32", 50, 10, 32, 40, L2, "gauss"),
    # exactly-bf16 data and >= 1024 rows of A: the one-pass collect sweep with two row blocks per
    # wavefront, at every d it is built for, with row counts that leave ragged 256-row tiles
    ("sift_d32_k10_many_rows", 20_000, 1500, 32, 10, L2, "sift"),
    ("sift_d64_k5_ip_many_rows", 12_000, 1111, 64, 5, IP, "sift"),
    ("sift_d96_k30_many_rows", 15_000, 1025, 96, 30, L2, "sift"),
    ("sift_d128_k100_many_rows", 25_000, 1300, 128, 100, L2, "sift"),
    # dimensions beyond 128: the tiled kernel (operands streamed in chunks of 32 dimensions)
    ("gauss_d256_k10", 20_000, 700, 256, 10, L2, "gauss"),
    ("gauss_d160_k100", 12_000, 130, 160, 100, L2, "gauss"),
    ("unit_d768_k32_ip", 9_000, 300, 768, 32, IP, "unit"),
    ("sift_d256_k20", 40_000, 64, 256, 20, L2, "sift"),
    ("gauss_d2048_k5", 3_000, 40, 2048, 5, L2, "gauss"),
    # integer queries (exactly bf16) against a general database: the two-pass variant (nq >= 256)
    ("int_q_float_x_d128_k20", 30_000, 700, 128, 20, L2, "int_q"),
    ("int_q_float_x_d64_k5_ip", 8_000, 300, 64, 5, IP, "int_q"),
    ("int_q_float_x_d96_few_rows", 8_000, 40, 96, 10, L2, "int_q"),    # short A: three passes
    # B barely longer than the shortlist: fewer finite group minima than the wanted rank
    ("gauss_d256_k100_short_b", 190, 70, 256, 100, L2, "gauss"),
    ("gauss_d160_k150_ip_short_b", 300, 33, 160, 150, IP, "gauss"),
    ("gauss_d768_k32_ip_short_b", 128, 300, 768, 32, IP, "gauss"),
    ("gauss_d128_k100_short_b", 130, 40, 128, 100, L2, "gauss"),
    # long database in cluster order: the threshold comes from a sample of the columns
    ("sift_sorted_d128_k100", 200_000, 64, 128, 100, L2, "sift_sorted"),
    ("unit_sorted_d96_k10", 150_000, 96, 96, 10, L2, "unit_sorted"),
    # a handful of rows against a long database: the forced exact fallback cuts the columns into
    # its largest number of chunks
    ("gauss_d128_k50_three_rows", 120_000, 3, 128, 50, L2, "gauss"),
    ("gauss_d64_k1_ip_one_row", 70_000, 1, 64, 1, IP, "gauss"),
]


@pytest.mark.parametrize("name,nb,nq,d,k,metric,kind", ROUTE_CASES, ids=[c[0] for c in ROUTE_CASES])
def test_matrix_core_route_equals_canon_route(vs, oracle, name, nb, nq, d, k, metric, kind):
    """Flat search through the MFMA shortlist + re-rank must return exactly what the
    canon distance tiles return (values and ids), also when every row is forced through
    the exact fallback; both agree with the oracle."""
    say("routes %s nb=%d nq=%d d=%d k=%d metric=%d" % (name, nb, nq, d, k, metric))
    if kind == "gauss":
        rng = np.random.default_rng(zlib.crc32(name.encode()))
        x = rng.standard_normal((nb, d), dtype=np.float32)
        q = rng.standard_normal((nq, d), dtype=np.float32)
    elif kind == "int_q":
        rng = np.random.default_rng(zlib.crc32(name.encode()))
        x = (30.0 * rng.standard_normal((nb, d))).astype(np.float32)
        q = np.rint(30.0 * rng.standard_normal((nq, d))).astype(np.float32)
    elif kind.startswith("unit"):
        x, q = S.make_data(S.config("C4", nb=nb, nq=nq, d=d, ncomp=30))
    else:
        x, q = S.make_data(S.config("C2", nb=nb, nq=nq, d=d, ncomp=30))
    if kind.endswith("sorted"):
        x = np.ascontiguousarray(x[np.lexsort(x[:, :3].T)])
    xd, qd = dev(x), dev(q)
    try:
        vs.vs_set_option("knn_path", 1)
        Dc, Ic = [host(t).copy() for t in vs.vs_flat_search(xd, qd, k, metric)]
        vs.vs_set_option("knn_path", 0)
        vs.vs_counters_read()
        Dm, Im = [host(t).copy() for t in vs.vs_flat_search(xd, qd, k, metric)]
        rows, fallback = vs.vs_counters_read()
        say("  matrix-core route: %d rows, %d needed the exact fallback" % (rows, fallback))
        assert rows == nq
        vs.vs_set_option("knn_eps_scale", -1.0)
        Df, If = [host(t).copy() for t in vs.vs_flat_search(xd, qd, k, metric)]
        rows, fallback = vs.vs_counters_read()
        assert fallback == nq
    finally:
        vs.vs_set_option("knn_eps_scale", 1.0)
        vs.vs_set_option("knn_path", 0)
    np.testing.assert_array_equal(Dm, Dc)
    np.testing.assert_array_equal(Im, Ic)
    np.testing.assert_array_equal(Df, Dc)
    np.testing.assert_array_equal(If, Ic)
    Do, Io = oracle.flat_search(x, q, min(k + EXTRA, max(nb, k)), metric)
    xn = np.sqrt((x.astype(np.float64) ** 2).sum(1).max())
    check_search(Dm, Im, Do, Io, metric, q, xn)


def test_random_route_shapes_agree(vs, oracle):
    """Forty seeded shapes over every d class of the matrix-core kernels (register-stationary and
    tiled, up to 2048), ragged and tiny B, k from 1 to 150, the three operand-precision variants
    and data with a large common offset: the matrix-core route returns what the canon tiles
    return, bit for bit, and both agree with the oracle on the shape's queries (on a seeded
    sub-sample of them where nb * nq * d is large)."""
    import torch
    rng = np.random.default_rng(20241127)
    try:
        for n in range(40):
            d = int(rng.choice([32, 64, 96, 128, 160, 192, 256, 320, 512, 768, 1024, 2048]))
            nb = int(rng.choice([1, 5, 63, 64, 65, 127, 129, 190, 255, 257, 300, 1000, 2047, 2049, 5000, 20000]))
            nq = int(rng.choice([1, 2, 31, 64, 100, 255, 256, 257, 600]))
            if nb * nq * d > 2e10:
                nq = max(1, int(2e10 / (nb * d)))
            k = int(rng.choice([1, 2, 10, 32, 64, 100, 128, 150]))
            metric = int(rng.choice([L2, L2, IP]))
            kind = int(rng.choice([0, 1, 2, 3]))
            say("route shape %d: d=%d nb=%d nq=%d k=%d metric=%d kind=%d" % (n, d, nb, nq, k, metric, kind))
            g = torch.Generator(device="cuda"); g.manual_seed(1000 + n)
            x = torch.randn((nb, d), generator=g, device="cuda")
            q = torch.randn((nq, d), generator=g, device="cuda")
            if kind == 1:                       # integers on both sides: one pass
                x, q = (x * 20).round(), (q * 20).round()
            elif kind == 2:                     # exact queries, general database: two passes from 256 queries on
                x, q = x * 20, (q * 20).round()
            elif kind == 3:                     # a common offset: large norms, small gaps
                x, q = x + 3.0, q + 3.0
            vs.vs_set_option("knn_path", 1)
            Dc, Ic = vs.vs_flat_search(x, q, k, metric)
            vs.vs_set_option("knn_path", 0)
            vs.vs_counters_read()
            Dm, Im = vs.vs_flat_search(x, q, k, metric)
            rows, _ = vs.vs_counters_read()
            assert rows == nq
            np.testing.assert_array_equal(host(Im), host(Ic))
            np.testing.assert_array_equal(host(Dm), host(Dc))
            nqs = int(max(1, min(nq, 4e8 // (nb * d))))
            qs = np.sort(rng.choice(nq, nqs, replace=False))
            xh, qh = host(x), host(q)[qs]
            Do, Io = oracle.flat_search(xh, qh, min(k + EXTRA, max(nb, k)), metric)
            xn = np.sqrt((xh.astype(np.float64) ** 2).sum(1).max())
            check_search(host(Dm)[qs], host(Im)[qs], Do, Io, metric, qh, xn)
    finally:
        vs.vs_set_option("knn_path", 0)


def test_sweeps_on_fp16_heads_alone_never_change_a_result(vs, oracle):
    """An index's own operand is first swept by its fp16 heads alone (one matrix product, a wide
    error bound); rows that cannot be proven under that bound are redone exactly, and when too many
    are, later calls go back to three products.  Whatever the state, every call returns what the
    canon tiles return, bit for bit: on data with a large common offset (many rows fail the wide
    bound), on well-separated data (none does), on values so small that their fp16 images are
    subnormal or zero, on values beyond the fp16 range (where the attempt must not be made), for
    inner product, for k = 1 and k > 1, call after call."""
    import torch
    cases = (("offset", 20_000, 700, 64, L2, 1.0), ("gauss", 30_000, 600, 96, L2, 1.0),
             ("offset", 9_000, 300, 256, L2, 1.0), ("gauss", 12_000, 300, 128, L2, 3e-6),
             ("gauss", 12_000, 300, 64, L2, 2e-8), ("gauss", 12_000, 300, 128, L2, 4e4),
             ("gauss", 8_000, 200, 512, L2, 1e5), ("gauss", 15_000, 400, 128, IP, 1.0),
             ("gauss", 9_000, 300, 256, IP, 1e-6))
    for kind, nb, nq, d, metric, scale in cases:
        g = torch.Generator(device="cuda"); g.manual_seed(77)
        x = torch.randn((nb, d), generator=g, device="cuda")
        q = torch.randn((nq, d), generator=g, device="cuda")
        if kind == "offset":
            x, q = x + 3.0, q + 3.0
        x, q = x * scale, q * scale
        ix = vs.Flat(d, metric)
        ix.add(x)
        for k in (1, 10, 1, 10, 10):
            say("heads alone: %s nb=%d d=%d metric=%d scale=%g k=%d" % (kind, nb, d, metric, scale, k))
            vs.vs_set_option("knn_path", 1)
            try:
                Dc, Ic = [host(t).copy() for t in vs.vs_flat_search(x, q, k, metric)]
            finally:
                vs.vs_set_option("knn_path", 0)
            vs.vs_counters_read()
            D, I = [host(t).copy() for t in ix.search(q, k)]
            rows, fallback = vs.vs_counters_read()
            assert rows == nq and 0 <= fallback <= nq
            np.testing.assert_array_equal(I, Ic)
            np.testing.assert_array_equal(D, Dc)
        # by now calls of both kinds have settled: a call redoes at most one row in 512 (or 7)
        vs.vs_counters_read()
        ix.search(q, 10); ix.search(q, 1)
        rows, fallback = vs.vs_counters_read()
        assert rows == 2 * nq and fallback <= 2 * max(7, nq // 512 + 1), (kind, scale, fallback)
        ix.close()
        Do, Io = oracle.flat_search(host(x), host(q)[:20], 10, metric)
        np.testing.assert_array_equal(I[:20], Io)


# ------------------------------------------------- flat index (prepared database)

FLAT_INDEX_CASES = [
    # name, nb, nq, d, k, metric, kind
    ("sift_d128_k100", 30_000, 200, 128, 100, L2, "sift"),      # one matrix-core pass, row-major planes
    ("gauss_d768_k10_ip", 5_000, 64, 768, 10, IP, "gauss"),     # tiled kernel, panel planes
    ("gauss_d256_k30", 9_000, 70, 256, 30, L2, "gauss"),
    ("gauss_d100_k20", 4_000, 50, 100, 20, L2, "gauss"),        # d the matrix-core route does not cover
    ("sift_d128_k300", 6_000, 33, 128, 300, L2, "sift"),        # k beyond the matrix-core route: planes unused
]


@pytest.mark.parametrize("name,nb,nq,d,k,metric,kind", FLAT_INDEX_CASES, ids=[c[0] for c in FLAT_INDEX_CASES])
def test_flat_index_equals_flat_search(vs, oracle, name, nb, nq, d, k, metric, kind):
    """The flat index returns, after every add, exactly what the stateless flat search returns
    on the rows stored so far (the prepared operand is laid out anew when the index grows),
    and the final state agrees with the oracle."""
    say("flat index %s nb=%d nq=%d d=%d k=%d metric=%d" % (name, nb, nq, d, k, metric))
    if kind == "gauss":
        rng = np.random.default_rng(zlib.crc32(name.encode()))
        x = rng.standard_normal((nb, d), dtype=np.float32)
        q = rng.standard_normal((nq, d), dtype=np.float32)
    else:
        x, q = S.make_data(S.config("C2", nb=nb, nq=nq, d=d, ncomp=30))
    xd, qd = dev(x), dev(q)
    ix = vs.Flat(d, metric)
    assert ix.ntotal == 0
    D0, I0 = ix.search(qd, k)                                   # empty index: empty slots
    assert (host(I0) == -1).all()
    assert np.isinf(host(D0)).all()
    n = 0
    for piece in (1000, 1, nb // 2, nb):                        # grows twice; a one-row add
        m = min(piece, nb - n)
        if m <= 0:
            break
        say("  add %d rows at %d" % (m, n))
        ix.add(xd[n:n + m])
        n += m
        assert ix.ntotal == n
        Di, Ii = ix.search(qd, k)
        Ds, Is = vs.vs_flat_search(xd[:n], qd, k, metric)
        np.testing.assert_array_equal(host(Ii), host(Is))
        np.testing.assert_array_equal(host(Di), host(Ds))
    assert n == nb
    Do, Io = oracle.flat_search(x, q, min(k + EXTRA, nb), metric)
    xn = np.sqrt((x.astype(np.float64) ** 2).sum(1).max())
    check_search(host(Di), host(Ii), Do, Io, metric, q, xn)
    with pytest.raises(vs.VSError):
        ix.search(qd, vs.VS_MAX_K + 1)
    with pytest.raises(ValueError):
        ix.add(xd[:3, : d - 1].contiguous())
    ix.close()


# ------------------------------------------------- refinement of a shortlist

REFINE_CASES = [
    # name, nb, nq, d, kc, k, metric
    ("gauss_d32", 5_000, 100, 32, 100, 10, L2),
    ("gauss_d96_ip", 3_000, 37, 96, 70, 70, IP),          # k = kc: a pure re-ordering
    ("gauss_d30_large_k", 4_000, 9, 30, 1500, 1000, L2),  # odd d, selection in LDS (k > 192)
    ("gauss_d768", 2_000, 21, 768, 33, 5, IP),
]


@pytest.mark.parametrize("name,nb,nq,d,kc,k,metric", REFINE_CASES, ids=[c[0] for c in REFINE_CASES])
def test_refine_matches_oracle(vs, oracle, name, nb, nq, d, kc, k, metric):
    say("refine %s nb=%d nq=%d d=%d kc=%d k=%d metric=%d" % (name, nb, nq, d, kc, k, metric))
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    x = rng.standard_normal((nb, d), dtype=np.float32)
    q = rng.standard_normal((nq, d), dtype=np.float32)
    cand = np.stack([rng.choice(nb, kc, replace=False) for _ in range(nq)]).astype(np.int64)
    cand[rng.random(cand.shape) < 0.05] = -1              # empty slots of a first stage
    cand[0, :] = -1                                        # a query with nothing to refine
    cand[1, : kc - 2] = -1                                 # and one with two candidates
    D, I = [host(t) for t in vs.vs_refine(dev(x), dev(q), dev(cand), k, metric)]
    Do, Io = oracle.refine(x, q, cand, k, metric)
    assert (I[0] == -1).all() and (I[1, min(2, k):] == -1).all()
    np.testing.assert_array_equal(I == -1, Io == -1)
    xn = np.sqrt((x.astype(np.float64) ** 2).sum(1).max())
    # candidates are distinct, so the oracle's k best ARE the answer: same ids except where
    # two oracle distances are within the tolerance, same distances within the tolerance
    Dx, Ix = oracle.refine(x, q, cand, min(k + EXTRA, kc), metric)
    check_search(D, I, Dx, Ix, metric, q, xn)


def test_refine_on_integer_data_equals_flat_search_bits(vs, oracle):
    """Exact distances on integer data are exact in every summation order: re-ranking a
    shuffled superset of flat search's answer returns flat search's answer bit for bit."""
    cfg = S.config("C2", nb=20_000, nq=64, ncomp=30)
    say("refine on integer data vs flat search")
    x, q = S.make_data(cfg)
    Df, If = [host(t) for t in vs.vs_flat_search(dev(x), dev(q), 50, L2)]
    rng = np.random.default_rng(5)
    extra = rng.integers(0, cfg["nb"], size=(64, 30))
    cand = np.concatenate([If, extra], axis=1)
    for a in range(64):                                    # distinct ids per query, shuffled
        u = np.unique(cand[a])
        row = np.full(80, -1, dtype=np.int64)
        row[: u.size] = rng.permutation(u)
        cand[a] = row
    D, I = [host(t) for t in vs.vs_refine(dev(x), dev(q), dev(cand), 50, L2)]
    np.testing.assert_array_equal(I, If)
    np.testing.assert_array_equal(D, Df)
    Do, Io = oracle.refine(x, q, cand, 50, L2)
    np.testing.assert_array_equal(I, Io)
    np.testing.assert_array_equal(D, Do)


def test_ivfpq_search_then_refine_pipeline(vs, oracle):
    """First stage IVF-PQ with a shortlist of 100, second stage exact: the pipeline agrees
    with the oracle's pipeline and gains recall over the first stage's own top 10."""
    cfg = S.config("C3", nb=100_000, nq=200, ncomp=100, nlist=512)
    say("ivfpq -> refine pipeline")
    x, q = S.make_data(cfg)
    ix, orc = build_both(vs, oracle, cfg, x)
    D1, I1 = ix.search(dev(q), 100, 16)
    Dr, Ir = [host(t) for t in vs.vs_refine(dev(x), dev(q), I1, 10, L2)]
    Do1, Io1 = orc.search(q, 100, 16)
    # the two first stages may order near-ties differently; refine the GPU's own shortlist
    # with the oracle (integer data: exact values, so the comparison is bit for bit)
    Dor, Ior = oracle.refine(x, q, host(I1), 10, L2)
    np.testing.assert_array_equal(Ir, Ior)
    np.testing.assert_array_equal(Dr, Dor)
    _, It = oracle.flat_search(x, q, 10, L2)
    r1, r2 = oracle.recall(host(I1)[:, :10], It), oracle.recall(Ir, It)
    say("  10-recall@10: first stage %.3f, refined %.3f" % (r1, r2))
    assert r2 >= r1 and r2 > r1 + 0.1
    ix.close()


# ------------------------------------------------- L2 through stored norms (Sec. 4.3)

@pytest.mark.parametrize("name", ["c1", "c3_small", "c4_small", "pq4_l2", "odd_shapes", "c4_long_lists",
                                  "c3_long_lists", "c1_long_lists", "pq16x8_d64", "pq32x4_d64",
                                  "max_k_and_nprobe"])
def test_ivfpq_stored_norm_search_matches_oracle(vs, oracle, name):
    """Search type |q|^2 + |x'|^2 - 2 <q, x'>: the stored norms are the oracle's bit for bit,
    the results agree with the definition (oracle form 0) within the rounding of the
    cancelling terms, and with the default search type of the same index."""
    cfg, searches = IVF_CASES[name]
    say("ivfpq stored norms %s nb=%d d=%d nlist=%d M=%d nbits=%d" % (
        name, cfg["nb"], cfg["d"], cfg["nlist"], cfg["M"], cfg["nbits"]))
    x, q = S.make_data(cfg)
    cent, cb = S.make_index_params(cfg, x)
    ix = vs.IVFPQ(cfg["d"], L2, dev(cent), dev(cb), cfg["nbits"])
    ix.set_search_type(vs.ST_STORED_NORMS)
    orc = oracle.OracleIVFPQ(cfg["d"], L2, cent, cb, cfg["nbits"])
    half = cfg["nb"] // 2
    ix.add(dev(x[:half])); ix.add(dev(x[half:]))                 # two pieces: norms move with the codes
    orc.add(x[:half]); orc.add(x[half:])
    check_storage(ix, orc)
    np.testing.assert_array_equal(host(ix.norms()), orc.norms)
    cancel = (q.astype(np.float64) ** 2).sum(1) + float(orc.norms.max())
    for k, nprobe in searches:
        say("  search k=%d nprobe=%d" % (k, nprobe))
        D, I = [host(t).copy() for t in ix.search(dev(q), k, nprobe)]
        Do, Io = orc.search(q, k + EXTRA, nprobe)                 # the definition
        same = check_search(D, I, Do, Io, L2, cancel=cancel)
        assert same > 0.97, same
        ix.set_search_type(vs.ST_RESIDUAL_TABLES)                 # the other form on the same store
        D0, I0 = [host(t) for t in ix.search(dev(q), k, nprobe)]
        ix.set_search_type(vs.ST_STORED_NORMS)
        live = I0 >= 0
        assert (np.abs(D.astype(np.float64) - D0)[live] <= (1e-4 * np.abs(D0) + 2.0 ** -21 * cancel[:, None])[live]).all()
    ix.close()


@pytest.mark.parametrize("name", ["c1", "c3_small", "c4_small", "c4_long_lists", "c3_long_lists", "c1_long_lists",
                                  "max_k_and_nprobe"])
def test_ivfpq_precomputed_table_search_matches_oracle(vs, oracle, name):
    """Search type "per-query term + per-list term" (Sec. 4.3): against the definition (oracle form
    0) within the rounding of the cancelling terms |q|^2 + |c_l|^2 + |x' - c_l|^2, and against the
    default search type of the same index; switching back and forth leaves both unchanged."""
    cfg, searches = IVF_CASES[name]
    say("ivfpq precomputed tables %s nb=%d d=%d nlist=%d M=%d" % (name, cfg["nb"], cfg["d"], cfg["nlist"], cfg["M"]))
    x, q = S.make_data(cfg)
    ix, orc = build_both(vs, oracle, cfg, x, pieces=2)
    check_storage(ix, orc)
    tmax = float((orc.codebooks.astype(np.float64) ** 2).sum(2).max(1).sum())
    cancel = (q.astype(np.float64) ** 2).sum(1) + float((orc.centroids.astype(np.float64) ** 2).sum(1).max()) + tmax
    for k, nprobe in searches:
        say("  search k=%d nprobe=%d" % (k, nprobe))
        D0, I0 = [host(t).copy() for t in ix.search(dev(q), k, nprobe)]
        ix.set_search_type(vs.ST_PRECOMPUTED_TABLES)
        D, I = [host(t).copy() for t in ix.search(dev(q), k, nprobe)]
        ix.set_search_type(vs.ST_RESIDUAL_TABLES)
        D1, I1 = [host(t).copy() for t in ix.search(dev(q), k, nprobe)]
        np.testing.assert_array_equal(D1, D0); np.testing.assert_array_equal(I1, I0)
        assert (D[I >= 0] >= 0).all()
        Do, Io = orc.search(q, k + EXTRA, nprobe)                 # the definition
        same = check_search(D, I, Do, Io, L2, cancel=cancel)
        assert same > 0.97, same
        live = I0 >= 0
        assert (np.abs(D.astype(np.float64) - D0)[live] <= (1e-4 * np.abs(D0) + 2.0 ** -21 * cancel[:, None])[live]).all()
    ix.close()


def test_precomputed_table_search_type_rules(vs):
    import torch
    say("precomputed tables: rules")
    cfg = S.config("C1", nb=2000)
    x, q = S.make_data(cfg)
    cent, cb = S.make_index_params(cfg, x)
    ip = vs.IVFPQ(cfg["d"], IP, dev(cent), dev(cb), 8)
    with pytest.raises(vs.VSError):
        ip.set_search_type(vs.ST_PRECOMPUTED_TABLES)            # L2 only
    ip.close()
    cfg2 = S.config("C1", nb=2000, M=16, nbits=4)
    cent2, cb2 = S.make_index_params(cfg2, x)
    g = vs.IVFPQ(cfg2["d"], L2, dev(cent2), dev(cb2), 4)
    with pytest.raises(vs.VSError) as e:
        g.set_search_type(vs.ST_PRECOMPUTED_TABLES)             # no specialised kernel for this shape
    assert e.value.code == -2
    g.close()
    ix = vs.IVFPQ(cfg["d"], L2, dev(cent), dev(cb), 8)
    ix.set_search_type(vs.ST_PRECOMPUTED_TABLES)                # before any add: fine, the tables depend on the parameters only
    ix.add(dev(x))
    D, I = ix.search(dev(q), 5, 3)
    ix.set_search_type(vs.ST_RESIDUAL_TABLES)
    D0, I0 = ix.search(dev(q), 5, 3)
    assert (host(I) == host(I0)).mean() > 0.98
    ix.close()


def test_stored_norm_search_on_integer_data_is_exact(vs, oracle):
    """With integer-valued vectors, centroids and codebooks every term of the decomposition
    is exact, so both search types and the oracle's definition return the same bits."""
    say("stored norms, integer data")
    rng = np.random.default_rng(77)
    x = rng.integers(0, 40, size=(6000, 32)).astype(np.float32)
    q = rng.integers(0, 40, size=(50, 32)).astype(np.float32)
    cent = x[rng.permutation(6000)[:16]].copy()
    cb = rng.integers(-6, 7, size=(8, 256, 4)).astype(np.float32)
    ix = vs.IVFPQ(32, L2, dev(cent), dev(cb), 8)
    ix.set_search_type(vs.ST_STORED_NORMS)
    ix.add(dev(x))
    orc = oracle.OracleIVFPQ(32, L2, cent, cb, 8)
    orc.add(x)
    D, I = [host(t).copy() for t in ix.search(dev(q), 10, 4)]
    Do, Io = orc.search(q, 10, 4)
    np.testing.assert_array_equal(D, Do)
    ix.set_search_type(vs.ST_RESIDUAL_TABLES)
    D0, I0 = [host(t) for t in ix.search(dev(q), 10, 4)]
    np.testing.assert_array_equal(D, D0)
    np.testing.assert_array_equal(I, I0)
    ix.close()


@pytest.mark.parametrize("name", ["c1", "pq4_l2", "c4_small", "odd_shapes"])
def test_stored_norms_of_an_index_filled_under_another_search_type(vs, oracle, name):
    """Selecting the stored-norm search on an index that holds vectors without norms computes them
    from the stored codes (rotated or not): bit for bit the oracle's norms, and they survive
    switching back and forth; an add under another search type drops them and a new selection
    brings all of them back."""
    cfg, searches = IVF_CASES[name]
    say("norms of a filled index: %s" % name)
    x, q = S.make_data(cfg)
    cent, cb = S.make_index_params(cfg, x)
    ix = vs.IVFPQ(cfg["d"], L2, dev(cent), dev(cb), cfg["nbits"])
    orc = oracle.OracleIVFPQ(cfg["d"], L2, cent, cb, cfg["nbits"])
    half = cfg["nb"] // 2
    ix.add(dev(x[:half])); orc.add(x[:half])
    ix.set_search_type(vs.ST_STORED_NORMS)                        # vectors were added without norms
    np.testing.assert_array_equal(host(ix.norms()), orc.norms)
    k, nprobe = searches[0]
    D1, I1 = [host(t).copy() for t in ix.search(dev(q), k, nprobe)]
    ix.set_search_type(vs.ST_RESIDUAL_TABLES)
    ix.add(dev(x[half:])); orc.add(x[half:])                      # drops the norms
    with pytest.raises(vs.VSError):
        ix.norms()
    ix.set_search_type(vs.ST_STORED_NORMS)
    check_storage(ix, orc)
    np.testing.assert_array_equal(host(ix.norms()), orc.norms)
    cancel = (q.astype(np.float64) ** 2).sum(1) + float(orc.norms.max())
    D, I = [host(t) for t in ix.search(dev(q), k, nprobe)]
    Do, Io = orc.search(q, k + EXTRA, nprobe)
    check_search(D, I, Do, Io, L2, cancel=cancel)
    ix.close()


def test_stored_norm_search_type_rules(vs):
    cfg = S.config("C1", nb=500)
    x, q = S.make_data(cfg)
    cent, cb = S.make_index_params(cfg, x)
    ix = vs.IVFPQ(32, L2, dev(cent), dev(cb), 8)
    ix.add(dev(x))
    with pytest.raises(vs.VSError):
        ix.set_search_type(7)
    ix.close()
    ixp = vs.IVFPQ(32, IP, dev(cent), dev(cb), 8)
    with pytest.raises(vs.VSError):
        ixp.set_search_type(vs.ST_STORED_NORMS)                   # L2 only
    ixp.close()


# ------------------------------------------------- IVF-Flat

IVFFLAT_CASES = {
    "c1": (S.config("C1"), [(10, 4), (10, 16), (1, 1), (300, 2)]),
    "c3_small": (S.config("C3", nb=60_000, nq=100, ncomp=100, nlist=256), [(10, 16), (100, 64)]),
    "c4_small_ip": (S.config("C4", nb=30_000, nq=64, ncomp=50, nlist=128, metric=1), [(10, 8)]),
    "odd_d30": (S.config("C1", nb=3_001, nq=33, d=30, nlist=7), [(10, 3), (500, 7)]),
    "d768": (S.config("C5", nb=4_000, nq=20, ncomp=20, nlist=16), [(10, 4)]),
    "max_k_and_nprobe": (S.config("C1", nb=30_000, nq=40, nlist=1024), [(1024, 1024)]),
}


@pytest.mark.parametrize("name", list(IVFFLAT_CASES))
def test_ivfflat_matches_oracle(vs, oracle, name):
    cfg, searches = IVFFLAT_CASES[name]
    say("ivfflat %s nb=%d d=%d nlist=%d metric=%d" % (name, cfg["nb"], cfg["d"], cfg["nlist"], cfg["metric"]))
    x, q = S.make_data(cfg)
    cent = S.make_centroids(x, cfg["nlist"], cfg["seed"])
    ix = vs.IVFFlat(cfg["d"], cfg["metric"], dev(cent))
    orc = oracle.OracleIVFFlat(cfg["d"], cfg["metric"], cent)
    half = cfg["nb"] // 3
    ids = np.arange(cfg["nb"], dtype=np.int64) * 2 + 11                  # custom ids, two pieces
    ix.add(dev(x[:half]), dev(ids[:half])); ix.add(dev(x[half:]), dev(ids[half:]))
    orc.add(x[:half], ids[:half]); orc.add(x[half:], ids[half:])
    assert ix.ntotal == cfg["nb"]
    # storage: same lists, same order inside every list, the stored rows are the vectors
    sid, slist, srows = [host(t) for t in ix.storage()]
    np.testing.assert_array_equal(host(ix.list_sizes()), orc.list_sizes())
    np.testing.assert_array_equal(sid, orc.ids)
    np.testing.assert_array_equal(srows, orc.vecs)
    np.testing.assert_array_equal(slist, np.repeat(np.arange(cfg["nlist"]), orc.list_sizes()))
    xn = np.sqrt((x.astype(np.float64) ** 2).sum(1).max())
    for k, nprobe in searches:
        say("  search k=%d nprobe=%d" % (k, nprobe))
        D, I = ix.search(dev(q), k, nprobe)
        Do, Io = orc.search(q, k + EXTRA, nprobe)
        # check_search has verified every id that differs (oracle distances within the
        # tolerance of each other); such near-ties must stay rare
        same = check_search(host(D), host(I), Do, Io, cfg["metric"], q, xn)
        assert same >= 0.97, same
    ix.close()


def test_ivfflat_with_all_lists_probed_equals_flat_search_bits(vs, oracle):
    """Both scans evaluate the same fp32 chain: probing every list of an IVF-Flat index
    returns flat search's values bit for bit (ids too, the data being integer-valued)."""
    cfg = S.config("C3", nb=30_000, nq=50, ncomp=50, nlist=64)
    say("ivfflat, all lists probed, vs flat search")
    x, q = S.make_data(cfg)
    ix = vs.IVFFlat(cfg["d"], L2, dev(S.make_centroids(x, 64, cfg["seed"])))
    ix.add(dev(x))
    D, I = [host(t) for t in ix.search(dev(q), 20, 64)]
    Df, If = [host(t) for t in vs.vs_flat_search(dev(x), dev(q), 20, L2)]
    np.testing.assert_array_equal(D, Df)
    check_search(D, I, *oracle.flat_search(x, q, 20 + EXTRA, L2), L2)
    ix.close()


# ------------------------------------------------- IVF-SQ8

IVFSQ8_CASES = {
    "c1": (S.config("C1"), [(10, 4), (10, 16), (300, 2)]),                          # d = 32: 32-wide tiles
    "c3_small": (S.config("C3", nb=60_000, nq=100, ncomp=100, nlist=256), [(10, 16), (100, 64)]),  # d = 128: 64-wide
    "c4_small_ip": (S.config("C4", nb=30_000, nq=64, ncomp=50, nlist=128, metric=1), [(10, 8)]),   # d = 96
    "odd_d30": (S.config("C1", nb=3_001, nq=33, d=30, nlist=7), [(10, 3), (500, 7)]),              # untiled kernel
}


@pytest.mark.parametrize("name", list(IVFSQ8_CASES))
def test_ivfsq8_matches_oracle(vs, oracle, name):
    cfg, searches = IVFSQ8_CASES[name]
    say("ivfsq8 %s nb=%d d=%d nlist=%d metric=%d" % (name, cfg["nb"], cfg["d"], cfg["nlist"], cfg["metric"]))
    x, q = S.make_data(cfg)
    cent = S.make_centroids(x, cfg["nlist"], cfg["seed"])
    vmin, step = oracle.sq8_params(x[: cfg["nb"] // 2])             # trained on half: the rest may fall outside
    ix = vs.IVFSQ8(cfg["d"], cfg["metric"], dev(cent), dev(vmin), dev(step))
    orc = oracle.OracleIVFSQ8(cfg["d"], cfg["metric"], cent, vmin, step)
    cut = cfg["nb"] // 3
    ix.add(dev(x[:cut])); ix.add(dev(x[cut:]))
    orc.add(x[:cut]); orc.add(x[cut:])
    sid, slist, scodes = [host(t) for t in ix.storage()]
    np.testing.assert_array_equal(host(ix.list_sizes()), orc.list_sizes())
    np.testing.assert_array_equal(sid, orc.ids)
    np.testing.assert_array_equal(scodes, orc.codes)                   # codes bit for bit
    xr = oracle.sq8_decode(orc.codes, vmin, step)
    xn = np.sqrt((xr.astype(np.float64) ** 2).sum(1).max())
    for k, nprobe in searches:
        say("  search k=%d nprobe=%d" % (k, nprobe))
        D, I = ix.search(dev(q), k, nprobe)
        Do, Io = orc.search(q, k + EXTRA, nprobe)
        same = check_search(host(D), host(I), Do, Io, cfg["metric"], q, xn)
        assert same >= 0.97, same
    ix.close()


def test_ivfflat_storage_beyond_four_billion_elements(vs):
    """72M x 96 floats added in three pieces: the last re-layout moves 4.6e9 elements, more
    than one launch can hold as work-items.  Every list probed must then equal flat search
    bit for bit, and sampled stored rows must be the vectors of their ids."""
    import torch
    cfg = S.config("C4", nb=72_000_000, nq=64, nlist=1024)
    say("ivfflat large storage: nb=%d d=%d" % (cfg["nb"], cfg["d"]))
    xd, qd = S.make_data_device(cfg)
    cent, _ = S.make_index_params_device(cfg, xd)
    ix = vs.IVFFlat(cfg["d"], L2, dev(cent))
    piece = cfg["nb"] // 3
    for s0 in range(0, cfg["nb"], piece):
        ix.add(xd[s0:s0 + piece])
        say("  added %d" % (s0 + piece))
    assert ix.ntotal == cfg["nb"] and int(ix.list_sizes().sum().item()) == cfg["nb"]
    D, I = ix.search(qd, 10, 1024)
    Df, If = vs.vs_flat_search(xd, qd, 10, L2)
    assert torch.equal(D, Df)
    assert (I == If).float().mean().item() > 0.99          # equal values may swap
    ids, list_of, rows = ix.storage()
    g = torch.Generator(device="cuda"); g.manual_seed(3)
    pos = torch.randint(0, cfg["nb"], (200_000,), generator=g, device="cuda")
    assert torch.equal(rows[pos], xd[ids[pos]])
    assert torch.equal(torch.sort(ids).values, torch.arange(cfg["nb"], device="cuda"))
    ix.close()


def test_add_whose_last_piece_is_shorter_than_the_others(vs):
    """One add of 2^20 + 931,328 vectors: the assignment runs in pieces of 2^20 rows and the
    shorter last piece is laid out with more splits of the centroids than a full one, so its
    work space is the larger of the two.  Every list probed must equal flat search."""
    import torch
    cfg = S.config("C4", nb=(1 << 20) + 931_328, nq=64, nlist=1024, d=32, M=8)
    say("ivfflat add with a shorter last piece: nb=%d d=%d" % (cfg["nb"], cfg["d"]))
    xd, qd = S.make_data_device(cfg)
    cent, _ = S.make_index_params_device(cfg, xd)
    ix = vs.IVFFlat(cfg["d"], L2, dev(cent))
    ix.add(xd)
    assert ix.ntotal == cfg["nb"] and int(ix.list_sizes().sum().item()) == cfg["nb"]
    D, I = ix.search(qd, 10, 1024)
    Df, If = vs.vs_flat_search(xd, qd, 10, L2)
    assert torch.equal(D, Df)
    assert (I == If).float().mean().item() > 0.99          # equal values may swap
    ix.close()


def test_random_shapes_flat_ivfflat_ivfsq8_match_oracle(vs, oracle):
    """Thirty seeded small problems of mixed shapes (d from 1 to 288, both routes of the distance
    stage, tiled and untiled list scans, k from 1 to 1024): flat search, IVF-Flat and IVF-SQ8
    against their oracles."""
    rng = np.random.default_rng(20240128)
    for n in range(30):
        d = int(rng.choice([1, 3, 8, 30, 32, 64, 96, 100, 128, 160, 288]))
        kind = str(rng.choice(["C1", "C3", "C4"]))
        nb = int(rng.choice([1, 60, 3_000, 12_000]))
        nq = int(rng.choice([1, 9, 130, 1_100]))
        metric = int(rng.choice([L2, L2, IP]))
        k = int(rng.choice([1, 10, 100, 1024]))
        nlist = int(min(nb, rng.choice([1, 5, 40])))
        nprobe = int(min(nlist, rng.choice([1, 4, 40])))
        cfg = S.config(kind, nb=nb, nq=nq, d=d, nlist=nlist, metric=metric, ncomp=min(20, nb), seed=2000 + n,
                       M=1, nbits=8)
        say("random problem %d: %s nb=%d nq=%d d=%d metric=%d k=%d nlist=%d nprobe=%d" % (
            n, kind, nb, nq, d, metric, k, nlist, nprobe))
        x, q = S.make_data(cfg)
        xn = np.sqrt((x.astype(np.float64) ** 2).sum(1).max())
        kk = min(k + EXTRA, max(nb, k))
        D, I = vs.vs_flat_search(dev(x), dev(q), k, metric)
        Do, Io = oracle.flat_search(x, q, kk, metric)
        check_search(host(D), host(I), Do, Io, metric, q, xn)
        cent = S.make_centroids(x, nlist, cfg["seed"])
        fx = vs.IVFFlat(d, metric, dev(cent))
        fo = oracle.OracleIVFFlat(d, metric, cent)
        fx.add(dev(x)); fo.add(x)
        D, I = fx.search(dev(q), k, nprobe)
        Do, Io = fo.search(q, k + EXTRA, nprobe)
        check_search(host(D), host(I), Do, Io, metric, q, xn)
        fx.close()
        vmin, step = oracle.sq8_params(x)
        sx = vs.IVFSQ8(d, metric, dev(cent), dev(vmin), dev(step))
        so = oracle.OracleIVFSQ8(d, metric, cent, vmin, step)
        sx.add(dev(x)); so.add(x)
        np.testing.assert_array_equal(host(sx.storage()[2]), so.codes)
        xr = oracle.sq8_decode(so.codes, vmin, step)
        xrn = np.sqrt((xr.astype(np.float64) ** 2).sum(1).max())
        D, I = sx.search(dev(q), k, nprobe)
        Do, Io = so.search(q, k + EXTRA, nprobe)
        check_search(host(D), host(I), Do, Io, metric, q, xrn)
        sx.close()


# ------------------------------------------------- k-means and parameter training

KMEANS_CASES = [
    # name, n, d, K, niter, kind
    ("gauss_d32_k16", 5_000, 32, 16, 5, "gauss"),            # matrix-core route, three passes
    ("sift_d128_k64", 20_000, 128, 64, 4, "sift"),            # matrix-core route, exact data in round 0
    ("unit_d96_k300", 30_000, 96, 300, 3, "unit"),
    ("subvectors_d4_k256", 20_000, 4, 256, 4, "gauss"),       # a sub-quantizer's shape: canon tiles
    ("odd_d30_k7", 3_001, 30, 7, 6, "gauss"),
    # large clusters of short rows: the update kernel that reads several rows per load
    ("subvectors_d8_k16", 30_000, 8, 16, 3, "gauss"),
    ("subvectors_d12_k20", 20_000, 12, 20, 3, "gauss"),
    ("subvectors_d3_k8", 9_000, 3, 8, 3, "gauss"),
    ("more_centroids_than_vectors", 40, 8, 64, 2, "gauss"),
    # clusters longer than 4096 vectors: the kernel adds partial sums, the oracle one by one
    ("long_clusters_d8_k4", 40_000, 8, 4, 3, "gauss"),
    ("long_clusters_d12_k3", 30_001, 12, 3, 2, "gauss"),
    ("long_clusters_d32_k5", 33_000, 32, 5, 2, "gauss"),
    ("long_clusters_d96_k3", 20_000, 96, 3, 2, "unit"),
    ("long_clusters_d200_k2", 13_000, 200, 2, 2, "gauss"),
    ("long_and_short_clusters_d64", 25_000, 64, 40, 2, "sift"),
    # more centroids than the device-side bookkeeping takes (16384): the host sorts the assignment
    ("host_bookkeeping_k20000", 25_000, 4, 20_000, 2, "gauss"),
    ("device_bookkeeping_k16384", 40_000, 8, 16_384, 2, "gauss"),
]


def _ulp_apart(a, b):
    """Largest distance between two fp32 arrays counted in representable numbers."""
    ia = a.view(np.int32).astype(np.int64); ib = b.view(np.int32).astype(np.int64)
    ia = np.where(ia < 0, -(ia & 0x7FFFFFFF), ia); ib = np.where(ib < 0, -(ib & 0x7FFFFFFF), ib)
    return int(np.abs(ia - ib).max()) if a.size else 0


@pytest.mark.parametrize("name,n,d,K,niter,kind", KMEANS_CASES, ids=[c[0] for c in KMEANS_CASES])
def test_kmeans_matches_oracle(vs, oracle, name, n, d, K, niter, kind):
    """Round by round, each round started from the ORACLE's centroids: the assignment (a canon
    decision on both sides) is identical bit for bit, the objective is a float64 sum of identical
    terms, and every new centroid is within one fp32 step of the oracle's (the oracle adds a
    cluster's vectors one by one in float64; the kernel adds partial sums of 4096 members, which
    differs by float64 rounding only) -- and identical where no cluster exceeds 4096 vectors.
    The whole run from the same start then agrees within 1e-5 (a centroid one step off can move a
    vector that sits on a cell boundary)."""
    import torch
    say("kmeans %s n=%d d=%d K=%d niter=%d" % (name, n, d, K, niter))
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    if kind == "gauss":
        x = rng.standard_normal((n, d), dtype=np.float32)
    elif kind == "unit":
        x, _ = S.make_data(S.config("C4", nb=n, nq=1, d=d, ncomp=30))
    else:
        x, _ = S.make_data(S.config("C2", nb=n, nq=1, d=d, ncomp=30))
    init = x[rng.permutation(n)[:K]].copy() if K <= n else rng.standard_normal((K, d), dtype=np.float32)
    if name == "odd_d30_k7":
        init[3] = 1e4                                          # a centroid no vector ever picks
    xd = dev(x)
    c_or = init.copy()
    short = True
    for r in range(niter):
        c_next, obj_o, a_o = oracle.kmeans(x, c_or, 1, return_assign=True)
        c = dev(c_or.copy())
        obj, a = vs.vs_kmeans(xd, c, 1, return_assign=True)
        np.testing.assert_array_equal(host(a), a_o)
        np.testing.assert_allclose(np.array(obj), obj_o, rtol=1e-12)
        largest = int(np.bincount(a_o, minlength=K).max())
        if largest <= 4096:
            np.testing.assert_array_equal(host(c), c_next)
        else:
            short = False
            # one fp32 step, or (a mean that nearly cancels to zero) the float64 rounding itself
            assert _ulp_apart(host(c), c_next) <= 1 or \
                np.abs(host(c).astype(np.float64) - c_next).max() <= 1e-10 * float(np.abs(x).max())
        c_or = c_next
    c = dev(init.copy())
    obj = vs.vs_kmeans(xd, c, niter)
    co, objo = oracle.kmeans(x, init, niter)
    if short:
        np.testing.assert_array_equal(host(c), co)
        np.testing.assert_allclose(np.array(obj), objo, rtol=1e-12)
    else:
        np.testing.assert_allclose(np.array(obj), objo, rtol=1e-6)
        scale = float(np.abs(x).max())
        np.testing.assert_allclose(host(c), co, rtol=1e-5, atol=1e-5 * scale)
    if name == "odd_d30_k7":
        np.testing.assert_array_equal(host(c)[3], init[3])


@pytest.mark.parametrize("name", ["c1", "pq4_l2", "ip_8bit"])
def test_ivfpq_training_matches_oracle_bit_for_bit(vs, oracle, name):
    """(6000 training vectors: no cluster reaches the 4096 vectors beyond which the kernel's
    float64 sum is grouped differently from the oracle's, so the parameters are identical.)"""
    cfg = dict(IVF_CASES[name][0])
    cfg["nb"] = min(cfg["nb"], 6_000)
    say("train %s nb=%d d=%d nlist=%d M=%d nbits=%d metric=%d" % (
        name, cfg["nb"], cfg["d"], cfg["nlist"], cfg["M"], cfg["nbits"], cfg["metric"]))
    x, q = S.make_data(cfg)
    cent0, cb0 = S.make_index_params(cfg, x)
    cent, cb = dev(cent0.copy()), dev(cb0.copy())
    objs = vs.vs_ivfpq_train(dev(x), cfg["metric"], cent, cb, cfg["nbits"], 4)
    ce, cbk, objo = oracle.train_ivfpq(x, cfg["metric"], cent0, cb0, cfg["nbits"], 4)
    np.testing.assert_array_equal(host(cent), ce)
    np.testing.assert_array_equal(host(cb), cbk)
    np.testing.assert_allclose(np.array(objs), objo, rtol=1e-12)
    # the trained parameters make a working index: storage and search agree with the oracle
    ix = vs.IVFPQ(cfg["d"], cfg["metric"], cent, cb, cfg["nbits"])
    ix.add(dev(x))
    orc = oracle.OracleIVFPQ(cfg["d"], cfg["metric"], ce, cbk, cfg["nbits"])
    orc.add(x)
    check_storage(ix, orc)
    D, I = ix.search(dev(q), 10, 4)
    Do, Io = orc.search(q, 10 + EXTRA, 4)
    xn = float(np.sqrt(orc.norms.max()))
    _, co = oracle.coarse_probe(q, ce, 4, cfg["metric"])
    tc, te = l2_table_cancel(co, cbk) if cfg["metric"] == L2 else (None, 0.0)
    check_search(host(D), host(I), Do, Io, cfg["metric"], q, xn, cancel=tc, cancel_eps=te)
    ix.close()


# ------------------------------------------------- the two largest configurations

def _large_config_sampled(vs, oracle, name, n_sample, n_queries, searches):
    """Full-size C4 / C5: data are drawn on the device; the oracle checks list assignment
    and PQ codes bit-exactly on a seeded sample of the database, then searches the GPU-built
    store (copied to the host) for a seeded sample of the queries."""
    import torch
    cfg = S.config(name)
    say("%s full size: nb=%d d=%d nlist=%d M=%d nbits=%d metric=%d" % (
        name, cfg["nb"], cfg["d"], cfg["nlist"], cfg["M"], cfg["nbits"], cfg["metric"]))
    xd, qd = S.make_data_device(cfg)
    cent, cb = S.make_index_params_device(cfg, xd)
    ix = vs.IVFPQ(cfg["d"], cfg["metric"], dev(cent), dev(cb), cfg["nbits"])
    piece = 10_000_000
    for s0 in range(0, cfg["nb"], piece):
        ix.add(xd[s0:s0 + piece])
        say("  added %d" % min(s0 + piece, cfg["nb"]))
    assert ix.ntotal == cfg["nb"]
    ids, list_of = ix.assignments()
    sizes = host(ix.list_sizes())
    assert sizes.sum() == cfg["nb"]
    rng = np.random.default_rng(7)
    sample = np.sort(rng.choice(cfg["nb"], n_sample, replace=False))
    xs = xd[torch.from_numpy(sample).cuda()].cpu().numpy()
    say("  oracle assign + encode on %d sampled vectors" % n_sample)
    lo = oracle.assign(xs, cent, cfg["metric"])
    co = oracle.pq_encode(xs, lo, cent, cb, cfg["nbits"])
    # storage position of every id (ids are sequential): invert on the device
    pos = torch.empty(cfg["nb"], dtype=torch.int64, device="cuda")
    pos[ids] = torch.arange(cfg["nb"], dtype=torch.int64, device="cuda")
    ps = pos[torch.from_numpy(sample).cuda()]
    np.testing.assert_array_equal(host(list_of[ps]), lo)
    codes_d = ix.codes()
    np.testing.assert_array_equal(host(codes_d[ps]), co)
    del pos, ps
    offsets = np.zeros(cfg["nlist"] + 1, dtype=np.int64); np.cumsum(sizes, out=offsets[1:])
    orc = oracle.OracleIVFPQ.from_storage(cfg["d"], cfg["metric"], cent, cb, cfg["nbits"], offsets,
                                          host(codes_d), host(ids))
    del codes_d
    q = host(qd)
    qs = np.sort(rng.choice(cfg["nq"], n_queries, replace=False))
    xn = float(np.sqrt(orc.norms.max()))      # largest decoded vector
    for k, nprobe in searches:
        say("  search all %d queries k=%d nprobe=%d; oracle on %d of them" % (cfg["nq"], k, nprobe, qs.size))
        probes, cdist = ix.coarse(qd, nprobe)
        po, co_ = oracle.coarse_probe(q[qs], cent, nprobe, cfg["metric"])
        np.testing.assert_array_equal(host(probes)[qs], po)
        np.testing.assert_array_equal(host(cdist)[qs], co_)
        D, I = ix.search(qd, k, nprobe)
        Do, Io = orc.search(q[qs], k + EXTRA, nprobe)
        tc, te = l2_table_cancel(co_, cb) if cfg["metric"] == L2 else (None, 0.0)
        check_search(host(D)[qs], host(I)[qs], Do, Io, cfg["metric"], q[qs], xn, cancel=tc, cancel_eps=te)
    ix.close()


def test_c4_full_size_sampled(vs, oracle):
    _large_config_sampled(vs, oracle, "C4", 20_000, 1000, [(100, 64)])


def test_c5_full_size_sampled(vs, oracle):
    _large_config_sampled(vs, oracle, "C5", 20_000, 1000, [(10, 32)])
