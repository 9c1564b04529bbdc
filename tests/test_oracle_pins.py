"""Pins for the CPU oracle: each test checks it against something other than
itself -- the paper's definitions evaluated another way (numpy float64
library routines), closed forms, invariants, exhaustive search on tiny inputs.
No GPU needed."""
import itertools

import numpy as np
import pytest

import synth_inputs as S

L2, IP = 0, 1


def np_pairwise(q, x, metric):
    q64, x64 = q.astype(np.float64), x.astype(np.float64)
    if metric == L2:
        return ((q64[:, None, :] - x64[None, :, :]) ** 2).sum(-1)
    return q64 @ x64.T


def np_topk(dist, k, metric):
    """Eq. 2 with numpy: stable argsort on the fp32-rounded distances."""
    d32 = dist.astype(np.float32)
    key = d32 if metric == L2 else -d32
    idx = np.argsort(key, axis=1, kind="stable")[:, :k]
    return np.take_along_axis(d32, idx, axis=1), idx


# --------------------------------------------------------------------- O1 flat

@pytest.mark.parametrize("metric", [L2, IP])
def test_flat_matches_numpy_library_route(oracle, metric):
    rng = np.random.default_rng(1)
    x = rng.standard_normal((700, 24), dtype=np.float32)
    q = rng.standard_normal((33, 24), dtype=np.float32)
    D, I = oracle.flat_search(x, q, 10, metric)
    Dn, In = np_topk(np_pairwise(q, x, metric), 10, metric)
    np.testing.assert_array_equal(I, In)
    np.testing.assert_allclose(D, Dn, rtol=1e-6)


def test_flat_closed_form_grid(oracle):
    # Database = points (i, 0) for i = 0..19, query at the origin: the squared
    # distance of point i is i*i (METRIC_L2 is the squared distance).
    x = np.stack([np.arange(20, dtype=np.float32), np.zeros(20, dtype=np.float32)], axis=1)
    q = np.zeros((1, 2), dtype=np.float32)
    D, I = oracle.flat_search(x, q, 5, L2)
    assert I[0].tolist() == [0, 1, 2, 3, 4]
    assert D[0].tolist() == [0.0, 1.0, 4.0, 9.0, 16.0]
    # inner product with q = (1, 0): score i, best = largest
    q = np.array([[1.0, 0.0]], dtype=np.float32)
    D, I = oracle.flat_search(x, q, 3, IP)
    assert I[0].tolist() == [19, 18, 17]
    assert D[0].tolist() == [19.0, 18.0, 17.0]


def test_flat_k1_is_eq1_argmin(oracle):
    rng = np.random.default_rng(2)
    x = rng.standard_normal((500, 16), dtype=np.float32)
    q = rng.standard_normal((40, 16), dtype=np.float32)
    _, I = oracle.flat_search(x, q, 1, L2)
    np.testing.assert_array_equal(I[:, 0], np_pairwise(q, x, L2).argmin(1))


def test_flat_ties_go_to_smaller_id_and_padding(oracle):
    x = np.array([[1, 0], [0, 1], [-1, 0], [0, -1]], dtype=np.float32)  # all at distance 1
    q = np.zeros((1, 2), dtype=np.float32)
    D, I = oracle.flat_search(x, q, 6, L2)
    assert I[0].tolist() == [0, 1, 2, 3, -1, -1]
    assert D[0, :4].tolist() == [1.0] * 4 and np.isposinf(D[0, 4:]).all()
    D, I = oracle.flat_search(x, q, 6, IP)
    assert I[0].tolist() == [0, 1, 2, 3, -1, -1] and np.isneginf(D[0, 4:]).all()


def test_cosine_l2_ip_equivalence_on_unit_vectors(oracle):
    # Table "metric equivalences": on unit vectors ||q-x||^2 = 2 - 2<q,x>, so
    # L2 and IP searches return the same neighbours.
    cfg = S.config("C4", nb=3000, nq=50, ncomp=20)
    x, q = S.make_data(cfg)
    Dl, Il = oracle.flat_search(x, q, 10, L2)
    Di, Ii = oracle.flat_search(x, q, 10, IP)
    np.testing.assert_allclose(Dl, 2.0 - 2.0 * Di, atol=2e-6)
    # ids agree wherever neighbouring scores are not within rounding of a tie
    gap_ok = np.abs(np.diff(Di.astype(np.float64), axis=1)) > 1e-6
    same = Il == Ii
    assert same[:, 1:-1][gap_ok[:, :-1] & gap_ok[:, 1:]].all()
    assert same.mean() > 0.99


def test_canon_equals_exact_on_integer_data(oracle):
    # SIFT-like data are small integers: every partial sum is an integer below
    # 2^24, so fp32 in any order, the canon chain and fp64 agree bit for bit.
    cfg = S.config("C2", nb=400, nq=20, ncomp=5)
    x, q = S.make_data(cfg)
    assert (x == np.rint(x)).all() and x.min() >= 0 and x.max() <= 255
    exact = np_pairwise(q, x, L2)
    assert exact.max() < 2 ** 24
    for a in range(5):
        for i in range(0, 400, 37):
            assert float(oracle.canon_l2(q[a], x[i])) == exact[a, i]
            assert float(oracle.canon_ip(q[a], x[i])) == float(np_pairwise(q, x, IP)[a, i])
    D, _ = oracle.flat_search(x, q, 7, L2)
    np.testing.assert_array_equal(D, np.sort(exact, axis=1)[:, :7].astype(np.float32))


def test_canon_is_the_sequential_fma_chain(oracle):
    # a = (1, 2^-12), b = 0: the chain is fma(2^-12, 2^-12, 1) = 1 + 2^-24,
    # which rounds to 1 in fp32 (ties to even) -- an fp64 accumulation
    # would keep the low term.
    a = np.array([1.0, 2.0 ** -12], dtype=np.float32)
    b = np.zeros(2, dtype=np.float32)
    assert float(oracle.canon_l2(a, b)) == 1.0
    # fused: fma(x, x, -0.0...) keeps the exact product before the single
    # rounding: (1 + 2^-12)^2 = 1 + 2^-11 + 2^-24 -> fp32 gives 1 + 2^-11
    a = np.array([1.0 + 2.0 ** -12], dtype=np.float32)
    assert float(oracle.canon_l2(a, np.zeros(1, np.float32))) == 1.0 + 2.0 ** -11
    # ... and a non-zero accumulator joins before that single rounding:
    # 2^-24 + (1 + 2^-11 + 2^-24) = 1 + 2^-11 + 2^-23 exactly, whereas rounding the
    # product first would lose both 2^-24 terms to ties-to-even.
    a = np.array([2.0 ** -12, 1.0 + 2.0 ** -12], dtype=np.float32)
    assert float(oracle.canon_l2(a, np.zeros(2, np.float32))) == 1.0 + 2.0 ** -11 + 2.0 ** -23
    assert float(oracle.canon_ip(a, a)) == 1.0 + 2.0 ** -11 + 2.0 ** -23
    # order of summation is index order: big first swallows the small ones
    a = np.array([4096.0, 1.0, 1.0], dtype=np.float32)  # 2^24 + 1 + 1
    assert float(oracle.canon_l2(a, np.zeros(3, np.float32))) == 2.0 ** 24
    a = np.array([1.0, 1.0, 4096.0], dtype=np.float32)
    assert float(oracle.canon_l2(a, np.zeros(3, np.float32))) == 2.0 ** 24 + 2.0


# ------------------------------------------------------------ O2/O6 assignment

def test_assign_is_flat_search_over_centroids(oracle):
    # Sec. 5.1: the probed lists are the nprobe nearest centroids "as in Eq. 2".
    cfg = S.config("C3", nb=3000, nq=64, ncomp=10, nlist=40)
    x, q = S.make_data(cfg)
    cent = S.make_centroids(x, 40, cfg["seed"])
    a = oracle.assign(x, cent, L2)
    _, I1 = oracle.flat_search(cent, x, 1, L2)          # integer data: exact, no rounding issue
    np.testing.assert_array_equal(a, I1[:, 0])
    probes, cd = oracle.coarse_probe(q, cent, 8, L2)
    D8, I8 = oracle.flat_search(cent, q, 8, L2)
    np.testing.assert_array_equal(probes, I8)
    np.testing.assert_array_equal(cd, D8)
    # centroids that are database rows are their own nearest centroid (distance 0)
    a_c = oracle.assign(cent, cent, L2)
    d_self = np_pairwise(cent, cent, L2)
    np.testing.assert_array_equal(a_c, d_self.argmin(1))


def test_assign_ip_metric_is_argmax(oracle):
    rng = np.random.default_rng(5)
    x = rng.integers(-8, 9, size=(300, 12)).astype(np.float32)   # integers: exact arithmetic
    cent = rng.integers(-8, 9, size=(17, 12)).astype(np.float32)
    a = oracle.assign(x, cent, IP)
    np.testing.assert_array_equal(a, np_pairwise(x, cent, IP).argmax(1))


def test_assign_tie_goes_to_smaller_list(oracle):
    cent = np.array([[1, 0], [0, 1], [1, 0]], dtype=np.float32)      # list 0 and 2 identical
    x = np.array([[1, 0], [0.5, 0.5]], dtype=np.float32)
    assert oracle.assign(x, cent, L2).tolist() == [0, 0]
    assert oracle.assign(x, cent, IP).tolist() == [0, 0]


# ------------------------------------------------------------------ O4 encode

def test_pq_with_one_subquantizer_is_a_plain_vq(oracle):
    # Quantizer hierarchy (Sec. 4.1): PQ with M = 1 is the k-means quantizer, so
    # encoding with a zero coarse centroid equals assignment to the same table.
    rng = np.random.default_rng(7)
    table = rng.standard_normal((256, 6), dtype=np.float32)
    x = rng.standard_normal((500, 6), dtype=np.float32)
    zero_c = np.zeros((1, 6), dtype=np.float32)
    codes = oracle.pq_encode(x, np.zeros(500, np.int32), zero_c, table[None], 8)
    np.testing.assert_array_equal(codes[:, 0].astype(np.int32), oracle.assign(x, table, L2))


def _exact_code_case(rng, nlist, M, K, dsub, n):
    """x = centroid + concatenated codewords, everything on a dyadic grid so
    that all sums and differences are exact in fp32."""
    d = M * dsub
    cent = rng.integers(-64, 64, size=(nlist, d)).astype(np.float32) * 8.0   # well separated
    cb = np.empty((M, K, dsub), dtype=np.float32)
    for m in range(M):   # distinct codewords per sub-quantizer, small vs. centroid spacing
        flat = rng.permutation(7 ** dsub)[:K]
        digits = np.stack([(flat // 7 ** u) % 7 for u in range(dsub)], axis=1)
        cb[m] = (digits - 3).astype(np.float32) * 0.25
    lists = rng.integers(0, nlist, size=n)
    codes = rng.integers(0, K, size=(n, M))
    x = cent[lists].copy()
    for m in range(M):
        x[:, m * dsub:(m + 1) * dsub] += cb[m][codes[:, m]]
    return cent, cb, lists.astype(np.int32), codes, x


@pytest.mark.parametrize("nbits", [8, 4])
def test_encode_closed_form_when_residual_is_a_codeword(oracle, nbits):
    rng = np.random.default_rng(11)
    K = 1 << nbits
    M, dsub = 6, 3
    cent, cb, lists, codes, x = _exact_code_case(rng, 9, M, K, dsub, 400)
    got_lists = oracle.assign(x, cent, L2)
    # centroid spacing (>= 8) dwarfs the residuals (<= 0.75 per component) unless two
    # random centroids coincide; then ties go to the smaller one
    np.testing.assert_array_equal(np.abs(cent[got_lists] - cent[lists]).max(1) == 0, True)
    got = oracle.pq_encode(x, got_lists, cent, cb, nbits)
    if nbits == 8:
        np.testing.assert_array_equal(got, codes.astype(np.uint8))
    else:  # byte i = c_{2i} | c_{2i+1} << 4
        packed = (codes[:, 0::2] | (codes[:, 1::2] << 4)).astype(np.uint8)
        np.testing.assert_array_equal(got, packed)
        assert got.shape[1] == M * 4 // 8          # code size = M * ceil(log2 K) bits
    dec = oracle.pq_decode(got, got_lists, cent, cb, nbits)
    np.testing.assert_array_equal(dec, x.astype(np.float64))   # zero reconstruction error


def test_encode_duplicate_codeword_takes_smaller_index(oracle):
    cb = np.zeros((1, 16, 2), dtype=np.float32)
    cb[0, 5] = cb[0, 9] = [1.0, 1.0]
    cb[0, 0] = [9.0, 9.0]
    cb[0, 1:5] = 7.0; cb[0, 6:9] = 7.0; cb[0, 10:] = 7.0
    x = np.array([[1.0, 1.0]], dtype=np.float32)
    codes = oracle.pq_encode(np.concatenate([x, x], 1), np.zeros(1, np.int32),
                             np.zeros((1, 4), np.float32), np.concatenate([cb, cb]), 4)
    assert codes.tolist() == [[5 | (5 << 4)]]


def test_encode_minimises_reconstruction_error_exhaustively(oracle):
    rng = np.random.default_rng(13)
    M, K, dsub, nlist = 2, 16, 2, 3
    d = M * dsub
    cent = rng.standard_normal((nlist, d), dtype=np.float32)
    cb = rng.standard_normal((M, K, dsub), dtype=np.float32)
    x = rng.standard_normal((40, d), dtype=np.float32)
    lists = oracle.assign(x, cent, L2)
    codes = oracle.pq_encode(x, lists, cent, cb, 4)
    dec = oracle.pq_decode(codes, lists, cent, cb, 4)
    err = ((dec - x) ** 2).sum(1)
    for i in range(40):
        best = np.inf
        for j0, j1 in itertools.product(range(K), repeat=2):
            cand = cent[lists[i]].astype(np.float64) + np.concatenate([cb[0, j0], cb[1, j1]])
            best = min(best, ((cand - x[i]) ** 2).sum())
        assert err[i] <= best * (1 + 1e-6) + 1e-12


def test_decode_layout_M_K_dsub(oracle):
    # codebooks[m][j] is the j-th codeword of sub-quantizer m, dsub floats.
    M, K, dsub = 3, 256, 2
    cb = np.zeros((M, K, dsub), dtype=np.float32)
    for m in range(M):
        for j in range(K):
            cb[m, j] = [100 * m + j, -(100 * m + j)]
    cent = np.array([[1, 2, 3, 4, 5, 6]], dtype=np.float32)
    codes = np.array([[7, 200, 31]], dtype=np.uint8)
    dec = oracle.pq_decode(codes, np.zeros(1, np.int32), cent, cb, 8)
    assert dec[0].tolist() == [1 + 7, 2 - 7, 3 + 300, 4 - 300, 5 + 231, 6 - 231]


# -------------------------------------------------------------- O7 ADC, O8 select

@pytest.mark.parametrize("metric", [L2, IP])
def test_coarse_probe_with_fewer_probes_than_lists_is_flat_search_over_centroids(oracle, metric):
    # Sec. 5.1: the probed lists are the nprobe nearest centroids "as in Eq. 2".  Integer data, so the
    # canon fp32 chain, the float64 sum and numpy agree bit for bit: the probes, their order and
    # their values must be those of a flat search over the centroids (argmax for IP).
    rng = np.random.default_rng(51)
    cent = rng.integers(-9, 10, size=(40, 10)).astype(np.float32)
    q = rng.integers(-9, 10, size=(60, 10)).astype(np.float32)
    for nprobe in (1, 5, 17):
        probes, cd = oracle.coarse_probe(q, cent, nprobe, metric)
        Df, If = oracle.flat_search(cent, q, nprobe, metric)
        np.testing.assert_array_equal(probes, If)
        np.testing.assert_array_equal(cd, Df)
        Dn, In = np_topk(np_pairwise(q, cent, metric), nprobe, metric)
        np.testing.assert_array_equal(probes, In)
        np.testing.assert_array_equal(cd, Dn)
    if metric == IP:   # a plausible mistake: L2 ordering under the IP metric picks other lists
        p_l2, _ = oracle.coarse_probe(q, cent, 5, L2)
        p_ip, _ = oracle.coarse_probe(q, cent, 5, IP)
        assert (p_l2 != p_ip).any()


@pytest.mark.parametrize("metric,nbits", [(IP, 8), (IP, 4), (L2, 8)])
def test_ivfpq_search_with_fewer_probes_than_lists_is_numpy_over_the_probed_members(oracle, metric, nbits):
    # nprobe < nlist: the candidates of a query are exactly the members of its probed lists
    # (probes from numpy, not from the oracle), scored on the decoded vectors, best first.
    cfg, x, q, ix = _c1_index(oracle, metric, nbits, nb=2500, nq=40)
    nprobe, k = 3, 12
    D, I = ix.search(q, k, nprobe)
    dec = oracle.pq_decode(ix.add_codes, ix.add_list_of, ix.centroids, ix.codebooks, nbits)
    cd = np_pairwise(q, ix.centroids, metric).astype(np.float32)
    order = np.argsort(cd if metric == L2 else -cd, axis=1, kind="stable")[:, :nprobe]
    full = np_pairwise(q, dec, metric)
    for a in range(q.shape[0]):
        member = np.isin(ix.add_list_of, order[a])
        cand = np.flatnonzero(member)
        d32 = full[a, cand].astype(np.float32)
        o = np.lexsort((ix.add_ids[cand], d32 if metric == L2 else -d32))[:k]
        np.testing.assert_array_equal(I[a], ix.add_ids[cand][o])
        np.testing.assert_allclose(D[a], d32[o], rtol=1e-6)
    if metric == IP:   # the per-list bias <q, c_l> matters: without the centroid the scores differ
        assert not np.allclose(D, np.take_along_axis((q.astype(np.float64) @ (dec - ix.centroids[ix.add_list_of]).T), I, 1), rtol=1e-3)


@pytest.mark.parametrize("nbits", [8, 4])
def test_inner_product_index_with_l2_assignment_is_numpy_with_l2_lists_and_ip_scores(oracle, nbits):
    # Sec. 5.1, maximum inner product search: lists chosen by L2 (at add and at search), scores by
    # inner product on the decoded vectors.  Everything from numpy: the L2-nearest centroid of every
    # vector, the nprobe L2-nearest lists of every query, inner products with the reconstructions.
    # The centroids get very different norms, so that L2 and inner-product assignment disagree.
    cfg = S.config("C1", nb=2500, nq=40)
    x, q = S.make_data(cfg)
    M = cfg["M"] if nbits == 8 else 16
    cent = S.make_centroids(x, cfg["nlist"], cfg["seed"]) * np.linspace(0.3, 3.0, cfg["nlist"], dtype=np.float32)[:, None]
    cb = S.make_codebooks(x, cent, M, nbits, cfg["seed"])
    ix = oracle.OracleIVFPQ(cfg["d"], IP, cent, cb, nbits, coarse_metric=L2)
    ix.add(x)
    by_l2 = np.argmin(np_pairwise(x, cent, L2), axis=1)
    by_ip = np.argmax(np_pairwise(x, cent, IP), axis=1)
    np.testing.assert_array_equal(ix.add_list_of, by_l2)
    assert (by_l2 != by_ip).mean() > 0.3                      # the option changes the index
    nprobe, k = 3, 12
    D, I = ix.search(q, k, nprobe)
    dec = oracle.pq_decode(ix.add_codes, ix.add_list_of, ix.centroids, ix.codebooks, nbits)
    order = np.argsort(np_pairwise(q, cent, L2).astype(np.float32), axis=1, kind="stable")[:, :nprobe]
    full = np_pairwise(q, dec, IP)
    for a in range(q.shape[0]):
        cand = np.flatnonzero(np.isin(ix.add_list_of, order[a]))
        s32 = full[a, cand].astype(np.float32)
        o = np.lexsort((ix.add_ids[cand], -s32))[:k]
        np.testing.assert_array_equal(I[a], ix.add_ids[cand][o])
        np.testing.assert_allclose(D[a], s32[o], rtol=1e-6)
    # the table form (form 1: bias <q, c_l> + sum of per-query table entries) agrees with it
    D1, I1 = ix.search(q, k, nprobe, form=1)
    np.testing.assert_allclose(D1, D, rtol=1e-4, atol=1e-4)
    # and the default (coarse metric = index metric) is a different index
    ix2 = oracle.OracleIVFPQ(cfg["d"], IP, cent, cb, nbits)
    ix2.add(x)
    np.testing.assert_array_equal(ix2.add_list_of, by_ip)


@pytest.mark.parametrize("metric", [IP, L2])
def test_ivfsq8_search_with_fewer_probes_than_lists_is_numpy_over_the_probed_members(oracle, metric):
    rng = np.random.default_rng(53)
    x = rng.standard_normal((2000, 12)).astype(np.float32)
    q = rng.standard_normal((30, 12)).astype(np.float32)
    cent = x[rng.permutation(2000)[:14]].copy()
    vmin, step = oracle.sq8_params(x)
    ix = oracle.OracleIVFSQ8(12, metric, cent, vmin, step)
    ix.add(x)
    nprobe, k = 4, 9
    D, I = ix.search(q, k, nprobe)
    dec = oracle.sq8_decode(ix.add_codes, vmin, step)
    cd = np_pairwise(q, cent, metric).astype(np.float32)
    order = np.argsort(cd if metric == L2 else -cd, axis=1, kind="stable")[:, :nprobe]
    full = np_pairwise(q, dec, metric)
    for a in range(q.shape[0]):
        cand = np.flatnonzero(np.isin(ix.add_list_of, order[a]))
        d32 = full[a, cand].astype(np.float32)
        o = np.lexsort((ix.add_ids[cand], d32 if metric == L2 else -d32))[:k]
        np.testing.assert_array_equal(I[a], ix.add_ids[cand][o])
        np.testing.assert_allclose(D[a], d32[o], rtol=1e-6)


def _c1_index(oracle, metric=L2, nbits=8, **kw):
    cfg = S.config("C1", **kw)
    x, q = S.make_data(cfg)
    M = cfg["M"] if nbits == 8 else 16
    cent = S.make_centroids(x, cfg["nlist"], cfg["seed"])
    cb = S.make_codebooks(x, cent, M, nbits, cfg["seed"])
    ix = oracle.OracleIVFPQ(cfg["d"], metric, cent, cb, nbits)
    ix.add(x)
    return cfg, x, q, ix


@pytest.mark.parametrize("metric,nbits", [(L2, 8), (IP, 8), (L2, 4), (IP, 4)])
def test_adc_equals_distance_to_decoded_vector(oracle, metric, nbits):
    # Eq. 10: the ADC distance is the distance from q to D(C(x)); Eq. 14: the sum
    # of table look-ups equals it.  Probe all lists => the result must equal a
    # flat search over the decoded database, and the LUT form must agree.
    cfg, x, q, ix = _c1_index(oracle, metric, nbits, nb=2000, nq=30)
    D0, I0 = ix.search(q, 10, ix.nlist, form=0)
    D1, I1 = ix.search(q, 10, ix.nlist, form=1)
    dec = oracle.pq_decode(ix.add_codes, ix.add_list_of, ix.centroids, ix.codebooks, nbits)
    Dn, In = np_topk(np_pairwise(q, dec, metric), 10, metric)
    np.testing.assert_array_equal(I0, In)
    np.testing.assert_allclose(D0, Dn, rtol=1e-6)
    scale = (q.astype(np.float64) ** 2).sum(1, keepdims=True) + 1.0
    assert (np.abs(D1.astype(np.float64) - D0) <= 1e-5 * np.maximum(np.abs(D0), scale)).all()
    assert (I1 == I0).mean() > 0.98


@pytest.mark.parametrize("nbits", [8, 4])
def test_split_tables_form_equals_the_definition(oracle, nbits):
    # Sec. 4.3: the (query, list) table is the sum of a per-query and a per-list term plus the
    # coarse distance.  Against form 0 (distance to the decoded vector in float64) within the
    # rounding of the cancelling terms |q|^2 + |c|^2 + |t|^2, and exactly on integer data.
    cfg, x, q, ix = _c1_index(oracle, L2, nbits, nb=2000, nq=30)
    D0, I0 = ix.search(q, 10, 5, form=0)
    D3, I3 = ix.search(q, 10, 5, form=3)
    scale = (q.astype(np.float64) ** 2).sum(1, keepdims=True) + float((ix.centroids.astype(np.float64) ** 2).sum(1).max()) + 10.0
    assert (np.abs(D3.astype(np.float64) - D0) <= 1e-6 * scale).all()
    assert (I3 == I0).mean() > 0.98
    rng = np.random.default_rng(31)
    xi = rng.integers(-12, 13, size=(1500, 8)).astype(np.float32)
    qi = rng.integers(-12, 13, size=(20, 8)).astype(np.float32)
    cent = xi[:6].copy()
    cb = rng.integers(-6, 7, size=(4, 1 << nbits, 2)).astype(np.float32)
    io = oracle.OracleIVFPQ(8, L2, cent, cb, nbits)
    io.add(xi)
    Da, Ia = io.search(qi, 7, 3, form=0)
    Db, Ib = io.search(qi, 7, 3, form=3)
    np.testing.assert_array_equal(Da, Db)          # integers: every term is exact in fp32
    np.testing.assert_array_equal(Ia, Ib)


def test_exact_codes_and_all_probes_reproduce_flat_search(oracle):
    rng = np.random.default_rng(17)
    cent, cb, lists, codes, x = _exact_code_case(rng, 9, 6, 256, 3, 1500)
    q = (x[rng.integers(0, 1500, 25)] + rng.integers(-2, 3, size=(25, 18)) * 0.125).astype(np.float32)
    ix = oracle.OracleIVFPQ(18, L2, cent, cb, 8)
    ix.add(x)
    D, I = ix.search(q, 10, 9)
    Df, If = oracle.flat_search(x, q, 10, L2)
    np.testing.assert_array_equal(D, Df)         # dyadic data: exact in fp64 either way
    # duplicates in x (same list, same codes) are equal-distance ties: compare up to ties
    for a in range(25):
        assert sorted(zip(D[a].tolist(), I[a].tolist())) == sorted(zip(Df[a].tolist(), If[a].tolist()))
    assert oracle.recall(I, If) == 1.0 and oracle.recall(I, If, 1) == 1.0


def test_probe_count_monotonicity_and_scanned_count(oracle):
    cfg, x, q, ix = _c1_index(oracle)
    sizes = ix.list_sizes()
    assert sizes.sum() == cfg["nb"]
    prev = None
    for nprobe in (1, 2, 4, 8, 16, 99):
        D, I, nscanned, probes = ix.search(q, 10, nprobe, return_stats=True)
        assert probes.shape[1] == min(nprobe, 16)                 # clamped to nlist
        np.testing.assert_array_equal(nscanned, sizes[probes].sum(1))   # Eq. N_distances, scan term
        pr, _ = oracle.coarse_probe(q, ix.centroids, nprobe)
        np.testing.assert_array_equal(probes, pr)
        if prev is not None:   # a superset of candidates can only improve every rank
            assert (D <= prev).all()
        prev = D
        assert (np.diff(D, axis=1) >= 0).all()
    # balanced-list estimate of the scan term: nprobe * N / nlist times the imbalance factor
    imbalance = (sizes.astype(np.float64) ** 2).sum() * 16 / sizes.sum() ** 2
    assert 1.0 <= imbalance < 3.0


def test_select_equals_full_sort_of_candidates(oracle):
    cfg, x, q, ix = _c1_index(oracle, nb=3000, nq=20)
    D, I, _, probes = ix.search(q, 25, 3, return_stats=True)
    dec = oracle.pq_decode(ix.add_codes, ix.add_list_of, ix.centroids, ix.codebooks, 8)
    for a in range(20):
        cand = np.flatnonzero(np.isin(ix.add_list_of, probes[a]))
        dist = np_pairwise(q[a:a + 1], dec[cand], L2)[0].astype(np.float32)
        order = np.lexsort((cand, dist))[:25]
        np.testing.assert_array_equal(I[a], cand[order])
        np.testing.assert_allclose(D[a], dist[order], rtol=1e-6)


def test_fewer_candidates_than_k_pads_with_minus_one(oracle):
    cfg, x, q, ix = _c1_index(oracle, nb=40, nq=5)
    D, I, nscanned, _ = ix.search(q, 30, 2, return_stats=True)
    for a in range(5):
        n = int(nscanned[a])
        assert n < 30
        assert (I[a, :n] >= 0).all() and (I[a, n:] == -1).all() and np.isposinf(D[a, n:]).all()


def test_add_in_pieces_and_custom_ids(oracle):
    cfg, x, q, ix = _c1_index(oracle, nb=1200, nq=10)
    ix2 = oracle.OracleIVFPQ(cfg["d"], L2, ix.centroids, ix.codebooks, 8)
    ids = np.arange(1200, dtype=np.int64) * 3 + 5
    ix2.add(x[:500], ids[:500])
    ix2.add(x[500:], ids[500:])
    D, I = ix.search(q, 10, 4)
    D2, I2 = ix2.search(q, 10, 4)
    np.testing.assert_array_equal(D, D2)
    np.testing.assert_array_equal(I * 3 + 5, I2)
    ix3 = oracle.OracleIVFPQ(cfg["d"], L2, ix.centroids, ix.codebooks, 8)
    ix3.add(x[:500]); ix3.add(x[500:])        # sequential ids continue from ntotal
    np.testing.assert_array_equal(ix3.search(q, 10, 4)[1], I)


def test_recall_definitions(oracle):
    It = np.array([[1, 2, 3, 4]])
    assert oracle.recall(np.array([[4, 3, 2, 1]]), It) == 1.0
    assert oracle.recall(np.array([[9, 1, 8, 7]]), It) == 0.25
    assert oracle.recall(np.array([[9, 1, 8, 7]]), It, 1) == 1.0      # 1-recall@4
    assert oracle.recall(np.array([[2, 9, 8, -1]]), It, 1) == 0.0


# ------------------------------------------------------------- refinement

@pytest.mark.parametrize("metric", [L2, IP])
def test_refine_matches_numpy_on_the_shortlist(oracle, metric):
    # Sec. 3.5: the second stage computes accurate distances only for the shortlist.
    rng = np.random.default_rng(21)
    x = rng.standard_normal((300, 12), dtype=np.float32)
    q = rng.standard_normal((9, 12), dtype=np.float32)
    cand = np.stack([rng.choice(300, 40, replace=False) for _ in range(9)]).astype(np.int64)
    D, I = oracle.refine(x, q, cand, 7, metric)
    full = np_pairwise(q, x, metric).astype(np.float32)
    for a in range(9):
        c = np.sort(cand[a])                             # ascending ids: stable sort = ties to the smaller id
        v = full[a, c]
        order = np.argsort(v if metric == L2 else -v, kind="stable")[:7]
        np.testing.assert_array_equal(I[a], c[order])
        np.testing.assert_allclose(D[a], v[order], rtol=1e-6)


def test_refine_with_every_row_listed_is_flat_search(oracle):
    rng = np.random.default_rng(22)
    x = rng.standard_normal((120, 8), dtype=np.float32)
    q = rng.standard_normal((6, 8), dtype=np.float32)
    cand = np.stack([rng.permutation(120) for _ in range(6)]).astype(np.int64)
    D, I = oracle.refine(x, q, cand, 15, L2)
    Df, If = oracle.flat_search(x, q, 15, L2)
    np.testing.assert_array_equal(I, If)
    np.testing.assert_array_equal(D, Df)


def test_refine_skips_empty_slots_pads_and_breaks_ties_by_id(oracle):
    x = np.array([[0, 0], [3, 0], [0, 3], [1, 0], [5, 5]], dtype=np.float32)
    q = np.zeros((1, 2), dtype=np.float32)
    cand = np.array([[2, -1, 1, 7, 3, -1]], dtype=np.int64)      # 7 is not a row of x
    D, I = oracle.refine(x, q, cand, 5, L2)
    assert I[0].tolist() == [3, 1, 2, -1, -1]                    # rows 1 and 2 tie at 9: smaller id first
    assert D[0, :3].tolist() == [1.0, 9.0, 9.0] and np.isposinf(D[0, 3:]).all()
    D, I = oracle.refine(x, q + 1, cand, 2, IP)                  # q = (1, 1): scores 3, 3, 1
    assert I[0].tolist() == [1, 2] and D[0].tolist() == [3.0, 3.0]


def test_refining_an_ivfpq_shortlist_never_loses_recall(oracle):
    # A true k-nearest neighbour that is in the shortlist is among the k exact best of the
    # shortlist, so k-recall@k after refinement >= k-recall@k of the first stage's own top k.
    cfg, x, q, ix = _c1_index(oracle, nb=3000, nq=40)
    _, It = oracle.flat_search(x, q, 10, L2)
    D1, I1 = ix.search(q, 60, 4)
    Dr, Ir = oracle.refine(x, q, I1, 10, L2)
    assert oracle.recall(Ir, It) >= oracle.recall(I1[:, :10], It)
    assert oracle.recall(Ir, It) > oracle.recall(I1[:, :10], It) + 0.05     # and here it gains
    # refined distances are exact distances: they equal flat search's wherever the id matches
    Df, If = oracle.flat_search(x, q, 3000, L2)
    for a in range(40):
        pos = {int(i): j for j, i in enumerate(If[a])}
        for j in range(10):
            assert Dr[a, j] == Df[a, pos[int(Ir[a, j])]]


# ------------------------------------------------------------------ k-means

def _np_lloyd_round(x, c):
    """One round written with numpy in float64 (only used on integer data, where the
    nearest centroid is the same in every arithmetic)."""
    d2 = ((x[:, None, :].astype(np.float64) - c[None, :, :].astype(np.float64)) ** 2).sum(-1)
    a = d2.argmin(axis=1)                                   # first minimum = smaller centroid number
    new = c.copy()
    for j in range(c.shape[0]):
        if (a == j).any():
            new[j] = x[a == j].astype(np.float64).mean(axis=0).astype(np.float32)
    return new, d2.min(axis=1).mean()


def test_kmeans_round_is_assign_then_mean(oracle):
    # Sec. 4.1: k-means applies Lloyd's two conditions in turn.
    rng = np.random.default_rng(31)
    x = rng.integers(-20, 21, size=(400, 6)).astype(np.float32)
    c0 = x[rng.permutation(400)[:7]].copy()
    c, obj = oracle.kmeans(x, c0, 3)
    ref = c0
    for r in range(3):
        ref, o = _np_lloyd_round(x, ref)
        # round 0 works on integers (exact); later centroids are fractions, so the fp32 chain
        # of the reported objective is within fp32 rounding of the float64 value
        assert abs(obj[r] - o) <= (1e-12 if r == 0 else 1e-6) * max(1.0, o)
    np.testing.assert_allclose(c, ref, rtol=1e-6, atol=0)
    # the nearest-centroid rule is or_assign's
    a = oracle.assign(x, c0)
    first = np.stack([x[a == j].astype(np.float64).mean(0) if (a == j).any() else c0[j] for j in range(7)])
    np.testing.assert_allclose(oracle.kmeans(x, c0, 1)[0], first.astype(np.float32), rtol=1e-6)


def test_code_sizes_the_paper_states(oracle):
    """tests/golden/code_sizes.txt holds the code sizes the paper gives as numbers.  The oracle's
    encoders must produce codes of those sizes (for the parameters they support, 4 and 8 bits: the
    paper's rule M * ceil(log2 K) bits, checked on its own PQ6x10 example first), and a code must use
    all of its bytes: vectors built from the last codeword of every sub-quantizer fill every byte."""
    import math, os
    recs = []
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "code_sizes.txt")):
        if line.strip() and not line.startswith("#"):
            f = line.split()
            recs.append((f[0], dict(kv.split("=") for kv in f[1:] if "=" in kv and not kv.startswith("(")), line))
    kinds = {r[0] for r in recs}
    assert kinds == {"pq", "sq8", "kmeans", "ids"}
    rule = lambda M, K: M * math.ceil(math.log2(K))                  # Sec. 4.1, in bits
    for kind, kv, line in recs:
        if kind == "pq":
            assert rule(int(kv["M"]), 1 << int(kv["nbits"])) == int(kv["bits"]), line
        elif kind == "kmeans":
            assert rule(1, int(kv["K"])) == 8 * int(kv["bytes"]), line
        elif kind == "ids":
            assert math.ceil(math.log2(int(kv["N"]))) == int(kv["bits"]), line
        elif kind == "sq8":
            d = int(kv["d"])
            x = np.linspace(-1, 1, 2 * d, dtype=np.float32).reshape(2, d)
            vmin, step = oracle.sq8_params(x)
            codes = oracle.sq8_encode(x, vmin, step)
            assert codes.dtype == np.uint8 and codes.shape == (2, int(kv["bytes"])), line
    # the same rule for the product quantizers the oracle supports, on its encoder's output
    rng = np.random.default_rng(5)
    for M, nbits, dsub in ((6, 8, 2), (16, 8, 1), (8, 4, 3), (64, 4, 1)):
        K, d = 1 << nbits, M * dsub
        cb = rng.standard_normal((M, K, dsub)).astype(np.float32)
        cent = np.zeros((1, d), np.float32)
        x = np.stack([cb[:, 0, :].reshape(d), cb[:, K - 1, :].reshape(d)])   # first / last codeword everywhere
        codes = oracle.pq_encode(x, np.zeros(2, np.int32), cent, cb, nbits)
        assert codes.shape[1] * 8 == rule(M, K)
        assert (codes[0] == 0).all() and (codes[1] == 0xFF).all()            # every bit of every byte is used


def test_kmeans_mean_of_a_long_cluster_is_the_correctly_rounded_mean(oracle):
    """The update adds a centroid's vectors one after the other in float64.  A float64 sum of
    10,000 fp32 values of comparable size is within 1e-12 relative of the exact sum, so the fp32
    mean equals the correctly rounded mean of exact rational arithmetic in all but a vanishing
    share of components -- checked here against Python's exact fractions, and against numpy's
    pairwise float64 sum to the last fp32 bit but one."""
    from fractions import Fraction
    rng = np.random.default_rng(77)
    x = rng.standard_normal((10_000, 3)).astype(np.float32) + np.float32(5.0)   # one cluster, far from 0
    c0 = np.array([[5.0, 5.0, 5.0], [-50.0, -50.0, -50.0]], np.float32)          # the second gets nothing
    c, _ = oracle.kmeans(x, c0, 1)
    np.testing.assert_array_equal(c[1], c0[1])
    for t in range(3):
        exact = sum((Fraction(float(v)) for v in x[:, t]), Fraction(0)) / x.shape[0]
        assert c[0, t] == np.float32(float(exact)), (t, c[0, t], float(exact))
    ref = (x.astype(np.float64).sum(0) / x.shape[0]).astype(np.float32)
    assert np.all(np.abs(c[0].view(np.int32) - ref.view(np.int32)) <= 1)


def test_kmeans_sum_runs_in_training_set_order(oracle):
    """The float64 sum of a cluster is a running sum over the training set in its given order (no
    blocks, no pairwise tree, not reversed): values whose float64 sum depends on the order tell
    the orders apart.  From the left, 2^60 + 1 absorbs the 1, - 2^60 gives 0, + 1 gives 1: mean
    1/4.  A pairwise tree gives (2^60 + 1) + (-2^60 + 1) = 0, and so does the reversed order."""
    big = np.float32(2.0 ** 60)
    x = np.array([[big], [1.0], [-big], [1.0]], np.float32)
    c, _ = oracle.kmeans(x, np.array([[0.0]], np.float32), 1)
    assert c[0, 0] == np.float32(0.25)
    x2 = np.array([[1.0], [1.0], [big], [-big]], np.float32)     # both ones absorbed: 2^60 - 2^60
    c2, _ = oracle.kmeans(x2, np.array([[0.0]], np.float32), 1)
    assert c2[0, 0] == np.float32(0.0)


def test_kmeans_reported_assignment_is_the_last_rounds(oracle):
    rng = np.random.default_rng(78)
    x = rng.integers(-20, 21, size=(3000, 6)).astype(np.float32)
    c0 = x[rng.permutation(3000)[:11]].copy()
    c2, _ = oracle.kmeans(x, c0, 2)
    c3, _, a3 = oracle.kmeans(x, c0, 3, return_assign=True)
    np.testing.assert_array_equal(a3, oracle.assign(x, c2, L2))               # step (1) of round 3 starts from c2
    np.testing.assert_array_equal(a3, np_pairwise(x, c2, L2).argmin(1))       # integer data: exact either way
    for j in range(11):
        if (a3 == j).any():
            np.testing.assert_array_equal(c3[j], x[a3 == j].astype(np.float64).mean(0).astype(np.float32))


def test_kmeans_objective_never_increases(oracle):
    # Both of Lloyd's steps can only lower the mean squared error.
    rng = np.random.default_rng(32)
    x = rng.standard_normal((3000, 10), dtype=np.float32)
    c0 = x[:25].copy()
    c, obj = oracle.kmeans(x, c0, 12)
    assert (np.diff(obj) <= 1e-7 * obj[:-1]).all(), obj
    assert obj[-1] < 0.9 * obj[0]
    # the objective reported for a round is the MSE of assigning to that round's input centroids
    a = oracle.assign(x, c0)
    mse0 = ((x.astype(np.float64) - c0[a].astype(np.float64)) ** 2).sum(1).mean()
    assert abs(obj[0] - mse0) <= 1e-6 * mse0


def test_kmeans_finds_separated_blobs_and_stays_there(oracle):
    rng = np.random.default_rng(33)
    centres = np.array([[0, 0], [100, 0], [0, 100], [100, 100]], dtype=np.float32)
    lab = rng.integers(0, 4, size=800)
    x = (centres[lab] + rng.standard_normal((800, 2))).astype(np.float32)
    init = np.stack([x[np.flatnonzero(lab == j)[0]] for j in range(4)])       # one point of each blob
    c, obj = oracle.kmeans(x, init, 4)
    means = np.stack([x[lab == j].astype(np.float64).mean(0) for j in range(4)]).astype(np.float32)
    np.testing.assert_allclose(c, means, rtol=1e-6)
    c2, obj2 = oracle.kmeans(x, c, 3)                                          # a fixed point
    np.testing.assert_array_equal(c2, c)
    assert (obj2 == obj2[0]).all()


def test_kmeans_degenerate_cases(oracle):
    rng = np.random.default_rng(34)
    x = rng.standard_normal((50, 4), dtype=np.float32)
    c, obj = oracle.kmeans(x, x, 2)                     # one centroid per point: zero error, nothing moves
    np.testing.assert_array_equal(c, x)
    assert (obj == 0).all()
    far = np.concatenate([x[:3], np.full((1, 4), 1e6, dtype=np.float32)])
    c, _ = oracle.kmeans(x, far, 3)                      # the far centroid never gets a vector: it stays
    np.testing.assert_array_equal(c[3], far[3])
    assert not np.array_equal(c[:3], far[:3])
    dup = np.stack([x[0], x[0], x[1]])                   # identical centroids: the smaller number takes all
    c, _ = oracle.kmeans(x, dup, 1)
    np.testing.assert_array_equal(c[1], x[0])
    c, obj = oracle.kmeans(x, x[:5], 0)                  # no round: the initial centroids come back
    np.testing.assert_array_equal(c, x[:5])


def test_trained_parameters_lower_the_quantization_error(oracle):
    # Training = k-means for the coarse quantizer and for every sub-quantizer on residual
    # sub-vectors: each of them lowers its own MSE, and the PQ reconstruction error drops.
    cfg = S.config("C1", nb=4000, nq=20)
    x, q = S.make_data(cfg)
    cent0, cb0 = S.make_index_params(cfg, x)
    cent, cb, objs = oracle.train_ivfpq(x, L2, cent0, cb0, 8, 6)
    assert (np.diff(objs, axis=1) <= 1e-7 * objs[:, :-1]).all()
    def recon_mse(ce, cbk):
        a = oracle.assign(x, ce)
        codes = oracle.pq_encode(x, a, ce, cbk, 8)
        xr = oracle.pq_decode(codes, a, ce, cbk, 8)
        return ((x.astype(np.float64) - xr) ** 2).sum(1).mean()
    assert recon_mse(cent, cb) < 0.8 * recon_mse(cent0, cb0)
    # the residual k-means saw exactly x - c[assign]: its first objective is the MSE of coding
    # the residual slices with the initial codebook
    a = oracle.assign(x, cent)
    res = x - cent[a]
    for m in (0, 5):
        sl = res[:, m * 4:(m + 1) * 4]
        d2 = ((sl[:, None, :].astype(np.float64) - cb0[m][None].astype(np.float64)) ** 2).sum(-1).min(1)
        assert abs(objs[1 + m, 0] - d2.mean()) <= 1e-5 * d2.mean()


# ------------------------------------------------------------------ IVF-Flat

def _ivfflat(oracle, nb=2000, nq=30, metric=L2, nlist=16):
    cfg = S.config("C1", nb=nb, nq=nq, nlist=nlist, metric=metric)
    x, q = S.make_data(cfg)
    cent = S.make_centroids(x, nlist, cfg["seed"])
    ix = oracle.OracleIVFFlat(cfg["d"], metric, cent)
    ix.add(x)
    return x, q, cent, ix


@pytest.mark.parametrize("metric", [L2, IP])
def test_ivfflat_with_all_lists_probed_is_flat_search(oracle, metric):
    # Sec. 5.1: the inverted file only restricts which vectors are compared with the query.
    x, q, cent, ix = _ivfflat(oracle, metric=metric)
    D, I = ix.search(q, 12, 16)
    Df, If = oracle.flat_search(x, q, 12, metric)
    np.testing.assert_array_equal(I, If)
    np.testing.assert_array_equal(D, Df)


def test_ivfflat_visits_exactly_the_probed_lists(oracle):
    x, q, cent, ix = _ivfflat(oracle)
    a = oracle.assign(x, cent)
    prev = 0.0
    _, It = oracle.flat_search(x, q, 10, L2)
    for nprobe in (1, 3, 8, 16):
        D, I, nscanned, probes = ix.search(q, 10, nprobe, return_stats=True)
        po, _ = oracle.coarse_probe(q, cent, nprobe, L2)
        np.testing.assert_array_equal(probes, po)
        full = np_pairwise(q, x, L2).astype(np.float32)
        for qi in range(q.shape[0]):
            members = np.flatnonzero(np.isin(a, probes[qi]))          # ascending ids
            assert nscanned[qi] == members.size
            v = full[qi, members]
            order = np.argsort(v, kind="stable")[:10]
            np.testing.assert_array_equal(I[qi, :order.size], members[order])
            np.testing.assert_allclose(D[qi, :order.size], v[order], rtol=1e-6)
        r = oracle.recall(I, It)
        assert r >= prev                                               # more lists never lose a neighbour
        prev = r
    assert prev == 1.0


def test_ivfflat_add_in_pieces_custom_ids_and_padding(oracle):
    x, q, cent, ix = _ivfflat(oracle, nb=300)
    ix2 = oracle.OracleIVFFlat(32, L2, cent)
    ids = np.arange(300, dtype=np.int64) * 7 + 3
    ix2.add(x[:100], ids[:100]); ix2.add(x[100:], ids[100:])
    D, I = ix.search(q, 5, 4)
    D2, I2 = ix2.search(q, 5, 4)
    np.testing.assert_array_equal(D, D2)
    np.testing.assert_array_equal(I * 7 + 3, I2)
    np.testing.assert_array_equal(ix.list_sizes(), ix2.list_sizes())
    D, I, nscanned, _ = ix.search(q, 200, 1, return_stats=True)       # k larger than one list
    for qi in range(q.shape[0]):
        n = int(nscanned[qi])
        assert (I[qi, :n] >= 0).all() and (I[qi, n:] == -1).all() and np.isposinf(D[qi, n:]).all()


# ------------------------------------------- L2 through stored norms (Sec. 4.3)

def test_stored_norm_is_the_squared_norm_of_the_decoded_vector(oracle):
    cfg, x, q, ix = _c1_index(oracle, nb=500, nq=4)
    xr = oracle.pq_decode(ix.codes, np.repeat(np.arange(ix.nlist, dtype=np.int32), ix.list_sizes()),
                          ix.centroids, ix.codebooks, 8)
    np.testing.assert_allclose(ix.norms, (xr ** 2).sum(1), rtol=2e-6)
    # on integer-valued parameters every step is exact: the fp32 chain equals the float64 value
    rng = np.random.default_rng(41)
    cent = rng.integers(-9, 10, size=(4, 8)).astype(np.float32)
    cb = rng.integers(-5, 6, size=(2, 16, 4)).astype(np.float32)
    codes = rng.integers(0, 256, size=(50, 1)).astype(np.uint8)          # two 4-bit codes per byte
    lo = rng.integers(0, 4, size=50).astype(np.int32)
    nrm = oracle.pq_norms(codes, lo, cent, cb, 4)
    dec = oracle.pq_decode(codes, lo, cent, cb, 4)
    np.testing.assert_array_equal(nrm.astype(np.float64), (dec ** 2).sum(1))


def test_norm_decomposition_form_agrees_with_the_definition(oracle):
    # ||q - x'||^2 = ||q||^2 + ||x'||^2 - 2 <q, x'>: form 2 against form 0, within the
    # rounding of the cancelling terms; identical ranking apart from near-ties
    cfg, x, q, ix = _c1_index(oracle, nb=3000, nq=30)
    D0, I0 = ix.search(q, 10, 4, form=0)
    D2, I2 = ix.search(q, 10, 4, form=2)
    scale = (q.astype(np.float64) ** 2).sum(1)[:, None] + float(ix.norms.max())
    assert (np.abs(D2.astype(np.float64) - D0) <= 4e-7 * scale).all()
    assert (I0 == I2).mean() > 0.98
    # exact on integer data: same bits as the definition
    rng = np.random.default_rng(42)
    xi = rng.integers(0, 30, size=(400, 8)).astype(np.float32)
    qi = rng.integers(0, 30, size=(7, 8)).astype(np.float32)
    cent = xi[:5].copy()
    cb = rng.integers(-4, 5, size=(4, 256, 2)).astype(np.float32)
    ixi = oracle.OracleIVFPQ(8, L2, cent, cb, 8)
    ixi.add(xi)
    Da, Ia = ixi.search(qi, 6, 5, form=0)
    Db, Ib = ixi.search(qi, 6, 5, form=2)
    np.testing.assert_array_equal(Da, Db)
    np.testing.assert_array_equal(Ia, Ib)


# ------------------------------------------------------------ scalar quantizer, IVF-SQ8

def test_sq8_cells_codes_and_reconstruction(oracle):
    # Sec. 4.1: a uniform quantizer per component; scale and offset decide what is reconstructed.
    vmin = np.array([0.0, -1.0], dtype=np.float32)
    step = np.array([1.0, 0.5], dtype=np.float32)              # cells [j, j + 1) and [-1 + j / 2, ...)
    x = np.array([[0.0, -1.0], [0.999, -0.75], [1.0, -0.5], [255.5, 126.9], [256.0, 127.0],
                  [-3.0, -9.0], [1e9, 1e9]], dtype=np.float32)
    codes = oracle.sq8_encode(x, vmin, step)
    assert codes.tolist() == [[0, 0], [0, 0], [1, 1], [255, 255], [255, 255], [0, 0], [255, 255]]
    dec = oracle.sq8_decode(codes, vmin, step)
    assert dec.tolist() == [[0.5, -0.75], [0.5, -0.75], [1.5, -0.25], [255.5, 126.75], [255.5, 126.75],
                            [0.5, -0.75], [255.5, 126.75]]
    # inside the range the reconstruction is the nearest cell middle: error at most step / 2,
    # and re-encoding a reconstruction gives the same code (a fixed point)
    rng = np.random.default_rng(51)
    xr = rng.uniform(-4, 9, size=(2000, 6)).astype(np.float32)
    lo, st = oracle.sq8_params(xr)
    c = oracle.sq8_encode(xr, lo, st)
    r = oracle.sq8_decode(c, lo, st)
    assert (np.abs(r.astype(np.float64) - xr) <= st.astype(np.float64) * 0.5 * (1 + 1e-5) + 1e-6).all()
    np.testing.assert_array_equal(oracle.sq8_encode(r, lo, st), c)
    assert c.min() == 0 and c.max() == 255                       # the range is used from end to end


def test_ivfsq8_is_ivfflat_over_the_reconstructions(oracle):
    # The index only replaces every stored vector by its reconstruction.
    cfg = S.config("C1", nb=2500, nq=25)
    x, q = S.make_data(cfg)
    cent = S.make_centroids(x, 16, cfg["seed"])
    lo, st = oracle.sq8_params(x)
    ix = oracle.OracleIVFSQ8(32, L2, cent, lo, st)
    ix.add(x[:1000]); ix.add(x[1000:])
    xr = oracle.sq8_decode(oracle.sq8_encode(x, lo, st), lo, st)
    a = oracle.assign(x, cent)                                   # lists come from the ORIGINAL vectors
    for nprobe in (3, 16):
        D, I, nscanned = ix.search(q, 10, nprobe, return_stats=True)
        po, _ = oracle.coarse_probe(q, cent, nprobe, L2)
        full = np_pairwise(q, xr, L2).astype(np.float32)
        for qi in range(q.shape[0]):
            members = np.flatnonzero(np.isin(a, po[qi]))
            assert nscanned[qi] == members.size
            v = full[qi, members]
            order = np.argsort(v, kind="stable")[:10]
            np.testing.assert_array_equal(I[qi], members[order])
            np.testing.assert_allclose(D[qi], v[order], rtol=1e-6)
    # with 256 cells per component the quantization error is small: most exact neighbours survive
    _, It = oracle.flat_search(x, q, 10, L2)
    assert oracle.recall(ix.search(q, 10, 16)[1], It) > 0.9
