"""Comparison rules between the HIP path and the CPU oracle.

  - list assignments and PQ codes: bit-exact, compared as the map
    id -> (list, code bytes) because the order inside a list is storage detail;
  - distances: |gpu - oracle| <= 1e-4 * max(|oracle|, s) where s is the
    magnitude of the terms that cancel (inner product: ||q|| * max ||x||;
    L2: none, the squared distance is a sum of non-negative terms -- except for the
    search type that evaluates |q|^2 + |x'|^2 - 2 <q, x'> (Sec. 4.3), whose terms do
    cancel: there `cancel` = |q|^2 + max |x'|^2 per query enters with the fp32 rounding
    that decomposition can cost, 2^-21 of it, instead of a relative share);
  - ids: identical, except that a GPU id may differ from the oracle's id at
    the same rank when the ORACLE distances of the two candidates are within
    that tolerance of each other.  To see candidates just past rank k the
    oracle is run with a few extra ranks.
"""
import numpy as np

REL_TOL = 1e-4
EXTRA = 16


def tolerance(D_or, metric, q=None, xnorm_max=None, cancel=None):
    tol = REL_TOL * np.abs(D_or.astype(np.float64))
    if metric == 1:
        qn = np.sqrt((q.astype(np.float64) ** 2).sum(1, keepdims=True))
        tol = np.maximum(tol, REL_TOL * qn * float(xnorm_max))
    if cancel is not None:
        tol = tol + 2.0 ** -21 * np.asarray(cancel, dtype=np.float64).reshape(-1, 1)
    return tol


def check_search(D_gpu, I_gpu, D_or, I_or, metric, q=None, xnorm_max=None, cancel=None):
    """D_or/I_or come from the oracle with k + EXTRA ranks (or more); D_gpu/I_gpu have k.
    Returns the fraction of (query, rank) slots whose id equals the oracle's."""
    D_gpu = np.asarray(D_gpu); I_gpu = np.asarray(I_gpu)
    nq, k = D_gpu.shape
    assert D_or.shape[1] >= k
    Do, Io = D_or[:, :k].astype(np.float64), I_or[:, :k]
    tol_all = tolerance(D_or, metric, q, xnorm_max, cancel)
    tol = tol_all[:, :k]
    # empty slots agree
    empty_o = Io < 0
    assert ((I_gpu < 0) == empty_o).all(), "empty-slot pattern differs"
    assert np.isinf(D_gpu[empty_o]).all()
    live = ~empty_o
    err = np.abs(D_gpu.astype(np.float64) - Do)
    bad = live & ~(err <= tol)
    assert not bad.any(), "distance off by %g (tol %g) at %s" % (
        err[bad].max(), tol[bad].min(), np.argwhere(bad)[0])
    # ordered best first
    dd = np.diff(D_gpu.astype(np.float64), axis=1)
    ok = (dd >= 0) if metric == 0 else (dd <= 0)
    assert (ok | ~live[:, 1:]).all(), "results are not ordered best first"
    # ids
    mism = live & (I_gpu != Io)
    for a, j in np.argwhere(mism):
        pos = np.flatnonzero(I_or[a] == I_gpu[a, j])
        assert pos.size >= 1, "query %d rank %d: id %d is not among the oracle's top %d" % (
            a, j, I_gpu[a, j], I_or.shape[1])
        d_other = float(D_or[a, pos[0]])
        assert abs(d_other - Do[a, j]) <= tol_all[a, j] + tol_all[a, pos[0]], \
            "query %d rank %d: id %d (oracle distance %r) displaced id %d (%r)" % (
                a, j, I_gpu[a, j], d_other, Io[a, j], Do[a, j])
    # no duplicates among live results
    for a in range(nq):
        ids = I_gpu[a][I_gpu[a] >= 0]
        assert ids.size == np.unique(ids).size, "duplicate ids in query %d" % a
    return 1.0 - mism.sum() / max(1, live.sum())


def storage_map(ids, list_of, codes):
    """id -> (list, code bytes), as arrays sorted by id."""
    ids = np.asarray(ids); order = np.argsort(ids, kind="stable")
    return ids[order], np.asarray(list_of)[order], np.asarray(codes)[order]
