"""Comparison rules between the HIP path and the CPU oracle.

  - list assignments and PQ codes: bit-exact, compared as the map
    id -> (list, code bytes) because the order inside a list is storage detail;
  - distances: |gpu - oracle| <= 1e-4 * max(|oracle|, s) where s is the
    magnitude of the terms that cancel (inner product: ||q|| * max ||x||;
    L2: none for the definition itself, the squared distance is a sum of non-negative
    terms -- but the compressed-domain forms of Sec. 4.3 expand the square, and their
    terms do cancel: `cancel` = the magnitude of the cancelling terms per query enters
    with the fp32 rounding the expansion can cost, `cancel_eps` of it (default 2^-21),
    instead of a relative share.  For the stored-norm search type cancel = |q|^2 +
    max |x'|^2; for look-up tables built as |r_m|^2 + |t|^2 - 2 <r_m, t> it is the
    largest probed |q - c_l|^2 plus the largest decoded residual norm, see
    l2_table_cancel);
  - ids: identical, except that a GPU id may differ from the oracle's id at
    the same rank when the ORACLE distances of the two candidates are within
    that tolerance (one tolerance, the larger of the two candidates') of each other.  To see candidates just past rank k the
    oracle is run with a few extra ranks.
"""
import numpy as np

REL_TOL = 1e-4
EXTRA = 16


def tolerance(D_or, metric, q=None, xnorm_max=None, cancel=None, cancel_eps=2.0 ** -21):
    tol = REL_TOL * np.abs(D_or.astype(np.float64))
    if metric == 1:
        qn = np.sqrt((q.astype(np.float64) ** 2).sum(1, keepdims=True))
        tol = np.maximum(tol, REL_TOL * qn * float(xnorm_max))
    if cancel is not None:
        tol = tol + cancel_eps * np.asarray(cancel, dtype=np.float64).reshape(-1, 1)
    return tol


def l2_table_cancel(coarse_dist, codebooks):
    """(cancel, cancel_eps) for L2 look-up tables whose entries are evaluated as
    (|r_m|^2 + |t|^2) + sum_u r_u (-2 t_u), r = q - c_l (Sec. 4.3's expansion applied to one
    sub-vector): every entry carries at most (dsub + 2) roundings of 2^-24 relative to
    |r_m|^2 + |t|^2 + 2 |<r_m, t>| <= 2 (|r_m|^2 + |t|^2); summed over m that is
    (dsub + 2) 2^-23 (|q - c_l|^2 + |t|^2), bounded per query by the largest probed coarse
    distance and the largest residual reconstruction sum_m max_j |T_m[j]|^2."""
    cb = np.asarray(codebooks, dtype=np.float64)
    tmax = float((cb ** 2).sum(2).max(1).sum())
    cd = np.asarray(coarse_dist, dtype=np.float64)
    cd = np.where(np.isfinite(cd), cd, 0.0)
    return cd.max(1) + tmax, (cb.shape[2] + 2) * 2.0 ** -23


def check_search(D_gpu, I_gpu, D_or, I_or, metric, q=None, xnorm_max=None, cancel=None,
                 cancel_eps=2.0 ** -21):
    """D_or/I_or come from the oracle with k + EXTRA ranks (or more); D_gpu/I_gpu have k.
    Returns the fraction of (query, rank) slots whose id equals the oracle's."""
    D_gpu = np.asarray(D_gpu); I_gpu = np.asarray(I_gpu)
    nq, k = D_gpu.shape
    assert D_or.shape[1] >= k
    Do, Io = D_or[:, :k].astype(np.float64), I_or[:, :k]
    tol_all = tolerance(D_or, metric, q, xnorm_max, cancel, cancel_eps)
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
        assert abs(d_other - Do[a, j]) <= max(tol_all[a, j], tol_all[a, pos[0]]), \
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
