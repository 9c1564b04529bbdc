"""The search entry point that allocates nothing (vs_ivfpq_search_static), through the C ABI:
its results equal vs_ivfpq_search's bit for bit, on two calls in a row (the second with a
smaller input, so stale contents of the shared static work space would show), for both metrics
and a probe-split launch; a batch whose work space exceeds the static buffer is refused."""
import ctypes
import sys

import numpy as np
import pytest

import synth_inputs as S

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def vs():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2401_08281_amd as vs
    vs.lib()
    return vs


def _raw_search(vs, fn, ix, q, k, nprobe):
    """Calls fn(handle, q, nq, k, nprobe, out_dist, out_ids, stream) on raw device pointers."""
    import torch
    nq = q.shape[0]
    D = torch.full((nq, k), 7.0, dtype=torch.float32, device="cuda")
    I = torch.full((nq, k), 7, dtype=torch.int64, device="cuda")
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = fn(ix.h, ctypes.c_void_p(q.data_ptr()), nq, k, nprobe, ctypes.c_void_p(D.data_ptr()),
            ctypes.c_void_p(I.data_ptr()), st)
    torch.cuda.synchronize()
    return rc, D.cpu().numpy(), I.cpu().numpy()


@pytest.mark.parametrize("name,cfg,k,nprobe", [
    ("c1_l2", S.config("C1"), 10, 4),
    ("c4_small_l2", S.config("C4", nb=50_000, nq=100, ncomp=100, nlist=256), 100, 64),
    ("c5_small_ip_4bit", S.config("C5", nb=20_000, nq=100, ncomp=50, nlist=128), 10, 32),
], ids=["c1_l2", "c4_small_l2", "c5_small_ip_4bit"])
def test_static_search_equals_search_on_two_calls_in_a_row(vs, name, cfg, k, nprobe):
    import torch
    say("no-alloc %s nb=%d nq=%d d=%d nlist=%d k=%d nprobe=%d" % (
        name, cfg["nb"], cfg["nq"], cfg["d"], cfg["nlist"], k, nprobe))
    L = vs.lib()
    x, q = S.make_data(cfg)
    cent, cb = S.make_index_params(cfg, x)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    ix = vs.IVFPQ(cfg["d"], cfg["metric"], t(cent), t(cb), cfg["nbits"])
    ix.add(t(x))
    qd = t(q)
    # first call: the whole batch; second call: a smaller one (7 queries: the probes are split
    # over several workgroups per query and merged), then one query
    for nq in (q.shape[0], 7, 1):
        qs = qd[:nq].contiguous()
        rc0, D0, I0 = _raw_search(vs, L.vs_ivfpq_search, ix, qs, k, nprobe)
        rc1, D1, I1 = _raw_search(vs, L.vs_ivfpq_search_static, ix, qs, k, nprobe)
        assert rc0 == 0 and rc1 == 0, L.vs_last_error()
        np.testing.assert_array_equal(I1, I0)
        np.testing.assert_array_equal(D1.view(np.uint32), D0.view(np.uint32))
        assert (I1 != 7).all()                      # every output slot was written
    ix.close()


def test_static_search_refuses_a_batch_beyond_its_work_space(vs):
    import torch
    say("no-alloc: a batch beyond the static work space")
    L = vs.lib()
    cfg = S.config("C3", nb=20_000, nq=10, ncomp=20, nlist=4096)
    x, _ = S.make_data(cfg)
    cent, cb = S.make_index_params(cfg, x)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    ix = vs.IVFPQ(cfg["d"], 0, t(cent), t(cb), 8)
    ix.add(t(x))
    q = torch.zeros((20_000, cfg["d"]), dtype=torch.float32, device="cuda")
    rc, D, I = _raw_search(vs, L.vs_ivfpq_search_static, ix, q, 10, 64)
    assert rc == -1 and b"work space" in L.vs_last_error()
    assert (I == 7).all()                           # nothing ran
    rc, _, _ = _raw_search(vs, L.vs_ivfpq_search_static, ix, q[:0], 10, 64)
    assert rc == 0                                  # no queries: no-op
    ix.close()
