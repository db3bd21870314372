"""knn_search_static: the entry point that allocates nothing (its workspace is a static device
array inside the library).  Checked through the C ABI against knn_search -- the existing entry
point, handed a caller's workspace of the same size, takes the same plan and must give the same
bits -- and against the CPU oracle, on two calls in a row, the second with a smaller input (the
array keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from oracle import compare
from paper_0906_0231_amd import api, workloads

pytestmark = pytest.mark.gpu
RTOL = 1e-5


def _say(msg):
    print(msg, flush=True)


def _static(lib, Q, R, k, metric, off):
    nq, d = Q.shape
    idx = torch.empty((nq, k), dtype=torch.int32, device="cuda")
    dist = torch.empty((nq, k), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    st = lib.knn_search_static(Q.data_ptr(), nq, R.data_ptr(), R.shape[0], d, k, api.METRICS[metric], off,
                               idx.data_ptr(), dist.data_ptr(), stream)
    assert st == api.KNN_OK, lib.knn_status_string(st).decode() + " " + lib.knn_last_device_error().decode()
    return idx, dist


def _existing(lib, Q, R, k, metric, off, ws):
    nq, d = Q.shape
    idx = torch.empty((nq, k), dtype=torch.int32, device="cuda")
    dist = torch.empty((nq, k), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    st = lib.knn_search(Q.data_ptr(), nq, R.data_ptr(), R.shape[0], d, k, api.METRICS[metric], off,
                        idx.data_ptr(), dist.data_ptr(), ws.data_ptr(), ws.numel(), stream)
    assert st == api.KNN_OK
    return idx, dist


@pytest.mark.parametrize("metric", ["sqeuclidean", "cosine", "l1"])
def test_static_scratch_two_calls_in_a_row(metric):
    assert torch.cuda.is_available(), "this test needs the GPU"
    lib = api.load_library()
    ws = torch.empty(api.STATIC_SCRATCH_BYTES, dtype=torch.uint8, device="cuda")
    # first call: several query tiles and reference slices, ragged tails; second: smaller in every size
    cases = [(3000, 9000, 48, 20, 1500), (700, 2100, 33, 7, -1)]
    for nq, nr, d, k, off in cases:
        _say(f"  static scratch {metric} nq={nq} nr={nr} d={d} k={k} self_offset={off}")
        R = workloads.mixture(nr, d, 8, seed=100 + nr)
        Q = R[off:off + nq].contiguous() if off >= 0 else workloads.gaussian(nq, d, seed=101 + nq)
        Rd, Qd = R.cuda(), Q.cuda()
        plan = api.knn_plan(nq, nr, d, k, metric, workspace_bytes=api.STATIC_SCRATCH_BYTES)
        _say(f"    {plan}")
        assert plan.workspace_bytes <= api.STATIC_SCRATCH_BYTES
        s_idx, s_dist = _static(lib, Qd, Rd, k, metric, off)
        e_idx, e_dist = _existing(lib, Qd, Rd, k, metric, off, ws)
        torch.cuda.synchronize()
        assert torch.equal(s_idx, e_idx) and torch.equal(s_dist, e_dist)
        self_idx = np.arange(nq) + off if off >= 0 else None
        o_idx, o_dist, o_next = oracle.search(Q.numpy(), R.numpy(), k, metric, self_idx=self_idx)
        rep = compare.check(Q.numpy(), R.numpy(), metric, o_idx, o_dist, o_next, s_idx.cpu().numpy(),
                            s_dist.cpu().numpy(), self_idx=self_idx, rtol=RTOL)
        _say(f"    {rep}")
        assert rep.ok, str(rep)


def test_static_scratch_refuses_what_does_not_fit():
    """Sizes whose smallest plan needs more than the array: KNN_ENOMEM, nothing enqueued (the
    check is on the host, before any pointer is touched)."""
    lib = api.load_library()
    one = ctypes.c_void_p(256)
    assert api.knn_workspace_bytes_min(1 << 20, 1 << 20, 256, 10) > api.STATIC_SCRATCH_BYTES
    st = lib.knn_search_static(one, 1 << 20, one, 1 << 20, 256, 10, 0, -1, one, one, None)
    assert st == api.KNN_ENOMEM
    assert lib.knn_search_static(None, 10, one, 100, 8, 3, 0, -1, one, one, None) == api.KNN_EINVAL
    assert lib.knn_search_static(one, 10, one, 100, 8, 101, 0, -1, one, one, None) == api.KNN_EINVAL


def test_static_scratch_under_graph_capture():
    """A caller that cannot allocate because it is being captured into a HIP graph: the call is
    recorded once and replayed on new inputs, with the program's own eager work and
    synchronisations between the replays; every replay must give what the eager call gives.
    (The library enqueues kernels only -- no memset or copy nodes.)"""
    assert torch.cuda.is_available(), "this test needs the GPU"
    from paper_0906_0231_amd import knn_search, knn_search_static
    nq, nr, d, k = 1000, 5000, 40, 12
    R = workloads.mixture(nr, d, 6, seed=900).cuda()
    Q = torch.empty((nq, d), dtype=torch.float32, device="cuda")
    idx = torch.empty((nq, k), dtype=torch.int32, device="cuda")
    dist = torch.empty((nq, k), dtype=torch.float32, device="cuda")
    Q.copy_(workloads.gaussian(nq, d, seed=901).cuda())
    knn_search_static(Q, R, k, out=(idx, dist))            # first use of the array on this device: outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        knn_search_static(Q, R, k, out=(idx, dist))
    for rep in range(4):
        Qh = workloads.gaussian(nq, d, seed=910 + rep) * (1.0 + rep)
        Q.copy_(Qh.cuda())
        idx.fill_(-7)
        dist.fill_(-1.0)
        g.replay()
        torch.cuda.synchronize()
        eager = knn_search(Q, R, k)
        torch.cuda.synchronize()
        assert torch.equal(idx, eager.idx) and torch.equal(dist, eager.dist), f"replay {rep} differs from the eager call"
        o_idx, o_dist, o_next = oracle.search(Qh.numpy(), R.cpu().numpy(), k, "sqeuclidean")
        rep_ = compare.check(Qh.numpy(), R.cpu().numpy(), "sqeuclidean", o_idx, o_dist, o_next, idx.cpu().numpy(),
                             dist.cpu().numpy(), rtol=RTOL)
        assert rep_.ok, str(rep_)
