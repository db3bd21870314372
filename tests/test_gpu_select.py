"""Parity of knn_select (batched partial sort, the paper's Phase 2 as a routine of its own,
Sect. 6) with the CPU oracle.  Values are copies and ties go to the lower column, so the
match must be bit-exact."""
import numpy as np
import pytest
import torch

import oracle
from paper_0906_0231_amd import api, knn_select

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the GPU"
    api.load_library()


def _check(A_host, k, A_dev=None):
    A_dev = torch.from_numpy(A_host).cuda() if A_dev is None else A_dev
    idx, val = knn_select(A_dev, k)
    torch.cuda.synchronize()
    o_idx, o_val = oracle.select(A_host, k)
    assert np.array_equal(idx.cpu().numpy(), o_idx)
    assert np.array_equal(val.cpu().numpy().view(np.uint32), o_val.view(np.uint32))


@pytest.mark.parametrize("m,n,k", [
    (7, 5000, 10), (300, 1000, 1), (1, 100000, 100), (3, 33, 33), (64, 70001, 32),
    (5, 2049, 128), (1000, 257, 16), (2, 1, 1), (17, 4096, 64),
])
def test_select_shapes(m, n, k):
    print(f"  select m={m} n={n} k={k}", flush=True)
    rng = np.random.default_rng(m * 7 + n)
    _check(rng.standard_normal((m, n)).astype(np.float32), k)


def test_select_ties_and_order():
    """Heavily tied data (values on a grid of 64 levels), descending and ascending rows."""
    rng = np.random.default_rng(1)
    A = (rng.integers(0, 64, size=(40, 30000)) / 8).astype(np.float32)
    A[0] = np.arange(30000, 0, -1, dtype=np.float32)      # every element beats the threshold
    A[1] = np.arange(30000, dtype=np.float32)
    A[2] = 3.0                                            # all equal
    _check(A, 20)


def test_select_signed_zeros():
    """-0 and +0 are the same value: they tie (lower column first) and each is returned with its
    own sign, as a copy of the entry."""
    rng = np.random.default_rng(3)
    A = rng.integers(0, 3, size=(30, 5000)).astype(np.float32)
    A[rng.random(A.shape) < 0.3] *= -1.0           # -0.0 where the entry was 0
    assert np.signbit(A[A == 0]).any() and (~np.signbit(A[A == 0])).any()
    _check(A, 40)


def test_select_strided_and_unaligned_rows():
    rng = np.random.default_rng(2)
    big = rng.standard_normal((50, 9001)).astype(np.float32)
    dev = torch.from_numpy(big).cuda()
    _check(np.ascontiguousarray(big[:, :7000]), 12, dev[:, :7000])       # lda > n, lda odd
    _check(np.ascontiguousarray(big[:, 3:8003]), 12, dev[:, 3:8003])     # rows not 16-byte aligned


def test_select_large():
    """The shape the benchmark times: a 1 GiB slab."""
    g = torch.Generator(device="cpu").manual_seed(5)
    A = torch.randn(1024, 262144, generator=g)
    print("  select 1024 x 262144", flush=True)
    _check(A.numpy(), 10, A.cuda())


def test_select_errors():
    A = torch.zeros(4, 100, device="cuda")
    with pytest.raises(api.KnnError) as e:
        knn_select(A, 101)
    assert e.value.status == api.KNN_EINVAL
    with pytest.raises(api.KnnError) as e:
        knn_select(torch.zeros(4, 1000, device="cuda"), 129)
    assert e.value.status == api.KNN_EUNSUPPORTED
