"""The entry point that allocates nothing (ocean_row_products_noalloc) against ocean_row_products, through
the C ABI: two calls in a row on the same GPU, the second with a smaller input, so that what the first call
left in the library's fixed scratch array must not leak into the second."""
import numpy as np
import pytest

from paper_2604_19004_amd import workloads as W
from paper_2604_19004_amd.workloads import CSR

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ob():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2604_19004_amd import binding
    binding.load()
    return binding


def _both(ob, A, B):
    import torch
    dA, dB = ob.to_device(A), ob.to_device(B)
    ref, total, mx = ob.row_products(dA, dB)
    prod = torch.full((A.rows,), -7, dtype=torch.int64, device="cuda:0")
    totals = torch.full((3,), -7, dtype=torch.int64, device="cuda:0")
    import gc
    gc.collect()                                     # (tensors of earlier tests may still be waiting for the collector)
    before = torch.cuda.memory_allocated()
    ob.row_products_noalloc(dA, dB, prod, totals)
    assert torch.cuda.memory_allocated() <= before   # nothing was obtained through the caller's allocator either
    torch.cuda.synchronize()
    assert torch.equal(prod, ref), "prod differs from ocean_row_products"
    assert totals.cpu().tolist() == [total, mx, 0]
    return total


def test_no_alloc_matches_existing_entry_point_twice_second_smaller(ob):
    ob.init()
    A1, B1, _ = W.make("rmat", small=True)          # power-law: long rows go through the row list in scratch
    A2, B2, _ = W.make("laplacian", small=True)
    t1 = _both(ob, A1, B1)
    A3 = CSR(300, A1.cols, A1.row_ptr[:301].copy(), A1.col_idx[:int(A1.row_ptr[300])].copy(),
             A1.val[:int(A1.row_ptr[300])].copy())  # the first 300 rows of the first input: fewer rows, fewer long rows
    t3 = _both(ob, A3, B1)
    t2 = _both(ob, A2, B2)
    assert t3 < t1 and t2 > 0


def test_no_alloc_rejects_sizes_beyond_its_scratch(ob):
    import torch
    m = ob.NOALLOC_MAX_ROWS + 1
    A = ob.DeviceCSR(m, 4, torch.zeros(m + 1, dtype=torch.int64, device="cuda:0"),
                     torch.zeros(0, dtype=torch.int32, device="cuda:0"), torch.zeros(0, dtype=torch.float64, device="cuda:0"))
    B = ob.to_device(CSR(4, 4, np.zeros(5, np.int64), np.zeros(0, np.int32), np.zeros(0)))
    prod = torch.zeros(m, dtype=torch.int64, device="cuda:0")
    totals = torch.zeros(3, dtype=torch.int64, device="cuda:0")
    with pytest.raises(ob.OceanError) as e:
        ob.row_products_noalloc(A, B, prod, totals)
    assert e.value.code == 1 and "OCEAN_NOALLOC_MAX_ROWS" in str(e.value)
