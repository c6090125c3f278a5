"""sw_gemm_static: the product on the library's own static scratch, for callers that cannot allocate.

Through the C ABI, against sw_gemm_ex (same kernels, same step order: the results must be the same bits), on two
calls in a row, the second with a smaller input, so that what the first call left in the scratch is there when
the second runs.  The array is shared by all calls on the GPU and keeps its contents between them.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_1202_3173_amd import binding as sw
from paper_1202_3173_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _reference(n, A, B, levels, schedule):
    need = sw.sw_plan_memory(n, levels, schedule)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=DEV)
    C = torch.full((n, n), float("nan"), dtype=torch.float64, device=DEV)
    sw.sw_set_overlap(0)
    try:
        sw.sw_gemm_ex(n, A, n, B, n, C, n, levels, schedule, ws)
    finally:
        sw.sw_set_overlap(1)
    torch.cuda.synchronize()
    return C


def _pair(n, seed, dist="uniform"):
    return inputs.device_pair(dict(n=n, seed=seed, dist=dist), DEV)


def test_two_calls_in_a_row_second_smaller(oracle):
    # first call: 2048, three steps, 130 MB of the 134 MB scratch
    n1, l1, s1 = 2048, 3, "DDB"
    assert sw.sw_plan_memory(n1, l1, s1) <= sw.SW_STATIC_SCRATCH_BYTES
    A1, B1 = _pair(n1, 21)
    C1 = torch.full((n1, n1), float("nan"), dtype=torch.float64, device=DEV)
    sw.sw_gemm_static(n1, A1, n1, B1, n1, C1, n1, l1, s1)
    # second call straight after, smaller, odd size (zero-padded copies inside the scratch), other step order
    n2, l2, s2 = 1001, 2, "BD"
    A2, B2 = _pair(n2, 22)
    C2 = torch.full((n2, n2), float("nan"), dtype=torch.float64, device=DEV)
    sw.sw_gemm_static(n2, A2, n2, B2, n2, C2, n2, l2, s2)
    torch.cuda.synchronize()
    assert torch.equal(C1, _reference(n1, A1, B1, l1, s1))
    assert torch.equal(C2, _reference(n2, A2, B2, l2, s2))
    # and against the oracle, to the stated bar
    ref = oracle.gemm(A2.cpu().numpy(), B2.cpu().numpy(), l2)
    tol = 1e-10 * n2 * float(A2.abs().max()) * float(B2.abs().max())
    assert float(np.max(np.abs(C2.cpu().numpy() - ref))) <= tol


def test_integers_exact_and_planner_choice():
    for n, levels in ((1536, 2), (768, 3), (256, 1)):
        A, B = _pair(n, 5 + levels, "integer")
        C = torch.full((n, n), float("nan"), dtype=torch.float64, device=DEV)
        sw.sw_gemm_static(n, A, n, B, n, C, n, levels, None)       # the planner's order for the scratch size
        torch.cuda.synchronize()
        assert torch.equal(C, A @ B)
    # depth left to the library as well
    n = 1024
    A, B = _pair(n, 9, "integer")
    C = torch.full((n, n), float("nan"), dtype=torch.float64, device=DEV)
    sw.sw_gemm_static(n, A, n, B, n, C, n, -1, None)
    torch.cuda.synchronize()
    assert torch.equal(C, A @ B)


def test_views_with_leading_dimensions():
    n, ld = 640, 900
    g = torch.Generator(device=DEV).manual_seed(3)
    big = [torch.randint(-8, 9, (n, ld), generator=g, device=DEV, dtype=torch.int32).to(torch.float64) for _ in range(2)]
    Cb = torch.full((n, ld), -7.0, dtype=torch.float64, device=DEV)
    sw.sw_gemm_static(n, big[0], ld, big[1], ld, Cb, ld, 2, "DB")
    torch.cuda.synchronize()
    assert torch.equal(Cb[:, :n], big[0][:, :n] @ big[1][:n, :n])
    assert bool((Cb[:, n:] == -7.0).all())                          # nothing written beyond the n columns


def test_too_large_is_refused_before_anything_runs():
    n = 8192
    A = torch.zeros((n, n), dtype=torch.float64, device=DEV)
    C = torch.full((n, n), 3.0, dtype=torch.float64, device=DEV)
    with pytest.raises(sw.SwError) as e:
        sw.sw_gemm_static(n, A, n, A, n, C, n, 2, "DD")
    assert e.value.code == sw.SW_ENOMEM and "static scratch" in str(e.value)
    with pytest.raises(sw.SwError) as e:
        sw.sw_gemm_static(n, A, n, A, n, C, n, 3, None)             # not even the all-DFS order fits
    assert e.value.code == sw.SW_ENOMEM and "static scratch" in str(e.value)
    torch.cuda.synchronize()
    assert bool((C == 3.0).all())
    # the classical product needs no workspace and is not limited by the scratch
    n = 512
    A, B = _pair(n, 1, "integer")
    C = torch.empty((n, n), dtype=torch.float64, device=DEV)
    sw.sw_gemm_static(n, A, n, B, n, C, n, 0, "")
    torch.cuda.synchronize()
    assert torch.equal(C, A @ B)


def test_device_memory_is_not_allocated_by_a_call():
    n = 1024
    A, B = _pair(n, 2, "integer")
    C = torch.empty((n, n), dtype=torch.float64, device=DEV)
    sw.sw_gemm_static(n, A, n, B, n, C, n, 2, "DB")                 # first use: the address is looked up
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for _ in range(3):
        sw.sw_gemm_static(n, A, n, B, n, C, n, 2, "DB")
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 == free0
    assert torch.equal(C, A @ B)
