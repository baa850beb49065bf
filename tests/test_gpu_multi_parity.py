"""GPU parity of f3m_kmvm_multi (several right-hand sides with one plan): every column must equal the
single product f3m_kmvm of that column (same sums, another order in the near field: <= 2e-6 relative),
and one configuration is checked against the CPU oracle directly (<= 1e-5)."""
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2202_01085_amd import f3m, inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def rel(a, b):
    return float(torch.linalg.norm(a.double() - b.double()) / torch.linalg.norm(b.double()))


def columns(m, n, seed):
    return torch.stack([inputs.rhs_normal(n, seed + j) for j in range(m)]).contiguous()


@pytest.mark.parametrize("m", [1, 2, 3, 4, 7])
def test_multi_equals_single_products_on_the_fused_path(m):
    n = 600_000                                   # 32768 leaf boxes: enough tiles for the grouped near field
    say("f3m_kmvm_multi n=%d D=3 m=%d" % (n, m))
    X = inputs.points_uniform(n, 3, 801).to(DEV)
    B = columns(m, n, 810).to(DEV)
    plan = f3m.Plan(X, 0.5, 4, 2.0)
    assert plan.info().depth == 5
    Y = plan.kmvm_multi(B)
    torch.cuda.synchronize()
    for j in range(m):
        yj = plan.kmvm(B[j])
        e = rel(Y[j], yj)
        assert e <= 2e-6, (j, e)
    assert torch.equal(Y, plan.kmvm_multi(B))     # repeatable
    if m == 3:
        T = oracle.Tree(X.cpu().numpy(), zeta=128)
        yo = torch.from_numpy(T.apply(B[1].cpu().numpy(), 0.5, 4))
        e = rel(Y[1].cpu(), yo)
        say("  column 1 against the CPU F3M: %.3e" % e)
        assert e <= 1e-5


def test_multi_two_sets_and_strided_columns():
    say("f3m_kmvm_multi with two point sets and padded leading dimensions")
    nx, ny, m = 700_000, 300_000, 3
    X = inputs.points_uniform(nx, 3, 821).to(DEV)
    Yp = (inputs.points_normal(ny, 3, 822) * 0.3 + 0.5).to(DEV).contiguous()
    plan = f3m.Plan(X, 0.4, 4, 2.0, Y=Yp)
    ldb, ldy = ny + 37, nx + 5                     # columns that are not back to back
    Bbuf = torch.zeros(m * ldb, device=DEV)
    Ybuf = torch.full((m * ldy,), 9.0, device=DEV)
    cols = columns(m, ny, 830).to(DEV)
    for j in range(m):
        Bbuf[j * ldb:j * ldb + ny] = cols[j]
    import ctypes
    st = f3m.lib().f3m_kmvm_multi(plan._h, ctypes.c_void_p(Bbuf.data_ptr()), ldb, ctypes.c_void_p(Ybuf.data_ptr()), ldy, m,
                                  ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == 0
    torch.cuda.synchronize()
    for j in range(m):
        yj = plan.kmvm(cols[j])
        assert rel(Ybuf[j * ldy:j * ldy + nx], yj) <= 2e-6
        assert torch.all(Ybuf[j * ldy + nx:(j + 1) * ldy] == 9.0)      # the gaps are left alone


@pytest.mark.parametrize("n,D,p,kw", [(30_000, 3, 4, {}),                       # too few tiles for the grouped kernel
                                      (40_000, 2, 5, {}),                       # D != 3
                                      (50_000, 3, 4, dict(small_field=64)),     # small field
                                      (20_000, 5, 2, dict(max_depth=2))])
def test_multi_falls_back_to_single_products(n, D, p, kw):
    say("f3m_kmvm_multi fallback n=%d D=%d %s" % (n, D, kw))
    X = inputs.points_normal(n, D, 840 + D).to(DEV)
    B = columns(3, n, 850).to(DEV)
    plan = f3m.Plan(X, 0.7, p, 2.0, leaf_max=32, **kw)
    Y = plan.kmvm_multi(B)
    torch.cuda.synchronize()
    for j in range(3):
        assert torch.equal(Y[j], plan.kmvm(B[j]))  # the very same kernels


def test_multi_edge_cases():
    say("f3m_kmvm_multi edge cases")
    X = inputs.points_uniform(5_000, 3, 861).to(DEV)
    plan = f3m.Plan(X, 1.0, 4, 2.0)
    assert plan.kmvm_multi(torch.empty((0, 5_000), device=DEV)).shape == (0, 5_000)      # no columns
    with pytest.raises(ValueError):
        plan.kmvm_multi(torch.zeros((2, 4_999), device=DEV))
    import ctypes
    fake = ctypes.c_void_p(4096)
    assert f3m.lib().f3m_kmvm_multi(plan._h, fake, 4_999, fake, 5_000, 2, None) == 1          # ldb too small
    assert f3m.lib().f3m_kmvm_multi(plan._h, fake, 5_000, fake, 100, 2, None) == 1            # ldy too small
    assert f3m.lib().f3m_kmvm_multi(plan._h, fake, 5_000, fake, 5_000, -1, None) == 1
    two = f3m.Plan(X, 1.0, 4, 2.0, Y=X[:0])
    Y = two.kmvm_multi(torch.empty((2, 0), device=DEV), Y=torch.full((2, 5_000), 3.0, device=DEV))
    torch.cuda.synchronize()
    assert torch.count_nonzero(Y).item() == 0                                                # no sources: zeros
