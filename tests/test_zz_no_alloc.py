"""direct_kmvm_rows_f64_static, the entry point that allocates nothing, against direct_kmvm_rows_f64
(same kernels, same slicing of the sources: the results must be the same bits) and against the CPU
oracle's exact rows, on two calls in a row, the second with a smaller input, so that stale partial
sums of the first call in the shared static array would show."""
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


def test_rows_static_equals_allocating_entry_point_two_calls_in_a_row():
    cases = [
        # n, D, rows, seed: the first has 12 source slices and three row blocks, the second one slice and one block
        (50_000, 3, 150, 7001),
        (3_000, 3, 37, 7002),
    ]
    for n, D, m, seed in cases:
        X = inputs.points_normal(n, D, seed)
        b = inputs.rhs_normal(n, seed + 50)
        rows = inputs.sample_rows(n, m, seed + 100)
        gamma = 0.3
        say("direct_kmvm_rows_f64_static n=%d D=%d rows=%d" % (n, D, m))
        Xd, bd, rd = X.to(DEV).contiguous(), b.to(DEV).contiguous(), rows.to(DEV).contiguous()
        y_static = torch.full((m,), float("nan"), dtype=torch.float64, device=DEV)
        f3m.direct_kmvm_rows_f64_static(Xd, bd, gamma, rd, y_static)
        y_alloc = f3m.direct_kmvm_rows_f64(Xd, bd, gamma, rd)
        torch.cuda.synchronize()
        ys, ya = y_static.cpu().numpy(), y_alloc.cpu().numpy()
        assert np.array_equal(ys, ya)
        want = oracle.rows(X.numpy(), b.numpy(), float(np.float32(gamma)), rows.numpy())
        assert np.linalg.norm(ys - want) <= 1e-12 * np.linalg.norm(want)
        assert np.max(np.abs(ys - want)) <= 1e-11 * np.max(np.abs(want))


def test_rows_static_refuses_more_rows_than_its_scratch_holds():
    n = 1000
    X = inputs.points_uniform(n, 2, 7003).to(DEV)
    b = inputs.rhs_normal(n, 7004).to(DEV)
    m = 16384 + 1
    rows = torch.zeros(m, dtype=torch.int64, device=DEV)
    y64 = torch.zeros(m, dtype=torch.float64, device=DEV)
    say("direct_kmvm_rows_f64_static refuses m=%d" % m)
    with pytest.raises(f3m.F3MError) as e:
        f3m.direct_kmvm_rows_f64_static(X, b, 1.0, rows, y64)
    assert e.value.status == 3
    # at the limit it runs
    rows = (torch.arange(16384, dtype=torch.int64, device=DEV) % n).contiguous()
    y64 = torch.zeros(16384, dtype=torch.float64, device=DEV)
    f3m.direct_kmvm_rows_f64_static(X, b, 1.0, rows, y64)
    want = f3m.direct_kmvm_rows_f64(X, b, 1.0, rows)
    torch.cuda.synchronize()
    assert torch.equal(y64, want)
