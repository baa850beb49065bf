"""Writes tests/golden/config<k>_rows.txt: CPU-oracle values of a few rows of a full-size configuration.

At n = 1e7 (D = 7, 2187 nodes per box) and n = 1e9 the CPU oracle needs minutes and tens of gigabytes even for a
subset of the rows, so the GPU tests do not run it: this script does, once, and the tests compare the GPU result
with the stored numbers.  It calls the CPU oracle and the seeded input generators only -- never the HIP library.

For every stored row: the CPU F3M value (Appendix E, Algorithm 1, restricted to the boxes that hold the rows; same
bits as the full product) and the exact fp64 sum (Sec. 5, first paragraph: the reference the error is measured
against).  For the first boxes: per depth the rank of the box that holds the row, the lengths of its near and far
rows and a checksum of their columns, for the bit-exact comparison of the interaction lists.

    python tests/golden/make_full_size_rows.py 5 [--rows 256] [--out FILE]     (needs about 80 GB of memory)
    python tests/golden/make_full_size_rows.py 4 [--boxes 2] [--out FILE]
"""
import argparse
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2202_01085_amd import inputs  # noqa: E402

LIST_BOXES = 64      # rows whose interaction rows are stored as checksums
MASK = (1 << 64) - 1


def list_checksum(cols):
    """order-dependent 64-bit checksum of a row of box ranks"""
    h = 0
    for c in cols:
        h = (h * 1000003 + int(c) + 1) & MASK
    return h


def say(*a):
    print(*a, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("config", type=int, choices=[3, 4, 5])
    ap.add_argument("--rows", type=int, default=256, help="sampled rows (configurations 3 and 5)")
    ap.add_argument("--boxes", type=int, default=2, help="leaf boxes whose points are the rows (configuration 4)")
    ap.add_argument("--n", type=int, default=None, help="a reduced n of the same recipe (trial runs)")
    ap.add_argument("--out", default=None)
    args = ap.parse_args()
    k = args.config
    out = args.out or os.path.join(os.path.dirname(os.path.abspath(__file__)), "config%d_rows.txt" % k)
    oracle.set_verbose(True)
    t0 = time.time()
    X, b, cfg = inputs.make_config(k, n=args.n)
    X, b = X.numpy(), b.numpy()
    n, D = X.shape
    gamma = float(np.float32(cfg["lengthscale"]))          # the lengthscale as a float, as the C ABI of the library takes it
    p, theta, zeta = cfg["p"], cfg["theta"], 128
    say("configuration %d: n=%d D=%d generated in %.0f s" % (k, n, D, time.time() - t0))
    seed_rows = inputs.sample_rows(n, args.rows if k != 4 else args.boxes, 3000 + k).numpy()
    if k == 4:
        # the rows are all points of the leaf boxes that hold the first sampled rows: r^2 = 4.8e6 kernel values per far
        # pair and thousands of far pairs per box make every further target box cost minutes
        T0 = oracle.Tree(X, theta=theta, zeta=zeta, rows=seed_rows)
        perm, starts = T0.perm(), T0.boxes(T0.L)[1]
        inv_pos = {int(r): int(np.flatnonzero(perm == r)[0]) for r in seed_rows}
        rows = []
        for r in seed_rows:
            a = int(np.searchsorted(starts, inv_pos[int(r)], side="right") - 1)
            rows.extend(perm[starts[a]:starts[a + 1]].tolist())
        rows = np.array(sorted(set(rows)), dtype=np.int64)
        del T0
    else:
        rows = seed_rows
    say("%d rows" % rows.size)
    t0 = time.time()
    T = oracle.Tree(X, theta=theta, zeta=zeta, rows=rows)
    say("tree: depth %d, %.0f s" % (T.L, time.time() - t0))
    t0 = time.time()
    yf = T.apply_rows(b, gamma, p, rows)
    say("CPU F3M rows: %.0f s" % (time.time() - t0))
    t0 = time.time()
    ye = np.empty(rows.size)
    step = 16
    for i in range(0, rows.size, step):
        ye[i:i + step] = oracle.rows(X, b, gamma, rows[i:i + step])
        say("exact rows %d/%d, %.0f s" % (min(i + step, rows.size), rows.size, time.time() - t0))
    err = np.linalg.norm(yf - ye) / np.linalg.norm(ye)
    say("CPU F3M against the exact rows: relative L2 %.3e" % err)

    # box-order positions of the rows whose lists are stored
    perm = T.perm()
    lrows = rows[:LIST_BOXES]
    pos = np.empty(lrows.size, dtype=np.int64)
    want = {int(r): i for i, r in enumerate(lrows)}
    for c0 in range(0, n, 1 << 26):
        chunk = perm[c0:c0 + (1 << 26)]
        for h in np.flatnonzero(np.isin(chunk, lrows)):
            pos[want[int(chunk[h])]] = c0 + int(h)
    del perm
    with open(out, "w") as f:
        f.write("# configuration %d of the benchmark set: n=%d D=%d nodes/dim=%d lengthscale=%r far ratio=%g zeta=%d\n"
                % (k, n, D, p, gamma, theta, zeta))
        f.write("# written by tests/golden/make_full_size_rows.py from the CPU oracle (oracle/), %d threads\n"
                % oracle.num_threads())
        f.write("# depth %d; CPU F3M against exact on these rows: relative L2 %.6e\n" % (T.L, err))
        f.write("# rows: index, CPU F3M value (Appendix E Algorithm 1), exact fp64 sum (Sec. 5 first paragraph)\n")
        for r, a, e in zip(rows, yf, ye):
            f.write("row %d %.17g %.17g\n" % (r, a, e))
        f.write("# lists: row index, depth, rank of the box holding the row, near count, near checksum, far count, "
                "far checksum\n")
        for l in range(1, T.L + 1):
            starts = T.boxes(l)[1]
            nptr, ncol = T.interactions(l, 0)
            fptr, fcol = T.interactions(l, 1)
            seen = set()
            for i in range(lrows.size):
                a = int(np.searchsorted(starts, pos[i], side="right") - 1)
                if a in seen:                       # one record per box and depth
                    continue
                seen.add(a)
                f.write("list %d %d %d %d %d %d %d\n" % (lrows[i], l, a, nptr[a + 1] - nptr[a],
                                                        list_checksum(ncol[nptr[a]:nptr[a + 1]]), fptr[a + 1] - fptr[a],
                                                        list_checksum(fcol[fptr[a]:fptr[a + 1]])))
    say("wrote", out)


if __name__ == "__main__":
    main()
