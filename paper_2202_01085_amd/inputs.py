"""Seeded synthetic inputs shared by the tests, the oracle harness and bench.py.

Nothing of the method's arithmetic lives here: only point clouds, right-hand
sides and row samples.  Every value is a pure function of (seed, element
index) through a counter-based 64-bit integer mix, so a result does not depend
on the device, the chunking or the thread count.  The data sets stand in for
the paper's Uniform / Normal / Clustered sets (Sec. 5 "KMVM experiments",
Appendix A): iid Uniform[0,1]^D, iid N(0, I_D), and an equal-weight mixture of
isotropic unit Gaussians whose means are Uniform[-5,5]^D.
"""
import math

import torch

_M1 = -7046029254386353131          # 0x9E3779B97F4A7C15 as int64
_M2 = -4658895280553007687          # 0xBF58476D1CE4E5B9
_M3 = -7723592293110705685          # 0x94D049BB133111EB
_CHUNK = 1 << 24


def _lsr(x, k):
    """logical shift right of an int64 tensor"""
    return (x >> k) & ((1 << (64 - k)) - 1)


def _wrap64(v):
    """python int -> the int64 it wraps to"""
    v &= (1 << 64) - 1
    return v - (1 << 64) if v >= (1 << 63) else v


def _mix(counter, seed):
    """splitmix64 finaliser of (counter + (seed+1) * golden), int64 wrap-around arithmetic"""
    z = counter + _wrap64((seed + 1) * _M1)
    z = (z ^ _lsr(z, 30)) * _M2
    z = (z ^ _lsr(z, 27)) * _M3
    return z ^ _lsr(z, 31)


def _u24(counter, seed):
    """top 24 bits of the mix as an integer tensor in [0, 2^24)"""
    return _lsr(_mix(counter, seed), 40)


def _chunks(total):
    for lo in range(0, total, _CHUNK):
        yield lo, min(total, lo + _CHUNK)


def uniform(count, seed, device="cpu"):
    """count fp32 values in [0,1): top 24 bits of the mix times 2^-24 (exact in fp32)."""
    out = torch.empty(count, dtype=torch.float32, device=device)
    for lo, hi in _chunks(count):
        c = torch.arange(lo, hi, dtype=torch.int64, device=device)
        out[lo:hi] = _u24(c, seed).to(torch.float32) * (2.0 ** -24)
    return out


def normal(count, seed, device="cpu"):
    """count fp32 N(0,1) values: Box-Muller in fp64 on two 24-bit uniforms, rounded to fp32."""
    out = torch.empty(count, dtype=torch.float32, device=device)
    for lo, hi in _chunks(count):
        c = torch.arange(lo, hi, dtype=torch.int64, device=device)
        u1 = (_u24(2 * c, seed).to(torch.float64) + 1.0) * (2.0 ** -24)      # (0,1]
        u2 = _u24(2 * c + 1, seed).to(torch.float64) * (2.0 ** -24)          # [0,1)
        z = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)
        out[lo:hi] = z.to(torch.float32)
    return out


def points_uniform(n, D, seed, device="cpu"):
    return uniform(n * D, seed, device).view(n, D)


def points_normal(n, D, seed, device="cpu"):
    return normal(n * D, seed, device).view(n, D)


def points_mixture(n, D, seed, components=10, device="cpu"):
    """equal-weight mixture of `components` unit isotropic Gaussians, means Uniform[-5,5]^D"""
    means = (uniform(components * D, seed + 7919, device) * 10.0 - 5.0).view(components, D)
    x = normal(n * D, seed, device).view(n, D)
    for lo, hi in _chunks(n):
        c = torch.arange(lo, hi, dtype=torch.int64, device=device)
        comp = _u24(c, seed + 104729) % components
        x[lo:hi] += means[comp]
    return x


def rhs_normal(n, seed, device="cpu"):
    return normal(n, seed, device)


def sample_rows(n, m, seed):
    """m distinct row indices in [0,n), ascending, int64 numpy-compatible CPU tensor"""
    m = min(m, n)
    picked = set()
    c = 0
    while len(picked) < m:
        need = m - len(picked)
        idx = torch.arange(c, c + 2 * need + 16, dtype=torch.int64)
        c += idx.numel()
        cand = (_lsr(_mix(idx, seed), 1) % n).tolist()
        for v in cand:
            if len(picked) < m:
                picked.add(v)
    return torch.tensor(sorted(picked), dtype=torch.int64)


# The workloads of the benchmark configuration list, by 1-based index k.
# Seeds: X 1000+k, b 2000+k, sampled rows 3000+k.
CONFIGS = {
    1: dict(n=20_000, D=3, dist="uniform", lengthscale=1.0, p=4, theta=2.0),
    2: dict(n=1_000_000, D=3, dist="normal", lengthscale=0.1, p=4, theta=2.0),
    3: dict(n=100_000_000, D=3, dist="uniform", lengthscale=1.0, p=4, theta=2.0),
    4: dict(n=10_000_000, D=7, dist="mixture", lengthscale=1.0, p=3, theta=2.0),
    5: dict(n=1_000_000_000, D=3, dist="uniform", lengthscale=1.0, p=4, theta=2.0),
}


def make_config(k, n=None, device="cpu"):
    """(X, b, cfg) of configuration k, optionally at a reduced n of the same recipe."""
    cfg = dict(CONFIGS[k])
    if n is not None:
        cfg["n"] = int(n)
    gen = {"uniform": points_uniform, "normal": points_normal, "mixture": points_mixture}[cfg["dist"]]
    X = gen(cfg["n"], cfg["D"], 1000 + k, device=device)
    b = rhs_normal(cfg["n"], 2000 + k, device=device)
    return X, b, cfg
