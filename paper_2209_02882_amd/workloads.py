"""Seeded synthetic SpMM inputs.

This module only *draws inputs*: CSR structure (rowptr, colidx), values and the
dense operand B.  It holds none of the arithmetic of the method under test and
is the one piece of code that both the CPU oracle's tests and the HIP path's
tests/bench use, so that the two sides see identical bytes.

The paper evaluates on the sparse-matrix collection of the DA-SpMM work
(Section 7, "Experiment settings"), which is not available offline.  The five
workloads below stand in for it; each is fully determined by its seed.

All matrices: int32 0-based rowptr / colidx, column indices sorted ascending
and distinct inside each row, fp32 values, B row-major contiguous fp32.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

__all__ = [
    "SpmmProblem",
    "make_problem",
    "WORKLOADS",
    "csr_from_lengths",
    "uniform_fixed_degree",
    "powerlaw_rows",
    "stencil27",
    "rmat",
    "skewed_rows",
    "fill_values",
    "dense_operand",
    "RECIPES",
    "recipe",
    "Tensor3Problem",
    "make_tensor3",
    "TENSOR_WORKLOADS",
]


@dataclass
class SpmmProblem:
    """One SpMM instance  C[M,N] = A_csr[M,K] * B[K,N]  (inputs only)."""

    name: str
    M: int
    K: int
    N: int
    rowptr: np.ndarray  # int32 [M+1]
    colidx: np.ndarray  # int32 [nnz]
    vals: np.ndarray  # float32 [nnz]
    B: np.ndarray  # float32 [K, N] row-major

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])

    def minimal_bytes(self) -> int:
        """A read once + rowptr + B read once + C written once."""
        return self.nnz * 8 + (self.M + 1) * 4 + self.K * self.N * 4 + self.M * self.N * 4

    def flops(self) -> int:
        return 2 * self.nnz * self.N

    def row_stats(self) -> dict:
        ln = np.diff(self.rowptr.astype(np.int64))
        return {
            "M": self.M,
            "K": self.K,
            "N": self.N,
            "nnz": self.nnz,
            "max_row": int(ln.max()) if ln.size else 0,
            "mean_row": float(ln.mean()) if ln.size else 0.0,
            "empty_rows": int((ln == 0).sum()),
        }


# --------------------------------------------------------------------------
# structure generators
# --------------------------------------------------------------------------

def _rowptr_from_lengths(lengths: np.ndarray) -> np.ndarray:
    rowptr = np.zeros(lengths.size + 1, dtype=np.int64)
    np.cumsum(lengths, out=rowptr[1:])
    if rowptr[-1] >= 2**31:
        raise ValueError("nnz does not fit int32")
    return rowptr.astype(np.int32)


def csr_from_lengths(rng: np.random.Generator, lengths: np.ndarray, K: int):
    """Rows of the given lengths, each with uniformly random *distinct* columns.

    Draw with replacement, drop duplicates, and top the short rows up with new
    draws until every row has its length.  The procedure is symmetric under
    any relabelling of the columns, so each row's column set is a uniform
    random subset of its size.  Returns (rowptr int32, colidx int32 sorted
    ascending inside each row).
    """
    lengths = np.asarray(lengths, dtype=np.int64)
    M = lengths.size
    if lengths.size and int(lengths.max()) > K:
        raise ValueError("row longer than K cannot have distinct columns")
    rows = np.repeat(np.arange(M, dtype=np.int64), lengths)
    keys = rows * K + rng.integers(0, K, size=rows.size, dtype=np.int64)
    del rows
    keys = np.unique(keys)
    while True:
        have = np.bincount(keys // K, minlength=M).astype(np.int64)
        deficit = lengths - have
        if not deficit.any():
            break
        r2 = np.repeat(np.arange(M, dtype=np.int64), deficit)
        k2 = r2 * K + rng.integers(0, K, size=r2.size, dtype=np.int64)
        keys = np.unique(np.concatenate([keys, k2]))
    colidx = (keys % K).astype(np.int32)
    return _rowptr_from_lengths(lengths), colidx


def uniform_fixed_degree(rng, M: int, K: int, degree: int):
    return csr_from_lengths(rng, np.full(M, degree, dtype=np.int64), K)


def _zipf_mandelbrot_shift(exponent: float, lo: int, hi: int, mean: float) -> float:
    """Shift q such that P(l) ~ (l+q)^-exponent on [lo,hi] has the given mean."""
    ell = np.arange(lo, hi + 1, dtype=np.float64)

    def m(q):
        w = (ell + q) ** (-exponent)
        return float((ell * w).sum() / w.sum())

    a, b = 0.0, 64.0
    for _ in range(80):
        mid = 0.5 * (a + b)
        if m(mid) < mean:
            a = mid
        else:
            b = mid
    return 0.5 * (a + b)


def powerlaw_rows(rng, M: int, K: int, exponent=2.1, lo=1, hi=4096, mean=16.0):
    """Row lengths from a truncated Zipf-Mandelbrot law, columns uniform distinct.

    A plain truncated Zipf(2.1) on [1,4096] has mean 4, not the ~16 the
    workload statement asks for; the shift q (about 2.84) restores mean 16
    while keeping min 1, max 4096 and the 2.1 tail exponent.
    """
    q = _zipf_mandelbrot_shift(exponent, lo, hi, mean)
    ell = np.arange(lo, hi + 1, dtype=np.float64)
    w = (ell + q) ** (-exponent)
    cdf = np.cumsum(w / w.sum())
    cdf[-1] = 1.0
    lengths = lo + np.searchsorted(cdf, rng.random(M), side="right")
    lengths = np.minimum(lengths, hi).astype(np.int64)
    return csr_from_lengths(rng, lengths, K)


def stencil27(n: int):
    """27-point stencil on an n^3 grid, natural ordering x + n*y + n^2*z,
    neighbours clipped at the faces (no wrap-around)."""
    M = n * n * n
    idx = np.arange(M, dtype=np.int64)
    x = idx % n
    y = (idx // n) % n
    z = idx // (n * n)
    cols = np.empty((M, 27), dtype=np.int32)
    mask = np.empty((M, 27), dtype=bool)
    j = 0
    for dz in (-1, 0, 1):
        okz = (z + dz >= 0) & (z + dz < n)
        for dy in (-1, 0, 1):
            oky = okz & (y + dy >= 0) & (y + dy < n)
            for dx in (-1, 0, 1):
                ok = oky & (x + dx >= 0) & (x + dx < n)
                mask[:, j] = ok
                cols[:, j] = (idx + dx + n * dy + n * n * dz).astype(np.int32)
                j += 1
    lengths = mask.sum(axis=1).astype(np.int64)
    colidx = cols[mask]  # row-major selection keeps ascending order per row
    return _rowptr_from_lengths(lengths), colidx


def rmat(rng, scale: int, raw_edges: int, a=0.57, b=0.19, c=0.19, d=0.05):
    """R-MAT edges (directed, self loops kept, no vertex permutation, no
    noise), duplicates removed.  One 16-bit uniform draw per level per edge
    picks the quadrant."""
    assert abs(a + b + c + d - 1.0) < 1e-9
    M = 1 << scale
    ta = int(round(a * 65536))
    tab = int(round((a + b) * 65536))
    tabc = int(round((a + b + c) * 65536))
    row = np.zeros(raw_edges, dtype=np.int64)
    col = np.zeros(raw_edges, dtype=np.int64)
    for _ in range(scale):
        u = rng.integers(0, 65536, size=raw_edges, dtype=np.uint16)
        rbit = u >= tab  # quadrants c, d: lower half of rows
        cbit = ((u >= ta) & (u < tab)) | (u >= tabc)  # quadrants b, d
        row = (row << 1) | rbit
        col = (col << 1) | cbit
    keys = np.unique((row << scale) | col)
    del row, col
    r = keys >> scale
    colidx = (keys & (M - 1)).astype(np.int32)
    lengths = np.bincount(r, minlength=M).astype(np.int64)
    return _rowptr_from_lengths(lengths), colidx


def skewed_rows(rng, M: int, K: int, heavy_frac=0.01, light=(1, 8), heavy=(2000, 20000)):
    """heavy_frac of the rows (at seeded uniformly random positions) are long,
    the rest are short; columns uniform distinct."""
    n_heavy = int(round(M * heavy_frac))
    lengths = rng.integers(light[0], light[1] + 1, size=M, dtype=np.int64)
    pos = rng.choice(M, size=n_heavy, replace=False)
    lengths[pos] = rng.integers(heavy[0], heavy[1] + 1, size=n_heavy, dtype=np.int64)
    lengths = np.minimum(lengths, K)
    return csr_from_lengths(rng, lengths, K)


# --------------------------------------------------------------------------
# values
# --------------------------------------------------------------------------

def fill_values(rng, n: int, integer: bool) -> np.ndarray:
    if integer:
        return rng.integers(-2, 3, size=n).astype(np.float32)
    return (rng.random(n, dtype=np.float32) * np.float32(2.0) - np.float32(1.0)).astype(np.float32)


def dense_operand(seed: int, K: int, N: int, integer: bool) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed))
    return fill_values(rng, K * N, integer).reshape(K, N)


# --------------------------------------------------------------------------
# the five named workloads
# --------------------------------------------------------------------------

# name -> (seed, default N)
WORKLOADS = {
    "uniform10": (1001, 32),
    "uniform10_int": (1001, 32),
    "powerlaw": (1002, 64),
    "stencil27": (1003, 128),
    "rmat": (1004, 32),
    "skewed": (1005, 256),
}

# one line per workload on how it is drawn (printed by the benchmark next to the measured statistics)
RECIPES = {
    "uniform10": "exactly 10 uniform distinct columns per row",
    "uniform10_int": "exactly 10 uniform distinct columns per row; values and B uniform on {-2..2}",
    "powerlaw": "row lengths Zipf-Mandelbrot P(l) ~ (l+q)^-2.1 on [1,4096] with the shift q = %.3f that gives mean 16 "
                "(a plain Zipf(2.1) has mean 4); columns uniform distinct",
    "stencil27": "27-point stencil on a cube in natural order, faces clipped; random values",
    "rmat": "R-MAT (0.57, 0.19, 0.19, 0.05), no permutation, no noise, self loops kept, duplicates removed",
    "skewed": "1 % of the rows, at seeded random positions, hold 2,000-20,000 entries, the rest 1-8; columns uniform distinct",
}


def recipe(name: str) -> str:
    text = RECIPES[name]
    return text % _zipf_mandelbrot_shift(2.1, 1, 4096, 16.0) if "%.3f" in text else text


# raw R-MAT edge count whose de-duplicated size is 50M +- 2% at scale 21
RMAT_SCALE = 21
RMAT_RAW_EDGES = 52_300_000


def make_problem(name: str, N: int | None = None, scale_down: int = 1) -> SpmmProblem:
    """Build a named workload.  `scale_down` > 1 shrinks M (and the R-MAT edge
    count / stencil edge) for quick tests while keeping the row-length law."""
    if name not in WORKLOADS:
        raise KeyError(f"unknown workload {name!r}; have {sorted(WORKLOADS)}")
    seed, defN = WORKLOADS[name]
    N = defN if N is None else int(N)
    rng = np.random.Generator(np.random.PCG64(seed))
    integer = name.endswith("_int")
    if name.startswith("uniform10"):
        M = K = max(16, 1024 // scale_down)
        rowptr, colidx = uniform_fixed_degree(rng, M, K, 10)
    elif name == "powerlaw":
        M = K = max(4096, 65536 // scale_down)
        rowptr, colidx = powerlaw_rows(rng, M, K)
    elif name == "stencil27":
        n = max(4, int(round(100 / scale_down ** (1 / 3))))
        rowptr, colidx = stencil27(n)
        M = K = n ** 3
    elif name == "rmat":
        sc = RMAT_SCALE
        raw = RMAT_RAW_EDGES
        s = scale_down
        while s > 1:
            sc -= 1
            raw //= 2
            s //= 2
        rowptr, colidx = rmat(rng, sc, raw)
        M = K = 1 << sc
    elif name == "skewed":
        M = K = max(20000, 500000 // scale_down)
        hi = min(20000, K // 8)  # shrunken copies keep long rows well below K
        rowptr, colidx = skewed_rows(rng, M, K, heavy=(min(2000, hi // 10), hi))
    else:  # pragma: no cover
        raise AssertionError(name)
    vals = fill_values(rng, int(rowptr[-1]), integer)
    B = dense_operand(seed + 100, K, N, integer)
    return SpmmProblem(name, M, K, N, rowptr, colidx, vals, B)


def sddmm_left_operand(p: SpmmProblem, integer: bool | None = None) -> np.ndarray:
    """The M x J dense operand X1 of an SDDMM on problem p's pattern (J = p.N;
    the K x J operand X2T is p.B).  Seeded per workload (seed + 200)."""
    seed, _ = WORKLOADS[p.name]
    if integer is None:
        integer = p.name.endswith("_int")
    return dense_operand(seed + 200, p.M, p.N, integer)


def sddmm_minimal_bytes(p: SpmmProblem) -> int:
    """colidx, vals read once, out written once, rowptr, X1 and X2T read once."""
    return p.nnz * 12 + (p.M + 1) * 4 + p.M * p.N * 4 + p.K * p.N * 4


# --------------------------------------------------------------------------
# third-order tensors (MTTKRP, TTM)
# --------------------------------------------------------------------------

@dataclass
class Tensor3Problem:
    """A third-order sparse tensor A[I, K, L] as compressed sparse fibers plus
    the dense operands of MTTKRP and TTM (inputs only).

    Slice i (first index, dense) owns the fibers fptr[i] .. fptr[i+1]-1; fiber
    f has second index fidx[f] and owns the entries eptr[f] .. eptr[f+1]-1;
    entry p has third index eidx[p] and value vals[p].  Second indices are
    sorted and distinct inside a slice, third indices inside a fiber; no fiber
    is empty, slices may be.  X1 is [K, J] and X2 is [L, J] (MTTKRP:
    Y[i,j] = sum A[i,k,l] X1[k,j] X2[l,j]); for TTM along the third index the
    dense operand is X2 (Y[i,k,:] = sum_l A[i,k,l] X2[l,:]).
    """

    name: str
    I: int
    K: int
    L: int
    J: int
    fptr: np.ndarray  # int32 [I+1]
    fidx: np.ndarray  # int32 [F]
    eptr: np.ndarray  # int32 [F+1]
    eidx: np.ndarray  # int32 [E]
    vals: np.ndarray  # float32 [E]
    X1: np.ndarray  # float32 [K, J]
    X2: np.ndarray  # float32 [L, J]

    @property
    def fibers(self) -> int:
        return int(self.fptr[-1])

    @property
    def nnz(self) -> int:
        return int(self.eptr[-1])

    def mttkrp_minimal_bytes(self) -> int:
        """entries, fibers and slice pointers read once, both factor matrices read once, Y written once."""
        return (self.nnz * 8 + self.fibers * 8 + 4 + (self.I + 1) * 4
                + (self.K + self.L) * self.J * 4 + self.I * self.J * 4)

    def mttkrp_flops(self) -> int:
        """one multiply-add per entry and column, one more per fiber and column"""
        return 2 * self.J * (self.nnz + self.fibers)

    def stats(self) -> dict:
        fl = np.diff(self.fptr.astype(np.int64))
        el = np.diff(self.eptr.astype(np.int64))
        return {
            "I": self.I, "K": self.K, "L": self.L, "J": self.J, "fibers": self.fibers, "nnz": self.nnz,
            "max_fibers_per_slice": int(fl.max()) if fl.size else 0,
            "empty_slices": int((fl == 0).sum()),
            "max_entries_per_fiber": int(el.max()) if el.size else 0,
        }


# name -> (seed, I, K, L, J, mean fibers per slice, longest fiber)
TENSOR_WORKLOADS = {
    "tensor3_small": (2001, 512, 256, 320, 32, 4.0, 12),
    "tensor3_small_int": (2001, 512, 256, 320, 32, 4.0, 12),
    "tensor3": (2002, 262_144, 65_536, 65_536, 32, 8.0, 16),
    "tensor3_skewed": (2003, 262_144, 65_536, 65_536, 32, 4.0, 16),
}
# name -> (share of the slices that are heavy, their fewest and most fibers): slices that differ in size by four
# orders of magnitude, the case the nnz-balanced schedule is for
TENSOR_HEAVY_SLICES = {"tensor3_skewed": (0.001, 2_000, 20_000)}


def make_tensor3(name: str, J: int | None = None) -> Tensor3Problem:
    """Seeded random tensor: the number of fibers of a slice is geometric with
    the given mean, minus one with probability 1/8 (so some slices are empty and
    a few are many times longer than the mean; tensor3_skewed: one slice in a thousand
    has 2,000 to 20,000 fibers instead); a fiber holds 1 .. longest entries,
    uniformly; second and third indices are uniform distinct subsets."""
    if name not in TENSOR_WORKLOADS:
        raise KeyError(f"unknown tensor workload {name!r}; have {sorted(TENSOR_WORKLOADS)}")
    seed, I, K, L, defJ, mean_fibers, longest = TENSOR_WORKLOADS[name]
    J = defJ if J is None else int(J)
    integer = name.endswith("_int")
    rng = np.random.Generator(np.random.PCG64(seed))
    fibers = rng.geometric(1.0 / mean_fibers, size=I).astype(np.int64)
    fibers -= rng.random(I) < 0.125
    if name in TENSOR_HEAVY_SLICES:
        share, fewest, most = TENSOR_HEAVY_SLICES[name]
        heavy = rng.random(I) < share
        fibers[heavy] = rng.integers(fewest, most + 1, size=int(heavy.sum()))
    fibers = np.minimum(fibers, K)
    fptr, fidx = csr_from_lengths(rng, fibers, K)
    entries = rng.integers(1, longest + 1, size=int(fptr[-1])).astype(np.int64)
    eptr, eidx = csr_from_lengths(rng, entries, L)
    vals = fill_values(rng, int(eptr[-1]), integer)
    X1 = dense_operand(seed + 100, K, J, integer)
    X2 = dense_operand(seed + 200, L, J, integer)
    return Tensor3Problem(name, I, K, L, J, fptr, fidx, eptr, eidx, vals, X1, X2)
