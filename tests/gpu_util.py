"""Helpers shared by the GPU parity tests: compare device results with the
CPU oracle."""
import numpy as np
import torch

import oracle
from paper_2209_02882_amd.device import GR_POINTS, POINTS, DeviceProblem  # noqa: F401

TOL = 1e-5  # |C - C_ref| <= TOL * (|A| |B|) elementwise, fp32 atomics reorder sums

def full_reference(p):
    return oracle.spmm_csr(p.M, p.K, p.N, p.rowptr, p.colidx, p.vals, p.B, nthreads=8)


def assert_close(C_gpu, C_ref, BND, exact=False, what=""):
    """exact: compare as IEEE values (so -0 == +0); else the fp32 tolerance."""
    got = C_gpu.detach().cpu().numpy().astype(np.float64)
    assert not np.isnan(got).any(), f"{what}: NaN left in C (element never written)"
    if exact:
        bad = got != C_ref
    else:
        bad = np.abs(got - C_ref) > TOL * BND
    if bad.any():
        i, k = np.argwhere(bad)[0]
        raise AssertionError(
            f"{what}: {int(bad.sum())} elements off; first at ({i},{k}): got {got[i, k]!r}, "
            f"want {C_ref[i, k]!r}, bound {BND[i, k]!r}")


def sample_rows(p, n_random=2000, n_longest=40, seed=0):
    ln = np.diff(p.rowptr.astype(np.int64))
    rng = np.random.default_rng(seed)
    rows = set(rng.integers(0, p.M, size=n_random).tolist())
    rows.update(np.argsort(ln)[-n_longest:].tolist())
    rows.update([0, 1, p.M - 2, p.M - 1])
    empty = np.nonzero(ln == 0)[0][:50]
    rows.update(empty.tolist())
    return np.array(sorted(rows), dtype=np.int64)
