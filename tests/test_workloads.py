"""The seeded input generators: structure and reproducibility (CPU only)."""
import numpy as np
import pytest

from paper_2209_02882_amd import workloads as wl


def check_csr(p):
    assert p.rowptr.dtype == np.int32 and p.colidx.dtype == np.int32
    assert p.vals.dtype == np.float32 and p.B.dtype == np.float32
    assert p.rowptr[0] == 0 and p.rowptr.shape == (p.M + 1,)
    ln = np.diff(p.rowptr.astype(np.int64))
    assert (ln >= 0).all()
    assert p.colidx.shape == (p.nnz,) and p.vals.shape == (p.nnz,)
    assert p.colidx.min() >= 0 and p.colidx.max() < p.K
    # sorted ascending and distinct inside each row
    d = np.diff(p.colidx.astype(np.int64))
    row_start = np.zeros(p.nnz, dtype=bool)
    starts = p.rowptr[:-1][ln > 0]
    row_start[starts] = True
    assert (d[~row_start[1:]] > 0).all()
    assert p.B.shape == (p.K, p.N) and p.B.flags["C_CONTIGUOUS"]
    return ln


def test_uniform10():
    p = wl.make_problem("uniform10")
    ln = check_csr(p)
    assert p.M == p.K == 1024 and p.N == 32 and (ln == 10).all() and p.nnz == 10240
    assert p.vals.min() >= -1 and p.vals.max() < 1
    q = wl.make_problem("uniform10")
    assert np.array_equal(p.colidx, q.colidx) and np.array_equal(p.vals, q.vals) and np.array_equal(p.B, q.B)


def test_uniform10_integer_variant():
    p = wl.make_problem("uniform10_int")
    check_csr(p)
    assert set(np.unique(p.vals)) <= {-2.0, -1.0, 0.0, 1.0, 2.0}
    assert set(np.unique(p.B)) <= {-2.0, -1.0, 0.0, 1.0, 2.0}


def test_powerlaw_row_length_law():
    p = wl.make_problem("powerlaw")
    ln = check_csr(p)
    assert p.M == 65536 and p.N == 64
    assert ln.min() >= 1 and ln.max() <= 4096
    assert 14.0 < ln.mean() < 18.5
    assert 0.2 < (ln == 1).mean() < 0.3


def test_stencil_small_and_count_formula():
    rowptr, colidx = wl.stencil27(6)
    ln = np.diff(rowptr)
    assert rowptr[-1] == (3 * 6 - 2) ** 3
    assert set(np.unique(ln)) == {8, 12, 18, 27}
    # interior point 1+6+36: neighbours are the 27 offsets
    i = 1 + 6 + 36
    got = colidx[rowptr[i]:rowptr[i + 1]]
    want = sorted(i + dx + 6 * dy + 36 * dz for dz in (-1, 0, 1) for dy in (-1, 0, 1) for dx in (-1, 0, 1))
    assert list(got) == want


def test_rmat_small():
    p = wl.make_problem("rmat", scale_down=64)
    ln = check_csr(p)
    assert p.M == 1 << 15
    assert (ln == 0).sum() > 0 and ln.max() > 50 * max(1.0, ln.mean())


def test_skewed_small():
    p = wl.make_problem("skewed", scale_down=25)
    ln = check_csr(p)
    heavy = ln >= 250
    assert heavy.sum() == round(p.M * 0.01)
    assert ln[~heavy].min() >= 1 and ln[~heavy].max() <= 8
    assert ln[heavy].max() <= 2500


def test_distinct_columns_when_rows_are_nearly_full():
    rng = np.random.default_rng(0)
    rowptr, colidx = wl.csr_from_lengths(rng, np.array([5, 0, 4, 5]), 5)
    assert list(np.diff(rowptr)) == [5, 0, 4, 5]
    assert list(colidx[:5]) == [0, 1, 2, 3, 4]
    with pytest.raises(ValueError):
        wl.csr_from_lengths(rng, np.array([6]), 5)


def test_every_workload_has_a_recipe_line():
    for name in wl.WORKLOADS:
        assert isinstance(wl.recipe(name), str) and wl.recipe(name)
    assert "2.838" in wl.recipe("powerlaw")
