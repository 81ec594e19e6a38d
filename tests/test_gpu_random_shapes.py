"""Seeded random shapes, row-length mixes and tuning knobs against the oracle:
every SpMM point, a third of the (g, r) points and every SDDMM point per case,
exact on integer-valued inputs."""
import numpy as np
import pytest
import torch

import oracle
from paper_2209_02882_amd import binding
from paper_2209_02882_amd import workloads as wl

from gpu_util import GR_POINTS, POINTS, DeviceProblem

pytestmark = pytest.mark.gpu


def draw_case(seed):
    rng = np.random.default_rng(seed)
    M = int(rng.choice([1, 2, 7, 63, 64, 65, 300, 1025, 5000]))
    K = int(rng.choice([1, 5, 64, 1000, 70000]))
    N = int(rng.choice([1, 2, 4, 5, 8, 12, 16, 32, 36, 64, 100, 128, 200, 256, 384]))
    kind = str(rng.choice(["short", "mixed", "long", "empty_heavy"]))
    if kind == "short":
        ln = rng.integers(0, 6, M)
    elif kind == "mixed":
        ln = np.where(rng.random(M) < 0.05, rng.integers(100, 3000, M), rng.integers(0, 20, M))
    elif kind == "long":
        ln = rng.integers(500, 5000, M) if M <= 300 else rng.integers(0, 60, M)
    else:
        ln = np.where(rng.random(M) < 0.9, 0, rng.integers(1, 400, M))
    ln = np.minimum(ln, K)
    rowptr, colidx = wl.csr_from_lengths(rng, ln.astype(np.int64), K)
    vals = wl.fill_values(rng, colidx.size, True)
    B = wl.fill_values(rng, K * N, True).reshape(K, N)
    # per-call knobs of sgap_spmm_csr_cfg (drawn in this order, so that a seed keeps its case)
    knobs = {
        "nnz_tile": int(rng.choice([0, 0, 256, 512, 2048])),
        "long_row_min": int(rng.choice([0, 0, 50, 1000])),
        "window_kb": int(rng.choice([0, 1, 16])),
    }
    knobs["block_size"] = int(rng.choice([0, 128, 256, 512]))
    knobs["max_long_rows"] = int(rng.choice([0, 3, 700]))
    X1 = wl.fill_values(rng, M * N, True).reshape(M, N)
    return wl.SpmmProblem(f"random {kind}", M, K, N, rowptr, colidx, vals, B), X1, knobs


@pytest.mark.parametrize("seed", range(100, 148))
def test_random_case(seed):
    p, X1, knobs = draw_case(seed)
    print(f"seed {seed}: {p.name} M={p.M} K={p.K} N={p.N} nnz={p.nnz} knobs={knobs}", flush=True)
    C_ref, _ = oracle.spmm_csr(p.M, p.K, p.N, p.rowptr, p.colidx, p.vals, p.B, nthreads=8, bound=False)
    dp = DeviceProblem(p)
    C = dp.new_output()
    for pt in POINTS:
        cfg = binding.make_config(*pt, **knobs)
        ws = dp.workspace_for(cfg)
        for hint in (None, -1):  # the host knows the number of stored entries, or does not
            C.fill_(float("nan"))
            dp.launch_cfg(C, cfg, ws, nnz_hint=hint)
            got = C.cpu().numpy().astype(np.float64)
            assert np.array_equal(got, C_ref), f"seed {seed} {pt} nnz_hint={hint}"
    for g, r in GR_POINTS[::3]:
        got = dp.run_cfg(binding.make_config(g, "parallel", "row_split", reduce_size=r, block_size=knobs["block_size"]))
        assert np.array_equal(got.cpu().numpy().astype(np.float64), C_ref), f"seed {seed} g={g} r={r}"
    if p.nnz:
        ref, _ = oracle.sddmm_csr(p.M, p.K, p.N, p.rowptr, p.colidx, p.vals, X1, p.B, nthreads=8, bound=False)
        X1d = torch.from_numpy(X1).cuda()
        for st in ("parallel", "serial"):
            for g in binding.GROUP_SIZES:
                got = dp.run_sddmm_windows(X1d, g, st, knobs["long_row_min"], knobs["window_kb"],
                                           knobs["max_long_rows"]).cpu().numpy().astype(np.float64)
                assert np.array_equal(got, ref), f"seed {seed} sddmm g={g} {st}"
