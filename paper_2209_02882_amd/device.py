"""Device-side plumbing for tests and the benchmark: upload a problem into
HBM (torch tensors as device memory) and run one design-space point through
the C ABI.  No arithmetic of the method lives here."""
from __future__ import annotations

import torch

from . import binding

# every (group_size, strategy, schedule) point of the design space
POINTS = [(g, st, sc) for sc in ("row_split", "nnz_balanced") for st in ("parallel", "serial")
          for g in binding.GROUP_SIZES]
# the points {<1/g row, c col>, r} with the reduction narrower than the tiling
GR_POINTS = [(g, r) for g in binding.GROUP_SIZES for r in binding.GROUP_SIZES if r < g]


class DeviceProblem:
    """`arena=True` puts rowptr, colidx, vals, B and one C into ONE device allocation, packed one after the
    other at 512-byte boundaries.  Results do not depend on it; the time of kernels that gather at random
    does (one mapping for the translation caches instead of five, and streams that are read in step do not
    start at the same offset of a 2-MiB page): R-MAT 0.86 ms with five allocations, 0.75 ms in one
    allocation at 2-MiB boundaries, 0.70 ms packed."""

    def __init__(self, p, device="cuda:0", arena=False):
        self.p = p
        dev = torch.device(device)
        self._C = None
        hosts = [("rowptr", p.rowptr), ("colidx", p.colidx), ("vals", p.vals), ("B", p.B)]
        if not arena:
            for name, h in hosts:
                setattr(self, name, torch.from_numpy(h).to(dev))
            return
        align = 512
        sizes = [h.nbytes for _, h in hosts] + [p.M * p.N * 4]
        offsets, end = [], 0
        for nb in sizes:
            offsets.append(end)
            end = (end + nb + align - 1) // align * align
        self.arena = torch.empty(max(end, align), dtype=torch.uint8, device=dev)
        for (name, h), off in zip(hosts, offsets):
            t = self.arena[off:off + h.nbytes].view(torch.from_numpy(h).dtype).view(h.shape)
            t.copy_(torch.from_numpy(h))
            setattr(self, name, t)
        self._C = self.arena[offsets[4]:offsets[4] + sizes[4]].view(torch.float32).view(p.M, p.N)

    def new_output(self, poison=False):
        """A C for this problem: the arena's own the first time it is asked for, a fresh tensor otherwise."""
        if self._C is not None:
            C, self._C = self._C, None
        else:
            C = torch.empty((self.p.M, self.p.N), dtype=torch.float32, device=self.rowptr.device)
        if poison:
            C.fill_(float("nan"))
        return C

    def launch(self, C, group, strategy, schedule, nnz_hint=None, stream=None):
        """Enqueue C = A*B for one point (asynchronous)."""
        p = self.p
        binding.sgap_spmm_csr_ex(p.M, p.K, p.N, self.rowptr, self.colidx, self.vals, self.B, C,
                                 group, binding.STRATEGIES[strategy], binding.SCHEDULES[schedule],
                                 nnz_hint=nnz_hint, stream=stream)

    def workspace_for(self, config):
        """Device workspace (uint8 tensor) of the size the configuration needs, or None."""
        p = self.p
        size = binding.sgap_spmm_csr_workspace_size(p.M, p.K, p.N, config)
        return torch.empty(size, dtype=torch.uint8, device=self.rowptr.device) if size else None

    def launch_cfg(self, C, config, workspace=None, nnz_hint=None, stream=None):
        """Enqueue C = A*B for one configuration (asynchronous)."""
        p = self.p
        binding.sgap_spmm_csr_cfg(p.M, p.K, p.N, self.rowptr, self.colidx, self.vals, self.B, C, config,
                                  nnz_hint=nnz_hint, workspace=workspace, stream=stream)

    def run_cfg(self, config, workspace=None, poison=True, C=None):
        if C is None:
            C = self.new_output()
        if poison:
            C.fill_(float("nan"))
        if workspace is None:
            workspace = self.workspace_for(config)
        self.launch_cfg(C, config, workspace)
        torch.cuda.synchronize()
        return C

    def launch_gr(self, C, group, reduce_size, nnz_hint=None, stream=None):
        """Enqueue the row-split point with `group` lanes per row reducing in
        sub-groups of `reduce_size` lanes (asynchronous)."""
        p = self.p
        binding.sgap_spmm_csr_gr(p.M, p.K, p.N, self.rowptr, self.colidx, self.vals, self.B, C,
                                 group, reduce_size, nnz_hint=nnz_hint, stream=stream)

    def run_gr(self, group, reduce_size, poison=True):
        C = self.new_output(poison)
        self.launch_gr(C, group, reduce_size)
        torch.cuda.synchronize()
        return C

    def launch_sddmm(self, X1, out, group, strategy, nnz_hint=None, stream=None):
        """Enqueue out[p] = vals[p] * <X1[row(p)], B[colidx[p]]> (B serves as the
        transposed second dense operand); asynchronous."""
        p = self.p
        binding.sgap_sddmm_csr(p.M, p.K, p.N, self.rowptr, self.colidx, self.vals, X1, self.B, out,
                               group, binding.STRATEGIES[strategy], nnz_hint=nnz_hint, stream=stream)

    def run_sddmm_windows(self, X1, group, strategy, long_row_min, window_kb=0, max_long_rows=0, poison=True):
        p = self.p
        out = torch.empty(p.nnz, dtype=torch.float32, device=self.rowptr.device)
        if poison:
            out.fill_(float("nan"))
        size = binding.sgap_sddmm_csr_workspace_size(p.K, p.N, window_kb, max_long_rows)
        ws = torch.empty(size, dtype=torch.uint8, device=self.rowptr.device) if size else None
        binding.sgap_sddmm_csr_windows(p.M, p.K, p.N, self.rowptr, self.colidx, self.vals, X1, self.B, out, group,
                                       binding.STRATEGIES[strategy], long_row_min, window_kb, max_long_rows,
                                       workspace=ws)
        torch.cuda.synchronize()
        return out

    def run_sddmm(self, X1, group, strategy, poison=True):
        out = torch.empty(self.p.nnz, dtype=torch.float32, device=self.rowptr.device)
        if poison:
            out.fill_(float("nan"))
        self.launch_sddmm(X1, out, group, strategy)
        torch.cuda.synchronize()
        return out

    def run(self, group, strategy, schedule, poison=True, C=None, nnz_hint=None):
        """Run one point to completion; by default C starts filled with NaN so
        that any element the kernels fail to write is visible."""
        if C is None:
            C = self.new_output()
        if poison:
            C.fill_(float("nan"))
        self.launch(C, group, strategy, schedule, nnz_hint=nnz_hint)
        torch.cuda.synchronize()
        return C


class DeviceTensor3:
    """A Tensor3Problem uploaded into HBM, with launchers for MTTKRP and for TTM
    along the third index."""

    def __init__(self, p, device="cuda:0"):
        self.p = p
        dev = torch.device(device)
        for name in ("fptr", "fidx", "eptr", "eidx", "vals", "X1", "X2"):
            setattr(self, name, torch.from_numpy(getattr(p, name)).to(dev))

    def launch_mttkrp(self, Y, group, strategy, schedule="row_split", stream=None):
        p = self.p
        binding.sgap_mttkrp_csf_ex(p.I, p.K, p.L, p.J, self.fptr, self.fidx, self.eptr, self.eidx, self.vals,
                                   self.X1, self.X2, Y, group, binding.STRATEGIES[strategy],
                                   binding.SCHEDULES[schedule], stream=stream)

    def run_mttkrp(self, group, strategy, schedule="row_split", poison=True):
        Y = torch.empty((self.p.I, self.p.J), dtype=torch.float32, device=self.fptr.device)
        if poison:
            Y.fill_(float("nan"))
        self.launch_mttkrp(Y, group, strategy, schedule)
        torch.cuda.synchronize()
        return Y

    def launch_ttm(self, Yf, group, strategy, schedule, stream=None):
        """Yf[f, :] = sum over fiber f's entries of vals * X2[eidx, :] (X2 serves as TTM's dense operand)."""
        p = self.p
        binding.sgap_ttm_csf(p.fibers, p.L, p.J, self.eptr, self.eidx, self.vals, self.X2, Yf, group,
                             binding.STRATEGIES[strategy], binding.SCHEDULES[schedule], stream=stream)

    def run_ttm(self, group, strategy, schedule, poison=True):
        Yf = torch.empty((self.p.fibers, self.p.J), dtype=torch.float32, device=self.fptr.device)
        if poison:
            Yf.fill_(float("nan"))
        self.launch_ttm(Yf, group, strategy, schedule)
        torch.cuda.synchronize()
        return Yf
