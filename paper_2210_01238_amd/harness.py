"""Small convenience layer over the binding for tests, the smoke check and the
benchmark: owns device buffers (PyTorch is used for device memory and streams
only) and moves padded global arrays in and out.  No arithmetic happens here.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

from . import binding as B

_TORCH_DT = {np.dtype(np.float64): torch.float64, np.dtype(np.float32): torch.float32}
_J_DT = {np.dtype(np.float64): B.JACOBI_F64, np.dtype(np.float32): B.JACOBI_F32}


# Options every JacobiRun starts with (explicit keyword options override them).  Empty: the library's defaults.
DEFAULT_OPTIONS: dict = {}


def _stream() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


class JacobiRun:
    """A plan plus two ping-pong grids on the current CUDA (HIP) device."""

    def __init__(self, dims: Sequence[int], tiles: Sequence[int], dtype=np.float64, **options: int):
        if not torch.cuda.is_available():
            raise RuntimeError("libjacobi needs a GPU; there is no CPU path")
        self.dims = tuple(int(d) for d in dims)
        self.tiles = tuple(int(t) for t in tiles)
        self.np_dtype = np.dtype(dtype)
        self.plan = B.jacobi_create(self.dims, self.tiles, _J_DT[self.np_dtype])
        for k, v in {**DEFAULT_OPTIONS, **options}.items():
            B.jacobi_set_option(self.plan, k, v)
        self.nbytes = B.jacobi_grid_bytes(self.plan)
        # contents deliberately left uninitialised: padding and stale halos may hold anything
        self.a = torch.empty(self.nbytes, dtype=torch.uint8, device="cuda")
        self.b = torch.empty(self.nbytes, dtype=torch.uint8, device="cuda")
        self.cur = self.a
        self.padded_shape = tuple(d + 2 for d in self.dims)

    # -- data movement -------------------------------------------------------
    def other(self) -> torch.Tensor:
        return self.b if self.cur is self.a else self.a

    def load(self, padded: np.ndarray) -> None:
        """Upload a padded global array and scatter it into the current grid."""
        assert padded.shape == self.padded_shape and padded.dtype == self.np_dtype
        g = torch.from_numpy(np.ascontiguousarray(padded)).cuda()
        self.load_device(g)

    def load_device(self, g: torch.Tensor) -> None:
        assert g.is_cuda and g.is_contiguous() and tuple(g.shape) == self.padded_shape
        assert g.dtype == _TORCH_DT[self.np_dtype]
        self.cur = self.a
        B.jacobi_scatter(self.plan, g.data_ptr(), self.cur.data_ptr(), _stream())
        torch.cuda.current_stream().synchronize()  # g may be freed by the caller afterwards

    def fetch_device(self) -> torch.Tensor:
        g = torch.empty(self.padded_shape, dtype=_TORCH_DT[self.np_dtype], device="cuda")
        B.jacobi_gather(self.plan, self.cur.data_ptr(), g.data_ptr(), _stream())
        return g

    def fetch(self) -> np.ndarray:
        return self.fetch_device().cpu().numpy()

    # -- the hot path ----------------------------------------------------------
    def sweep(self, iters: int) -> None:
        fin = B.jacobi_sweep(self.plan, self.cur.data_ptr(), self.other().data_ptr(), iters, _stream())
        self.cur = self.a if fin == self.a.data_ptr() else self.b

    def sweep_tasks(self, iters: int, tiles_per_task: int, nstreams: int) -> None:
        """sweep(iters) executed as per-tile-group tasks over several streams."""
        fin = B.jacobi_sweep_tasks(self.plan, self.cur.data_ptr(), self.other().data_ptr(), iters,
                                   tiles_per_task, nstreams, _stream())
        self.cur = self.a if fin == self.a.data_ptr() else self.b

    def sweep_residual(self, iters: int, out: torch.Tensor) -> None:
        """sweep(iters), and `out` (1-element float64 CUDA tensor) receives the residual norm
        of the field as it was BEFORE these iterations."""
        fin = B.jacobi_sweep_residual(self.plan, self.cur.data_ptr(), self.other().data_ptr(), iters,
                                      out.data_ptr(), _stream())
        self.cur = self.a if fin == self.a.data_ptr() else self.b

    def exchange(self) -> None:
        B.halo_exchange(self.plan, self.cur.data_ptr(), _stream())

    def residual(self) -> float:
        return B.residual_norm_host(self.plan, self.cur.data_ptr(), _stream())

    def residual_async(self, out: torch.Tensor) -> None:
        """out: a 1-element float64 CUDA tensor that receives the norm."""
        B.residual_norm(self.plan, self.cur.data_ptr(), out.data_ptr(), _stream())

    def run(self, iters: int, residual_every: int = 0, fuse_residual: bool = False) -> List[float]:
        """iters iterations with a residual after every residual_every-th one.

        fuse_residual: the whole schedule as ONE jacobi_run call (each residual but the last is
        then taken from the first update of the NEXT block of iterations instead of a stand-alone
        reduction pass) - what the benchmark times; otherwise jacobi_sweep / residual_norm pairs."""
        res: List[float] = []
        if residual_every <= 0:
            self.sweep(iters)
            return res
        nres = iters // residual_every
        dev = torch.zeros(max(nres, 1), dtype=torch.float64, device="cuda")
        if fuse_residual:
            # the library's own schedule: one call
            fin = B.jacobi_run(self.plan, self.cur.data_ptr(), self.other().data_ptr(), iters, residual_every,
                               dev.data_ptr(), _stream())
            self.cur = self.a if fin == self.a.data_ptr() else self.b
        else:
            done = 0
            while done < iters:
                n = min(residual_every, iters - done)
                self.sweep(n)
                done += n
                if done % residual_every == 0:
                    k = done // residual_every - 1
                    self.residual_async(dev[k:k + 1])
        torch.cuda.current_stream().synchronize()
        return dev[:nres].cpu().tolist()

    def set_option(self, key: str, value: int) -> None:
        B.jacobi_set_option(self.plan, key, value)

    def close(self) -> None:
        if self.plan is not None:
            torch.cuda.synchronize()
            B.jacobi_destroy(self.plan)
            self.plan = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
