"""Device-memory helpers on top of torch (allocation, upload, streams) -- plumbing, no arithmetic.

Matrices handed to the library are column-major.  A column-major m x n FP64 matrix with leading dimension
m is represented by a contiguous torch tensor of shape (n, m): tensor[j, i] = M(i, j).
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding


def to_device_colmajor(M: np.ndarray) -> torch.Tensor:
    """numpy (rows, cols) array -> device tensor of shape (cols, rows) holding it column-major."""
    return torch.from_numpy(np.ascontiguousarray(M.T)).to("cuda")


def from_device_colmajor(T: torch.Tensor) -> np.ndarray:
    return T.cpu().numpy().T


class Workspace:
    """Owns the library's work memory (allocated once, outside any timed region) and binds the current stream."""

    def __init__(self, nbytes: int):
        self.buf = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda")
        assert self.buf.data_ptr() % 256 == 0
        binding.ozaki_set_stream(torch.cuda.current_stream().cuda_stream)
        binding.ozaki_set_workspace(self.buf, self.buf.numel())

    @classmethod
    def for_problem(cls, m, n, k, slice_format, num_slices, k_block, minimum: bool = False, scaled: bool = False,
                    pair_set: int = binding.PAIRS_TRIANGLE) -> "Workspace":
        if scaled:
            nbytes = binding.ozaki_workspace_bytes_scaled(m, n, k, slice_format, num_slices, k_block)
        else:
            nbytes = binding.ozaki_workspace_bytes_ex(m, n, k, slice_format, num_slices, k_block, pair_set, minimum)
        if nbytes == 0 and m and n and k:
            raise ValueError("infeasible or invalid problem")
        return cls(nbytes)

    def close(self):
        binding.ozaki_set_workspace(None, 0)
        self.buf = None
