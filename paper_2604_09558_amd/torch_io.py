"""PyTorch as plumbing: device memory for sources, outputs and index tables.

Nothing here computes: arrays of stored bits go to the GPU unchanged and come back unchanged.
"""
from __future__ import annotations

import numpy as np
import torch

TORCH_DTYPE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def to_device(arr: np.ndarray, dtype: str, device="cuda:0") -> torch.Tensor:
    """Stored bits (float32 / float16 / uint16-for-bf16) -> device tensor of the same bits."""
    arr = np.ascontiguousarray(arr)
    if dtype == "bf16":
        assert arr.dtype == np.uint16
        return torch.from_numpy(arr.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(arr).to(device)


def to_host_bits(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> numpy array of stored bits (uint16 for bf16)."""
    t = t.detach().contiguous().cpu()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def to_host_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


class DeviceWorkload:
    """Sources and index tables of a workload resident on the GPU, plus the specs the
    descriptor builder needs (shape, dtype, device address)."""

    def __init__(self, wl, device="cuda:0", share=None):
        """`share`: another DeviceWorkload whose device tensors are used for the sources of the
        same name (two stages of one pipeline working on the same buffers)."""
        self.wl = wl
        self.device = device
        shared = share.tensors if share is not None else {}
        self.tensors = {k: shared[k] if k in shared else to_device(v, wl.dtype, device) for k, v in wl.sources.items()}
        self.tables = {k: torch.from_numpy(np.ascontiguousarray(v, dtype=np.int32)).to(device)
                       for k, v in wl.index_tables.items()}

    def specs(self):
        return {k: (tuple(t.shape), self.wl.dtype, t.data_ptr()) for k, t in self.tensors.items()}

    def table_ptrs(self):
        return {k: t.data_ptr() for k, t in self.tables.items()}

    def build(self, result: str):
        from . import binding
        return binding.build_chain(self.wl.chain, self.specs(), result, self.wl.index_tables, self.table_ptrs())

    def empty(self, shape, dtype=None):
        return torch.empty(tuple(int(s) for s in shape), dtype=TORCH_DTYPE[dtype or self.wl.dtype], device=self.device)
