"""Glue between the synthetic workloads and the library binding: device tensors for a kernel."""
from __future__ import annotations

import numpy as np

from . import api
from . import workloads as wl


def to_device(arr: np.ndarray, dtype: int):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(arr)).cuda()
    return t.to(torch.bfloat16) if dtype == wl.BF16 else t


def output_shape(kernel: wl.Kernel):
    s = kernel.shape
    if kernel.is_conv():
        return (s.n, s.k, s.ho, s.wo)
    if kernel.cls == wl.CLS_BATCH_MATMUL:
        return (s.batch, s.m, s.n)
    return (s.m, s.n)


def max_workspace_bytes(kernel: wl.Kernel, max_split: int = 32) -> int:
    b, m, n, _ = kernel.gemm_extents()
    if kernel.cls == wl.CLS_DWCONV_BIAS_RELU6:
        return 0
    return 4 * max_split * b * m * n


def device_kernel(kernel: wl.Kernel, seed: int, inputs: dict | None = None, max_split: int = 32) -> api.DeviceKernel:
    """Upload a kernel's seeded inputs and allocate its output and split-K workspace."""
    import torch
    host = inputs if inputs is not None else wl.make_inputs(kernel, seed)
    dt = kernel.shape.dtype
    tensors = {k: to_device(v, dt) for k, v in host.items()}
    out_key = "c" if kernel.cls == wl.CLS_BATCH_MATMUL else "y"
    tensors[out_key] = torch.zeros(output_shape(kernel), dtype=api.torch_dtype(dt), device="cuda")
    return api.DeviceKernel(kernel.cls, kernel.shape, tensors, kernel.use_count, kernel.name,
                            max_workspace_bytes(kernel, max_split))
