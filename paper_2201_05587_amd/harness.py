"""Glue between the synthetic workloads and the library binding: device tensors for a kernel."""
from __future__ import annotations

import numpy as np

from . import api
from . import workloads as wl


def to_device(arr: np.ndarray, dtype: int):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(arr)).cuda()
    return t.to(torch.bfloat16) if dtype == wl.BF16 else t


def to_library_layout(kernel: wl.Kernel, name: str, arr: np.ndarray) -> np.ndarray:
    """Permute a tensor from the operator definition's index order to the library's storage order.

    The workloads (and the paper's listings) index convolution tensors as
    [n,c,h,w] / [k,c,r,s]; the library stores them channels-last, [n,h,w,c] /
    [k,r,s,c] ([r,s,c] for depthwise filters).  A pure permutation: no value changes.
    """
    if not kernel.is_conv() or name == "bias":
        return arr
    if name == "w" and kernel.cls == wl.CLS_DWCONV_BIAS_RELU6:
        return np.ascontiguousarray(arr[:, 0].transpose(1, 2, 0))
    return np.ascontiguousarray(arr.transpose(0, 2, 3, 1))


def output_in_definition_order(kernel: wl.Kernel, y):
    """The library's output tensor viewed in the definition's index order ([n,k,Ho,Wo] for conv)."""
    return y.permute(0, 3, 1, 2) if kernel.is_conv() else y


def output_shape(kernel: wl.Kernel):
    """Shape of the output as the library stores it."""
    s = kernel.shape
    if kernel.is_conv():
        return (s.n, s.ho, s.wo, s.k)
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
    tensors = {k: to_device(to_library_layout(kernel, k, v), dt) for k, v in host.items()}
    out_key = "c" if kernel.cls == wl.CLS_BATCH_MATMUL else "y"
    tensors[out_key] = torch.zeros(output_shape(kernel), dtype=api.torch_dtype(dt), device="cuda")
    return api.DeviceKernel(kernel.cls, kernel.shape, tensors, kernel.use_count, kernel.name,
                            max_workspace_bytes(kernel, max_split))
