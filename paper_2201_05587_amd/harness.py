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


def device_kernel(kernel: wl.Kernel, seed: int, inputs: dict | None = None, max_split: int = 32,
                  cold_mb: float = 0.0, cold_min_mb: float = 0.0) -> api.DeviceKernel:
    """Upload a kernel's seeded inputs and allocate its output and split-K workspace.

    cold_mb > 0 adds copies of every tensor (weights too: a network's layers do not share them) until all sets
    together hold that many megabytes; the timing functions then rotate through them, so that every launch
    reads its operands from memory (the caches hold 8 x 4 MB of L2 and 256 MB on the memory side).  Kernels
    whose tensors take less than cold_min_mb get no copies: what fits the L2s a kernel finds there inside a
    network, just written by its producer, and timing it on one set ranks records with far less noise."""
    import torch
    host = inputs if inputs is not None else wl.make_inputs(kernel, seed)
    dt = kernel.shape.dtype
    tensors = {k: to_device(to_library_layout(kernel, k, v), dt) for k, v in host.items()}
    out_key = "c" if kernel.cls == wl.CLS_BATCH_MATMUL else "y"
    tensors[out_key] = torch.zeros(output_shape(kernel), dtype=api.torch_dtype(dt), device="cuda")
    n_alt = 0
    if cold_mb > 0 and kernel.algorithmic_bytes() >= cold_min_mb * 1e6:
        n_alt = int(min(400, max(1, -(-cold_mb * 1e6 // kernel.algorithmic_bytes()))))
    alternates = [{name: t.clone() for name, t in tensors.items()} for _ in range(n_alt)]
    return api.DeviceKernel(kernel.cls, kernel.shape, tensors, kernel.use_count, kernel.name,
                            max_workspace_bytes(kernel, max_split), alternates)


def bottleneck_chain(k_reduce: wl.Kernel, k_conv: wl.Kernel, k_expand: wl.Kernel, blocks: int, seed: int):
    """Residual bottleneck blocks wired output-to-input (paper Section 5.5: kernels run in their network context).

    Each block is reduce (1x1) -> conv (3x3) -> expand (1x1 + residual + ReLU); the block's input is the
    expand kernel's residual and the next block's input.  Every block reuses the same three filters
    (timing and parity do not depend on the values).  Returns (device kernels in launch order, the
    kernels they instantiate, host inputs: block input x0 and the three kernels' weights and biases).
    """
    import torch
    sr, sc, se = k_reduce.shape, k_conv.shape, k_expand.shape
    assert (sr.n, sr.ho, sr.wo, sr.k) == (sc.n, sc.h, sc.w, sc.c) and (sc.n, sc.ho, sc.wo, sc.k) == (se.n, se.h, se.w, se.c)
    assert (se.n, se.ho, se.wo, se.k) == (sr.n, sr.h, sr.w, sr.c) and k_expand.cls == wl.CLS_CONV2D_BIAS_ADD_RELU
    dt = sr.dtype
    host = {"reduce": wl.make_inputs(k_reduce, seed), "conv": wl.make_inputs(k_conv, seed + 100),
            "expand": wl.make_inputs(k_expand, seed + 200)}
    dev = {name: {t: to_device(to_library_layout(k, t, v), dt) for t, v in inp.items() if t in ("w", "bias")}
           for (name, inp), k in zip(host.items(), (k_reduce, k_conv, k_expand))}
    x0 = host["reduce"]["x"]
    tdt = api.torch_dtype(dt)
    ping = to_device(to_library_layout(k_reduce, "x", x0), dt)
    pong = torch.zeros_like(ping)
    y1 = torch.zeros(output_shape(k_reduce), dtype=tdt, device="cuda")
    y2 = torch.zeros(output_shape(k_conv), dtype=tdt, device="cuda")
    dks, kinds = [], []
    for b in range(blocks):
        src, dst = (ping, pong) if b % 2 == 0 else (pong, ping)
        wiring = ((k_reduce, "reduce", dict(x=src, y=y1)), (k_conv, "conv", dict(x=y1, y=y2)),
                  (k_expand, "expand", dict(x=y2, res=src, y=dst)))
        for k, name, io in wiring:
            tensors = dict(dev[name], **io)
            dks.append(api.DeviceKernel(k.cls, k.shape, tensors, 1, f"{k.name}@block{b}", max_workspace_bytes(k, 8)))
            kinds.append(k)
    return dks, kinds, dict(x0=x0, **{name: {t: inp[t] for t in ("w", "bias")} for name, inp in host.items()})
