"""Synthetic, seeded workloads: kernel shapes and input tensors.

This module holds no arithmetic of the method.  It lists the kernel shapes the
evaluation networks of the paper have (Section 5.1: ImageNet CNNs at batch 1,
224x224; Table 1 for ResNet18; BERT-shaped dense and batch-matmul kernels;
MobileNetV2-shaped depthwise and pointwise kernels) and draws input tensors
from a counter-based generator.  Datasets and trained weights are not needed:
timing and parity do not depend on the values.

Both the CPU oracle's tests and the GPU library's tests take their inputs from
here, so the two sides see the same bytes.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

# kernel classes (paper Section 4.2); letters are the paper's labels where it gives one
CLS_CONV2D_ADD = 0            # A
CLS_CONV2D_BIAS_RELU = 1      # E
CLS_CONV2D_BIAS_ADD_RELU = 2  # F
CLS_CONV2D_BIAS_RELU6 = 3
CLS_DENSE_ADD = 4             # D
CLS_DENSE_BIAS_RELU = 5
CLS_DENSE_BIAS_GELU = 6
CLS_BATCH_MATMUL = 7
CLS_DWCONV_BIAS_RELU6 = 8
CLASS_NAMES = ["conv2d_add", "conv2d_bias_relu", "conv2d_bias_add_relu", "conv2d_bias_relu6", "dense_add",
               "dense_bias_relu", "dense_bias_gelu", "batch_matmul", "dwconv_bias_relu6"]
CONV_CLASSES = (0, 1, 2, 3)
DENSE_CLASSES = (4, 5, 6)

F32, BF16 = 0, 1
ACT_NONE, ACT_RELU, ACT_RELU6, ACT_GELU = 0, 1, 2, 3
CLASS_ACT = {0: ACT_NONE, 1: ACT_RELU, 2: ACT_RELU, 3: ACT_RELU6, 4: ACT_NONE, 5: ACT_RELU, 6: ACT_GELU,
             7: ACT_NONE, 8: ACT_RELU6}


@dataclass(frozen=True)
class ConvShape:
    n: int
    c: int
    h: int
    w: int
    k: int
    r: int
    s: int
    stride_h: int = 1
    stride_w: int = 1
    pad_h: int = 0
    pad_w: int = 0
    dtype: int = F32

    @property
    def ho(self):
        return (self.h + 2 * self.pad_h - self.r) // self.stride_h + 1

    @property
    def wo(self):
        return (self.w + 2 * self.pad_w - self.s) // self.stride_w + 1


@dataclass(frozen=True)
class GemmShape:
    batch: int
    m: int
    n: int
    k: int
    trans_b: int = 1
    dtype: int = F32


@dataclass
class Kernel:
    """One fused kernel of a network: its class, its shape and how often the network uses it."""
    cls: int
    shape: object
    use_count: int = 1
    name: str = ""

    def is_conv(self):
        return self.cls in CONV_CLASSES or self.cls == CLS_DWCONV_BIAS_RELU6

    def gemm_extents(self):
        s = self.shape
        if self.cls == CLS_DWCONV_BIAS_RELU6:
            return (1, s.ho, s.wo, s.n * s.c)
        if self.is_conv():
            return (1, s.n * s.ho * s.wo, s.k, s.c * s.r * s.s)
        return (s.batch, s.m, s.n, s.k)

    def flops(self) -> float:
        s = self.shape
        if self.cls == CLS_DWCONV_BIAS_RELU6:
            return 2.0 * s.n * s.c * s.ho * s.wo * s.r * s.s
        b, m, n, k = self.gemm_extents()
        return 2.0 * b * m * n * k

    def algorithmic_bytes(self) -> float:
        """Compulsory traffic: every input, weight, bias, residual read once, the output written once."""
        s = self.shape
        e = 4 if s.dtype == F32 else 2
        if self.is_conv():
            out = s.n * s.k * s.ho * s.wo
            wts = s.c * s.r * s.s if self.cls == CLS_DWCONV_BIAS_RELU6 else s.k * s.c * s.r * s.s
            res = out if self.cls == CLS_CONV2D_BIAS_ADD_RELU else 0
            return e * (s.n * s.c * s.h * s.w + wts + s.k + res + out)
        b, m, n, k = self.gemm_extents()
        bias = 0 if self.cls == CLS_BATCH_MATMUL else n
        return e * (b * m * k + b * n * k + bias + b * m * n)


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=int(seed) & 0xFFFFFFFFFFFFFFFF))


def to_bf16_values(a: np.ndarray) -> np.ndarray:
    """Round float32 values to bf16-representable float32 values (library conversion, ties to even)."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


def make_inputs(kernel: Kernel, seed: int) -> dict:
    """float32 numpy inputs of a kernel; for bf16 kernels the values are bf16-representable.

    Distributions: activations U(-1, 1) (N(0,1) for the BERT-shaped kernels),
    weights N(0, 1/sqrt(fan_in)), bias U(-0.1, 0.1), residual U(-1, 1).
    """
    s = kernel.shape
    out = {}
    if kernel.is_conv():
        dw = kernel.cls == CLS_DWCONV_BIAS_RELU6
        fan_in = (1 if dw else s.c) * s.r * s.s
        out["x"] = _rng(seed + 0).uniform(-1.0, 1.0, (s.n, s.c, s.h, s.w)).astype(np.float32)
        wshape = (s.c, 1, s.r, s.s) if dw else (s.k, s.c, s.r, s.s)
        out["w"] = (_rng(seed + 1).standard_normal(wshape) / np.sqrt(fan_in)).astype(np.float32)
        out["bias"] = _rng(seed + 2).uniform(-0.1, 0.1, (s.k,)).astype(np.float32)
        if kernel.cls == CLS_CONV2D_BIAS_ADD_RELU:
            out["res"] = _rng(seed + 3).uniform(-1.0, 1.0, (s.n, s.k, s.ho, s.wo)).astype(np.float32)
    elif kernel.cls == CLS_BATCH_MATMUL:
        out["a"] = _rng(seed + 0).standard_normal((s.batch, s.m, s.k)).astype(np.float32)
        bshape = (s.batch, s.n, s.k) if s.trans_b else (s.batch, s.k, s.n)
        out["b"] = (_rng(seed + 1).standard_normal(bshape) / np.sqrt(s.k)).astype(np.float32)
    else:
        out["x"] = _rng(seed + 0).standard_normal((s.m, s.k)).astype(np.float32)
        out["w"] = (_rng(seed + 1).standard_normal((s.n, s.k)) / np.sqrt(s.k)).astype(np.float32)
        out["bias"] = _rng(seed + 2).uniform(-0.1, 0.1, (s.n,)).astype(np.float32)
    if s.dtype == BF16:
        out = {k: to_bf16_values(v) for k, v in out.items()}
    return out


def seed_for(cfg: int, kernel_index: int) -> int:
    return 0x5EED0000 + cfg * 1000 + kernel_index * 10


# ---- network-shaped kernel sets -------------------------------------------------------------------
def _conv(cls, n, c, hw, k, f, stride, dtype, use=1, name=""):
    pad = f // 2
    return Kernel(cls, ConvShape(n, c, hw, hw, k, f, f, stride, stride, pad, pad, dtype), use, name)


def cfg1_target() -> Kernel:
    return _conv(CLS_CONV2D_BIAS_RELU, 1, 64, 56, 64, 3, 1, F32, 1, "conv3x3_64_64_56")


def cfg1_donor() -> Kernel:
    return _conv(CLS_CONV2D_BIAS_RELU, 1, 128, 28, 128, 3, 1, F32, 1, "conv3x3_128_128_28")


def resnet18_kernels(batch: int = 1, dtype: int = F32) -> List[Kernel]:
    """The conv and dense kernels of paper Table 1 (pooling classes B and C carry ~0% of the time).

    Table 1's second shape column is [C_out, C_in, H_out, W_out]; filter sizes
    follow the ResNet definition: class-A rows are the 1x1/stride-2 projections,
    row 4 is the 7x7/stride-2 stem, all others are 3x3 with stride 2 where the
    map halves.
    """
    A, E, Fc = CLS_CONV2D_ADD, CLS_CONV2D_BIAS_RELU, CLS_CONV2D_BIAS_ADD_RELU
    ks = [
        _conv(A, batch, 256, 14, 512, 1, 2, dtype, 1, "r18_k1_proj_256_512"),
        _conv(A, batch, 128, 28, 256, 1, 2, dtype, 1, "r18_k2_proj_128_256"),
        _conv(A, batch, 64, 56, 128, 1, 2, dtype, 1, "r18_k3_proj_64_128"),
        _conv(E, batch, 3, 224, 64, 7, 2, dtype, 1, "r18_k4_stem"),
        _conv(E, batch, 64, 56, 64, 3, 1, dtype, 2, "r18_k6_64_64_56"),
        _conv(Fc, batch, 64, 56, 64, 3, 1, dtype, 2, "r18_k7_64_64_56_res"),
        _conv(E, batch, 64, 56, 128, 3, 2, dtype, 1, "r18_k8_64_128_s2"),
        _conv(E, batch, 128, 28, 128, 3, 1, dtype, 1, "r18_k9_128_128_28"),
        _conv(Fc, batch, 128, 28, 128, 3, 1, dtype, 2, "r18_k10_128_128_28_res"),
        _conv(E, batch, 128, 28, 256, 3, 2, dtype, 1, "r18_k11_128_256_s2"),
        _conv(E, batch, 256, 14, 256, 3, 1, dtype, 1, "r18_k12_256_256_14"),
        _conv(Fc, batch, 256, 14, 256, 3, 1, dtype, 2, "r18_k13_256_256_14_res"),
        _conv(E, batch, 256, 14, 512, 3, 2, dtype, 1, "r18_k14_256_512_s2"),
        _conv(E, batch, 512, 7, 512, 3, 1, dtype, 1, "r18_k15_512_512_7"),
        _conv(Fc, batch, 512, 7, 512, 3, 1, dtype, 2, "r18_k16_512_512_7_res"),
        Kernel(CLS_DENSE_ADD, GemmShape(1, batch, 1000, 512, 1, dtype), 1, "r18_k18_dense_512_1000"),
    ]
    return ks


def resnet50_kernels(batch: int = 1, dtype: int = F32, with_dense: bool = True) -> List[Kernel]:
    """ResNet-50-shaped conv kernels: stem + 4 stages of bottlenecks, stride on the 3x3 conv.

    That variant reproduces the class counts the paper's Table 2 gives for
    ResNet50: 16 kernels of class E, 4 of class A (projections) and 4 of the
    conv+bias+residual+ReLU class.
    """
    A, E, Fc = CLS_CONV2D_ADD, CLS_CONV2D_BIAS_RELU, CLS_CONV2D_BIAS_ADD_RELU
    ks = [_conv(E, batch, 3, 224, 64, 7, 2, dtype, 1, "r50_stem")]
    widths, blocks, spatial = [64, 128, 256, 512], [3, 4, 6, 3], [56, 28, 14, 7]
    cin = 64
    for st, (wd, nb, sp) in enumerate(zip(widths, blocks, spatial)):
        cout = wd * 4
        first_stride = 1 if st == 0 else 2
        sp_in = sp * first_stride
        tag = f"r50_s{st + 1}"
        # first block: 1x1 reduce at the incoming resolution, 3x3 (strided), 1x1 expand + residual, projection
        ks.append(_conv(E, batch, cin, sp_in, wd, 1, 1, dtype, 1, f"{tag}_b1_reduce_{cin}_{wd}"))
        ks.append(_conv(E, batch, wd, sp_in, wd, 3, first_stride, dtype, 1, f"{tag}_b1_3x3_s{first_stride}"))
        ks.append(_conv(Fc, batch, wd, sp, cout, 1, 1, dtype, nb, f"{tag}_expand_{wd}_{cout}_res"))
        ks.append(_conv(A, batch, cin, sp_in, cout, 1, first_stride, dtype, 1, f"{tag}_proj_{cin}_{cout}"))
        # remaining blocks
        ks.append(_conv(E, batch, cout, sp, wd, 1, 1, dtype, nb - 1, f"{tag}_reduce_{cout}_{wd}"))
        if first_stride != 1:
            ks.append(_conv(E, batch, wd, sp, wd, 3, 1, dtype, nb - 1, f"{tag}_3x3"))
        else:
            ks[-4].use_count += nb - 1  # stage 1: every 3x3 has the same shape
        cin = cout
    if with_dense:
        ks.append(Kernel(CLS_DENSE_ADD, GemmShape(1, batch, 1000, 2048, 1, dtype), 1, "r50_dense_2048_1000"))
    return ks


def bert_kernels(seq: int = 128, batch: int = 8, hidden: int = 768, heads: int = 12, ffn: int = 3072,
                 dtype: int = BF16) -> List[Kernel]:
    """BERT-base-shaped encoder kernels: dense hidden->hidden, hidden->ffn(+GELU), ffn->hidden, QK^T, PV."""
    tokens, hd = seq * batch, hidden // heads
    return [
        Kernel(CLS_DENSE_ADD, GemmShape(1, tokens, hidden, hidden, 1, dtype), 4, f"dense_{hidden}_{hidden}"),
        Kernel(CLS_DENSE_BIAS_GELU, GemmShape(1, tokens, ffn, hidden, 1, dtype), 1, f"dense_{hidden}_{ffn}_gelu"),
        Kernel(CLS_DENSE_ADD, GemmShape(1, tokens, hidden, ffn, 1, dtype), 1, f"dense_{ffn}_{hidden}"),
        Kernel(CLS_DENSE_BIAS_RELU, GemmShape(1, tokens, ffn, hidden, 1, dtype), 1, f"dense_{hidden}_{ffn}_relu"),
        Kernel(CLS_BATCH_MATMUL, GemmShape(batch * heads, seq, seq, hd, 1, dtype), 1, "bmm_qk"),
        Kernel(CLS_BATCH_MATMUL, GemmShape(batch * heads, seq, hd, seq, 0, dtype), 1, "bmm_pv"),
    ]


def mobilenetv2_kernels(batch: int = 1, dtype: int = F32) -> List[Kernel]:
    """MobileNetV2-shaped depthwise 3x3 (+bias+ReLU6) and pointwise 1x1 kernels.

    Built from the network's (expansion t, channels c, repeats n, stride s)
    stage rule at 224x224 input: expand 1x1 (ReLU6), depthwise 3x3 (ReLU6),
    project 1x1 (linear).
    """
    stages = [(1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2), (6, 96, 3, 1), (6, 160, 3, 2),
              (6, 320, 1, 1)]
    ks: List[Kernel] = []
    seen = {}

    def add(k: Kernel):
        key = (k.cls, k.shape)
        if key in seen:
            seen[key].use_count += 1
        else:
            seen[key] = k
            ks.append(k)

    cin, sp = 32, 112
    for t, c, n, s in stages:
        for i in range(n):
            stride = s if i == 0 else 1
            hidden = cin * t
            if t != 1:
                add(_conv(CLS_CONV2D_BIAS_RELU6, batch, cin, sp, hidden, 1, 1, dtype, 1, f"pw_expand_{cin}_{hidden}_{sp}"))
            add(Kernel(CLS_DWCONV_BIAS_RELU6,
                       ConvShape(batch, hidden, sp, sp, hidden, 3, 3, stride, stride, 1, 1, dtype), 1,
                       f"dw_{hidden}_{sp}_s{stride}"))
            sp_out = sp // stride
            add(_conv(CLS_CONV2D_ADD, batch, hidden, sp_out, c, 1, 1, dtype, 1, f"pw_project_{hidden}_{c}_{sp_out}"))
            cin, sp = c, sp_out
    add(_conv(CLS_CONV2D_BIAS_RELU6, batch, 320, 7, 1280, 1, 1, dtype, 1, "pw_head_320_1280"))
    return ks


def synthetic_network(index: int, batch: int = 32, dtype: int = BF16, kernels: int = 30,
                      exclude: Optional[set] = None) -> List[Kernel]:
    """A random CNN-shaped kernel list of the conv/dense classes, used as a donor network.

    Channel counts are multiples of 32 up to 2048, spatial sizes 112..7, filters
    1x1..7x7, strides 1 or 2; classes are drawn mostly from E, then A, F and D,
    like the mixes of the paper's Table 2.  Shapes in ``exclude`` are skipped: an
    identical shape would be a native schedule, not a transferred one.
    """
    rng = _rng(0xD0000 + index)
    out: List[Kernel] = []
    tries = 0
    while len(out) < kernels and tries < 100 * kernels:
        tries += 1
        u = rng.random()
        cls = CLS_CONV2D_BIAS_RELU if u < 0.6 else CLS_CONV2D_ADD if u < 0.75 else \
            CLS_CONV2D_BIAS_ADD_RELU if u < 0.95 else CLS_DENSE_ADD
        if cls == CLS_DENSE_ADD:
            k = Kernel(cls, GemmShape(1, batch, int(rng.integers(1, 65)) * 32, int(rng.integers(1, 65)) * 32, 1,
                                      dtype), 1, f"syn{index}_dense{len(out)}")
        else:
            sp = int(rng.choice([112, 56, 28, 14, 7]))
            f = int(rng.choice([1, 1, 3, 3, 3, 5, 7]))
            stride = int(rng.choice([1, 1, 1, 2]))
            # keep a kernel's work in the range of the networks' layers (at most ~8 GFLOP at batch 32)
            cmax = {112: 4, 56: 8, 28: 16, 14: 32, 7: 64}[sp]
            cin, cout = int(rng.integers(1, cmax + 1)) * 32, int(rng.integers(1, cmax + 1)) * 32
            if f >= 5:
                cin = min(cin, 128)
            k = _conv(cls, batch, cin, sp, cout, f, stride, dtype, 1, f"syn{index}_conv{len(out)}")
        if exclude is not None and (k.cls, k.shape) in exclude:
            continue
        out.append(k)
    return out
