"""Thin ctypes binding of libtt (argument marshalling only; every step runs in the library).

Names mirror ``include/tt.h``.  Tensors are torch tensors on the GPU (PyTorch is
used for device memory and streams only); their ``data_ptr()`` and the current
stream's handle are what crosses the boundary.  There is no CPU fallback: if the
shared library is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, byref, c_double, c_float, c_int32, c_int64, c_size_t, c_void_p

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtt.so")

# classes, dtypes, status codes, sketches (same values as tt.h)
(TT_CONV2D_ADD, TT_CONV2D_BIAS_RELU, TT_CONV2D_BIAS_ADD_RELU, TT_CONV2D_BIAS_RELU6, TT_DENSE_ADD,
 TT_DENSE_BIAS_RELU, TT_DENSE_BIAS_GELU, TT_BATCH_MATMUL, TT_DWCONV_BIAS_RELU6) = range(9)
TT_NUM_CLASSES = 9
TT_F32, TT_BF16 = 0, 1
TT_OK, TT_ERR_INVALID_SCHEDULE, TT_ERR_CLASS_MISMATCH, TT_ERR_BAD_ARG = 0, -1, -2, -3
TT_ERR_WORKSPACE, TT_ERR_UNSUPPORTED, TT_ERR_HIP = -4, -5, -6
TT_SK_MFMA, TT_SK_GEMV, TT_SK_DWCONV, TT_SK_DIRECT = range(4)
TT_STRICT_DIVISIBLE = 1
CONV_CLASSES = (0, 1, 2, 3)
DENSE_CLASSES = (4, 5, 6)


class tt_conv_shape(Structure):
    _fields_ = [(n, c_int32) for n in ("n", "c", "h", "w", "k", "r", "s", "stride_h", "stride_w", "pad_h",
                                       "pad_w", "dtype")]


class tt_gemm_shape(Structure):
    _fields_ = [(n, c_int32) for n in ("batch", "m", "n", "k", "trans_b", "dtype")]


class tt_schedule(Structure):
    _fields_ = [(n, c_int32) for n in ("cls", "sketch", "tile_m", "tile_n", "tile_k", "wave_m", "wave_n",
                                       "mfma", "split_k", "order", "vec", "unroll", "stages", "id")]
    _fields_ += [("donor_shape", c_int32 * 12), ("donor_us", c_float)]

    KNOBS = ("cls", "sketch", "tile_m", "tile_n", "tile_k", "wave_m", "wave_n", "mfma", "split_k", "order",
             "vec", "unroll", "stages")

    def knobs(self):
        return {k: getattr(self, k) for k in self.KNOBS}

    def copy(self):
        out = tt_schedule()
        ctypes.memmove(byref(out), byref(self), ctypes.sizeof(tt_schedule))
        return out

    def __repr__(self):
        return "tt_schedule(" + ", ".join(f"{k}={v}" for k, v in self.knobs().items()) + f", id={self.id})"


class tt_plan(Structure):
    _fields_ = [(n, c_int32) for n in (
        "status", "reason", "sketch", "batch", "M", "N", "K", "tile_m", "tile_n", "tile_k", "wave_m", "wave_n",
        "mfma", "tiles_m", "tiles_n", "k_tiles", "tail_m", "tail_n", "tail_k", "eff_split_k", "k_iters", "slabs",
        "eff_vec_a", "eff_vec_b", "eff_vec_c", "eff_unroll", "stages", "order", "grid", "block", "lds_bytes")]
    _fields_ += [("workspace_bytes", c_int64), ("variant_id", c_int32), ("reserved", c_int32)]

    # the fields the method defines (Sections 4.1, 4.2); the others describe this library's kernels
    METHOD_FIELDS = ("status", "reason", "sketch", "batch", "M", "N", "K", "tile_m", "tile_n", "tile_k", "wave_m",
                     "wave_n", "mfma", "tiles_m", "tiles_n", "k_tiles", "tail_m", "tail_n", "tail_k", "eff_split_k",
                     "k_iters", "slabs", "order", "grid", "block", "workspace_bytes")
    LIBRARY_FIELDS = ("eff_vec_a", "eff_vec_b", "eff_vec_c", "eff_unroll", "stages", "lds_bytes", "variant_id")

    def method(self):
        return {k: getattr(self, k) for k in self.METHOD_FIELDS}

    def runnable(self):
        """A valid plan that a kernel of this library implements."""
        return self.status == TT_OK and self.variant_id >= 0


class tt_kernel_desc(Structure):
    _fields_ = [("cls", c_int32), ("use_count", c_int32), ("shape", c_void_p), ("bufs", c_void_p * 5),
                ("ws", c_void_p), ("ws_bytes", c_size_t), ("alt_bufs", POINTER(c_void_p)), ("n_alt", c_int32)]


class tt_sweep_opts(Structure):
    _fields_ = [(n, c_int32) for n in ("warmup", "samples", "min_sample_us", "max_launches", "flags",
                                       "allow_slower_than_default", "pair_budget", "prioritise")]
    _fields_ += [("seed", ctypes.c_uint64)]


class tt_sweep_row(Structure):
    _fields_ = [(n, c_int32) for n in ("kernel", "chosen", "n_valid", "n_invalid", "n_other_class", "n_not_tried")]
    _fields_ += [("best_us", c_double), ("default_us", c_double)]


EXPORTS = ("tt_version", "tt_status_name", "tt_last_error", "tt_schedule_default", "tt_schedule_apply", "tt_plan_tile",
           "tt_debug_tile_map", "tt_debug_fast_div", "tt_debug_probe", "tt_conv2d_bias_relu", "tt_conv2d_bias_relu_noalloc", "tt_dense_bias_relu", "tt_batch_matmul", "tt_dwconv",
           "tt_transfer_sweep", "tt_sweep_plan", "tt_refine_space", "tt_refine", "tt_native_sweep", "tt_time_pair", "tt_run_kernels", "tt_schedule_space", "tt_sweep_select", "tt_variant_info", "tt_num_variants", "tt_select_donor")


def _load():
    # PyTorch owns the device memory and the streams that cross the boundary, so the library must
    # bind to the HIP runtime PyTorch has loaded: import it first, the loader then reuses that copy.
    import torch  # noqa: F401
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(or `make -C paper_2201_05587_amd/csrc`); there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    lib.tt_version.restype = ctypes.c_int
    lib.tt_status_name.restype = ctypes.c_char_p
    lib.tt_status_name.argtypes = [ctypes.c_int]
    lib.tt_last_error.restype = ctypes.c_char_p
    lib.tt_schedule_default.argtypes = [ctypes.c_int, c_void_p, POINTER(tt_schedule)]
    lib.tt_schedule_apply.argtypes = [POINTER(tt_schedule), ctypes.c_int, c_void_p, ctypes.c_int, POINTER(tt_plan)]
    lib.tt_plan_tile.argtypes = [POINTER(tt_plan), c_int64, POINTER(c_int32 * 8)]
    lib.tt_debug_tile_map.argtypes = [POINTER(tt_plan), c_void_p, c_void_p]
    lib.tt_conv2d_bias_relu.argtypes = [c_void_p] * 5 + [POINTER(tt_conv_shape), ctypes.c_int, POINTER(tt_schedule),
                                                         c_void_p, c_size_t, c_void_p]
    lib.tt_conv2d_bias_relu_noalloc.argtypes = [c_void_p] * 5 + [POINTER(tt_conv_shape), ctypes.c_int,
                                                                 POINTER(tt_schedule), c_void_p]
    lib.tt_dense_bias_relu.argtypes = [c_void_p] * 4 + [POINTER(tt_gemm_shape), ctypes.c_int, POINTER(tt_schedule),
                                                        c_void_p, c_size_t, c_void_p]
    lib.tt_batch_matmul.argtypes = [c_void_p] * 3 + [POINTER(tt_gemm_shape), POINTER(tt_schedule), c_void_p,
                                                     c_size_t, c_void_p]
    lib.tt_dwconv.argtypes = [c_void_p] * 4 + [POINTER(tt_conv_shape), POINTER(tt_schedule), c_void_p]
    lib.tt_transfer_sweep.argtypes = [POINTER(tt_kernel_desc), ctypes.c_int, POINTER(tt_schedule), ctypes.c_int,
                                      POINTER(tt_sweep_opts), c_void_p, POINTER(tt_sweep_row), POINTER(c_double),
                                      POINTER(c_int64), POINTER(c_double)]
    lib.tt_sweep_plan.argtypes = [POINTER(c_int32), POINTER(c_double), ctypes.c_int, POINTER(c_int32), ctypes.c_int,
                                  ctypes.c_int, ctypes.c_int, ctypes.c_uint64, POINTER(ctypes.c_uint8), POINTER(c_int64)]
    lib.tt_refine_space.argtypes = [POINTER(tt_schedule), POINTER(tt_schedule), ctypes.c_int]
    lib.tt_refine.argtypes = [POINTER(tt_kernel_desc), POINTER(tt_schedule), ctypes.c_int, POINTER(tt_sweep_opts), c_void_p,
                              POINTER(tt_schedule), POINTER(c_double), POINTER(c_double), POINTER(c_int32)]
    lib.tt_native_sweep.argtypes = [POINTER(tt_kernel_desc), ctypes.c_int, ctypes.c_int, POINTER(tt_sweep_opts),
                                    POINTER(tt_sweep_opts), c_void_p, POINTER(tt_schedule), POINTER(c_double),
                                    POINTER(c_double), POINTER(c_int32), POINTER(c_int32)]
    lib.tt_time_pair.argtypes = [POINTER(tt_kernel_desc), POINTER(tt_schedule), POINTER(tt_sweep_opts), c_void_p,
                                 POINTER(c_double), POINTER(c_double)]
    lib.tt_run_kernels.argtypes = [POINTER(tt_kernel_desc), POINTER(POINTER(tt_schedule)), ctypes.c_int, ctypes.c_int,
                                   c_void_p]
    lib.tt_schedule_space.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, POINTER(tt_schedule), ctypes.c_int]
    lib.tt_variant_info.argtypes = [ctypes.c_int, POINTER(c_int32 * 12)]
    lib.tt_sweep_select.argtypes = [POINTER(c_int32), ctypes.c_int, POINTER(c_int32), ctypes.c_int, POINTER(c_double),
                                    POINTER(c_double), ctypes.c_int, POINTER(tt_sweep_row)]
    lib.tt_select_donor.argtypes = [POINTER(c_double), ctypes.c_int, POINTER(c_int32), ctypes.c_int, POINTER(c_double),
                                    POINTER(c_int32)]
    for name in EXPORTS:
        if name not in ("tt_status_name", "tt_last_error", "tt_debug_fast_div"):
            getattr(lib, name).restype = ctypes.c_int
    lib.tt_debug_probe.argtypes = [ctypes.c_int, c_void_p, c_void_p, c_size_t, ctypes.c_int, c_void_p, POINTER(c_double)]
    lib.tt_debug_fast_div.restype = c_int64
    lib.tt_debug_fast_div.argtypes = [ctypes.c_uint32, ctypes.c_uint32]
    return lib


lib = _load()


class TTError(RuntimeError):
    def __init__(self, status, where):
        detail = lib.tt_last_error().decode() if status == TT_ERR_HIP else ""
        super().__init__(f"{where}: {status_name(status)} ({status}) {detail}")
        self.status = status


def status_name(status: int) -> str:
    return lib.tt_status_name(status).decode()


def _check(status, where):
    if status != TT_OK:
        raise TTError(status, where)


# ---- shapes and records ----------------------------------------------------------------------------
def to_c_shape(shape):
    """Accept a ctypes shape or any object with the fields of ConvShape / GemmShape."""
    if isinstance(shape, (tt_conv_shape, tt_gemm_shape)):
        return shape
    if hasattr(shape, "stride_h"):
        return tt_conv_shape(shape.n, shape.c, shape.h, shape.w, shape.k, shape.r, shape.s, shape.stride_h,
                             shape.stride_w, shape.pad_h, shape.pad_w, shape.dtype)
    return tt_gemm_shape(shape.batch, shape.m, shape.n, shape.k, shape.trans_b, shape.dtype)


def make_schedule(cls, sketch=TT_SK_MFMA, tile_m=64, tile_n=64, tile_k=16, wave_m=32, wave_n=32, mfma=16,
                  split_k=1, order=0, vec=4, unroll=1, stages=2, id=-1) -> tt_schedule:
    s = tt_schedule()
    for k, v in dict(cls=cls, sketch=sketch, tile_m=tile_m, tile_n=tile_n, tile_k=tile_k, wave_m=wave_m,
                     wave_n=wave_n, mfma=mfma, split_k=split_k, order=order, vec=vec, unroll=unroll,
                     stages=stages, id=id).items():
        setattr(s, k, v)
    return s


def tt_schedule_default(cls, shape) -> tt_schedule:
    out = tt_schedule()
    cs = to_c_shape(shape)
    _check(lib.tt_schedule_default(cls, ctypes.addressof(cs), byref(out)), "tt_schedule_default")
    return out


def tt_schedule_apply(sched, cls, shape, flags=0) -> tt_plan:
    """Returns the plan; plan.status carries the result (no exception for invalid records)."""
    plan = tt_plan()
    cs = to_c_shape(shape)
    lib.tt_schedule_apply(byref(sched) if sched is not None else None, cls, ctypes.addressof(cs), flags, byref(plan))
    return plan


def tt_plan_tile(plan, wg):
    out = (c_int32 * 8)()
    _check(lib.tt_plan_tile(byref(plan), wg, byref(out)), "tt_plan_tile")
    return list(out)


def tt_schedule_space(cls, dtype, level=1):
    n = lib.tt_schedule_space(cls, dtype, level, None, 0)
    if n < 0:
        raise TTError(n, "tt_schedule_space")
    arr = (tt_schedule * max(n, 1))()
    lib.tt_schedule_space(cls, dtype, level, arr, n)
    return [arr[i].copy() for i in range(n)]


def tt_sweep_select(kernel_cls, pool_cls, pair_us, default_us, allow_slower_than_default=False):
    nk, np_ = len(kernel_cls), len(pool_cls)
    kc = (c_int32 * max(nk, 1))(*kernel_cls)
    pc = (c_int32 * max(np_, 1))(*pool_cls)
    flat = [float(v) for row in pair_us for v in row]
    pu = (c_double * max(len(flat), 1))(*flat)
    du = (c_double * max(nk, 1))(*[float(v) for v in default_us])
    rows = (tt_sweep_row * max(nk, 1))()
    _check(lib.tt_sweep_select(kc, nk, pc, np_, pu, du, int(allow_slower_than_default), rows), "tt_sweep_select")
    return [(rows[i].chosen, rows[i].best_us, rows[i].n_valid, rows[i].n_invalid) for i in range(nk)]


# ---- device helpers (torch is plumbing: memory and streams) -----------------------------------------
def tt_select_donor(class_cost, donor_class_counts):
    """Eq. 1: (index of the best candidate model, score of every candidate).

    class_cost: sequence of the target's untuned time per class; donor_class_counts: one sequence of
    per-class kernel counts per candidate model.
    """
    nc, nd = len(class_cost), len(donor_class_counts)
    cost = (c_double * nc)(*[float(v) for v in class_cost])
    flat = [int(v) for row in donor_class_counts for v in row]
    assert len(flat) == nc * nd
    counts = (c_int32 * max(len(flat), 1))(*flat)
    scores = (c_double * max(nd, 1))()
    best = c_int32(-1)
    _check(lib.tt_select_donor(cost, nc, counts, nd, scores, byref(best)), "tt_select_donor")
    return int(best.value), [float(scores[i]) for i in range(nd)]


def _torch():
    import torch
    return torch


def _ptr(t):
    return None if t is None else c_void_p(t.data_ptr())


def _stream():
    return c_void_p(_torch().cuda.current_stream().cuda_stream)


def torch_dtype(dtype):
    torch = _torch()
    return torch.float32 if dtype == TT_F32 else torch.bfloat16


def workspace_bytes(sched, cls, shape) -> int:
    plan = tt_schedule_apply(sched if sched is not None else tt_schedule_default(cls, shape), cls, shape)
    return int(plan.workspace_bytes) if plan.status == TT_OK else 0


def _ws_for(sched, cls, shape, ws):
    if ws is not None:
        return ws
    need = workspace_bytes(sched, cls, shape)
    if need == 0:
        return None
    return _torch().empty(need, dtype=_torch().uint8, device="cuda")


def tt_conv2d_bias_relu(x, w, bias, residual, shape, cls, sched=None, ws=None, y=None):
    torch = _torch()
    cs = to_c_shape(shape)
    ho = (cs.h + 2 * cs.pad_h - cs.r) // cs.stride_h + 1
    wo = (cs.w + 2 * cs.pad_w - cs.s) // cs.stride_w + 1
    if y is None:
        y = torch.empty((cs.n, cs.k, ho, wo), dtype=x.dtype, device=x.device)
    ws = _ws_for(sched, cls, cs, ws)
    rc = lib.tt_conv2d_bias_relu(_ptr(x), _ptr(w), _ptr(bias), _ptr(residual), _ptr(y), byref(cs), cls,
                                 byref(sched) if sched is not None else None, _ptr(ws),
                                 0 if ws is None else ws.numel() * ws.element_size(), _stream())
    _check(rc, "tt_conv2d_bias_relu")
    return y


TT_STATIC_WORKSPACE_BYTES = 16 * 1024 * 1024


def tt_conv2d_bias_relu_noalloc(x, w, bias, residual, y, shape, cls, sched=None):
    """The conv operator with the library's static split-K workspace; `y` is the caller's (nothing is allocated)."""
    cs = to_c_shape(shape)
    rc = lib.tt_conv2d_bias_relu_noalloc(_ptr(x), _ptr(w), _ptr(bias), _ptr(residual), _ptr(y), byref(cs), cls,
                                         byref(sched) if sched is not None else None, _stream())
    return rc


def tt_dense_bias_relu(x, w, bias, shape, cls, sched=None, ws=None, y=None):
    torch = _torch()
    gs = to_c_shape(shape)
    if y is None:
        y = torch.empty((gs.m, gs.n), dtype=x.dtype, device=x.device)
    ws = _ws_for(sched, cls, gs, ws)
    rc = lib.tt_dense_bias_relu(_ptr(x), _ptr(w), _ptr(bias), _ptr(y), byref(gs), cls,
                                byref(sched) if sched is not None else None, _ptr(ws),
                                0 if ws is None else ws.numel() * ws.element_size(), _stream())
    _check(rc, "tt_dense_bias_relu")
    return y


def tt_batch_matmul(a, b, shape, sched=None, ws=None, c=None):
    torch = _torch()
    gs = to_c_shape(shape)
    if c is None:
        c = torch.empty((gs.batch, gs.m, gs.n), dtype=a.dtype, device=a.device)
    ws = _ws_for(sched, TT_BATCH_MATMUL, gs, ws)
    rc = lib.tt_batch_matmul(_ptr(a), _ptr(b), _ptr(c), byref(gs), byref(sched) if sched is not None else None,
                             _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(), _stream())
    _check(rc, "tt_batch_matmul")
    return c


def tt_dwconv(x, w, bias, shape, sched=None, y=None):
    torch = _torch()
    cs = to_c_shape(shape)
    ho = (cs.h + 2 * cs.pad_h - cs.r) // cs.stride_h + 1
    wo = (cs.w + 2 * cs.pad_w - cs.s) // cs.stride_w + 1
    if y is None:
        y = torch.empty((cs.n, cs.c, ho, wo), dtype=x.dtype, device=x.device)
    rc = lib.tt_dwconv(_ptr(x), _ptr(w), _ptr(bias), _ptr(y), byref(cs), byref(sched) if sched is not None else None,
                       _stream())
    _check(rc, "tt_dwconv")
    return y


def tt_debug_tile_map(plan):
    torch = _torch()
    out = torch.empty((plan.grid, 8), dtype=torch.int32, device="cuda")
    _check(lib.tt_debug_tile_map(byref(plan), _ptr(out), _stream()), "tt_debug_tile_map")
    torch.cuda.synchronize()
    return out.cpu().numpy()


TT_PROBE_LAUNCH_GAP_US, TT_PROBE_MFMA_BF16_TFLOPS, TT_PROBE_COPY_LINEAR_GBPS, TT_PROBE_COPY_TILED_GBPS, \
    TT_PROBE_L2_READ_GBPS = range(5)


def tt_debug_probe(which, src=None, dst=None, reps=10):
    """One hardware-rate figure (see tt.h); src and dst are device tensors where the probe needs them."""
    out = c_double(0.0)
    nbytes = (src if src is not None else dst)
    nbytes = nbytes.numel() * nbytes.element_size() if nbytes is not None else 0
    _check(lib.tt_debug_probe(which, _ptr(src) if src is not None else None, _ptr(dst) if dst is not None else None,
                              nbytes, reps, _stream(), byref(out)), "tt_debug_probe")
    return out.value


class DeviceKernel:
    """A target kernel with its tensors resident on the GPU, ready for timing and sweeps."""

    def __init__(self, cls, shape, tensors, use_count=1, name="", ws_bytes=0, alternates=()):
        """alternates: further tensor dicts of the same shapes, which the timing functions rotate through."""
        torch = _torch()
        self.cls, self.name, self.use_count = cls, name, use_count
        self.cshape = to_c_shape(shape)
        self.tensors = tensors  # dict name -> device tensor (kept alive here)
        self.alternates = list(alternates)
        self.ws = torch.empty(max(int(ws_bytes), 16), dtype=torch.uint8, device="cuda")
        if cls in CONV_CLASSES:
            order = ("x", "w", "bias", "res", "y")
        elif cls in DENSE_CLASSES or cls == TT_DWCONV_BIAS_RELU6:
            order = ("x", "w", "bias", "y", None)
        else:
            order = ("a", "b", "c", None, None)
        self.desc = tt_kernel_desc()
        self.desc.cls, self.desc.use_count = cls, use_count
        self.desc.shape = ctypes.addressof(self.cshape)
        for i, key in enumerate(order):
            t = tensors.get(key) if key else None
            self.desc.bufs[i] = None if t is None else t.data_ptr()
        self.desc.ws = self.ws.data_ptr()
        self.desc.ws_bytes = self.ws.numel()
        self.desc.n_alt = len(self.alternates)
        self._alt = (c_void_p * max(5 * len(self.alternates), 1))()
        for a, alt in enumerate(self.alternates):
            for i, key in enumerate(order):
                t = alt.get(key) if key else None
                self._alt[5 * a + i] = None if t is None else t.data_ptr()
        self.desc.alt_bufs = ctypes.cast(self._alt, POINTER(c_void_p)) if self.alternates else None

    def output(self):
        return self.tensors["c" if self.cls == TT_BATCH_MATMUL else "y"]

    def run(self, sched=None):
        """Enqueue the kernel once under `sched` (None = default) on the current stream."""
        d, s = self.desc, (byref(sched) if sched is not None else None)
        if self.cls in CONV_CLASSES:
            rc = lib.tt_conv2d_bias_relu(d.bufs[0], d.bufs[1], d.bufs[2], d.bufs[3], d.bufs[4], byref(self.cshape),
                                         self.cls, s, d.ws, d.ws_bytes, _stream())
        elif self.cls in DENSE_CLASSES:
            rc = lib.tt_dense_bias_relu(d.bufs[0], d.bufs[1], d.bufs[2], d.bufs[3], byref(self.cshape), self.cls, s,
                                        d.ws, d.ws_bytes, _stream())
        elif self.cls == TT_BATCH_MATMUL:
            rc = lib.tt_batch_matmul(d.bufs[0], d.bufs[1], d.bufs[2], byref(self.cshape), s, d.ws, d.ws_bytes,
                                     _stream())
        else:
            rc = lib.tt_dwconv(d.bufs[0], d.bufs[1], d.bufs[2], d.bufs[3], byref(self.cshape), s, _stream())
        return rc


def make_opts(warmup=3, samples=10, min_sample_us=200, max_launches=64, flags=0, allow_slower_than_default=0,
              pair_budget=0, prioritise=0, seed=0):
    return tt_sweep_opts(warmup, samples, min_sample_us, max_launches, flags, allow_slower_than_default, pair_budget,
                         prioritise, seed)


def tt_sweep_plan(kernel_cls, weight, pool_cls, pair_budget, prioritise=0, seed=0):
    """mask[k][p] (1 = evaluate) of a budgeted sweep; host only."""
    nk, np_ = len(kernel_cls), len(pool_cls)
    kc = (c_int32 * max(nk, 1))(*kernel_cls)
    pc = (c_int32 * max(np_, 1))(*pool_cls)
    w = (c_double * max(nk, 1))(*[float(v) for v in weight]) if weight is not None else None
    mask = (ctypes.c_uint8 * max(nk * np_, 1))()
    sel = c_int64(0)
    _check(lib.tt_sweep_plan(kc, w, nk, pc, np_, pair_budget, prioritise, seed, mask, byref(sel)), "tt_sweep_plan")
    return [[int(mask[k * np_ + p]) for p in range(np_)] for k in range(nk)], int(sel.value)


def tt_refine_space(base: tt_schedule):
    n = lib.tt_refine_space(byref(base), None, 0)
    if n < 0:
        raise TTError(n, "tt_refine_space")
    arr = (tt_schedule * max(n, 1))()
    lib.tt_refine_space(byref(base), arr, n)
    return [arr[i].copy() for i in range(n)]


def tt_refine(kernel, base: tt_schedule, rounds=2, opts=None):
    """(status, best record, best_us, base_us, pairs timed): local refinement of a record on a kernel."""
    best = tt_schedule()
    bu, su, tried = c_double(-1.0), c_double(-1.0), c_int32(0)
    rc = lib.tt_refine(byref(kernel.desc), byref(base), rounds, byref(opts) if opts is not None else None, _stream(),
                       byref(best), byref(bu), byref(su), byref(tried))
    return rc, best, bu.value, su.value, tried.value


def tt_native_sweep(kernel, level=1, finalists=4, explore=None, full=None):
    """(best record, best_us, default_us, n_valid, n_records): the exhaustive sweep of one kernel."""
    best = tt_schedule()
    bu, du, nv, nr = c_double(-1.0), c_double(-1.0), c_int32(0), c_int32(0)
    rc = lib.tt_native_sweep(byref(kernel.desc), level, finalists, byref(explore) if explore is not None else None,
                             byref(full) if full is not None else None, _stream(), byref(best), byref(bu), byref(du),
                             byref(nv), byref(nr))
    _check(rc, "tt_native_sweep")
    return best, bu.value, du.value, nv.value, nr.value


def tt_time_pair(kernel: DeviceKernel, sched=None, opts=None):
    """(status, median_us, min_us) of one (kernel, schedule) pair."""
    med, mn = c_double(-1.0), c_double(-1.0)
    rc = lib.tt_time_pair(byref(kernel.desc), byref(sched) if sched is not None else None,
                          byref(opts) if opts is not None else None, _stream(), byref(med), byref(mn))
    return rc, med.value, mn.value


def tt_transfer_sweep(kernels, pool, opts=None):
    """Run the sweep; returns (rows, pair_us[nk][np], evaluations, wall_seconds)."""
    nk, np_ = len(kernels), len(pool)
    descs = (tt_kernel_desc * max(nk, 1))()
    for i, k in enumerate(kernels):
        ctypes.memmove(byref(descs[i]), byref(k.desc), ctypes.sizeof(tt_kernel_desc))
    parr = (tt_schedule * max(np_, 1))()
    for i, s in enumerate(pool):
        ctypes.memmove(byref(parr[i]), byref(s), ctypes.sizeof(tt_schedule))
    rows = (tt_sweep_row * max(nk, 1))()
    pair = (c_double * max(nk * np_, 1))()
    evals, wall = c_int64(0), c_double(0.0)
    rc = lib.tt_transfer_sweep(descs, nk, parr, np_, byref(opts) if opts is not None else None, _stream(), rows, pair,
                               byref(evals), byref(wall))
    _check(rc, "tt_transfer_sweep")
    table = [[pair[k * np_ + p] for p in range(np_)] for k in range(nk)]
    out_rows = [dict(kernel=rows[i].kernel, chosen=rows[i].chosen, n_valid=rows[i].n_valid,
                     n_invalid=rows[i].n_invalid, n_other_class=rows[i].n_other_class,
                     n_not_tried=rows[i].n_not_tried, best_us=rows[i].best_us,
                     default_us=rows[i].default_us) for i in range(nk)]
    return out_rows, table, evals.value, wall.value


class KernelList:
    """Kernels and their chosen records marshalled once, for repeated network-shaped passes."""

    def __init__(self, kernels, scheds):
        self.kernels, self.scheds = list(kernels), [None if s is None else s.copy() for s in scheds]
        n = len(self.kernels)
        self.descs = (tt_kernel_desc * max(n, 1))()
        for i, k in enumerate(self.kernels):
            ctypes.memmove(byref(self.descs[i]), byref(k.desc), ctypes.sizeof(tt_kernel_desc))
        self.ptrs = (POINTER(tt_schedule) * max(n, 1))()
        for i, s in enumerate(self.scheds):
            if s is not None:
                self.ptrs[i] = ctypes.pointer(s)
        self.n = n

    def run(self, repeat=1):
        _check(lib.tt_run_kernels(self.descs, self.ptrs, self.n, repeat, _stream()), "tt_run_kernels")


VARIANT_INFO = ("dtype", "family", "tile_m", "tile_n", "tile_k", "wave_m", "wave_n", "mfma", "amode", "pipe",
                "stage_bytes", "k_granule")


def tt_variant_info(variant_id: int):
    info = (c_int32 * 12)()
    _check(lib.tt_variant_info(variant_id, byref(info)), "tt_variant_info")
    return list(info)


def variant_name(plan: tt_plan, shape=None) -> str:
    """Name of the kernel a plan launches, spelled like the demangled symbol rocprofv3 reports.

    `shape` (a conv shape) is needed only to tell the two depthwise kernels apart.
    """
    if plan.sketch == TT_SK_MFMA:
        info = tt_variant_info(plan.variant_id)
        if info[9] == 2:
            threads = (info[2] // info[5]) * (info[3] // info[6]) * 128
            per_thread = info[10] * (info[4] // 8) // threads   # patch items per thread and channel slice
            stride = shape.stride_h if shape is not None else 0
            return (f"tt::conv3x3_patch_kernel<{info[2]}, {info[3]}, {info[4]}, {info[5]}, {info[6]}, {stride}, "
                    f"{per_thread}>")
        if info[9] == 3:
            return "tt::gemm_stream_kernel<" + ", ".join(str(info[i]) for i in (0, 2, 3, 4, 5, 6, 7)) + ">"
        if info[9]:
            return "tt::contract_async_kernel<" + ", ".join(str(v) for v in info[:8]) + ">"
        return "tt::contract_kernel<" + ", ".join(str(v) for v in info[:9]) + ">"
    if plan.sketch == TT_SK_DWCONV:
        s = shape
        bound = 256 if plan.block <= 256 else 512 if plan.block <= 512 else 1024   # the instance's thread bound
        if (s is not None and plan.stages == 1 and s.stride_h == s.stride_w and s.stride_h in (1, 2)
                and s.n * s.h * s.w * s.c * 4 < 2 ** 31):
            return (f"tt::dwconv3x3_rows_kernel<{plan.wave_m}, {plan.wave_n}, {plan.eff_vec_a}, {s.stride_h}, "
                    f"{bound}>")
        return f"tt::dwconv3x3_kernel<{plan.wave_m}, {plan.wave_n}, {bound}>"
    return {TT_SK_GEMV: "tt::gemv_kernel", TT_SK_DIRECT: "tt::direct_kernel"}[plan.sketch]
