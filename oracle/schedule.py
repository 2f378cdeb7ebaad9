"""Integer-only oracle of schedule re-application, the workgroup index map and the sweep's selection.

TEST INFRASTRUCTURE ONLY: the product package never imports this module, and
this module imports nothing from the product.  Pure Python integers, no numpy.

What the paper fixes (Sections 4.1-4.3) and what is written out here:

* ``split`` / ``replay_split_chain``: the Split primitive in its two-argument
  form (Algorithm 1): the inner range is the factor, the outer range is derived
  from the loop being split.  Section 4.1's worked example is the rule: a split
  stored with absolute extents (4, 8) fits N = 32 only, while keeping the inner
  factor 8 and deriving the outer extent N / 8 is valid for every N that 8
  divides.  Section 4.2 adds the failure case: a factor larger than the loop
  gives invalid code.
* ``apply``: the same rule applied to a GPU schedule record.  Inner factors
  (workgroup tile, wave tile, MFMA edge, parallel split of the reduction) are
  kept, every outer extent is derived from the TARGET kernel's shape; a record
  of another kernel class is always invalid (Section 4.2).  The result is an
  integer *plan* holding what the method defines: validity and its reason,
  the GEMM view of the kernel (convolution: M = n * Ho * Wo, N = k,
  K = c * r * s), tiles, tails, the split of the reduction, grid and
  workspace.  How a kernel implementation stages its tiles (on-chip memory
  bytes, pipeline depth, access widths of the matrix-core sketch) is NOT
  modelled here: those fields belong to the library and are checked against
  what its kernels export.
* ``plan_tile``: workgroup id -> (batch, k-split, tile origin and clipped
  extents), a closed-form integer map; the device code must agree bit for bit.
* ``select`` / ``evaluation_count``: Section 4.3's sweep once the times are
  known: every kernel is tried with the default schedule and with every donor
  record of its class, invalid pairs are marked -1 and skipped, the fastest is
  kept, the default is the fallback.
* ``sweep_plan``: which pairs a sweep with a pair budget evaluates.  The paper
  only names the idea (Section 5.5: sample a subset of the schedules, "randomly
  or using some other selection heuristic"; Section 4.4.2: prioritise kernel
  classes by their potential); the rule written out here is this repository's
  reading: SplitMix64 keys per pair, the smallest keys are kept; with
  prioritisation kernels are served in order of their share of untuned time.
* ``refine_neighbours``: the one-knob neighbourhood of a record, for the local
  refinement the paper proposes as future work (Section 6).

Readings of points the paper leaves open are listed in the repository's design
notes; the ones that matter here: factors are compared against the fused GEMM
extents M, N, K; a non-dividing factor gets a guarded tail unless
``STRICT_DIVISIBLE`` is set; ties go to the default, then to the lowest pool
index.
"""
from __future__ import annotations

# ---- kernel classes (paper Section 4.2: a class is an operator sequence) -------------------------
CLS_CONV2D_ADD = 0            # paper class A: conv2d + per-channel vector, no activation
CLS_CONV2D_BIAS_RELU = 1      # paper class E (Algorithm 2)
CLS_CONV2D_BIAS_ADD_RELU = 2  # paper class F: + residual tensor
CLS_CONV2D_BIAS_RELU6 = 3     # pointwise/regular conv of MobileNetV2-shaped nets
CLS_DENSE_ADD = 4             # paper class D
CLS_DENSE_BIAS_RELU = 5
CLS_DENSE_BIAS_GELU = 6
CLS_BATCH_MATMUL = 7
CLS_DWCONV_BIAS_RELU6 = 8
NUM_CLASSES = 9

CONV_CLASSES = (CLS_CONV2D_ADD, CLS_CONV2D_BIAS_RELU, CLS_CONV2D_BIAS_ADD_RELU, CLS_CONV2D_BIAS_RELU6)
DENSE_CLASSES = (CLS_DENSE_ADD, CLS_DENSE_BIAS_RELU, CLS_DENSE_BIAS_GELU)

DT_F32, DT_BF16 = 0, 1

# ---- sketches: the loop-nest skeleton a record's factors refer to --------------------------------
SK_MFMA = 0     # workgroup tile -> wave tile -> MFMA block, LDS-staged K loop
SK_GEMV = 1     # dense only: one wave per few outputs, lanes split K, wave reduction
SK_DWCONV = 2   # depthwise only: (planes, rows, cols) tile per workgroup, micro-tile per thread
SK_DIRECT = 3   # any class: one thread per output element, unscheduled loop nest

# ---- status / reason codes -----------------------------------------------------------------------
OK = 0
ERR_INVALID_SCHEDULE = -1   # the paper's "-1" bar: the record does not fit this kernel
ERR_CLASS_MISMATCH = -2
ERR_BAD_ARG = -3

R_NONE = 0
R_FACTOR_GT_M = 1
R_FACTOR_GT_N = 2
R_FACTOR_GT_K = 3
R_NOT_DIVISIBLE = 4
R_SPLIT_K = 5
# 6 and 7 are the library's own resource reasons (on-chip memory, matrix-core K step): never produced here
R_GRID = 8
R_SKETCH_CLASS = 9

STRICT_DIVISIBLE = 1  # flag bit: Section 4.1's divisibility reading ({N : f | N})

XCDS = 8
GROUP_M = 8

RECORD_FIELDS = ("cls", "sketch", "tile_m", "tile_n", "tile_k", "wave_m", "wave_n", "mfma", "split_k",
                 "order", "vec", "unroll", "stages")
PLAN_FIELDS = ("status", "reason", "sketch", "batch", "M", "N", "K", "tile_m", "tile_n", "tile_k",
               "wave_m", "wave_n", "mfma", "tiles_m", "tiles_n", "k_tiles", "tail_m", "tail_n", "tail_k",
               "eff_split_k", "k_iters", "slabs", "order", "grid", "block", "workspace_bytes")


def ceil_div(a: int, b: int) -> int:
    return -(-a // b)


# ---- the Split primitive (paper Algorithm 1, Section 4.1) ----------------------------------------
def split(extent: int, factor: int, strict: bool = True):
    """Split(range, factor) -> (outer, inner): inner = factor, outer derived from the loop.

    Returns None when the split is invalid for this extent: a factor larger than
    the loop (Section 4.2) or, in the strict reading of Section 4.1, a factor
    that does not divide it.
    """
    if factor < 1 or extent < 1:
        raise ValueError("extent and factor must be positive")
    if factor > extent:
        return None
    if extent % factor:
        if strict:
            return None
        return (ceil_div(extent, factor), factor)
    return (extent // factor, factor)


def split_fixed(extent: int, outer: int, inner: int) -> bool:
    """Three-argument Split(range, outer, inner) with both extents stored: valid only if it covers the loop."""
    return outer * inner == extent


def replay_split_chain(extent: int, factors, strict: bool = True):
    """Replay a chain of two-argument splits, each one splitting the previous OUTER loop.

    ``factors`` lists the factors in the order the schedule applies them
    (innermost first, as Algorithm 1 writes them).  Returns the loop extents
    outermost first, or None if a step is invalid.
    """
    inner = []
    outer = extent
    for f in factors:
        res = split(outer, f, strict)
        if res is None:
            return None
        outer, kept = res
        inner.append(kept)
    return tuple([outer] + inner[::-1])


# ---- shapes --------------------------------------------------------------------------------------
def conv_shape(n, c, h, w, k, r, s, stride_h=1, stride_w=1, pad_h=0, pad_w=0, dtype=DT_F32):
    return dict(kind="conv", n=n, c=c, h=h, w=w, k=k, r=r, s=s, stride_h=stride_h, stride_w=stride_w,
                pad_h=pad_h, pad_w=pad_w, dtype=dtype)


def gemm_shape(batch, m, n, k, trans_b=0, dtype=DT_F32):
    return dict(kind="gemm", batch=batch, m=m, n=n, k=k, trans_b=trans_b, dtype=dtype)


def record(cls, sketch=SK_MFMA, tile_m=64, tile_n=64, tile_k=16, wave_m=32, wave_n=32, mfma=16, split_k=1,
           order=0, vec=4, unroll=1, stages=2):
    return dict(cls=cls, sketch=sketch, tile_m=tile_m, tile_n=tile_n, tile_k=tile_k, wave_m=wave_m,
                wave_n=wave_n, mfma=mfma, split_k=split_k, order=order, vec=vec, unroll=unroll, stages=stages)


def conv_out(size, filt, stride, pad):
    return (size + 2 * pad - filt) // stride + 1


def _is_pow2(v: int) -> bool:
    return v >= 1 and (v & (v - 1)) == 0


def _pow2_floor(v: int) -> int:
    p = 1
    while p * 2 <= v:
        p *= 2
    return p


def pow2_dividing(vmax: int, extent: int) -> int:
    """Largest power of two <= vmax that divides extent (vector-width reformulation)."""
    v = 1
    while v * 2 <= vmax and extent % (v * 2) == 0:
        v *= 2
    return v


def gemm_extents(cls: int, shape: dict):
    """(batch, M, N, K) of the contraction, or (1, Ho, Wo, planes) for depthwise; None if ill-formed."""
    if cls in CONV_CLASSES or cls == CLS_DWCONV_BIAS_RELU6:
        if shape.get("kind") != "conv":
            return None
        for f in ("n", "c", "h", "w", "k", "r", "s", "stride_h", "stride_w"):
            if shape[f] < 1:
                return None
        if shape["pad_h"] < 0 or shape["pad_w"] < 0:
            return None
        if shape["h"] + 2 * shape["pad_h"] < shape["r"] or shape["w"] + 2 * shape["pad_w"] < shape["s"]:
            return None
        ho = conv_out(shape["h"], shape["r"], shape["stride_h"], shape["pad_h"])
        wo = conv_out(shape["w"], shape["s"], shape["stride_w"], shape["pad_w"])
        if cls == CLS_DWCONV_BIAS_RELU6:
            if shape["k"] != shape["c"]:
                return None
            return (1, ho, wo, shape["n"] * shape["c"])
        # the fused GEMM view of Algorithm 2's loop nest: rows = output pixels, reduction = c * r * s
        return (1, shape["n"] * ho * wo, shape["k"], shape["c"] * shape["r"] * shape["s"])
    if shape.get("kind") != "gemm":
        return None
    for f in ("batch", "m", "n", "k"):
        if shape[f] < 1:
            return None
    if shape["trans_b"] not in (0, 1):
        return None
    if cls in DENSE_CLASSES and (shape["batch"] != 1 or shape["trans_b"] != 1):
        return None  # dense weights are stored [out, in]
    return (shape["batch"], shape["m"], shape["n"], shape["k"])


def _blank_plan():
    return {f: 0 for f in PLAN_FIELDS}


def _fail(plan, status, reason=R_NONE):
    out = _blank_plan()
    out["status"] = status
    out["reason"] = reason
    return out


def record_is_well_formed(rec: dict) -> bool:
    """Shape-independent consistency of a record (violations are argument errors, not transfer failures)."""
    sk = rec["sketch"]
    if rec["cls"] < 0 or rec["cls"] >= NUM_CLASSES or sk not in (SK_MFMA, SK_GEMV, SK_DWCONV, SK_DIRECT):
        return False
    if rec["split_k"] < 1 or rec["order"] < 0 or rec["order"] >= 6 or rec["vec"] not in (1, 2, 4, 8):
        return False
    if rec["unroll"] < 1 or rec["stages"] < 1 or rec["stages"] > (7 if sk == SK_MFMA else 2):
        return False
    tm, tn, tk, wm, wn, mf = (rec[f] for f in ("tile_m", "tile_n", "tile_k", "wave_m", "wave_n", "mfma"))
    if sk == SK_MFMA:
        if mf not in (16, 32):
            return False
        if not (_is_pow2(tm) and _is_pow2(tn) and 16 <= tm <= 256 and 16 <= tn <= 256):
            return False
        if tk not in (16, 32, 64, 128):
            return False
        if wm < mf or wn < mf or tm % wm or tn % wn or wm % mf or wn % mf:
            return False
        waves = (tm // wm) * (tn // wn)
        if waves not in (1, 2, 4, 8, 16):
            return False
        if wm * wn // 64 > 256:
            return False
        return True
    if mf != 0:
        return False
    if sk == SK_GEMV:
        if rec["split_k"] != 1 or tm < 1 or tm > 8 or wm != tm:
            return False
        if wn < 1 or wn > 8 or tn % wn or (tn // wn) not in (1, 2, 4, 8, 16):
            return False
        if tk % 64 or (tk // 64) not in (1, 2, 4, 8):
            return False
        return True
    if sk == SK_DWCONV:
        if rec["split_k"] != 1 or min(tm, tn, tk, wm, wn) < 1 or tm % wm or tn % wn:
            return False
        if wm > 8 or wn > 8:
            return False
        threads = tk * (tm // wm) * (tn // wn)
        return threads % 64 == 0 and 64 <= threads <= 1024
    # SK_DIRECT: a single knob-free record per class
    return tm == 1 and tn == 1 and tk == 1 and wm == 1 and wn == 1 and rec["split_k"] == 1


def apply(rec: dict, cls: int, shape: dict, flags: int = 0) -> dict:
    """Re-apply a schedule record to a target kernel (class, shape): plan or failure code."""
    plan = _blank_plan()
    if cls < 0 or cls >= NUM_CLASSES or not record_is_well_formed(rec):
        return _fail(plan, ERR_BAD_ARG)
    ext = gemm_extents(cls, shape)
    if ext is None or shape["dtype"] not in (DT_F32, DT_BF16):
        return _fail(plan, ERR_BAD_ARG)
    # Section 4.2: a schedule of another class transforms loops this kernel does not have.
    if rec["cls"] != cls:
        return _fail(plan, ERR_CLASS_MISMATCH)
    sk = rec["sketch"]
    is_dw = cls == CLS_DWCONV_BIAS_RELU6
    if (sk == SK_DWCONV) != is_dw and sk != SK_DIRECT:
        return _fail(plan, ERR_INVALID_SCHEDULE, R_SKETCH_CLASS)
    if sk == SK_GEMV and cls not in DENSE_CLASSES:
        return _fail(plan, ERR_INVALID_SCHEDULE, R_SKETCH_CLASS)

    strict = bool(flags & STRICT_DIVISIBLE)
    batch, M, N, K = ext
    plan.update(sketch=sk, batch=batch, M=M, N=N, K=K, order=rec["order"], mfma=rec["mfma"])

    if sk == SK_DIRECT:
        total = batch * M * N * (K if is_dw else 1)
        grid = ceil_div(total, 256)
        if grid >= 2 ** 31:
            return _fail(plan, ERR_INVALID_SCHEDULE, R_GRID)
        plan.update(tile_m=1, tile_n=1, tile_k=1, wave_m=1, wave_n=1, tiles_m=M, tiles_n=N, k_tiles=K,
                    tail_m=1, tail_n=1, tail_k=1, eff_split_k=1, k_iters=K, slabs=batch, grid=grid, block=256)
        if is_dw:
            plan.update(k_iters=1, slabs=K)
        return plan

    tm, tn, tk = rec["tile_m"], rec["tile_n"], rec["tile_k"]
    if sk == SK_DWCONV:
        # Vectorize on the plane axis, reformulated to the target (Section 4.1): a lane owns the widest
        # power-of-two group of channels, not above the record's width or one memory access, that divides
        # the channel count; the tile_k lanes of a workgroup then cover tile_k * ev planes.
        widest = 4 if shape["dtype"] == DT_F32 else 8  # elements of the widest single memory access
        tk *= pow2_dividing(min(rec["vec"], widest), shape["c"])
    # Inner factors are kept; a factor larger than the loop it splits is invalid (Section 4.2).
    for factor, extent, reason in ((tm, M, R_FACTOR_GT_M), (tn, N, R_FACTOR_GT_N), (tk, K, R_FACTOR_GT_K)):
        if factor > extent:
            return _fail(plan, ERR_INVALID_SCHEDULE, reason)
        if strict and extent % factor:
            return _fail(plan, ERR_INVALID_SCHEDULE, R_NOT_DIVISIBLE)
    # Outer extents are derived from the target (Section 4.1's Split(N, N/8, 8)), with a guarded tail.
    tiles_m, tiles_n, k_tiles = ceil_div(M, tm), ceil_div(N, tn), ceil_div(K, tk)
    plan.update(tile_m=tm, tile_n=tn, tile_k=tk, wave_m=rec["wave_m"], wave_n=rec["wave_n"],
                tiles_m=tiles_m, tiles_n=tiles_n, k_tiles=k_tiles, tail_m=M - (tiles_m - 1) * tm,
                tail_n=N - (tiles_n - 1) * tn, tail_k=K - (k_tiles - 1) * tk)

    if sk == SK_DWCONV:
        threads = rec["tile_k"] * (tm // rec["wave_m"]) * (tn // rec["wave_n"])
        grid = tiles_m * tiles_n * k_tiles
        if grid >= 2 ** 31:
            return _fail(plan, ERR_INVALID_SCHEDULE, R_GRID)
        plan.update(eff_split_k=1, k_iters=1, slabs=k_tiles, grid=grid, block=threads)
        return plan

    if sk == SK_GEMV:
        waves = tn // rec["wave_n"]
        grid = tiles_m * tiles_n * batch
        if grid >= 2 ** 31:
            return _fail(plan, ERR_INVALID_SCHEDULE, R_GRID)
        plan.update(eff_split_k=1, k_iters=k_tiles, slabs=batch, grid=grid, block=64 * waves)
        return plan

    # SK_MFMA.  Parallel split of the reduction: a split larger than the number of K tiles splits nothing.
    if rec["split_k"] > k_tiles:
        return _fail(plan, ERR_INVALID_SCHEDULE, R_SPLIT_K)
    if strict and k_tiles % rec["split_k"]:
        return _fail(plan, ERR_INVALID_SCHEDULE, R_NOT_DIVISIBLE)
    k_iters = ceil_div(k_tiles, rec["split_k"])
    eff_split_k = ceil_div(k_tiles, k_iters)  # no empty split
    waves = (tm // rec["wave_m"]) * (tn // rec["wave_n"])
    slabs = batch * eff_split_k
    grid = tiles_m * tiles_n * slabs
    if grid >= 2 ** 31:
        return _fail(plan, ERR_INVALID_SCHEDULE, R_GRID)
    plan.update(eff_split_k=eff_split_k, k_iters=k_iters, slabs=slabs, grid=grid, block=64 * waves,
                workspace_bytes=(4 * eff_split_k * batch * M * N) if eff_split_k > 1 else 0)
    return plan


def plan_tile(plan: dict, wg: int):
    """Workgroup id -> [slab_hi, slab_lo, m0, m_ext, n0, n_ext, k0, k_ext] for tiled sketches.

    slab_hi / slab_lo are (batch, k-split) for contractions and (plane tile, 0)
    for depthwise, whose k0 / k_ext give the first plane and the plane count.
    """
    if plan["status"] != OK or plan["sketch"] == SK_DIRECT or wg < 0 or wg >= plan["grid"]:
        return None
    G = plan["grid"]
    order = plan["order"]
    if order >= 3:
        # Workgroups are dealt round-robin to the XCDs; give each XCD a contiguous run of logical ids.
        per, rem = divmod(G, XCDS)
        x, j = wg % XCDS, wg // XCDS
        L = x * per + min(x, rem) + j
    else:
        L = wg
    tiles_m, tiles_n = plan["tiles_m"], plan["tiles_n"]
    T = tiles_m * tiles_n
    slab, t = divmod(L, T)
    base = order % 3
    if base == 0:      # M tiles fastest
        im, i_n = t % tiles_m, t // tiles_m
    elif base == 1:    # N tiles fastest
        i_n, im = t % tiles_n, t // tiles_n
    else:              # bands of GROUP_M M-tiles, M fastest inside a band
        width = GROUP_M * tiles_n
        first = (t // width) * GROUP_M
        gsize = min(tiles_m - first, GROUP_M)
        im = first + (t % width) % gsize
        i_n = (t % width) // gsize
    m0, n0 = im * plan["tile_m"], i_n * plan["tile_n"]
    m_ext, n_ext = min(plan["tile_m"], plan["M"] - m0), min(plan["tile_n"], plan["N"] - n0)
    if plan["sketch"] == SK_DWCONV:
        k0 = slab * plan["tile_k"]
        return [slab, 0, m0, m_ext, n0, n_ext, k0, min(plan["tile_k"], plan["K"] - k0)]
    if plan["sketch"] == SK_GEMV:
        return [slab, 0, m0, m_ext, n0, n_ext, 0, plan["K"]]
    b, z = divmod(slab, plan["eff_split_k"])
    kt0 = z * plan["k_iters"]
    kt1 = min(plan["k_tiles"], kt0 + plan["k_iters"])
    k0 = kt0 * plan["tile_k"]
    return [b, z, m0, m_ext, n0, n_ext, k0, min(plan["K"], kt1 * plan["tile_k"]) - k0]


def default_schedule(cls: int, shape: dict) -> dict:
    """The always-valid "untuned" record of a kernel (paper Section 4.3's default schedule)."""
    ext = gemm_extents(cls, shape)
    if ext is None:
        raise ValueError("ill-formed shape")
    batch, M, N, K = ext
    dt = shape["dtype"]
    vfull = 4 if dt == DT_F32 else 8
    direct = record(cls, SK_DIRECT, 1, 1, 1, 1, 1, 0, 1, 0, 1, 1, 1)
    if cls == CLS_DWCONV_BIAS_RELU6:
        if dt != DT_F32:
            return direct
        tk = min(64, _pow2_floor(K))
        tn = min(256 // tk, _pow2_floor(N))
        tm = min(256 // (tk * tn), _pow2_floor(M))
        if (tk * tm * tn) % 64 or tk * tm * tn < 64:
            return direct
        return record(cls, SK_DWCONV, tm, tn, tk, 1, 1, 0, 1, 0, 1, 1, 1)
    kmin = 16 if dt == DT_F32 else 32
    if M >= 16 and N >= 16 and K >= kmin:
        tm, tn = min(64, _pow2_floor(M)), min(64, _pow2_floor(N))
        return record(cls, SK_MFMA, tm, tn, kmin, min(tm, 32), min(tn, 32), 16, 1, 0, vfull, 1, 2)
    if cls in DENSE_CLASSES and K >= 64 and N >= 4:
        return record(cls, SK_GEMV, 1, 4, 256 if K >= 256 else 64, 1, 1, 0, 1, 0, 4, 1, 1)
    return direct


# ---- the sweep once times are known (paper Section 4.3) ------------------------------------------
NOT_TRIED = -3.0

def evaluation_count(kernel_classes, pool_classes) -> int:
    """Pairs a sweep evaluates: every kernel once with the default plus once per same-class donor."""
    return sum(1 + sum(1 for pc in pool_classes if pc == kc) for kc in kernel_classes)


def select(kernel_classes, pool_classes, pair_us, default_us, allow_slower_than_default=False):
    """Per kernel: (chosen pool index or -1 for the default, best time, #valid, #invalid).

    ``pair_us[k][p]`` is the measured time of kernel k under donor p, or a
    negative value when the pair is invalid.  Pairs of another class are never
    looked at.  Ties: the default wins, then the lowest pool index.
    """
    rows = []
    for k, kc in enumerate(kernel_classes):
        best_id, best = -1, default_us[k]
        if allow_slower_than_default:
            best = float("inf")
        n_valid = n_invalid = 0
        for p, pc in enumerate(pool_classes):
            if pc != kc:
                continue
            t = pair_us[k][p]
            if t == NOT_TRIED:      # left out by a pair budget: neither valid nor invalid
                continue
            if t < 0:
                n_invalid += 1
                continue
            n_valid += 1
            if t < best:
                best_id, best = p, t
        if best_id < 0:
            best = default_us[k]
        rows.append((best_id, best, n_valid, n_invalid))
    return rows


def model_selection_score(target_class_cost: dict, candidate_class_count: dict) -> float:
    """Paper Eq. 1: sum over the target's classes of P_c^2 * sqrt(|W_Tc|)."""
    return sum(p * p * (candidate_class_count.get(c, 0) ** 0.5) for c, p in target_class_cost.items())


# ---- cheaper sweeps (paper Sections 5.5 and 4.4.2: ideas only; the rule is this repository's) -----
MASK64 = (1 << 64) - 1


def splitmix64(x: int) -> int:
    """Output function of SplitMix64 (Steele, Lea, Flood 2014) applied to the counter x."""
    x = (x + 0x9E3779B97F4A7C15) & MASK64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & MASK64
    return x ^ (x >> 31)


def sweep_plan(kernel_classes, weights, pool_classes, pair_budget, prioritise=False, seed=0):
    """mask[k][p] = 1 for the (kernel, donor) pairs a budgeted sweep evaluates.

    Every same-class pair gets the key splitmix64(seed + k * np + p + 1).  Without
    prioritisation the ``pair_budget`` smallest keys are taken (a uniform sample
    without replacement).  With it, kernels are served by decreasing weight (their
    untuned time times their use count; ties: lower index), each taking all its pairs
    while the budget lasts; the kernel the budget runs out on keeps its smallest keys.
    """
    nk, np_ = len(kernel_classes), len(pool_classes)
    pairs = {k: [] for k in range(nk)}
    for k in range(nk):
        for p in range(np_):
            if pool_classes[p] == kernel_classes[k]:
                i = k * np_ + p
                pairs[k].append((splitmix64((seed + i + 1) & MASK64), i))
    total = sum(len(v) for v in pairs.values())
    mask = [[0] * np_ for _ in range(nk)]
    if pair_budget <= 0 or pair_budget >= total:
        chosen = [i for v in pairs.values() for _, i in v]
    elif not prioritise:
        chosen = [i for _, i in sorted(q for v in pairs.values() for q in v)[:pair_budget]]
    else:
        chosen, left = [], pair_budget
        for k in sorted(range(nk), key=lambda k: (-weights[k], k)):
            take = sorted(pairs[k])[:left] if len(pairs[k]) > left else pairs[k]
            chosen += [i for _, i in take]
            left -= len(take)
            if left <= 0:
                break
    for i in chosen:
        mask[i // np_][i % np_] = 1
    return mask


SPLIT_STEPS = (1, 2, 3, 4, 6, 8, 12, 16, 32)


def refine_neighbours(rec: dict):
    """Well-formed records that differ from ``rec`` in exactly one knob by one step (Section 6's outlook)."""
    out = []

    def consider(**change):
        r = dict(rec, **change)
        if r != rec and record_is_well_formed(r) and r not in out:
            out.append(r)

    if rec["sketch"] in (SK_MFMA, SK_DWCONV):
        for f in ("tile_m", "tile_n", "tile_k", "wave_m", "wave_n", "vec"):
            if rec[f] % 2 == 0:
                consider(**{f: rec[f] // 2})
            consider(**{f: rec[f] * 2})
        for order in range(6):
            consider(order=order)
        consider(stages=rec["stages"] - 1)
        consider(stages=rec["stages"] + 1)
        consider(unroll=1 if rec["unroll"] >= 2 else 8)
    if rec["sketch"] == SK_MFMA:
        consider(mfma=32 if rec["mfma"] == 16 else 16)
        if rec["split_k"] in SPLIT_STEPS:
            at = SPLIT_STEPS.index(rec["split_k"])
            for j in (at - 1, at + 1):
                if 0 <= j < len(SPLIT_STEPS):
                    consider(split_k=SPLIT_STEPS[j])
    return out
