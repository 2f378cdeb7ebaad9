#!/usr/bin/env python3
"""Write the instantiation slices and the variant table of the matrix-core contraction kernel.

Usage: gen_variants.py OUT_DIR [N_SLICES] [SET]

A variant is one compiled instance of the contraction kernel for a (data type,
operand family, workgroup tile, wave tile, matrix-core block, pipeline kind)
combination; the run-time knobs of a schedule record (split_k, order, vec,
unroll, the number of stages within a pipeline kind) do not need a variant of
their own.  SET = "full" (default) or "small" (a handful of
tiles, for quick development builds).
"""
import os
import sys

F32, BF16 = 0, 1
FAMILIES = (0, 1, 2)  # conv, gemm [M][K]x[N][K], gemm [M][K]x[K][N]

# (tile_m, tile_n, wave_m, wave_n)
TILES_FULL = [
    (16, 16, 16, 16), (64, 16, 16, 16), (128, 16, 32, 16),
    (16, 32, 16, 32), (32, 16, 32, 16), (16, 64, 16, 32), (64, 16, 32, 16),
    (32, 32, 16, 16), (32, 32, 32, 32), (64, 32, 32, 32), (32, 64, 32, 32), (128, 32, 32, 32),
    (32, 128, 32, 32), (256, 32, 64, 32), (64, 64, 32, 32), (128, 64, 64, 32),
    (64, 128, 32, 64), (256, 64, 64, 64), (64, 256, 64, 64), (128, 128, 64, 64), (128, 128, 64, 32),
    (256, 128, 128, 64), (256, 128, 64, 64), (128, 256, 64, 128), (128, 256, 64, 64),
    # the same workgroup tiles cut into more, smaller wave tiles: more waves per CU to hide latency
    # where a layer gives each CU only one or two workgroups
    (64, 64, 16, 32), (64, 64, 32, 16), (64, 128, 32, 32), (128, 64, 32, 32), (128, 128, 32, 32), (128, 128, 32, 64),
    (64, 64, 16, 16), (128, 64, 32, 16), (64, 128, 16, 32), (256, 64, 32, 32), (64, 256, 32, 32), (256, 128, 64, 32),
    (128, 256, 32, 64), (32, 128, 16, 32), (128, 32, 32, 16),
]
# tiles that also get a deep K slice (tile_k 128 for bf16, 64 for fp32): fewer, larger loads in flight
DEEP_K_TILES = {(64, 64, 16, 16), (128, 64, 32, 16), (64, 128, 16, 32), (128, 128, 32, 32), (128, 128, 32, 64), (64, 64, 16, 32), (64, 64, 32, 16), (64, 128, 32, 32), (128, 64, 32, 32), (64, 64, 32, 32), (64, 128, 32, 64), (128, 64, 64, 32), (128, 128, 64, 32), (128, 128, 64, 64),
                (32, 128, 32, 32), (128, 32, 32, 32), (256, 64, 64, 64), (64, 256, 64, 64), (32, 64, 32, 32),
                (64, 32, 32, 32), (256, 128, 64, 64), (128, 256, 64, 64)}
TILES_SMALL = [(16, 16, 16, 16), (32, 32, 16, 16), (64, 64, 32, 32), (128, 128, 64, 64), (256, 128, 128, 64),
               (16, 32, 16, 32), (32, 16, 32, 16), (16, 64, 16, 32), (64, 16, 32, 16), (32, 32, 32, 32),
               (32, 64, 32, 32), (64, 32, 32, 32)]


# 3x3 convolutions with the padded input patch in LDS (bf16, 32-blocks, two K groups per wave position):
# (tile_m, tile_n, channels per slice = tile_k, wave_m, wave_n, stride, patch items per thread and slice)
PATCH_TILES = [
    (128, 128, 64, 64, 64, 1, 6), (128, 64, 64, 64, 32, 1, 6), (128, 64, 64, 64, 64, 1, 7), (256, 64, 64, 64, 64, 1, 7),
    (64, 128, 64, 64, 64, 1, 7), (64, 64, 64, 64, 32, 1, 7), (64, 128, 64, 32, 64, 1, 4),
    (128, 128, 32, 64, 64, 1, 4),
    (128, 128, 32, 64, 64, 2, 6), (64, 128, 32, 64, 64, 2, 7), (64, 64, 32, 64, 32, 2, 7), (128, 64, 32, 64, 64, 2, 7),
]


# persistent contraction for short reductions (dense family; record knob stages = 7):
# (tile_m, tile_n, wave_m, wave_n), each with both matrix-core blocks and the tile_k list of its data type
STREAM_TILES = [(64, 128, 32, 64), (32, 128, 32, 32), (64, 64, 32, 32), (128, 64, 32, 32), (128, 128, 32, 64)]


def stream_variants():
    out = []
    for dt in (F32, BF16):
        for tm, tn, wm, wn in STREAM_TILES:
            assert (tm, tn, wm, wn) in TILES_FULL  # the record space lists a tile through its register-pipeline instance
            for mf in (16, 32):
                for tk in ((16, 32) if dt == F32 else (32, 64)):
                    if async_ok(dt, 1, tm, tn, tk, wm, wn, 0):
                        out.append((dt, 1, tm, tn, tk, wm, wn, mf, 0, 3, 0))
    return out


def patch_variants():
    seen, out = set(), []
    for tm, tn, ck, wm, wn, stride, pl in PATCH_TILES:
        key = (tm, tn, ck, wm, wn, stride)
        assert key not in seen, key  # one patch capacity per (tile, stride): the record does not carry it
        seen.add(key)
        threads = (tm // wm) * (tn // wn) * 128
        cpp = ck // 8
        assert (tn * cpp) % threads == 0 and (threads // 16) % cpp == 0, key  # the filter loader's conditions
        assert (pl * threads) % cpp == 0 and pl <= 7, key
        out.append((BF16, 0, tm, tn, ck, wm, wn, 32, 16, 2, stride, pl))
    return out


def spilling():
    """(kernel name, template arguments) of the instances listed in spilling_variants.txt."""
    import re
    out = set()
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "spilling_variants.txt")
    if os.path.exists(path):
        with open(path) as f:
            for ln in f:
                m = re.match(r"(\w+)<(.*)>", ln.strip())
                if m:
                    out.add((m.group(1), tuple(int(x) for x in m.group(2).split(","))))
    return out


def variants(which):
    tiles = TILES_SMALL if which == "small" else TILES_FULL
    out = []
    for dt in (F32, BF16):
        tks = (16, 32) if dt == F32 else (32, 64)
        for fam in FAMILIES:
            for tm, tn, wm, wn in tiles:
                for mf in (16, 32):
                    if wm % mf or wn % mf:
                        continue
                    deep = ((64,) if dt == F32 else (128,)) if (tm, tn, wm, wn) in DEEP_K_TILES else ()
                    for tk in tks + deep:
                        # conv kernels come in two copies: 16-byte gathers, and element-wise gathers for
                        # channel counts that do not fill 16-byte items
                        amodes = (0,) if fam != 0 else ((16, 4) if dt == F32 else (16, 2))
                        for am in amodes:
                            if am not in (0, 16) and tk not in tks:
                                continue  # the element-wise gather keeps much per-item state: no deep slices
                            out.append((dt, fam, tm, tn, tk, wm, wn, mf, am, 0, 0))
                            if async_ok(dt, fam, tm, tn, tk, wm, wn, am):
                                out.append((dt, fam, tm, tn, tk, wm, wn, mf, am, 1, 0))
    skip = spilling()
    out = [v for v in out if not (v[9] == 0 and ("contract_kernel", v[:9]) in skip)]
    patch = [v for v in patch_variants() if ("conv3x3_patch_kernel", (v[2], v[3], v[4], v[5], v[6], v[10], v[11])) not in skip]
    return out + patch + stream_variants()


def async_ok(dt, fam, tm, tn, tk, wm, wn, am):
    """Tiles the asynchronous (global -> LDS) pipeline can load: whole 16-byte items per thread, and the
    threads of a workgroup covering whole groups of 16 rows so that one swizzle serves all of a thread's items."""
    if not (fam == 1 or (fam == 0 and am == 16)):
        return False
    threads = (tm // wm) * (tn // wn) * 64
    cpr = tk * (4 if dt == F32 else 2) // 16
    return (tm * cpr) % threads == 0 and (tn * cpr) % threads == 0 and (threads // 16) % cpr == 0


def main():
    out_dir = sys.argv[1]
    n_slices = int(sys.argv[2]) if len(sys.argv) > 2 else 16
    which = sys.argv[3] if len(sys.argv) > 3 else "full"
    os.makedirs(out_dir, exist_ok=True)
    vs = variants(which)
    slices = [[] for _ in range(n_slices)]
    for i, v in enumerate(vs):
        slices[i % n_slices].append((i, v))
    for s, items in enumerate(slices):
        lines = ['// generated by gen_variants.py - do not edit', '#include "../contract.hip.h"',
                 '#include "../conv_patch.hip.h"', '#include "../stream_gemm.hip.h"', "namespace tt {"]
        for i, v in items:
            if v[9] == 2:
                args = ", ".join(str(x) for x in (v[2], v[3], v[4], v[5], v[6], v[10], v[11]))
                call, size, lds = (f"launch_conv_patch<{args}>", f"capacity_conv_patch<{args}>",
                                   f"lds_bytes_conv_patch<{args}>")
            elif v[9] == 3:
                args = ", ".join(str(x) for x in (v[0], v[2], v[3], v[4], v[5], v[6], v[7]))
                call, size, lds = (f"launch_gemm_stream<{args}>", f"requests_gemm_stream<{args}>",
                                   f"lds_bytes_gemm_stream<{args}>")
            elif v[9] == 1:
                args = ", ".join(str(x) for x in v[:8])
                call, size, lds = (f"launch_contract_async<{args}>", f"stage_bytes_contract_async<{args}>",
                                   f"lds_bytes_contract_async<{args}>")
            else:
                args = ", ".join(str(x) for x in v[:9])
                call, size, lds = f"launch_contract<{args}>", f"stage_bytes_contract<{args}>", f"lds_bytes_contract<{args}>"
            lines.append(f"int ttv_{i}(const ContractArgs &a, int grid, int lds, void *s) "
                         f"{{ return {call}(a, grid, lds, s); }}")
            lines.append(f"int tts_{i}() {{ return {size}(); }}")
            lines.append(f"int ttl_{i}(int stages) {{ return {lds}(stages); }}")
        lines.append("} // namespace tt")
        write_if_changed(os.path.join(out_dir, f"inst_{s:02d}.hip"), "\n".join(lines) + "\n")
    lines = ['// generated by gen_variants.py - do not edit', '#include "../tt_internal.h"', "namespace tt {"]
    for i, _ in enumerate(vs):
        lines.append(f"int ttv_{i}(const ContractArgs &, int, int, void *);")
        lines.append(f"int tts_{i}();")
        lines.append(f"int ttl_{i}(int);")
    lines.append("const Variant kVariants[] = {")
    for i, v in enumerate(vs):
        lines.append("    {" + ", ".join(str(x) for x in v[:11]) + f", ttv_{i}, tts_{i}, ttl_{i}}},")
    lines.append("};")
    lines.append(f"const int kNumVariants = {len(vs)};")
    lines.append("} // namespace tt")
    write_if_changed(os.path.join(out_dir, "variants_table.cpp"), "\n".join(lines) + "\n")
    print(f"{len(vs)} variants in {n_slices} slices ({which})")


def write_if_changed(path, text):
    if os.path.exists(path):
        with open(path) as f:
            if f.read() == text:
                return
    with open(path, "w") as f:
        f.write(text)


if __name__ == "__main__":
    main()
