"""Tile-configuration search for one convolution shape on the GPU at hand.

The paper picks the tile sizes of its kernels by exploring the design space per device
(Sec. 5: 256 x 8 tiles for the special case, Table 1 for the general case).  The library
compiles a handful of tile configurations per kernel and picks one by shape with rules
measured on MI355X; this module times every configuration of a given shape through the
C ABI (variant VARIANT_TILED_CFG0 + i) and reports them next to the library's own choice, so
that the rules can be checked or re-derived on another chip.

    python -m paper_1705_10591_amd.tune single H W K F
    python -m paper_1705_10591_amd.tune general N C H W K F
    python -m paper_1705_10591_amd.tune bf16 N C H W K F          (general case, bf16 inputs)
    python -m paper_1705_10591_amd.tune bf16-blocked N C H W K F  (the same, channel-blocked layout)
    python -m paper_1705_10591_amd.tune special N C H W K F       (general case with C <= 4: the tile
                                                                   configurations of the special-case
                                                                   kernel next to the general kernel)
    python -m paper_1705_10591_amd.tune table single|general|bf16|bf16-blocked
                                                                  (the shapes the rules were set on)
    python -m paper_1705_10591_amd.tune random single|general SEED COUNT
                                                                  (shapes drawn at random: the check of the rules
                                                                   on shapes they were not set on)
    python -m paper_1705_10591_amd.tune route SEED COUNT          (one image of one channel on shapes drawn at
                                                                   random: the library's choice, the special
                                                                   case's kernel and the general-case kernel)
    python -m paper_1705_10591_amd.tune units                     (special case: 16-byte against 4-byte units
                                                                   on the way out, the width-matching ablation)
    python -m paper_1705_10591_amd.tune writeback                 (general case: stores straight from the
                                                                   accumulators against the line-aligned
                                                                   write-back through LDS, per tile shape)
    python -m paper_1705_10591_amd.tune operands                  (the benchmark shapes on random inputs against
                                                                   the same launches on an input of zeros: what
                                                                   the chip's power management takes)
"""
from __future__ import annotations

import sys
import time

import torch

import paper_1705_10591_amd as dconv


def _time(fn, warm_ms: float = 40.0, steps: int = 20) -> float:
    t0 = time.perf_counter()
    n = 0
    while n < 3 or (time.perf_counter() - t0) * 1e3 < warm_ms:
        fn()
        n += 1
        if n % 8 == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def _config_count(kind: str) -> int:
    # the short-data-type kernel: 64 filters x 256 pixels and 128 x 512 staged through registers,
    # the same two and 128 x 384 staged directly into LDS
    if kind.startswith("bf16"):
        return 5
    # general case: configurations 0..11 (12..23 repeat them with the line-aligned write-back,
    # see `writeback`)
    return 12 if kind == "general" else dconv.tile_config_count(kind in ("single", "special"))


def tune(kind: str, dims, steps: int = 20):
    """Return [(label, ms or None)] for the library's choice and every tile configuration."""
    gen = torch.Generator(device="cuda").manual_seed(1705)
    if kind == "single":
        H, W, K, F = dims
        x = torch.rand(H, W, device="cuda", generator=gen)
        f = torch.rand(K, F, F, device="cuda", generator=gen) - 0.5
        out = torch.empty(K, H - F + 1, W - F + 1, device="cuda")
        call = lambda v: dconv.dconv_single_channel(x, f, out=out, variant=v)
    elif kind.startswith("bf16"):
        N, C, H, W, K, F = dims
        blocked = kind == "bf16-blocked"
        xs, fs = ((N, C // 16, H, W, 16), (K, C // 16, F, F, 16)) if blocked else ((N, H, W, C), (K, F, F, C))
        x = torch.rand(*xs, device="cuda", generator=gen).to(torch.bfloat16)
        f = ((torch.rand(*fs, device="cuda", generator=gen) - 0.5) * 0.1).to(torch.bfloat16)
        out = torch.empty(N, K, H - F + 1, W - F + 1, device="cuda")
        call = lambda v: dconv.dconv_general_half(x, f, out=out, variant=v, blocked=blocked)
    else:
        N, C, H, W, K, F = dims
        x = torch.rand(N, C, H, W, device="cuda", generator=gen)
        f = (torch.rand(K, C, F, F, device="cuda", generator=gen) - 0.5) * 0.1
        out = torch.empty(N, K, H - F + 1, W - F + 1, device="cuda")
        call = lambda v: dconv.dconv_general(x, f, out=out, variant=v)
    if kind == "special":
        rows = [("library choice", _time(lambda: call(dconv.VARIANT_AUTO), steps=steps)),
                ("general kernel", _time(lambda: call(dconv.VARIANT_TILED), steps=steps))]
        first = dconv.VARIANT_SPECIAL_CASE_CFG0
    else:
        rows = [("library choice", _time(lambda: call(dconv.VARIANT_AUTO), steps=steps))]
        first = dconv.VARIANT_TILED_CFG0
    for i in range(_config_count(kind)):
        v = first + i
        try:
            call(v)
        except dconv.DconvError as e:
            if e.status != dconv.STATUS_UNSUPPORTED:
                raise
            rows.append((f"configuration {i}", None))
            continue
        rows.append((f"configuration {i}", _time(lambda: call(v), steps=steps)))
    return rows


# The shapes the library's rules were derived from: (H, W, K, F) and (N, C, H, W, K, F).
TABLE_SINGLE = [(4096, 4096, 64, 5), (4096, 4096, 64, 3), (4096, 4096, 64, 7), (4096, 4096, 64, 11),
                (2048, 2048, 64, 5), (2048, 2048, 64, 9), (1024, 1024, 64, 5), (1024, 1024, 64, 9),
                (1024, 1024, 64, 3), (512, 512, 64, 3), (1080, 1920, 32, 3), (1080, 1920, 64, 7),
                (256, 256, 16, 3), (1536, 1536, 128, 3), (3000, 3000, 64, 5), (2048, 2048, 256, 5),
                (720, 1280, 96, 5),
                # images that 512-pixel tiles divide unevenly over the CUs
                (720, 1280, 64, 9), (1080, 1920, 64, 9), (1536, 1536, 64, 9), (1800, 1800, 64, 7),
                (1280, 1280, 32, 8), (900, 1600, 128, 11), (600, 800, 64, 7), (720, 1280, 32, 5),
                # up to 32 filters: one filter block, rows dealt to the waves
                (256, 256, 32, 5), (512, 512, 32, 3), (768, 768, 16, 3), (768, 768, 32, 5),
                (1024, 1024, 16, 3), (1024, 1024, 16, 5), (1024, 1024, 32, 7), (2048, 2048, 16, 3),
                # up to 16 filters: blocks of 16 filters (configurations 9 and 10); where the library
                # picks the vector-ALU kernel for few filters, its time is the first column's
                (4096, 4096, 16, 5), (4096, 4096, 8, 3), (2048, 2048, 16, 7), (1536, 1536, 8, 4),
                (1080, 1920, 12, 7), (720, 1280, 16, 5), (3000, 3000, 8, 5)]
TABLE_GENERAL = [(32, 64, 56, 56, 64, 3), (32, 256, 28, 28, 512, 3), (64, 3, 224, 224, 64, 11),
                 (32, 128, 56, 56, 128, 3), (32, 256, 14, 14, 256, 3), (16, 64, 112, 112, 128, 3),
                 (64, 32, 32, 32, 32, 3), (32, 96, 27, 27, 256, 5), (16, 64, 224, 224, 64, 3),
                 (64, 128, 28, 28, 128, 3), (16, 512, 14, 14, 512, 3), (32, 192, 13, 13, 384, 3),
                 (8, 3, 224, 224, 32, 3), (32, 16, 64, 64, 32, 5), (128, 64, 32, 32, 128, 3),
                 (32, 64, 56, 56, 64, 5), (32, 64, 56, 56, 64, 7), (32, 64, 56, 56, 256, 3),
                 (8, 128, 112, 112, 128, 3), (64, 512, 7, 7, 512, 3),
                 # few multiply-adds per output: the output stream is a large part of the time
                 (64, 8, 224, 224, 64, 3), (256, 8, 112, 112, 64, 3), (256, 16, 112, 112, 64, 3),
                 (512, 8, 56, 56, 128, 3), (256, 32, 112, 112, 64, 1),
                 # 1x1 layers
                 (128, 256, 28, 28, 256, 1), (64, 512, 14, 14, 512, 1), (512, 64, 56, 56, 128, 1),
                 (58, 64, 112, 112, 128, 1), (7, 256, 112, 112, 256, 1),
                 # fewer tiles than CUs (small batches of deep layers): tiles shared over channels
                 (1, 512, 14, 14, 512, 3), (1, 384, 20, 20, 384, 7), (4, 512, 17, 14, 448, 1),
                 (2, 384, 28, 28, 256, 5), (1, 256, 28, 28, 256, 3),
                 # filter counts that are not multiples of 64; 2x2 filters
                 (13, 64, 75, 75, 96, 3), (19, 256, 48, 48, 160, 3), (94, 8, 224, 224, 64, 2),
                 (108, 320, 30, 30, 128, 2)]

# Shapes for the comparison of the two write-backs: few multiply-adds per output element, maps
# narrower and wider than a column strip, outputs below and above the 256 MB memory-side cache;
# and the three benchmark shapes of the general case.
TABLE_WRITEBACK = [(64, 8, 224, 224, 64, 3), (64, 16, 224, 224, 64, 3), (64, 8, 130, 130, 64, 3),
                   (64, 16, 130, 130, 64, 3), (128, 8, 56, 56, 64, 3), (64, 16, 112, 112, 64, 3),
                   (256, 8, 112, 112, 64, 3), (256, 16, 112, 112, 64, 3), (512, 8, 56, 56, 128, 3),
                   (256, 32, 112, 112, 64, 1), (512, 64, 56, 56, 128, 1),
                   (64, 3, 224, 224, 64, 11), (32, 64, 56, 56, 64, 3), (32, 256, 28, 28, 512, 3)]


TABLE_BF16 = [(32, 64, 56, 56, 64, 3), (32, 256, 28, 28, 512, 3), (32, 128, 56, 56, 128, 3),
              (64, 64, 112, 112, 128, 3), (32, 64, 56, 56, 64, 5), (32, 128, 56, 56, 256, 5),
              (64, 256, 56, 56, 256, 3), (128, 512, 14, 14, 512, 1), (32, 64, 56, 56, 128, 7),
              (16, 512, 14, 14, 512, 3), (64, 128, 28, 28, 128, 3), (8, 128, 112, 112, 128, 3)]


KINDS = ("single", "general", "bf16", "bf16-blocked")     # with a table of shapes



def table(kind: str) -> None:
    """One line per shape: the library's choice and every configuration, in microseconds."""
    shapes = {"single": TABLE_SINGLE, "general": TABLE_GENERAL, "bf16": TABLE_BF16,
              "bf16-blocked": TABLE_BF16}[kind]
    n = _config_count(kind)
    print(f"# {kind}: microseconds per launch; columns: library choice, configurations 0..{n - 1} "
          "(n/a = cannot hold the shape), fastest configuration, library / fastest (below 1 where the "
          "library runs the shape on another kernel than the one whose configurations are listed)")
    for sh in shapes:
        rows = tune(kind, sh)
        lib, cfgs = rows[0][1], [ms for _, ms in rows[1:]]
        best = min(ms for ms in cfgs if ms is not None)
        cells = " ".join("    n/a" if ms is None else f"{ms * 1e3:7.1f}" for ms in cfgs)
        print(f"{'x'.join(map(str, sh)):24s} {lib * 1e3:7.1f} | {cells} | {cfgs.index(best):2d} {lib / best:5.2f}",
              flush=True)


def random_shapes(kind: str, seed: int, count: int):
    """Shapes drawn at random (Python's own generator, so the same seed gives the same shapes
    anywhere): images 400 to 3000 pixels on a side with 24 to 200 filters of 3x3 to 11x11 for
    the special case; layers of 3 to 512 channels, 16 to 512 filters of 1x1 to 7x7 on 7 x 7 to
    224 x 224 maps, 0.5 to 30 GFLOP, for the general case."""
    import random
    rng = random.Random(seed)
    shapes = []
    while len(shapes) < count:
        if kind == "single":
            H, W = rng.randint(400, 3000), rng.randint(400, 3000)
            K = rng.choice((24, 32, 48, 64, 96, 128, 200))
            F = rng.choice((3, 4, 5, 6, 7, 8, 9, 10, 11))
            if K * H * W * 4 <= 3e9:
                shapes.append((H, W, K, F))
            continue
        C = rng.choice((3, 6, 8, 12, 16, 24, 32, 48, 64, 96, 128, 160, 192, 256, 320, 384, 512))
        K = rng.choice((16, 32, 48, 64, 80, 96, 112, 128, 160, 192, 224, 256, 288, 320, 384, 448, 512))
        F = rng.choice((1, 2, 3, 3, 3, 4, 5, 5, 7))
        H = rng.choice((7, 8, 10, 13, 14, 17, 20, 24, 28, 30, 35, 40, 48, 56, 60, 64, 75, 96, 112,
                        128, 150, 224))
        W = H if rng.random() < 0.7 else rng.choice((14, 28, 40, 56, 80, 112, 160))
        if F > min(H, W):
            continue
        Ho, Wo = H - F + 1, W - F + 1
        N = max(1, min(512, int(rng.choice((0.5e9, 2e9, 8e9, 30e9)) / (2.0 * C * K * F * F * Ho * Wo))))
        if N * C * H * W * 4 <= 2e9 and N * K * Ho * Wo * 4 <= 2e9:
            shapes.append((N, C, H, W, K, F))
    return shapes


def random_table(kind: str, seed: int, count: int) -> None:
    """The library's choice against every tile configuration on shapes drawn at random; the
    lines of the shapes where the choice is 8 % or more above the fastest, and a summary."""
    n = _config_count(kind)
    print(f"# {kind}, {count} random shapes (seed {seed}): microseconds per launch; the library's choice and "
          f"the fastest of configurations 0..{n - 1} (the ablation excluded; where the library runs a shape on "
          "another kernel than the one with these configurations its time can be below the fastest); shapes "
          "listed where the choice is 8 % or more above the fastest")
    ratios = []
    for sh in random_shapes(kind, seed, count):
        rows = tune(kind, sh, steps=6)
        lib = rows[0][1]
        cfgs = [None if (kind == "single" and i == 7) else ms for i, (_, ms) in enumerate(rows[1:])]
        best = min(ms for ms in cfgs if ms is not None)
        ratios.append(lib / best)
        if lib / best >= 1.08:
            print(f"{'x'.join(map(str, sh)):28s} {lib * 1e3:8.1f} {best * 1e3:8.1f}  configuration "
                  f"{cfgs.index(best):2d}  {lib / best:5.2f}", flush=True)
    ratios.sort()
    m = len(ratios)
    print(f"# library / fastest over {m} shapes: mean {sum(ratios) / m:.3f}, median {ratios[m // 2]:.3f}, "
          f"90th percentile {ratios[(9 * m) // 10]:.3f}, worst {ratios[-1]:.2f}; "
          f"{sum(r >= 1.06 for r in ratios)} shapes 6 % or more above the fastest")


def route_table(seed: int, count: int) -> None:
    """One image of one channel: the library's choice against the special case's kernel (its own
    tile choice) and the general-case kernel (its own tile choice) on shapes drawn at random --
    images 64 to 4096 pixels on a side, 9 to 512 filters of 1x1 to 11x11.  Lists the shapes where
    the choice is 10 % or more above the faster of the two, and a summary."""
    import random
    rng = random.Random(seed)
    print(f"# one channel, {count} random shapes (seed {seed}): microseconds per launch of the library's choice, "
          "the special case's kernel and the general-case kernel; shapes listed where the choice is 10 % or "
          "more above the faster kernel")
    lib_r, special_r, general_r = [], [], []
    gen = torch.Generator(device="cuda").manual_seed(1705)
    done = 0
    while done < count:
        K = rng.choice((9, 12, 16, 17, 24, 32, 32, 40, 48, 64, 64, 80, 96, 128, 128, 160, 192, 224, 256, 320, 512))
        F = rng.randint(1, 11)
        H = rng.choice((64, 96, 128, 150, 224, 256, 384, 512, 768, 1024, 1536, 2048, 3000, 4096))
        W = H if rng.random() < 0.7 else rng.choice((100, 160, 320, 640, 1280, 1920))
        if F > min(H, W):
            continue
        Ho, Wo = H - F + 1, W - F + 1
        if K * Ho * Wo * 4 > 4.5e9 or K * Ho * Wo < 2e5:
            continue
        x = torch.rand(1, 1, H, W, device="cuda", generator=gen) * 2 - 1
        f = torch.rand(K, 1, F, F, device="cuda", generator=gen) * 2 - 1
        out = torch.empty(1, K, Ho, Wo, device="cuda")
        x1, f1, out1 = x[0, 0], f[:, 0], out[0]
        # (interleaved and repeated: the clock settles differently after a long and a short launch)
        t = [1e30, 1e30, 1e30]
        for _ in range(2):
            t[0] = min(t[0], _time(lambda: dconv.dconv_single_channel(x1, f1, out=out1), 8, 6))
            t[1] = min(t[1], _time(lambda: dconv.dconv_single_channel(x1, f1, out=out1, variant=dconv.VARIANT_TILED), 8, 6))
            t[2] = min(t[2], _time(lambda: dconv.dconv_general(x, f, out=out, variant=dconv.VARIANT_TILED), 8, 6))
        best = min(t[1:])
        lib_r.append(t[0] / best); special_r.append(t[1] / best); general_r.append(t[2] / best)
        if t[0] / best >= 1.10:
            print(f"{H}x{W}x{K}x{F:<3d} {t[0] * 1e3:9.1f} {t[1] * 1e3:9.1f} {t[2] * 1e3:9.1f}  choice "
                  f"{dconv.tile_choice(True, 1, 1, H, W, K, F):3d}  {t[0] / best:5.2f}", flush=True)
        del x, f, out, x1, f1, out1
        done += 1
    m = len(lib_r)
    mean = lambda r: sum(r) / len(r)
    print(f"# time / faster kernel's time over {m} shapes: library's choice mean {mean(lib_r):.3f} "
          f"({sum(r >= 1.10 for r in lib_r)} shapes 10 % or more above), special case's kernel alone {mean(special_r):.3f} "
          f"({sum(r >= 1.10 for r in special_r)}), general-case kernel alone {mean(general_r):.3f} "
          f"({sum(r >= 1.10 for r in general_r)})")


def writeback_table() -> None:
    """Per shape: the library's choice, the three tile shapes with stores straight from the
    accumulators (configurations 0..2) and with the line-aligned write-back (12..14)."""
    print("# general case, microseconds per launch: library choice | 64x128, 64x256, 32x256 tiles straight "
          "from the accumulators | the same through LDS in whole lines | bound = max(flops / 157.3 TFLOP/s, "
          "bytes / 8 TB/s) | output MB | best straight / best aligned")
    for sh in TABLE_WRITEBACK:
        N, C, H, W, K, F = sh
        gen = torch.Generator(device="cuda").manual_seed(1705)
        x = torch.rand(N, C, H, W, device="cuda", generator=gen)
        f = (torch.rand(K, C, F, F, device="cuda", generator=gen) - 0.5) * 0.1
        out = torch.empty(N, K, H - F + 1, W - F + 1, device="cuda")
        t = [_time(lambda: dconv.dconv_general(x, f, out=out, variant=v))
             for v in [dconv.VARIANT_AUTO] + [dconv.VARIANT_TILED_CFG0 + i for i in (0, 1, 2, 12, 13, 14)]]
        flops = 2.0 * out.numel() * C * F * F
        byts = 4.0 * (x.numel() + f.numel() + out.numel())
        bound = max(flops / 157.3e12, byts / 8e12) * 1e6
        print(f"{'x'.join(map(str, sh)):24s} {t[0] * 1e3:7.1f} | " + " ".join(f"{v * 1e3:7.1f}" for v in t[1:4]) + " | " +
              " ".join(f"{v * 1e3:7.1f}" for v in t[4:7]) + f" | {bound:7.1f} | {out.numel() * 4 / 1e6:6.0f} | "
              f"{min(t[1:4]) / min(t[4:7]):4.2f}", flush=True)
        del x, f, out
        torch.cuda.empty_cache()


def unit_table() -> None:
    """The paper's matched-against-unmatched experiment (Sec. 5.1: its 3x3 kernel is 19 % slower
    when a thread moves units narrower than the hardware serves best) inside the special-case
    kernel: tile configuration 0 moves 16 bytes per lane from the write-back strips to memory,
    configuration 7 is the same kernel moving 4 bytes per lane."""
    print("# special case, 64 filters, milliseconds per launch: 16-byte unit | 4-byte unit | ratio")
    for H, W, K, F in [(4096, 4096, 64, 1), (4096, 4096, 64, 3), (4096, 4096, 64, 5), (4096, 4096, 64, 7),
                       (2048, 2048, 64, 3)]:
        gen = torch.Generator(device="cuda").manual_seed(1705)
        x = torch.rand(H, W, device="cuda", generator=gen)
        f = torch.rand(K, F, F, device="cuda", generator=gen) - 0.5
        out = torch.empty(K, H - F + 1, W - F + 1, device="cuda")
        t = {}
        for rep in range(2):        # alternate, so that neither gets the warmer chip
            for name, cfg in (("16", 0), ("4", 7)):
                ms = _time(lambda: dconv.dconv_single_channel(x, f, out=out, variant=dconv.VARIANT_TILED_CFG0 + cfg),
                           warm_ms=60.0, steps=30)
                t[name] = min(ms, t.get(name, ms))
        print(f"{H}x{W}x{K}x{F:<3d} {t['16']:8.4f} | {t['4']:8.4f} | {t['4'] / t['16']:5.3f}", flush=True)
        del x, f, out
        torch.cuda.empty_cache()


def operand_table() -> None:
    """The same launch on an input of zeros: instructions, addresses and memory traffic are those of
    the random input, what the matrix cores and the memory draw is not, and the clock follows."""
    print("# milliseconds per launch, random filters: random input | input of zeros | ratio")
    rows = [("S2 F=%d" % F, (4096, 4096, 64, F)) for F in (3, 5, 7, 9, 11)]
    rows += [("G1", (64, 3, 224, 224, 64, 11)), ("G2", (32, 64, 56, 56, 64, 3)), ("G3", (32, 256, 28, 28, 512, 3)),
             ("G3 bf16", (32, 256, 28, 28, 512, 3)), ("G3 int8", (32, 256, 28, 28, 512, 3))]
    for name, sh in rows:
        gen = torch.Generator(device="cuda").manual_seed(1705)
        if len(sh) == 4:
            H, W, K, F = sh
            xs = [torch.rand(H, W, device="cuda", generator=gen), torch.zeros(H, W, device="cuda")]
            f = torch.rand(K, F, F, device="cuda", generator=gen) - 0.5
            out = torch.empty(K, H - F + 1, W - F + 1, device="cuda")
            call = lambda x: dconv.dconv_single_channel(x, f, out=out)
        else:
            N, C, H, W, K, F = sh
            if name.endswith("bf16") or name.endswith("int8"):
                if name.endswith("bf16"):
                    x = (torch.rand(N, H, W, C, device="cuda", generator=gen) - 0.5).to(torch.bfloat16)
                    f = (torch.rand(K, F, F, C, device="cuda", generator=gen) - 0.5).to(torch.bfloat16)
                    out = torch.empty(N, K, H - F + 1, W - F + 1, device="cuda")
                    call = lambda x: dconv.dconv_general_half(x, f, out=out)
                else:
                    x = torch.randint(-128, 128, (N, H, W, C), device="cuda", generator=gen, dtype=torch.int8)
                    f = torch.randint(-128, 128, (K, F, F, C), device="cuda", generator=gen, dtype=torch.int8)
                    out = torch.empty(N, K, H - F + 1, W - F + 1, device="cuda", dtype=torch.int32)
                    call = lambda x: dconv.dconv_general_i8(x, f, out=out)
                xs = [x, torch.zeros_like(x)]
            else:
                xs = [torch.rand(N, C, H, W, device="cuda", generator=gen), torch.zeros(N, C, H, W, device="cuda")]
                f = (torch.rand(K, C, F, F, device="cuda", generator=gen) - 0.5) * 0.1
                out = torch.empty(N, K, H - F + 1, W - F + 1, device="cuda")
                call = lambda x: dconv.dconv_general(x, f, out=out)
        t = [None, None]
        for rep in range(2):        # alternate, so that neither gets the warmer chip
            for i in (0, 1):
                ms = _time(lambda: call(xs[i]), warm_ms=80.0, steps=30)
                t[i] = ms if t[i] is None else min(t[i], ms)
        print(f"{name:10s} {t[0]:8.4f} | {t[1]:8.4f} | {t[0] / t[1]:5.3f}", flush=True)
        del xs, f, out
        torch.cuda.empty_cache()


def main(argv):
    if argv == ["operands"]:
        if not torch.cuda.is_available():
            print("tune needs a GPU", file=sys.stderr)
            return 2
        operand_table()
        return 0
    if argv == ["units"]:
        if not torch.cuda.is_available():
            print("tune needs a GPU", file=sys.stderr)
            return 2
        unit_table()
        return 0
    if argv == ["writeback"]:
        if not torch.cuda.is_available():
            print("tune needs a GPU", file=sys.stderr)
            return 2
        writeback_table()
        return 0
    if len(argv) == 4 and argv[0] == "random" and argv[1] in ("single", "general"):
        if not torch.cuda.is_available():
            print("tune needs a GPU", file=sys.stderr)
            return 2
        random_table(argv[1], int(argv[2]), int(argv[3]))
        return 0
    if len(argv) == 3 and argv[0] == "route":
        if not torch.cuda.is_available():
            print("tune needs a GPU", file=sys.stderr)
            return 2
        route_table(int(argv[1]), int(argv[2]))
        return 0
    if len(argv) == 2 and argv[0] == "table" and argv[1] in KINDS:
        if not torch.cuda.is_available():
            print("tune needs a GPU", file=sys.stderr)
            return 2
        table(argv[1])
        return 0
    if len(argv) < 2 or argv[0] not in KINDS + ("special",) or \
            len(argv) - 1 != (4 if argv[0] == "single" else 6):
        print(__doc__)
        return 2
    if not torch.cuda.is_available():
        print("tune needs a GPU", file=sys.stderr)
        return 2
    rows = tune(argv[0], [int(a) for a in argv[1:]])
    best = min((ms for label, ms in rows if ms is not None and label != "library choice"), default=None)
    for label, ms in rows:
        mark = " <- fastest" if ms is not None and ms == best and label != "library choice" else ""
        print(f"{label:18s} {'not applicable' if ms is None else f'{ms:9.4f} ms'}{mark}")
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
