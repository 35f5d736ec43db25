"""Tile-configuration search for one convolution shape on the GPU at hand.

The paper picks the tile sizes of its kernels by exploring the design space per device
(Sec. 5: 256 x 8 tiles for the special case, Table 1 for the general case).  The library
compiles a handful of tile configurations per kernel and picks one by shape with rules
measured on MI355X; this module times every configuration of a given shape through the
C ABI (variant VARIANT_TILED_CFG0 + i) and reports them next to the library's own choice, so
that the rules can be checked or re-derived on another chip.

    python -m paper_1705_10591_amd.tune single H W K F
    python -m paper_1705_10591_amd.tune general N C H W K F
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


def tune(kind: str, dims, steps: int = 20):
    """Return [(label, ms or None)] for the library's choice and every tile configuration."""
    gen = torch.Generator(device="cuda").manual_seed(1705)
    if kind == "single":
        H, W, K, F = dims
        x = torch.rand(H, W, device="cuda", generator=gen)
        f = torch.rand(K, F, F, device="cuda", generator=gen) - 0.5
        out = torch.empty(K, H - F + 1, W - F + 1, device="cuda")
        call = lambda v: dconv.dconv_single_channel(x, f, out=out, variant=v)
    else:
        N, C, H, W, K, F = dims
        x = torch.rand(N, C, H, W, device="cuda", generator=gen)
        f = (torch.rand(K, C, F, F, device="cuda", generator=gen) - 0.5) * 0.1
        out = torch.empty(N, K, H - F + 1, W - F + 1, device="cuda")
        call = lambda v: dconv.dconv_general(x, f, out=out, variant=v)
    rows = [("library choice", _time(lambda: call(dconv.VARIANT_AUTO), steps=steps))]
    for i in range(dconv.tile_config_count(kind == "single")):
        v = dconv.VARIANT_TILED_CFG0 + i
        try:
            call(v)
        except dconv.DconvError as e:
            if e.status != dconv.STATUS_UNSUPPORTED:
                raise
            rows.append((f"configuration {i}", None))
            continue
        rows.append((f"configuration {i}", _time(lambda: call(v), steps=steps)))
    return rows


def main(argv):
    if len(argv) < 2 or argv[0] not in ("single", "general") or \
            len(argv) - 1 != (4 if argv[0] == "single" else 6):
        print(__doc__)
        return 2
    if not torch.cuda.is_available():
        print("tune needs a GPU", file=sys.stderr)
        return 2
    rows = tune(argv[0], [int(a) for a in argv[1:]])
    best = min((ms for _, ms in rows[1:] if ms is not None), default=None)
    for label, ms in rows:
        mark = " <- fastest" if ms is not None and ms == best and label != "library choice" else ""
        print(f"{label:18s} {'not applicable' if ms is None else f'{ms:9.4f} ms'}{mark}")
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
