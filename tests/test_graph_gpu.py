"""The entry points under HIP graph capture: captured once, replayed several times.

Every entry point only enqueues kernels on the stream it is given, so a sequence of calls can be
captured into a graph and replayed without the launch cost of each call.  dconv_general may
allocate (and clear) its workspace on the first call that needs it on a stream, which is not
allowed while capturing: the calls are run once on the capture stream beforehand.

Each replay is checked against the eager results bit for bit (the kernels are deterministic,
shared tiles included), with the outputs cleared and eager work of the same library between the
replays, and the eager results against the oracle.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_1705_10591_amd as dconv
from helpers import assert_within_bound

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


def test_captured_graph_replays_match_eager_calls():
    shared = dconv.VARIANT_TILED_CFG0 + 2 * 3 + 1      # 64 x 256 tile, tiles shared between workgroups
    x1, f1 = wl.random_case(31, 1, 1, 200, 300, 16, 3)
    img, fs = x1[0, 0], f1[:, 0]
    xg, fg = wl.random_case(32, 2, 8, 30, 30, 70, 3)
    xs, fsh = wl.random_case(33, 3, 16, 28, 28, 130, 3)
    xh, fh = wl.random_case(34, 2, 32, 20, 23, 40, 3)
    x1g, f1g = wl.random_case(35, 1, 1, 64, 64, 128, 8)      # one channel that the general-case kernel runs
    xf, ff = wl.random_case(36, 3, 5, 40, 300, 3, 3)         # three filters: the few-filters kernel
    assert dconv.tile_choice(True, 1, 1, 64, 64, 128, 8) == dconv.CHOICE_GENERAL_CASE
    xhr, xhb = wl.to_16bit(xh, "bf16")              # rounded values for the oracle, bits for the device
    fhr, fhb = wl.to_16bit(fh, "bf16")

    d_img, d_fs, d_xg, d_fg, d_xs, d_fsh = map(dev, (img, fs, xg, fg, xs, fsh))
    d_xh, d_fh = (torch.from_numpy(np.ascontiguousarray(np.moveaxis(b, 1, -1)).view(np.int16))
                  .view(torch.bfloat16).to("cuda") for b in (xhb, fhb))       # channels last
    d_x1g, d_f1g, d_xf, d_ff = dev(x1g[0, 0]), dev(f1g[:, 0]), dev(xf), dev(ff)
    outs = [torch.empty(16, 198, 298, device="cuda"), torch.empty(2, 70, 28, 28, device="cuda"),
            torch.empty(3, 130, 26, 26, device="cuda"), torch.empty(2, 40, 18, 21, device="cuda"),
            torch.empty(128, 57, 57, device="cuda"), torch.empty(3, 3, 38, 298, device="cuda")]

    def enqueue():
        dconv.dconv_single_channel(d_img, d_fs, out=outs[0])
        dconv.dconv_general(d_xg, d_fg, out=outs[1])
        dconv.dconv_general(d_xs, d_fsh, out=outs[2], variant=shared)
        dconv.dconv_general_half(d_xh, d_fh, out=outs[3])
        dconv.dconv_single_channel(d_x1g, d_f1g, out=outs[4])
        dconv.dconv_general(d_xf, d_ff, out=outs[5], variant=dconv.VARIANT_FEW_FILTERS)

    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        enqueue()                      # on the capture stream: its workspace exists from here on
    s.synchronize()
    eager = [o.clone() for o in outs]

    print("capturing six launches into one graph", flush=True)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        enqueue()
    for rep in range(4):
        for o in outs:
            o.fill_(float("nan"))
        torch.cuda.synchronize()
        print(f"replay {rep}", flush=True)
        g.replay()
        torch.cuda.synchronize()
        for i, (o, e) in enumerate(zip(outs, eager)):
            assert torch.equal(o, e), f"replay {rep}, launch {i}"
        # eager work of the same kernels between replays (other buffers, default stream)
        other = dconv.dconv_general(d_xs, d_fsh, variant=shared)
        torch.cuda.synchronize()
        assert torch.equal(other, eager[2])

    acc, mag, _ = oracle.single_channel(img, fs)
    assert_within_bound(eager[0].cpu().numpy(), acc, mag, "single channel")
    for (x, f), e, what in (((xg, fg), eager[1], "general"), ((xs, fsh), eager[2], "general, shared tiles"),
                            ((x1g, f1g), eager[4][None], "one channel on the general kernel"),
                            ((xf, ff), eager[5], "general, few filters")):
        acc, mag, _ = oracle.general(x, f)
        assert_within_bound(e.cpu().numpy(), acc, mag, what)
    acc, mag, _ = oracle.general(xhr, fhr)
    assert_within_bound(eager[3].cpu().numpy(), acc, mag, "general bf16")


def test_graph_stays_valid_when_later_calls_on_its_stream_need_a_larger_workspace():
    """The workspace of a stream keeps its address: a graph that captured a small shared-tile
    launch is replayed after a much larger shared-tile call ran eagerly on the same stream."""
    shared = dconv.VARIANT_TILED_CFG0 + 3 * 3 + 1      # 64 x 256 tile, shared over seven workgroups
    xs, fs = wl.random_case(41, 3, 16, 28, 28, 130, 3)
    d_xs, d_fs = dev(xs), dev(fs)
    out_small = torch.empty(3, 130, 26, 26, device="cuda")
    big = wl.G3                                         # shares its tiles over the whole chip
    xb, fb = wl.make_inputs(big)
    d_xb, d_fb = dev(xb), dev(fb)
    out_big = torch.empty(big.out_shape(), device="cuda")
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        dconv.dconv_general(d_xs, d_fs, out=out_small, variant=shared)     # first use: allocates
    s.synchronize()
    eager_small = out_small.clone()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        dconv.dconv_general(d_xs, d_fs, out=out_small, variant=shared)
    for rep in range(3):
        with torch.cuda.stream(s):
            dconv.dconv_general(d_xb, d_fb, out=out_big)                   # needs the whole block
        s.synchronize()
        if rep == 0:
            eager_big = out_big.clone()
        assert torch.equal(out_big, eager_big)
        out_small.fill_(float("nan"))
        torch.cuda.synchronize()
        print(f"replay {rep} after the large call", flush=True)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_small, eager_small), f"replay {rep}"
    acc, mag, _ = oracle.general(xs, fs)
    assert_within_bound(eager_small.cpu().numpy(), acc, mag, "small shared-tile launch")
