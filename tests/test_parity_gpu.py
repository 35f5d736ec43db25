"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle.

Bar: integer-valued cases bit-exact; floating point within
|gpu - exact| <= 1e-5 * sum|x*w| per output element, where `exact` is the
oracle's fp64 sum.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_1705_10591_amd as dconv
from helpers import assert_within_bound

pytestmark = pytest.mark.gpu

SIMPLE, TILED, AUTO = dconv.VARIANT_SIMPLE, dconv.VARIANT_TILED, dconv.VARIANT_AUTO


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


def run_general(x, f, variant):
    print(f"general N,C,H,W={x.shape} K,F={f.shape[0]},{f.shape[-1]} variant={variant}", flush=True)
    out = dconv.dconv_general(dev(x), dev(f), variant=variant)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def run_single(img, f, variant):
    print(f"single H,W={img.shape} K,F={f.shape[0]},{f.shape[-1]} variant={variant}", flush=True)
    out = dconv.dconv_single_channel(dev(img), dev(f), variant=variant)
    torch.cuda.synchronize()
    return out.cpu().numpy()


# (N, C, H, W, K, F): several tiles, ragged tails, strips, image-boundary crossings
GENERAL_SHAPES = [
    (2, 3, 20, 23, 5, 3),
    (1, 8, 30, 30, 70, 3),       # more than 64 filters: the wide filter tile
    (3, 16, 28, 28, 130, 3),     # pixel blocks wrap over rows and images
    (2, 4, 40, 150, 33, 5),      # output wider than one column strip
    (1, 2, 12, 300, 8, 2),
    (2, 3, 37, 41, 64, 11),
    (1, 1, 9, 9, 1, 1),
    (2, 5, 16, 16, 3, 4),
    (1, 7, 20, 20, 9, 7),
    (5, 6, 8, 8, 4, 3),          # tiny images: one pixel block spans several images
    (3, 2, 5, 5, 4, 5),          # filter as large as the image: 1x1 output
    (1, 3, 14, 14, 2, 9),
    (1, 2, 13, 12, 3, 10),
    (2, 2, 11, 10, 2, 6),
    (1, 2, 12, 11, 2, 8),
    (7, 24, 9, 35, 96, 3),
    (1, 64, 20, 20, 64, 1),      # 1x1 filters: no spatial reuse at all
]


@pytest.mark.parametrize("variant", [SIMPLE, TILED], ids=["simple", "tiled"])
@pytest.mark.parametrize("shape", GENERAL_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_general_small_shapes(shape, variant):
    N, C, H, W, K, F = shape
    x, f = wl.random_case(100 + F, N, C, H, W, K, F)
    acc, mag, _ = oracle.general(x, f)
    got = run_general(x, f, variant)
    assert_within_bound(got, acc, mag, f"general {shape}")


# (H, W, K, F)
SINGLE_SHAPES = [
    (40, 300, 5, 3),
    (33, 31, 70, 5),
    (20, 20, 1, 1),
    (64, 600, 130, 7),
    (30, 40, 3, 11),
    (17, 17, 2, 2),
    (50, 50, 33, 9),
    (21, 260, 16, 4),
    (19, 22, 8, 6),
    (25, 140, 40, 8),
    (15, 15, 3, 10),
    (9, 9, 2, 9),               # 1x1 output
    (100, 515, 64, 5),          # three tiles across, ragged last one
    (40, 1030, 33, 3),          # last tile column only a few pixels wide
    (24, 700, 64, 5),           # row ends completed with the head of the next row
    (10, 2100, 32, 7),
    (35, 1200, 96, 3),
    (9, 1300, 70, 1),
]


@pytest.mark.parametrize("variant", [SIMPLE, TILED], ids=["simple", "tiled"])
@pytest.mark.parametrize("shape", SINGLE_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_single_channel_small_shapes(shape, variant):
    H, W, K, F = shape
    x, f = wl.random_case(200 + F, 1, 1, H, W, K, F)
    img, flt = x[0, 0], f[:, 0]
    acc, mag, _ = oracle.single_channel(img, flt)
    got = run_single(img, flt, variant)
    assert_within_bound(got, acc, mag, f"single {shape}")


def _tile_variants(single):
    """Every compiled tile configuration of the tiled kernel, forced."""
    return [dconv.VARIANT_TILED_CFG0 + i for i in range(dconv.tile_config_count(single))]


# shapes that exercise wide tiles, tall tiles, carried blocks and row ends in every configuration
SINGLE_CFG_SHAPES = [(33, 31, 70, 5), (24, 700, 64, 5), (21, 2300, 40, 3), (40, 1290, 33, 7),
                     (19, 1100, 96, 9), (12, 12, 3, 11), (70, 530, 130, 4)]


@pytest.mark.parametrize("shape", SINGLE_CFG_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_single_channel_every_tile_configuration(shape):
    H, W, K, F = shape
    x, f = wl.random_case(300 + F, 1, 1, H, W, K, F)
    img, flt = x[0, 0], f[:, 0]
    acc, mag, _ = oracle.single_channel(img, flt)
    xi, fi = wl.integer_case(30 + F, 1, 1, H, W, K, F)
    _, _, o32, _ = oracle.general(xi, fi, want32=True)
    for variant in _tile_variants(True):
        assert_within_bound(run_single(img, flt, variant), acc, mag, f"single {shape} variant {variant}")
        np.testing.assert_array_equal(run_single(xi[0, 0], fi[:, 0], variant), o32[0])


# shapes for every tile shape x schedule of the general kernel: channel counts that leave one,
# several and many chunks per tile (tiles shared by 2, by 3 and more workgroups, and whole),
# a channel count the chunk does not divide, more than 128 filters, several column strips
GENERAL_CFG_SHAPES = [(3, 16, 28, 28, 130, 3), (2, 3, 20, 23, 5, 3), (2, 37, 14, 14, 70, 3),
                      (1, 64, 20, 20, 64, 1), (2, 4, 40, 150, 33, 5), (2, 3, 37, 41, 64, 11),
                      (9, 24, 9, 35, 96, 3), (1, 7, 20, 20, 9, 7), (2, 19, 16, 16, 200, 2)]


@pytest.mark.parametrize("shape", GENERAL_CFG_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_general_every_tile_configuration(shape):
    N, C, H, W, K, F = shape
    x, f = wl.random_case(400 + F, N, C, H, W, K, F)
    acc, mag, _ = oracle.general(x, f)
    xi, fi = wl.integer_case(40 + F, N, C, H, W, K, F)
    _, _, o32, _ = oracle.general(xi, fi, want32=True)
    for variant in _tile_variants(False):
        got = run_general(x, f, variant)
        assert_within_bound(got, acc, mag, f"general {shape} variant {variant}")
        # the sum over channels of a shared tile is taken in a fixed order: same bits every time
        np.testing.assert_array_equal(run_general(x, f, variant), got)
        np.testing.assert_array_equal(run_general(xi, fi, variant), o32)


# shapes for the line-aligned write-back of the general kernel (tile configurations 12 to 23): maps
# smaller than a line (direct stores instead), tiles that span two and three images (a segment
# per image), column strips (a segment per strip row), filter counts that leave groups of eight
# incomplete, one output row
ALIGNED_SHAPES = [(6, 4, 7, 7, 20, 3), (5, 8, 16, 16, 37, 3), (9, 4, 14, 14, 70, 3), (2, 3, 30, 300, 13, 5),
                  (1, 8, 12, 500, 64, 3), (3, 16, 3, 90, 65, 3), (2, 2, 40, 41, 130, 11), (4, 16, 20, 20, 9, 1)]


@pytest.mark.parametrize("shape", ALIGNED_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_general_line_aligned_write_back(shape):
    """Whole tiles and tiles shared between workgroups, every tile shape, into an output buffer
    that starts mid-line between NaN guard bands; integer inputs bit for bit."""
    N, C, H, W, K, F = shape
    x, f = wl.random_case(1300 + C + K, N, C, H, W, K, F)
    acc, mag, _ = oracle.general(x, f)
    xi, fi = wl.integer_case(1350 + C + K, N, C, H, W, K, F)
    _, _, o32, _ = oracle.general(xi, fi, want32=True)
    Ho, Wo = H - F + 1, W - F + 1
    n_out, guard = N * K * Ho * Wo, 77
    xd, fd, xid, fid = dev(x), dev(f), dev(xi), dev(fi)
    for schedule in (0, 2, 3):
        for tile in range(3):
            variant = dconv.VARIANT_TILED_CFG0 + 12 + 3 * schedule + tile
            buf = torch.full((n_out + 2 * guard,), float("nan"), device="cuda")
            out = buf[guard:guard + n_out].view(N, K, Ho, Wo)
            print(f"aligned write-back {shape} variant {variant:#x}", flush=True)
            dconv.dconv_general(xd, fd, out=out, variant=variant)
            torch.cuda.synchronize()
            host = buf.cpu().numpy()
            assert np.isnan(host[:guard]).all() and np.isnan(host[guard + n_out:]).all(), "guard bands touched"
            assert_within_bound(host[guard:guard + n_out].reshape(N, K, Ho, Wo), acc, mag,
                                f"aligned write-back {shape} variant {variant:#x}")
            got = dconv.dconv_general(xid, fid, variant=variant)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(got.cpu().numpy(), o32)


@pytest.mark.parametrize("shape", [(9, 24, 9, 35, 96, 3), (4, 64, 28, 28, 128, 3)],
                         ids=lambda s: "x".join(map(str, s)))
def test_general_shared_tiles_repeat_exactly(shape):
    """Tiles summed by several workgroups meet in the workspace: the partial sums of every
    workgroup must have arrived before its arrival is counted.  Many launches in a row, every
    schedule that shares tiles, integer inputs (any lost or early-read word shows)."""
    N, C, H, W, K, F = shape
    xi, fi = wl.integer_case(90 + F, N, C, H, W, K, F)
    _, _, o32, _ = oracle.general(xi, fi, want32=True)
    want = torch.from_numpy(o32).to("cuda")
    xd, fd = dev(xi), dev(fi)
    out = torch.empty_like(want)
    shapes, schedules = 3, 4
    for tile in range(shapes):
        for schedule in (2, 3):
            variant = dconv.VARIANT_TILED_CFG0 + schedule * shapes + tile
            print(f"general shared tiles {shape} variant {variant} x40", flush=True)
            for _ in range(40):
                out.fill_(float("nan"))
                dconv.dconv_general(xd, fd, out=out, variant=variant)
                assert bool(torch.equal(out, want)), f"variant {variant}"


@pytest.mark.parametrize("shape", [(2, 8, 28, 28, 70, 3), (1, 3, 30, 140, 64, 11), (3, 6, 12, 12, 9, 5)],
                         ids=lambda s: "x".join(map(str, s)))
def test_general_integer_inputs_are_bit_exact(shape):
    N, C, H, W, K, F = shape
    x, f = wl.integer_case(1, N, C, H, W, K, F)
    _, _, o32, _ = oracle.general(x, f, want32=True)
    for variant in (SIMPLE, TILED):
        np.testing.assert_array_equal(run_general(x, f, variant), o32)


# odd reduction lengths per chunk (padding taps) with 5x5, 7x7, 9x9, 11x11 filters, three
# channels of 3x3; a filter count that is not a multiple of the filter tile
@pytest.mark.parametrize("shape", [(2, 2, 14, 15, 5, 5), (1, 3, 16, 16, 6, 3), (1, 2, 20, 21, 4, 11),
                                   (1, 1, 16, 40, 3, 7), (1, 2, 12, 30, 3, 9), (1, 1, 9, 9, 2, 1)],
                         ids=lambda s: "x".join(map(str, s)))
def test_general_non_finite_filter_stays_in_its_own_map(shape):
    """IEEE propagation: a NaN / Inf weight reaches the outputs of its own filter only.  The
    padding taps of the matrix-core steps sit next to other filters' weights in memory."""
    N, C, H, W, K, F = shape
    x, f = wl.random_case(77 + F, N, C, H, W, K, F)
    acc, mag, _ = oracle.general(x, f)
    for bad in range(K):
        fb = f.copy()
        fb[bad] = np.nan
        fb[bad, 0, 0, 0] = np.inf
        for variant in (SIMPLE, TILED) + tuple(_tile_variants(False)):
            got = run_general(x, fb, variant)
            assert not np.isfinite(got[:, bad]).any(), f"{shape} variant {variant}: filter {bad} finite"
            keep = [k for k in range(K) if k != bad]
            assert_within_bound(got[:, keep], acc[:, keep], mag[:, keep],
                                f"general {shape} variant {variant} with filter {bad} non-finite")


@pytest.mark.parametrize("shape", [(2, 2, 14, 15, 5, 5), (2, 3, 16, 16, 6, 3), (1, 2, 20, 21, 4, 11)],
                         ids=lambda s: "x".join(map(str, s)))
def test_general_non_finite_pixel_reaches_only_the_windows_that_hold_it(shape):
    N, C, H, W, K, F = shape
    x, f = wl.random_case(91 + F, N, C, H, W, K, F)
    acc, mag, _ = oracle.general(x, f)
    # (column 0 of a middle row sits right behind the end of the row above it in memory)
    for (n, c, y0, x0) in [(0, 0, 0, 0), (N - 1, C - 1, H - 1, W - 1), (0, C - 1, H // 2, W // 3),
                           (N - 1, 0, H // 2, 0), (0, C - 1, H - 1, 0)]:
        xb = x.copy()
        xb[n, c, y0, x0] = np.nan
        hit = np.zeros(acc.shape, dtype=bool)      # outputs whose window holds the pixel
        hit[n, :, max(0, y0 - F + 1):y0 + 1, max(0, x0 - F + 1):x0 + 1] = True
        for variant in (SIMPLE, TILED) + tuple(_tile_variants(False)):
            got = run_general(xb, f, variant)
            assert np.isnan(got[hit]).all(), f"{shape} variant {variant}: NaN pixel lost"
            clean = np.where(hit, acc.astype(np.float32), got)
            assert_within_bound(clean, acc, mag, f"general {shape} variant {variant} NaN pixel {(n, c, y0, x0)}")


@pytest.mark.parametrize("shape", [(60, 300, 40, 3), (40, 41, 64, 5), (30, 270, 7, 11)],
                         ids=lambda s: "x".join(map(str, s)))
def test_single_channel_integer_inputs_are_bit_exact(shape):
    H, W, K, F = shape
    x, f = wl.integer_case(2, 1, 1, H, W, K, F)
    _, _, o32, _ = oracle.general(x, f, want32=True)
    for variant in (SIMPLE, TILED):
        np.testing.assert_array_equal(run_single(x[0, 0], f[:, 0], variant), o32[0])


def test_filter_side_without_a_tiled_kernel_falls_back():
    x, f = wl.random_case(3, 1, 2, 40, 40, 3, 33)        # the tiled kernels end at 32 x 32
    acc, mag, _ = oracle.general(x, f)
    assert_within_bound(run_general(x, f, AUTO), acc, mag, "F=33 auto")
    with pytest.raises(dconv.DconvError) as e:
        run_general(x, f, TILED)
    assert e.value.status == dconv.STATUS_UNSUPPORTED
    acc, mag, _ = oracle.single_channel(x[0, 0], f[:, 0])
    assert_within_bound(run_single(x[0, 0], f[:, 0], AUTO), acc, mag, "F=33 single auto")


def test_single_channel_agrees_with_general_on_one_image_one_channel():
    x, f = wl.random_case(4, 1, 1, 70, 290, 48, 5)
    acc, mag, _ = oracle.general(x, f)
    a = run_single(x[0, 0], f[:, 0], AUTO)
    b = run_general(x, f, AUTO)
    assert_within_bound(a, acc[0], mag[0], "single")
    assert_within_bound(b, acc, mag, "general")


def test_output_guard_bands_stay_untouched_and_every_element_is_written():
    N, C, H, W, K, F = 2, 8, 28, 28, 40, 3
    x, f = wl.random_case(5, N, C, H, W, K, F)
    n_out = N * K * (H - F + 1) * (W - F + 1)
    pad = 4096
    buf = torch.full((n_out + 2 * pad,), float("nan"), device="cuda")
    out = buf[pad:pad + n_out].view(N, K, H - F + 1, W - F + 1)
    for variant in (SIMPLE, TILED):
        buf.fill_(float("nan"))
        dconv.dconv_general(dev(x), dev(f), out=out, variant=variant)
        torch.cuda.synchronize()
        assert torch.isnan(buf[:pad]).all() and torch.isnan(buf[pad + n_out:]).all()
        assert torch.isfinite(out).all()
    Hs, Ws, Ks, Fs = 45, 300, 20, 5
    xs, fs = wl.random_case(6, 1, 1, Hs, Ws, Ks, Fs)
    n_out = Ks * (Hs - Fs + 1) * (Ws - Fs + 1)
    buf = torch.full((n_out + 2 * pad,), float("nan"), device="cuda")
    out = buf[pad:pad + n_out].view(Ks, Hs - Fs + 1, Ws - Fs + 1)
    for variant in (SIMPLE, TILED):
        buf.fill_(float("nan"))
        dconv.dconv_single_channel(dev(xs[0, 0]), dev(fs[:, 0]), out=out, variant=variant)
        torch.cuda.synchronize()
        assert torch.isnan(buf[:pad]).all() and torch.isnan(buf[pad + n_out:]).all()
        assert torch.isfinite(out).all()


def test_runs_on_a_side_stream_and_is_repeatable():
    x, f = wl.random_case(7, 2, 8, 30, 30, 64, 3)
    acc, mag, _ = oracle.general(x, f)
    xd, fd = dev(x), dev(f)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        a = dconv.dconv_general(xd, fd)
        b = dconv.dconv_general(xd, fd)
    s.synchronize()
    assert torch.equal(a, b)
    assert_within_bound(a.cpu().numpy(), acc, mag, "side stream")


def test_python_binding_reports_bad_shapes():
    with pytest.raises(dconv.DconvError) as e:
        dconv.dconv_general(torch.zeros(1, 1, 4, 4, device="cuda"), torch.zeros(1, 1, 5, 5, device="cuda"))
    assert e.value.status == dconv.STATUS_BAD_SHAPE


# ---- the benchmark configurations at full size -------------------------------------------

def _sampled_check(w, out_dev, x, f, count, what):
    idx = wl.sample_indices(w.seed, w.out_elems, count)
    got = out_dev.reshape(-1)[torch.from_numpy(idx).to("cuda")].cpu().numpy()
    x4 = x.reshape(w.N, w.C, w.H, w.W)
    f4 = f.reshape(w.K, w.C, w.F, w.F)
    acc, mag = oracle.general_at(x4, f4, idx)
    return assert_within_bound(got, acc, mag, what)


def test_config_S1_whole_output():
    w = wl.S1
    img, f = wl.make_inputs(w)
    acc, mag, _ = oracle.single_channel(img, f)
    for variant in (AUTO, SIMPLE):
        assert_within_bound(run_single(img, f, variant), acc, mag, f"S1 variant {variant}")


@pytest.mark.parametrize("F", [5, 3, 7, 9, 11])
def test_config_S2_sampled_outputs(F):
    w = wl.S2_SWEEP[F] if F != 5 else wl.S2
    img, f = wl.make_inputs(w)
    print(f"S2 F={F}", flush=True)
    out = dconv.dconv_single_channel(dev(img), dev(f))
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
    _sampled_check(w, out, img, f, 40000, f"S2 F={F}")
    # rows and columns at tile seams and at the far edges, whole
    ys = [0, 15, 16, 17, w.Ho - 1]
    for k in (0, w.K - 1):
        for y in ys:
            idx = (k * w.Ho + y) * w.Wo + np.arange(w.Wo, dtype=np.int64)
            got = out.reshape(-1)[torch.from_numpy(idx).to("cuda")].cpu().numpy()
            acc, mag = oracle.general_at(img.reshape(1, 1, w.H, w.W), f.reshape(w.K, 1, F, F), idx)
            assert_within_bound(got, acc, mag, f"S2 F={F} row {y} of map {k}")
    del out


def test_config_S2_delta_filters_reproduce_the_shifted_image_exactly():
    w = wl.S2
    img, _ = wl.make_inputs(w)
    f = np.zeros(w.filt_shape(), np.float32)
    taps = [(k % w.F, (k // w.F) % w.F) for k in range(w.K)]
    for k, (a, b) in enumerate(taps):
        f[k, a, b] = 1.0
    imgd = dev(img)
    out = dconv.dconv_single_channel(imgd, dev(f))
    torch.cuda.synchronize()
    for k, (a, b) in enumerate(taps):
        assert torch.equal(out[k], imgd[a:a + w.Ho, b:b + w.Wo]), f"map {k} tap {(a, b)}"


def test_config_G1_sampled_outputs():
    w = wl.G1
    x, f = wl.make_inputs(w)
    print("G1", flush=True)
    out = dconv.dconv_general(dev(x), dev(f))
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
    _sampled_check(w, out, x, f, 60000, "G1")


def _delta_and_pair_filters(w, rng):
    """Filters with one unit tap, and filters with a unit tap plus a tap of weight 2 in another
    channel: out = x1 (exact), resp. x1 + 2 * x2 (one rounding whatever the order of additions,
    since every other term is an exact zero and 2 * x2 is exact)."""
    f = np.zeros(w.filt_shape(), np.float32)
    taps = []
    for k in range(w.K):
        c0, a, b = k % w.C, (k // w.C) % w.F, (k * 5 + k // 7) % w.F
        f[k, c0, a, b] = 1.0
        second = None
        if k % 2 == 1 and w.C > 1:
            c1 = int((c0 + 1 + rng.integers(0, w.C - 1)) % w.C)
            a1, b1 = int(rng.integers(0, w.F)), int(rng.integers(0, w.F))
            f[k, c1, a1, b1] = 2.0
            second = (c1, a1, b1)
        taps.append(((c0, a, b), second))
    return f, taps


@pytest.mark.parametrize("name", ["G1", "G3"])
def test_general_configs_delta_filters_whole_output_exact(name):
    """The whole output of the two large general-case configurations, compared on the device:
    unit-tap filters reproduce shifted crops of the input bit for bit, in every map, image, row
    and column, so no tile, strip, chunk or shared-tile boundary can hide a misplaced element."""
    w = wl.CONFIGS[name]
    x, _ = wl.make_inputs(w)
    f, taps = _delta_and_pair_filters(w, np.random.default_rng(w.seed))
    xd = dev(x)
    print(f"{name} delta filters", flush=True)
    out = torch.full(w.out_shape(), float("nan"), device="cuda")
    dconv.dconv_general(xd, dev(f), out=out)
    torch.cuda.synchronize()
    for k, ((c0, a, b), second) in enumerate(taps):
        want = xd[:, c0, a:a + w.Ho, b:b + w.Wo]
        if second is not None:
            c1, a1, b1 = second
            want = want + 2.0 * xd[:, c1, a1:a1 + w.Ho, b1:b1 + w.Wo]
        assert torch.equal(out[:, k], want), f"{name} map {k} taps {(c0, a, b)}, {second}"


def test_config_G1_whole_rows_at_seams():
    """Whole output rows of G1 at the first and last rows, around the middle (pixel tiles end
    anywhere along a row) and in images and maps at both ends, against the oracle."""
    w = wl.G1
    x, f = wl.make_inputs(w)
    out = dconv.dconv_general(dev(x), dev(f))
    torch.cuda.synchronize()
    idx = []
    for n in (0, 31, w.N - 1):
        for k in (0, 33, w.K - 1):
            for y in (0, 1, 106, 107, 108, w.Ho - 2, w.Ho - 1):
                idx.append(((n * w.K + k) * w.Ho + y) * w.Wo + np.arange(w.Wo, dtype=np.int64))
    idx = np.concatenate(idx)
    got = out.reshape(-1)[torch.from_numpy(idx).to("cuda")].cpu().numpy()
    acc, mag = oracle.general_at(x, f, idx)
    assert_within_bound(got, acc, mag, "G1 whole rows")


def test_plain_entry_points_called_directly():
    """dconv_single_channel and dconv_general as the header declares them (no variant argument),
    by ctypes with raw device pointers, against the oracle."""
    import ctypes
    lib = dconv.load_library()
    vp = ctypes.c_void_p
    st = vp(torch.cuda.current_stream().cuda_stream)
    x, f = wl.random_case(901, 1, 1, 70, 333, 37, 5)
    img, fs = dev(x[0, 0]), dev(f[:, 0])
    out = torch.full((37, 66, 329), float("nan"), device="cuda")
    rc = lib.dconv_single_channel(vp(img.data_ptr()), 70, 333, vp(fs.data_ptr()), 37, 5, vp(out.data_ptr()), st)
    assert rc == dconv.STATUS_OK
    torch.cuda.synchronize()
    acc, mag, _ = oracle.single_channel(x[0, 0], f[:, 0])
    assert_within_bound(out.cpu().numpy(), acc, mag, "dconv_single_channel by ctypes")
    x, f = wl.random_case(902, 3, 12, 31, 45, 70, 3)
    xd, fd = dev(x), dev(f)
    out = torch.full((3, 70, 29, 43), float("nan"), device="cuda")
    rc = lib.dconv_general(vp(xd.data_ptr()), 3, 12, 31, 45, vp(fd.data_ptr()), 70, 3, vp(out.data_ptr()), st)
    assert rc == dconv.STATUS_OK
    torch.cuda.synchronize()
    acc, mag, _ = oracle.general(x, f)
    assert_within_bound(out.cpu().numpy(), acc, mag, "dconv_general by ctypes")


@pytest.mark.parametrize("shape", [(1, 128, 20, 22, 8, 13), (2, 300, 14, 14, 5, 12), (1, 1024, 6, 7, 3, 5)],
                         ids=lambda s: "x".join(map(str, s)))
def test_fallback_kernel_long_reductions_stay_within_the_bound(shape):
    """The one-lane-per-output kernel on reductions of 10^4 and more terms of one sign (inputs in
    [0,1], the worst case for a running sum): its sums are taken level by level, so the error
    does not grow with the number of terms."""
    N, C, H, W, K, F = shape
    x, f = wl.random_case(950 + F, N, C, H, W, K, F, "u01", "u01")
    acc, mag, _ = oracle.general(x, f)
    ratio = assert_within_bound(run_general(x, f, SIMPLE), acc, mag, f"simple kernel {shape}")
    print(f"max err / mag = {ratio:.2e} over {C * F * F} terms", flush=True)
    if F > 11:
        assert_within_bound(run_general(x, f, AUTO), acc, mag, f"automatic choice {shape}")


def test_config_G2_whole_output():
    w = wl.G2
    x, f = wl.make_inputs(w)
    acc, mag, _ = oracle.general(x, f)
    assert_within_bound(run_general(x, f, AUTO), acc, mag, "G2")


def test_config_G3_sampled_outputs_and_one_image_whole():
    w = wl.G3
    x, f = wl.make_inputs(w)
    print("G3", flush=True)
    out = dconv.dconv_general(dev(x), dev(f))
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
    _sampled_check(w, out, x, f, 100000, "G3")
    acc, mag, _ = oracle.general(x[-1:], f[:64])
    assert_within_bound(out[-1, :64].cpu().numpy(), acc[0], mag[0], "G3 last image, 64 maps")


def test_config_G3_integer_inputs_bit_exact_on_samples():
    w = wl.G3
    x, f = wl.integer_case(9, w.N, w.C, w.H, w.W, w.K, w.F)
    out = dconv.dconv_general(dev(x), dev(f))
    torch.cuda.synchronize()
    idx = wl.sample_indices(99, w.out_elems, 50000)
    got = out.reshape(-1)[torch.from_numpy(idx).to("cuda")].cpu().numpy()
    acc, _ = oracle.general_at(x, f, idx)
    np.testing.assert_array_equal(got.astype(np.float64), acc)


# ---- the paper's other swept corners and the tile search ---------------------------------

@pytest.mark.parametrize("name", list(wl.PAPER_SWEEP))
def test_paper_sweep_shapes_sampled(name):
    w = wl.PAPER_SWEEP[name]
    x, f = wl.make_inputs(w)
    print(name, flush=True)
    if w.kind == "single":
        out = dconv.dconv_single_channel(dev(x), dev(f))
    else:
        out = dconv.dconv_general(dev(x), dev(f))
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
    _sampled_check(w, out, x, f, 30000, name)


def test_tile_search_reports_every_configuration():
    from paper_1705_10591_amd import tune
    rows = tune.tune("general", (2, 8, 28, 28, 70, 3), steps=2)
    assert len(rows) == 1 + 12          # (configurations 12..23 repeat them with the other write-back)
    assert all(ms is None or ms > 0 for _, ms in rows) and rows[0][1] is not None
    rows = tune.tune("single", (64, 600, 40, 5), steps=2)
    assert len(rows) == 1 + dconv.tile_config_count(True)


def _random_shapes(seed, count):
    """Seeded small shapes over the whole parameter range of the tiled kernels."""
    rng = np.random.default_rng(wl.SEED_BASE * 17 + seed)
    shapes = []
    while len(shapes) < count:
        F = int(rng.integers(1, 12))
        H = int(rng.integers(F, F + 40))
        W = int(rng.integers(F, F + (300 if len(shapes) % 5 == 0 else 60)))
        N = int(rng.integers(1, 5))
        C = int(rng.choice([1, 2, 3, 4, 5, 8, 12, 16, 17, 32]))
        K = int(rng.choice([1, 2, 7, 16, 33, 64, 65, 130, 200]))
        if N * C * H * W * K * F * F > 3e8:
            continue
        shapes.append((N, C, H, W, K, F))
    return shapes


def test_general_random_shapes_every_schedule():
    shapes = _random_shapes(1, 36)
    ncfg = dconv.tile_config_count(False)
    for idx, shape in enumerate(shapes):
        N, C, H, W, K, F = shape
        x, f = wl.random_case(500 + idx, N, C, H, W, K, F)
        acc, mag, _ = oracle.general(x, f)
        for variant in (AUTO, dconv.VARIANT_TILED_CFG0 + idx % ncfg, dconv.VARIANT_TILED_CFG0 + (idx * 5 + 3) % ncfg):
            try:
                got = run_general(x, f, variant)
            except dconv.DconvError as e:     # a forced configuration may not hold the shape
                assert e.status == dconv.STATUS_UNSUPPORTED and variant != AUTO
                continue
            assert_within_bound(got, acc, mag, f"general {shape} variant {variant}")


def test_single_channel_random_shapes_every_configuration():
    shapes = _random_shapes(2, 30)
    ncfg = dconv.tile_config_count(True)
    for idx, (N, C, H, W, K, F) in enumerate(shapes):
        W = W * 4 if idx % 3 == 0 else W          # some images wide enough for whole-line row ends
        x, f = wl.random_case(600 + idx, 1, 1, H, W, K, F)
        img, flt = x[0, 0], f[:, 0]
        acc, mag, _ = oracle.single_channel(img, flt)
        for variant in (AUTO, dconv.VARIANT_TILED_CFG0 + idx % ncfg):
            assert_within_bound(run_single(img, flt, variant), acc, mag,
                                f"single {(H, W, K, F)} variant {variant}")


# ---- the few-filters kernel of the single-channel case ----------------------------------

FEW = dconv.VARIANT_FEW_FILTERS
# (H, W, K, F): one and several filter groups, ragged tiles in both directions, row ends at
# every alignment, filter sides 1..7, a filter as large as the image
FEW_SHAPES = [(40, 300, 1, 3), (33, 31, 5, 5), (20, 20, 1, 1), (70, 600, 9, 7), (17, 17, 2, 2),
              (65, 515, 3, 4), (50, 263, 8, 6), (7, 7, 3, 7), (130, 258, 2, 5), (36, 1030, 4, 3)]


@pytest.mark.parametrize("shape", FEW_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_single_channel_few_filters_kernel(shape):
    H, W, K, F = shape
    x, f = wl.random_case(700 + F, 1, 1, H, W, K, F)
    img, flt = x[0, 0], f[:, 0]
    acc, mag, _ = oracle.single_channel(img, flt)
    assert_within_bound(run_single(img, flt, FEW), acc, mag, f"few-filters {shape}")
    xi, fi = wl.integer_case(70 + F, 1, 1, H, W, K, F)
    _, _, o32, _ = oracle.general(xi, fi, want32=True)
    np.testing.assert_array_equal(run_single(xi[0, 0], fi[:, 0], FEW), o32[0])


def test_few_filters_kernel_guard_bands_and_limits():
    Hs, Ws, Ks, Fs = 45, 300, 3, 5
    xs, fs = wl.random_case(8, 1, 1, Hs, Ws, Ks, Fs)
    n_out = Ks * (Hs - Fs + 1) * (Ws - Fs + 1)
    pad = 4096
    buf = torch.full((n_out + 2 * pad,), float("nan"), device="cuda")
    out = buf[pad:pad + n_out].view(Ks, Hs - Fs + 1, Ws - Fs + 1)
    dconv.dconv_single_channel(dev(xs[0, 0]), dev(fs[:, 0]), out=out, variant=FEW)
    torch.cuda.synchronize()
    assert torch.isnan(buf[:pad]).all() and torch.isnan(buf[pad + n_out:]).all()
    assert torch.isfinite(out).all()
    # filter sides above 7 and the general case are not its business
    x, f = wl.random_case(9, 1, 1, 20, 20, 2, 9)
    with pytest.raises(dconv.DconvError) as e:
        run_single(x[0, 0], f[:, 0], FEW)
    assert e.value.status == dconv.STATUS_UNSUPPORTED
    with pytest.raises(dconv.DconvError) as e:
        run_general(x, f, FEW)
    assert e.value.status == dconv.STATUS_UNSUPPORTED


def test_shared_tiles_on_two_streams_at_once_and_workspace_release():
    """Each stream has its own workspace: launches that overlap in time must not mix parts."""
    shapes = [(3, 16, 28, 28, 130, 3), (2, 37, 14, 14, 70, 3)]
    split = dconv.VARIANT_TILED_CFG0 + 2 * 3 + 1      # shared tiles, 64 x 256 tile
    cases = []
    for i, (N, C, H, W, K, F) in enumerate(shapes):
        x, f = wl.random_case(800 + i, N, C, H, W, K, F)
        acc, mag, _ = oracle.general(x, f)
        cases.append((dev(x), dev(f), acc, mag))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = [[], []]
    for rep in range(6):
        for si, s in enumerate(streams):
            with torch.cuda.stream(s):
                xd, fd, _, _ = cases[si]
                outs[si].append(dconv.dconv_general(xd, fd, variant=split))
    torch.cuda.synchronize()
    for si in range(2):
        _, _, acc, mag = cases[si]
        for o in outs[si]:
            assert_within_bound(o.cpu().numpy(), acc, mag, f"stream {si}")
            assert torch.equal(o, outs[si][0])
    dconv.release_workspace()
    xd, fd, acc, mag = cases[0]
    again = dconv.dconv_general(xd, fd, variant=split)
    torch.cuda.synchronize()
    assert torch.equal(again, outs[0][0])


# ---- a batch of one-channel images: the special-case kernel with the images as work items ----------

# (N, H, W, K, F): narrow and wide images (row ends completed across rows only on wide ones),
# several filter groups, image sizes whose planes start at every misalignment
BATCH_SHAPES = [(3, 20, 23, 5, 3), (4, 9, 700, 40, 5), (2, 37, 41, 130, 3), (5, 12, 330, 33, 7),
                (7, 8, 8, 4, 3), (2, 30, 270, 7, 11), (3, 6, 1500, 70, 1)]


@pytest.mark.parametrize("shape", BATCH_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_one_channel_batch_on_the_special_case_kernel(shape):
    N, H, W, K, F = shape
    x, f = wl.random_case(900 + N + K, N, 1, H, W, K, F)
    acc, mag, _ = oracle.general(x, f)
    xi, fi = wl.integer_case(950 + N + K, N, 1, H, W, K, F)
    acci, _, _ = oracle.general(xi, fi)
    variants = [dconv.VARIANT_SPECIAL_CASE] + [dconv.VARIANT_SPECIAL_CASE_CFG0 + i
                                               for i in range(dconv.tile_config_count(True))]
    for v in variants:
        assert_within_bound(run_general(x, f, v), acc, mag, f"batch {shape} variant {v:#x}")
        np.testing.assert_array_equal(run_general(xi, fi, v), acci.astype(np.float32))


def test_one_channel_batch_guard_bands_and_refusals():
    N, H, W, K, F = 3, 21, 340, 37, 5
    x, f = wl.random_case(970, N, 1, H, W, K, F)
    acc, mag, _ = oracle.general(x, f)
    total = N * K * (H - F + 1) * (W - F + 1)
    guard = 1001                      # an output buffer that starts in the middle of a 128-byte line
    buf = torch.full((total + 2 * guard,), float("nan"), device="cuda")
    out = buf[guard:guard + total].view(N, K, H - F + 1, W - F + 1)
    dconv.dconv_general(dev(x), dev(f), out=out, variant=dconv.VARIANT_SPECIAL_CASE)
    torch.cuda.synchronize()
    assert torch.isnan(buf[:guard]).all() and torch.isnan(buf[guard + total:]).all()
    assert_within_bound(out.cpu().numpy(), acc, mag, "batch with guard bands")
    # more channels than the special-case kernel is compiled for
    x2, f2 = wl.random_case(971, 2, 6, 12, 12, 3, 3)
    with pytest.raises(dconv.DconvError) as e:
        run_general(x2, f2, dconv.VARIANT_SPECIAL_CASE)
    assert e.value.status == dconv.STATUS_UNSUPPORTED


def test_one_channel_batch_automatic_choice_large_volume_sampled():
    """128 M outputs of 300-wide images with 3x3 filters: the automatic choice is the special-case
    kernel; checked on sampled outputs and against the general kernel on one image."""
    N, H, W, K, F = 24, 300, 302, 64, 3
    x, f = wl.random_case(980, N, 1, H, W, K, F)
    xd, fd = dev(x), dev(f)
    out = dconv.dconv_general(xd, fd)
    torch.cuda.synchronize()
    idx = wl.sample_indices(981, out.numel(), 20000)
    got = out.view(-1)[torch.from_numpy(idx).to("cuda")].cpu().numpy()
    acc, mag = oracle.general_at(x, f, idx)
    assert_within_bound(got, acc, mag, "one-channel batch, automatic choice")
    last = dconv.dconv_general(xd[N - 1:], fd, variant=TILED)           # the general kernel
    torch.cuda.synchronize()
    accl, magl, _ = oracle.general(x[N - 1:], f)
    assert_within_bound(out[N - 1:].cpu().numpy(), accl, magl, "last image, special-case kernel")
    assert_within_bound(last.cpu().numpy(), accl, magl, "last image, general kernel")


# ---- images so large that output planes lie more than 2 GiB apart ----------------------------------

@pytest.mark.parametrize("shape", [(1, 3, 4096, 4096, 64, 3),      # 4.3 GB of output from one image
                                   (2, 3, 2048, 2100, 160, 5)],    # 2.7 GB per image: runs image by image
                         ids=lambda s: "x".join(map(str, s)))
def test_general_large_images_sampled(shape):
    N, C, H, W, K, F = shape
    x, f = wl.random_case(990 + K, N, C, H, W, K, F)
    xd, fd = dev(x), dev(f)
    print(f"general {shape} automatic choice and tiled kernel", flush=True)
    out = dconv.dconv_general(xd, fd, variant=TILED)
    torch.cuda.synchronize()
    total = out.numel()
    idx = np.unique(np.concatenate([wl.sample_indices(991, total, 30000),
                                    np.arange(0, 4096), np.arange(total - 4096, total),
                                    # around the places where byte offsets cross 2 GiB and 4 GiB
                                    np.arange((1 << 29) - 2048, (1 << 29) + 2048),
                                    np.arange(min((1 << 30) - 2048, total - 4096), min((1 << 30) + 2048, total))]))
    got = out.view(-1)[torch.from_numpy(idx).to("cuda")].cpu().numpy()
    acc, mag = oracle.general_at(x, f, idx)
    assert_within_bound(got, acc, mag, f"general {shape}")
    auto = dconv.dconv_general(xd, fd)
    torch.cuda.synchronize()
    assert torch.equal(auto.view(-1)[torch.from_numpy(idx).to("cuda")], out.view(-1)[torch.from_numpy(idx).to("cuda")])


# ---- a few channels on the special-case kernel ---------------------------------------------------------

# (N, C, H, W, K, F)
FEW_CHANNEL_SHAPES = [(2, 3, 20, 23, 5, 3), (1, 3, 30, 700, 40, 3), (2, 2, 37, 41, 130, 5), (3, 4, 12, 330, 33, 5),
                      (4, 3, 8, 8, 4, 3), (1, 4, 9, 1500, 70, 1), (2, 3, 40, 300, 64, 5), (1, 2, 17, 290, 9, 4),
                      (2, 4, 11, 140, 20, 2)]


@pytest.mark.parametrize("shape", FEW_CHANNEL_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_few_channels_on_the_special_case_kernel(shape):
    N, C, H, W, K, F = shape
    x, f = wl.random_case(1000 + C + K, N, C, H, W, K, F)
    acc, mag, _ = oracle.general(x, f)
    xi, fi = wl.integer_case(1050 + C + K, N, C, H, W, K, F)
    acci, _, _ = oracle.general(xi, fi)
    ran = 0
    for v in [dconv.VARIANT_SPECIAL_CASE] + [dconv.VARIANT_SPECIAL_CASE_CFG0 + i for i in range(7)]:
        try:
            got = run_general(x, f, v)
        except dconv.DconvError as e:             # tile configurations 1 and 2 exist for one channel only
            assert e.status == dconv.STATUS_UNSUPPORTED and v in (dconv.VARIANT_SPECIAL_CASE_CFG0 + 1,
                                                                  dconv.VARIANT_SPECIAL_CASE_CFG0 + 2)
            continue
        ran += 1
        assert_within_bound(got, acc, mag, f"few channels {shape} variant {v:#x}")
        np.testing.assert_array_equal(run_general(xi, fi, v), acci.astype(np.float32))
    assert ran == 6


def test_few_channels_refusals():
    for shape in [(1, 5, 12, 12, 3, 3), (1, 3, 20, 20, 3, 7)]:       # too many channels, filter too large
        x, f = wl.random_case(1090, *shape)
        with pytest.raises(dconv.DconvError) as e:
            run_general(x, f, dconv.VARIANT_SPECIAL_CASE)
        assert e.value.status == dconv.STATUS_UNSUPPORTED


def test_few_channels_automatic_choice_large_volume_sampled():
    """266 M outputs from RGB images with 3x3 filters: the automatic choice is the special-case
    kernel; sampled outputs against the oracle, and the general kernel on the same samples."""
    N, C, H, W, K, F = 16, 3, 512, 512, 64, 3
    x, f = wl.random_case(1100, N, C, H, W, K, F)
    xd, fd = dev(x), dev(f)
    out = dconv.dconv_general(xd, fd)
    forced = dconv.dconv_general(xd, fd, variant=dconv.VARIANT_SPECIAL_CASE)
    torch.cuda.synchronize()
    assert torch.equal(out, forced)                 # the automatic choice is that kernel
    idx = wl.sample_indices(1101, out.numel(), 20000)
    sel = torch.from_numpy(idx).to("cuda")
    acc, mag = oracle.general_at(x, f, idx)
    assert_within_bound(out.view(-1)[sel].cpu().numpy(), acc, mag, "few channels, automatic choice")
    gen = dconv.dconv_general(xd, fd, variant=TILED)
    torch.cuda.synchronize()
    assert_within_bound(gen.view(-1)[sel].cpu().numpy(), acc, mag, "few channels, general kernel")


@pytest.mark.parametrize("W", [80, 95, 96, 97, 98, 99, 110, 127, 129, 130, 131, 159, 162, 191, 192, 193, 222, 256, 258, 287, 289, 319, 321])
def test_special_case_kernel_widths_around_the_row_end_rule(W):
    """From 192 output pixels of width on (128 with passes of 64 pixels, 96 with 32), the last pass of a row also
    writes the head of the next row: exact results and untouched guard bands on both sides of
    those limits, every tile size."""
    for (N, C, K, F, H) in ((2, 1, 40, 3, 9), (1, 3, 33, 3, 7), (1, 2, 64, 5, 9)):
        x, f = wl.integer_case(W + K, N, C, H, W, K, F)
        acc, _, _ = oracle.general(x, f)
        total = acc.size
        for i in (0, 3, 4, 5, 6):
            print(f"special-case kernel W={W} N,C,K,F,H={(N, C, K, F, H)} configuration {i}", flush=True)
            buf = torch.full((total + 2048,), float("nan"), device="cuda")
            out = buf[1001:1001 + total].view(acc.shape)          # starts mid-line
            dconv.dconv_general(dev(x), dev(f), out=out, variant=dconv.VARIANT_SPECIAL_CASE_CFG0 + i)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(out.cpu().numpy(), acc.astype(np.float32))
            assert torch.isnan(buf[:1001]).all() and torch.isnan(buf[1001 + total:]).all()


@pytest.mark.parametrize("K", [1, 4, 7, 8, 9, 12, 15, 16, 17, 24, 31, 32, 33, 40, 48])
def test_special_case_kernel_filter_counts_around_group_and_block_limits(K):
    """The write-back goes by groups of eight filters and by blocks of 32 or 16: filter counts on both
    sides of those limits (whole groups are stored without a test per filter, partial ones with),
    every tile configuration and the library's own choice, wide rows completed across row ends
    and narrow ones, exact results between guard bands that start mid-line."""
    for (H, W, F) in ((11, 700, 3), (9, 230, 5), (12, 90, 4)):
        x, f = wl.integer_case(900 + K + F, 1, 1, H, W, K, F)
        acc, _, _ = oracle.general(x, f)
        want = acc.astype(np.float32)[0]
        total = want.size
        img, flt = dev(x[0, 0]), dev(f[:, 0])
        for variant in [dconv.VARIANT_AUTO] + _tile_variants(True):
            print(f"special-case kernel K={K} H,W,F={(H, W, F)} variant {variant:#x}", flush=True)
            buf = torch.full((total + 2048,), float("nan"), device="cuda")
            out = buf[1003:1003 + total].view(want.shape)
            dconv.dconv_single_channel(img, flt, out=out, variant=variant)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(out.cpu().numpy(), want)
            assert torch.isnan(buf[:1003]).all() and torch.isnan(buf[1003 + total:]).all()


@pytest.mark.parametrize("K", [65, 96, 129, 160, 161, 192, 200, 225, 288, 353])
def test_special_case_kernel_leftover_filter_blocks(K):
    """Filter blocks beyond whole groups of four form a group of two and / or a group of one (three,
    five, six, seven ... blocks), and the groups of a tile are neighbouring work items: every tile
    configuration, one image and a batch with two to four channels, exact results between guard
    bands.  With one image of one channel and larger filters the library's own choice runs the
    leftover blocks as a launch of their own (64 + 32, 128 + 32, 128 + 64 + 32 filters ...)."""
    for (N, C, H, W, F) in ((1, 1, 9, 600, 3), (1, 1, 14, 140, 7), (1, 1, 12, 100, 9), (2, 3, 10, 300, 3), (3, 1, 8, 70, 5),
                            (2, 4, 7, 200, 2)):
        x, f = wl.integer_case(950 + K + F, N, C, H, W, K, F)
        want = oracle.general(x, f)[0].astype(np.float32)
        for variant in [dconv.VARIANT_SPECIAL_CASE] + [dconv.VARIANT_SPECIAL_CASE_CFG0 + i
                                                      for i in range(dconv.tile_config_count(True))]:
            print(f"special-case kernel K={K} {(N, C, H, W, F)} variant {variant:#x}", flush=True)
            buf = torch.full((want.size + 2048,), float("nan"), device="cuda")
            out = buf[1003:1003 + want.size].view(want.shape)
            try:
                dconv.dconv_general(dev(x), dev(f), out=out, variant=variant)
            except dconv.DconvError as e:          # (a configuration that cannot hold the shape)
                assert e.status == dconv.STATUS_UNSUPPORTED
                continue
            torch.cuda.synchronize()
            np.testing.assert_array_equal(out.cpu().numpy(), want)
            assert torch.isnan(buf[:1003]).all() and torch.isnan(buf[1003 + want.size:]).all()


ONE_CHANNEL_ON_THE_GENERAL_KERNEL = [(64, 64, 128, 8), (150, 150, 96, 5), (100, 333, 40, 11), (37, 700, 64, 9),
                                     (224, 224, 64, 3), (300, 61, 200, 6)]


@pytest.mark.parametrize("shape", ONE_CHANNEL_ON_THE_GENERAL_KERNEL, ids=lambda s: "x".join(map(str, s)))
def test_one_channel_where_the_library_runs_the_general_kernel(shape):
    """dconv_single_channel on shapes that the general-case kernel runs faster (narrow or short
    images, large filters): the same bits as dconv_general with one image of one channel, within
    the bound of the oracle, integer inputs exact, guard bands."""
    H, W, K, F = shape
    assert dconv.tile_choice(True, 1, 1, H, W, K, F) == dconv.CHOICE_GENERAL_CASE
    x, f = wl.random_case(7100 + K + F, 1, 1, H, W, K, F)
    acc, mag, _ = oracle.general(x, f)
    got = dconv.dconv_single_channel(dev(x[0, 0]), dev(f[:, 0]))
    same = dconv.dconv_general(dev(x), dev(f), variant=dconv.VARIANT_TILED)[0]
    plain = dconv.dconv_general(dev(x), dev(f))[0]
    torch.cuda.synchronize()
    assert torch.equal(got, same) and torch.equal(got, plain)
    assert_within_bound(got.cpu().numpy(), acc[0], mag[0], f"one channel on the general kernel {shape}")
    xi, fi = wl.integer_case(7200 + K + F, 1, 1, H, W, K, F)
    want = oracle.general(xi, fi)[0].astype(np.float32)[0]
    buf = torch.full((want.size + 2048,), float("nan"), device="cuda")
    out = buf[1001:1001 + want.size].view(want.shape)
    dconv.dconv_single_channel(dev(xi[0, 0]), dev(fi[:, 0]), out=out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), want)
    assert torch.isnan(buf[:1001]).all() and torch.isnan(buf[1001 + want.size:]).all()


def test_sixteen_filter_blocks_where_the_library_picks_them():
    """Shapes the dispatcher sends to the 16-filter matrix-core blocks (13 to 16 filters; 8 to 12 on
    images whose vector-ALU tiles do not cover the chip), at full size on sampled outputs, and the
    same launch with the configuration forced, bit for bit."""
    for (H, W, K, F) in ((1080, 1920, 12, 7), (1024, 1024, 16, 5), (720, 1280, 14, 4)):
        x, f = wl.random_case(1600 + K, 1, 1, H, W, K, F)
        img, flt = dev(x[0, 0]), dev(f[:, 0])
        got = dconv.dconv_single_channel(img, flt)
        forced = [dconv.dconv_single_channel(img, flt, variant=dconv.VARIANT_TILED_CFG0 + c) for c in (9, 10)]
        torch.cuda.synchronize()
        assert any(torch.equal(got, o) for o in forced), "the library's choice is one of the 16-filter configurations"
        rng = np.random.default_rng(K)
        Ho, Wo = H - F + 1, W - F + 1
        ks, ys, xs = rng.integers(0, K, 4000), rng.integers(0, Ho, 4000), rng.integers(0, Wo, 4000)
        xs[:200] = Wo - 1 - (xs[:200] % 40)                # row ends
        xs[200:400] = xs[200:400] % 40                     # row starts
        idx = ((ks * Ho + ys) * Wo + xs).astype(np.int64)
        acc, mag = oracle.general_at(x, f, idx)
        for o in [got] + forced:
            vals = o.cpu().numpy().reshape(-1)[idx]
            assert_within_bound(vals, acc, mag, f"16-filter blocks {(H, W, K, F)}")


@pytest.mark.parametrize("shape", [(1, 512, 14, 14, 512, 3), (1, 384, 20, 20, 192, 7), (4, 512, 17, 14, 448, 1),
                                   (2, 256, 9, 31, 96, 5), (1, 192, 12, 50, 160, 2), (3, 128, 28, 28, 64, 3),
                                   (1, 96, 33, 47, 320, 4), (2, 64, 10, 12, 256, 9)],
                         ids=lambda s: "x".join(map(str, s)))
def test_fewer_tiles_than_cus_integer_inputs_bit_exact(shape):
    """Small batches of deep layers: fewer tiles than CUs, so the launch shares every tile between a
    number of workgroups that it picks from the shape (ranges of chunks that start and end inside
    tiles, parts summed by the workgroup that arrives last).  Integer inputs, so every order of
    summation gives the same bits as the oracle; guard bands; each launch twice, because the
    counters of the shared tiles have to be back at zero for the next launch."""
    N, C, H, W, K, F = shape
    x, f = wl.integer_case(4100 + C + K, N, C, H, W, K, F)
    acc, _, _ = oracle.general(x, f)
    want = acc.astype(np.float32)
    xd, fd = dev(x), dev(f)
    for v in [dconv.VARIANT_AUTO] + [dconv.VARIANT_TILED_CFG0 + i for i in range(3)]:
        for rep in range(2):
            buf = torch.full((want.size + 2048,), float("nan"), device="cuda")
            out = buf[1024:1024 + want.size].view(want.shape)
            dconv.dconv_general(xd, fd, out=out, variant=v)
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy(), want), f"{shape} variant {v:#x} launch {rep}"
            assert torch.isnan(buf[:1024]).all() and torch.isnan(buf[1024 + want.size:]).all(), f"{shape}: guard bands"


# ---- the few-filters kernel of the general case -------------------------------------------

# (N, C, H, W, K, F): every tile shape of the kernel (256, 128 and 64 columns wide; four, two and
# one row per band: the tall bands need many tiles, hence the batches of small images), every
# compiled filter count, filter sides 1..7, ragged tiles, a filter as large as the image
GENERAL_FEW_SHAPES = [(400, 2, 20, 260, 3, 3), (200, 3, 20, 300, 7, 2), (3, 5, 40, 500, 4, 5), (800, 2, 12, 100, 1, 3),
                      (5, 4, 30, 120, 6, 4), (800, 2, 10, 60, 2, 3), (7, 8, 33, 40, 8, 7), (2, 16, 9, 700, 5, 1),
                      (1, 3, 50, 257, 3, 6), (2, 37, 7, 7, 2, 7), (1, 2, 130, 258, 1, 5),
                      # nine to sixteen filters (compiled for twelve and sixteen, one row per band)
                      (3, 4, 37, 300, 9, 3), (2, 3, 50, 130, 13, 7), (5, 6, 21, 70, 16, 5), (2, 7, 33, 257, 12, 1),
                      (3, 2, 30, 90, 11, 2), (1, 5, 40, 64, 15, 6), (2, 3, 35, 200, 10, 4), (1, 9, 16, 16, 14, 3)]


@pytest.mark.parametrize("shape", GENERAL_FEW_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_general_few_filters_kernel(shape):
    """Algorithm 2 with all filters in a thread's register tile, on the vector ALU: against the
    oracle within the bound, integer inputs bit for bit, guard bands, twice in a row."""
    N, C, H, W, K, F = shape
    x, f = wl.random_case(6100 + K + F, N, C, H, W, K, F)
    acc, mag, _ = oracle.general(x, f)
    assert_within_bound(run_general(x, f, FEW), acc, mag, f"general few-filters {shape}")
    xi, fi = wl.integer_case(6200 + K + F, N, C, H, W, K, F)
    want = oracle.general(xi, fi)[0].astype(np.float32)
    for rep in range(2):
        buf = torch.full((want.size + 2048,), float("nan"), device="cuda")
        out = buf[1024 + rep:1024 + rep + want.size].view(want.shape)      # (any 4-byte alignment)
        dconv.dconv_general(dev(xi), dev(fi), out=out, variant=FEW)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), want), f"{shape}: integer inputs"
        assert torch.isnan(buf[:1024 + rep]).all() and torch.isnan(buf[1024 + rep + want.size:]).all(), f"{shape}: guard bands"


def test_general_few_filters_kernel_limits_and_non_finite_inputs():
    x, f = wl.random_case(6300, 2, 3, 20, 70, 17, 3)
    with pytest.raises(dconv.DconvError) as e:              # seventeen filters
        run_general(x, f, FEW)
    assert e.value.status == dconv.STATUS_UNSUPPORTED
    x, f = wl.random_case(6301, 1, 2, 20, 70, 2, 8)
    with pytest.raises(dconv.DconvError) as e:              # 8 x 8 filters
        run_general(x, f, FEW)
    assert e.value.status == dconv.STATUS_UNSUPPORTED
    # a NaN pixel reaches exactly the windows that hold it, a NaN weight its own map only
    N, C, H, W, K, F = 2, 3, 24, 300, 4, 3
    x, f = wl.random_case(6302, N, C, H, W, K, F)
    x[1, 2, 10, 150] = np.nan
    got = run_general(x, f, FEW)
    bad = np.isnan(got)
    want = np.zeros_like(bad)
    want[1, :, 8:11, 148:151] = True
    assert np.array_equal(bad, want)
    x, f = wl.random_case(6303, N, C, H, W, K, F)
    f[2, 1, 0, 1] = np.inf
    got = run_general(x, f, FEW)
    assert np.isfinite(got[:, [0, 1, 3]]).all() and not np.isfinite(got[:, 2]).any()


def test_general_few_filters_where_the_library_picks_it():
    """Layers with one to sixteen filters that cover the chip, at full size on sampled outputs; the
    plain call and the forced kernel agree bit for bit."""
    for (N, C, H, W, K, F) in ((8, 16, 224, 224, 3, 5), (64, 32, 56, 56, 1, 3), (4, 32, 300, 512, 8, 3),
                               (15, 3, 384, 384, 10, 3), (21, 8, 96, 640, 12, 5), (64, 3, 128, 128, 16, 2),
                               (1, 3, 112, 112, 1, 5), (4, 3, 28, 28, 3, 3)):
        assert dconv.tile_choice(False, N, C, H, W, K, F) == dconv.CHOICE_FEW_FILTERS
        x, f = wl.random_case(6400 + K, N, C, H, W, K, F)
        got = dconv.dconv_general(dev(x), dev(f))
        forced = dconv.dconv_general(dev(x), dev(f), variant=FEW)
        torch.cuda.synchronize()
        assert torch.equal(got, forced)
        idx = wl.sample_indices(6400 + K, got.numel(), 20000)
        acc, mag = oracle.general_at(x, f, idx)
        assert_within_bound(got.cpu().numpy().reshape(-1)[idx], acc, mag, f"general few-filters {(N, C, H, W, K, F)}")


LARGE_FILTER_SHAPES = [(2, 3, 30, 40, 70, 13), (1, 8, 20, 50, 33, 12), (2, 16, 18, 18, 64, 16), (1, 2, 40, 41, 130, 14),
                       (3, 5, 15, 140, 9, 15), (1, 64, 16, 16, 40, 16), (1, 1, 70, 300, 24, 13), (4, 1, 33, 29, 5, 12),
                       (1, 3, 40, 60, 33, 17), (2, 4, 30, 70, 20, 21), (1, 2, 45, 50, 64, 24), (1, 1, 64, 200, 12, 25),
                       (1, 8, 36, 36, 70, 31), (2, 1, 40, 90, 16, 32), (1, 16, 34, 34, 8, 32), (1, 1, 50, 50, 3, 19)]


@pytest.mark.parametrize("shape", LARGE_FILTER_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_filters_of_12_to_32_on_the_general_kernel(shape):
    """Filters beyond 11 x 11 (up to 32 x 32) run on the general-case kernel, one to four filter
    rows of one channel per chunk: every tile shape and schedule against the oracle, integer inputs
    bit for bit, guard bands; with one channel and one image also through dconv_single_channel,
    which hands such filters to the same kernel."""
    N, C, H, W, K, F = shape
    x, f = wl.random_case(5200 + F + K, N, C, H, W, K, F)
    acc, mag, _ = oracle.general(x, f)
    xi, fi = wl.integer_case(5300 + F + K, N, C, H, W, K, F)
    want = oracle.general(xi, fi)[0].astype(np.float32)
    assert dconv.tile_choice(False, N, C, H, W, K, F) >= 0 or (N == 1 and C == 1)
    for v in [AUTO, dconv.VARIANT_TILED] + [dconv.VARIANT_TILED_CFG0 + i for i in range(12)]:
        assert_within_bound(run_general(x, f, v), acc, mag, f"general {shape} variant {v:#x}")
        buf = torch.full((want.size + 2048,), float("nan"), device="cuda")
        out = buf[1024:1024 + want.size].view(want.shape)
        dconv.dconv_general(dev(xi), dev(fi), out=out, variant=v)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), want), f"{shape} variant {v:#x}: integer inputs"
        assert torch.isnan(buf[:1024]).all() and torch.isnan(buf[1024 + want.size:]).all(), f"{shape}: guard bands"
    if N == 1 and C == 1:
        assert dconv.tile_choice(True, 1, 1, H, W, K, F) == dconv.CHOICE_GENERAL_CASE
        got = run_single(x[0, 0], f[:, 0], AUTO)
        assert_within_bound(got, acc[0], mag[0], f"single-channel {shape}")
        assert np.array_equal(run_single(xi[0, 0], fi[:, 0], AUTO), want[0])
        with pytest.raises(dconv.DconvError) as e:          # the special case's own kernels end at 11 x 11
            run_single(x[0, 0], f[:, 0], dconv.VARIANT_TILED)
        assert e.value.status == dconv.STATUS_UNSUPPORTED


def _variant_of_choice(c):
    return {dconv.CHOICE_FEW_FILTERS: dconv.VARIANT_FEW_FILTERS, dconv.CHOICE_SPECIAL_CASE: dconv.VARIANT_SPECIAL_CASE,
            dconv.CHOICE_SIMPLE: dconv.VARIANT_SIMPLE}.get(c, dconv.VARIANT_TILED_CFG0 + c)


def test_the_reported_choice_is_what_the_library_runs():
    """dconv_tile_choice names, on the host, the kernel and configuration the plain entry points
    launch: forcing what it names gives the plain call's output bit for bit (every kernel sums in
    an order that its configuration fixes), and the outputs are within the bound of the oracle.
    One shape for every branch of the dispatchers' rules that a small problem can reach."""
    single = [(256, 256, 16, 3), (300, 420, 3, 5), (700, 900, 12, 5), (600, 800, 64, 7), (720, 1280, 40, 9),
              (150, 2000, 64, 3), (512, 512, 32, 3), (640, 640, 128, 5), (96, 96, 8, 33), (1100, 1100, 8, 3), (120, 150, 8, 13),
              (800, 800, 96, 5), (1024, 1024, 16, 5), (256, 256, 1, 3), (500, 520, 2, 7)]
    general = [(2, 64, 30, 30, 64, 3), (3, 32, 20, 20, 32, 3), (2, 64, 40, 40, 96, 3), (1, 256, 14, 14, 256, 3),
               (1, 128, 20, 20, 128, 7), (4, 128, 17, 14, 192, 1), (8, 8, 60, 60, 64, 2), (2, 64, 30, 30, 128, 2),
               (40, 16, 7, 7, 64, 3), (2, 2, 200, 200, 16, 3), (1, 1, 200, 200, 64, 3), (2, 16, 40, 40, 8, 33),
               (16, 8, 96, 96, 64, 3), (1, 1, 700, 900, 64, 3)]
    seen = set()
    for i, (H, W, K, F) in enumerate(single):
        x, f = wl.random_case(3100 + i, 1, 1, H, W, K, F)
        c = dconv.tile_choice(True, 1, 1, H, W, K, F)
        seen.add(("single", c))
        got = dconv.dconv_single_channel(dev(x[0, 0]), dev(f[:, 0]))
        if c == dconv.CHOICE_GENERAL_CASE:     # (the general kernel's own entry point, one image of one channel)
            forced = dconv.dconv_general(dev(x), dev(f), variant=dconv.VARIANT_TILED)[0]
        else:
            forced = dconv.dconv_single_channel(dev(x[0, 0]), dev(f[:, 0]), variant=_variant_of_choice(c))
        torch.cuda.synchronize()
        assert torch.equal(got, forced), f"single-channel {(H, W, K, F)}: choice {c}"
        acc, mag, _ = oracle.general(x, f)
        assert_within_bound(got.cpu().numpy(), acc[0], mag[0], f"single-channel {(H, W, K, F)}")
    for i, (N, C, H, W, K, F) in enumerate(general):
        x, f = wl.random_case(3200 + i, N, C, H, W, K, F)
        c = dconv.tile_choice(False, N, C, H, W, K, F)
        seen.add(("general", c))
        got = dconv.dconv_general(dev(x), dev(f))
        forced = dconv.dconv_general(dev(x), dev(f), variant=_variant_of_choice(c))
        torch.cuda.synchronize()
        assert torch.equal(got, forced), f"general {(N, C, H, W, K, F)}: choice {c}"
        acc, mag, _ = oracle.general(x, f)
        assert_within_bound(got.cpu().numpy(), acc, mag, f"general {(N, C, H, W, K, F)}")
    # the shapes reach the three tile shapes and the other kernels of both entry points
    assert {("general", 0), ("general", 1), ("general", 2), ("general", dconv.CHOICE_SPECIAL_CASE),
            ("general", dconv.CHOICE_SIMPLE), ("single", dconv.CHOICE_FEW_FILTERS),
            ("single", dconv.CHOICE_SIMPLE), ("single", dconv.CHOICE_GENERAL_CASE)} <= seen, seen
    assert len({c for k, c in seen if k == "single" and c >= 0}) >= 5, seen


@pytest.mark.parametrize("side", [24000, 23100])
def test_single_channel_huge_images_sampled(side):
    """One 24000 x 24000 image (2.3 GB: input rows beyond 2 GiB, more than 4 GiB of output) on the
    few-filters kernel, whose row descriptors start at each row and are clamped to 31 bits; the
    matrix-core kernel addresses an output plane with 32-bit lane offsets and refuses it.  One
    23100 x 23100 image (2.13 GB, the largest it takes) on 32- and 16-filter blocks.  Sampled
    outputs, whole rows at the far end and at the seam between the maps."""
    H = W = side
    K, F = 2, 3
    rng = np.random.default_rng(side)
    img = rng.standard_normal((H, W), dtype=np.float32)
    flt = rng.standard_normal((K, F, F), dtype=np.float32)
    x4, f4 = img.reshape(1, 1, H, W), flt.reshape(K, 1, F, F)
    Ho, Wo = H - F + 1, W - F + 1
    total = K * Ho * Wo
    idx = np.unique(np.concatenate([wl.sample_indices(2401, total, 20000),
                                    np.arange(total - 2 * Wo, total),                  # the last rows, whole
                                    np.arange(Ho * Wo - 3000, Ho * Wo + 3000),         # the seam between the maps
                                    # around the input row whose byte offset crosses 2 GiB (if any)
                                    min((1 << 29) // W, Ho - 2) * Wo + np.arange(-3000, 3000)]))
    acc, mag = oracle.general_at(x4, f4, idx)
    xd, fd = dev(img), dev(flt)
    sel = torch.from_numpy(idx).to("cuda")
    if side == 24000:
        variants = (("few-filters kernel", dconv.VARIANT_FEW_FILTERS), ("library's choice", dconv.VARIANT_AUTO))
        with pytest.raises(dconv.DconvError) as e:
            dconv.dconv_single_channel(xd, fd, variant=dconv.VARIANT_TILED)
        assert e.value.status == dconv.STATUS_UNSUPPORTED
    else:
        variants = (("32-filter blocks", dconv.VARIANT_TILED_CFG0 + 0), ("16-filter blocks", dconv.VARIANT_TILED_CFG0 + 9),
                    ("library's choice", dconv.VARIANT_AUTO))
    for name, variant in variants:
        print(f"{side} x {side} image, {name}", flush=True)
        out = dconv.dconv_single_channel(xd, fd, variant=variant)
        torch.cuda.synchronize()
        assert_within_bound(out.view(-1)[sel].cpu().numpy(), acc, mag, f"{side}^2 image, {name}")
        del out
