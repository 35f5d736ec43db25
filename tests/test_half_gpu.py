"""Parity of the 16-bit (fp16 / bf16) general-case entry point with the fp64 oracle, through the C ABI.

The oracle is the same plain definition as for fp32, evaluated on the 16-bit values widened
to float32 (exact); layouts differ (channels innermost on the device), so the test transposes.
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
TORCH_TYPE = {"f16": torch.float16, "bf16": torch.bfloat16}
# the matrix-core kernel with its tile shape forced: 64 filters x 256 pixels, 128 x 512
# small and large tile staged through registers, small and large tile staged directly into LDS
# and a mid tile, 128 x 384, staged directly
TILE_SMALL, TILE_LARGE, TILE_SMALL_DIRECT, TILE_LARGE_DIRECT, TILE_MID_DIRECT = \
    (dconv.VARIANT_TILED_CFG0 + i for i in range(5))
TILES = (TILE_SMALL, TILE_LARGE, TILE_SMALL_DIRECT, TILE_LARGE_DIRECT, TILE_MID_DIRECT)
KERNELS = [TILED, SIMPLE, *TILES]


def dev16(bits_nchw_like: np.ndarray, kind: str) -> torch.Tensor:
    """uint16 patterns in [.., C, H, W] order -> device tensor in [.., H, W, C] order."""
    nhwc = np.ascontiguousarray(np.moveaxis(bits_nchw_like, 1, -1))
    return torch.from_numpy(nhwc.view(np.int16)).view(TORCH_TYPE[kind]).to("cuda")


def run_half(xb, fb, kind, variant):
    print(f"half {kind} N,C,H,W={xb.shape} K,F={fb.shape[0]},{fb.shape[-1]} variant={variant}", flush=True)
    out = dconv.dconv_general_half(dev16(xb, kind), dev16(fb, kind), variant=variant)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def rounded_case(seed, shape, kind, integer=False):
    N, C, H, W, K, F = shape
    x, f = (wl.integer_case if integer else wl.random_case)(seed, N, C, H, W, K, F)
    xr, xb = wl.to_16bit(x, kind)
    fr, fb = wl.to_16bit(f, kind)
    return xr, fr, xb, fb


# (N, C, H, W, K, F) with C a multiple of 16: the matrix-core kernel
HALF_SHAPES = [
    (2, 16, 20, 23, 5, 3),
    (1, 32, 30, 30, 70, 3),       # two filter tiles, ragged
    (3, 16, 28, 28, 130, 3),      # pixel blocks wrap over rows and images
    (2, 16, 24, 150, 33, 5),      # several column strips; row groups of 2, 2, 1
    (1, 48, 12, 300, 8, 2),
    (2, 16, 27, 31, 64, 11),      # one filter row per chunk
    (1, 64, 9, 9, 3, 1),
    (2, 32, 16, 16, 3, 4),
    (1, 16, 20, 20, 9, 7),
    (5, 16, 8, 8, 4, 3),          # tiny images: one pixel block spans several images
    (3, 16, 5, 5, 4, 5),          # filter as large as the image
    (1, 16, 14, 14, 2, 9),
    (1, 32, 13, 12, 3, 10),
    (2, 16, 11, 10, 2, 6),
    (1, 16, 12, 11, 2, 8),
    (7, 32, 9, 35, 96, 3),
]


@pytest.mark.parametrize("kind", ["f16", "bf16"])
@pytest.mark.parametrize("shape", HALF_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_half_small_shapes(shape, kind):
    xr, fr, xb, fb = rounded_case(900 + shape[-1], shape, kind)
    acc, mag, _ = oracle.general(xr, fr)
    for variant in KERNELS:
        got = run_half(xb, fb, kind, variant)
        assert_within_bound(got, acc, mag, f"half {kind} {shape} variant {variant}")


@pytest.mark.parametrize("kind", ["f16", "bf16"])
def test_half_fallback_kernel_long_reduction_of_one_sign(kind):
    """The one-lane-per-output kernel on 18 000 terms of one sign (the worst case for a running
    sum): it sums level by level, so the error stays within the bound."""
    shape = (1, 2000, 6, 7, 3, 3)
    N, C, H, W, K, F = shape
    x, f = wl.random_case(977, N, C, H, W, K, F, "u01", "u01")
    xr, xb = wl.to_16bit(x, kind)
    fr, fb = wl.to_16bit(f, kind)
    acc, mag, _ = oracle.general(xr, fr)
    assert_within_bound(run_half(xb, fb, kind, SIMPLE), acc, mag, f"half {kind} simple kernel {shape}")


@pytest.mark.parametrize("kind", ["f16", "bf16"])
@pytest.mark.parametrize("shape", [(2, 32, 28, 28, 70, 3), (1, 16, 30, 140, 64, 11), (3, 48, 12, 12, 9, 5)],
                         ids=lambda s: "x".join(map(str, s)))
def test_half_integer_inputs_are_bit_exact(shape, kind):
    xr, fr, xb, fb = rounded_case(3, shape, kind, integer=True)
    assert np.array_equal(xr, wl.integer_case(3, *shape)[0])        # small integers are representable
    _, _, o32, _ = oracle.general(xr, fr, want32=True)
    for variant in KERNELS:
        np.testing.assert_array_equal(run_half(xb, fb, kind, variant), o32)


@pytest.mark.parametrize("kind", ["f16", "bf16"])
@pytest.mark.parametrize("shape", [(2, 3, 20, 23, 5, 3), (1, 24, 14, 15, 7, 5), (2, 1, 9, 9, 2, 1)],
                         ids=lambda s: "x".join(map(str, s)))
def test_half_channel_counts_without_a_matrix_core_kernel_fall_back(shape, kind):
    xr, fr, xb, fb = rounded_case(17, shape, kind)
    acc, mag, _ = oracle.general(xr, fr)
    assert_within_bound(run_half(xb, fb, kind, AUTO), acc, mag, f"half {kind} {shape} auto")
    with pytest.raises(dconv.DconvError) as e:
        run_half(xb, fb, kind, TILED)
    assert e.value.status == dconv.STATUS_UNSUPPORTED


@pytest.mark.parametrize("kind", ["f16", "bf16"])
def test_half_non_finite_filter_stays_in_its_own_map(kind):
    shape = (2, 16, 14, 15, 5, 5)
    xr, fr, xb, fb = rounded_case(5, shape, kind)
    acc, mag, _ = oracle.general(xr, fr)
    inf_bits = {"f16": 0x7C00, "bf16": 0x7F80}[kind]
    for bad in (0, 2, 4):
        fbad = fb.copy()
        fbad[bad] = inf_bits + 1            # a NaN pattern
        fbad[bad, 0, 0, 0] = inf_bits
        for variant in TILES:
            got = run_half(xb, fbad, kind, variant)
            assert not np.isfinite(got[:, bad]).any()
            keep = [k for k in range(shape[4]) if k != bad]
            assert_within_bound(got[:, keep], acc[:, keep], mag[:, keep], f"half {kind} filter {bad} non-finite")


def test_half_output_guard_bands_stay_untouched():
    shape = (2, 16, 13, 29, 37, 3)
    N, C, H, W, K, F = shape
    xr, fr, xb, fb = rounded_case(8, shape, "f16")
    acc, mag, _ = oracle.general(xr, fr)
    Ho, Wo = H - F + 1, W - F + 1
    n_out, guard = N * K * Ho * Wo, 4096
    buf = torch.full((n_out + 2 * guard,), float("nan"), dtype=torch.float32, device="cuda")
    out = buf[guard:guard + n_out].view(N, K, Ho, Wo)
    for variant in TILES:
        buf.fill_(float("nan"))
        dconv.dconv_general_half(dev16(xb, "f16"), dev16(fb, "f16"), out=out, variant=variant)
        torch.cuda.synchronize()
        host = buf.cpu().numpy()
        assert np.isnan(host[:guard]).all() and np.isnan(host[guard + n_out:]).all()
        assert_within_bound(host[guard:guard + n_out].reshape(N, K, Ho, Wo), acc, mag, "half guard bands")


@pytest.mark.parametrize("variant", [TILED, *TILES],
                         ids=["auto", "small", "large", "small-direct", "large-direct", "mid-direct"])
@pytest.mark.parametrize("kind", ["f16", "bf16"])
@pytest.mark.parametrize("name", ["G2", "G3"])
def test_half_config_shapes_sampled(name, kind, variant):
    """The fp32 benchmark shapes G2 and G3 (channel counts 64 and 256) with 16-bit inputs."""
    w = wl.CONFIGS[name]
    x, f = wl.make_inputs(w)
    xr, xb = wl.to_16bit(x.reshape(w.N, w.C, w.H, w.W), kind)
    fr, fb = wl.to_16bit(f.reshape(w.K, w.C, w.F, w.F), kind)
    out = dconv.dconv_general_half(dev16(xb, kind), dev16(fb, kind), variant=variant)
    torch.cuda.synchronize()
    total = out.numel()
    idx = wl.sample_indices(31, total, 4000)
    got = out.view(-1)[torch.from_numpy(idx).to("cuda")].cpu().numpy()
    acc, mag = oracle.general_at(xr, fr, idx)
    assert_within_bound(got, acc, mag, f"half {kind} {name} sampled")


# ---- 8-bit integers: exact int32 sums, compared bit for bit -----------------------------------

def int8_case(seed, shape):
    N, C, H, W, K, F = shape
    rng = np.random.default_rng(1705 + seed)
    x = rng.integers(-128, 128, size=(N, C, H, W)).astype(np.int8)
    f = rng.integers(-128, 128, size=(K, C, F, F)).astype(np.int8)
    return x, f


def run_i8(x, f, variant):
    print(f"int8 N,C,H,W={x.shape} K,F={f.shape[0]},{f.shape[-1]} variant={variant}", flush=True)
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(np.moveaxis(a, 1, -1))).to("cuda")
    out = dconv.dconv_general_i8(to_dev(x), to_dev(f), variant=variant)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def exact_i8(x, f):
    """The oracle's fp64 sums are exact here (all terms are integers below 2**14, at most a few
    thousand of them)."""
    acc, _, _ = oracle.general(x.astype(np.float32), f.astype(np.float32))
    assert np.array_equal(acc, np.rint(acc))
    return acc.astype(np.int64)


I8_SHAPES = [
    (2, 32, 20, 23, 5, 3), (1, 64, 30, 30, 70, 3), (3, 32, 28, 28, 130, 3), (2, 32, 24, 150, 33, 5),
    (1, 96, 12, 300, 8, 2), (2, 32, 27, 31, 64, 11), (1, 64, 9, 9, 3, 1), (1, 32, 20, 20, 9, 7),
    (5, 32, 8, 8, 4, 3), (3, 32, 5, 5, 4, 5), (1, 32, 13, 12, 3, 10), (7, 64, 9, 35, 96, 3),
]


@pytest.mark.parametrize("shape", I8_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_int8_small_shapes_are_exact(shape):
    x, f = int8_case(shape[-1], shape)
    want = exact_i8(x, f)
    for variant in KERNELS:
        np.testing.assert_array_equal(run_i8(x, f, variant).astype(np.int64), want)


@pytest.mark.parametrize("shape", [(2, 3, 20, 23, 5, 3), (1, 48, 14, 15, 7, 5), (2, 16, 9, 9, 2, 1)],
                         ids=lambda s: "x".join(map(str, s)))
def test_int8_channel_counts_without_a_matrix_core_kernel_fall_back(shape):
    x, f = int8_case(11, shape)
    np.testing.assert_array_equal(run_i8(x, f, AUTO).astype(np.int64), exact_i8(x, f))
    with pytest.raises(dconv.DconvError) as e:
        run_i8(x, f, TILED)
    assert e.value.status == dconv.STATUS_UNSUPPORTED


def test_int8_extreme_values_do_not_overflow_early():
    """All pixels and weights at -128: the largest products; C*F*F*2**14 still fits int32."""
    shape = (1, 64, 12, 40, 3, 5)
    N, C, H, W, K, F = shape
    x = np.full((N, C, H, W), -128, np.int8)
    f = np.full((K, C, F, F), -128, np.int8)
    got = run_i8(x, f, TILED)
    assert (got == C * F * F * 16384).all()


@pytest.mark.parametrize("variant", [TILED, *TILES],
                         ids=["auto", "small", "large", "small-direct", "large-direct", "mid-direct"])
@pytest.mark.parametrize("name", ["G2", "G3"])
def test_int8_config_shapes_sampled(name, variant):
    w = wl.CONFIGS[name]
    x, f = int8_case(77, (w.N, w.C, w.H, w.W, w.K, w.F))
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(np.moveaxis(a, 1, -1))).to("cuda")
    out = dconv.dconv_general_i8(to_dev(x), to_dev(f), variant=variant)
    torch.cuda.synchronize()
    idx = wl.sample_indices(32, out.numel(), 4000)
    got = out.view(-1)[torch.from_numpy(idx).to("cuda")].cpu().numpy().astype(np.int64)
    acc, _ = oracle.general_at(x.astype(np.float32), f.astype(np.float32), idx)
    np.testing.assert_array_equal(got, acc.astype(np.int64))


# ---- the channel-blocked layout ------------------------------------------------------------------

def to_blocked(a_nchw_like: np.ndarray, cb: int) -> np.ndarray:
    """[X][C][A][B] -> [X][C/cb][A][B][cb]."""
    X, C, A, B = a_nchw_like.shape
    return np.ascontiguousarray(a_nchw_like.reshape(X, C // cb, cb, A, B).transpose(0, 1, 3, 4, 2))


@pytest.mark.parametrize("kind", ["f16", "bf16", "i8"])
@pytest.mark.parametrize("shape", [(2, 32, 20, 23, 5, 3), (3, 64, 28, 28, 130, 3), (2, 32, 24, 150, 33, 5),
                                   (2, 32, 27, 31, 64, 11), (5, 32, 8, 8, 4, 3), (1, 96, 13, 12, 3, 10),
                                   (1, 128, 9, 9, 3, 1)],
                         ids=lambda s: "x".join(map(str, s)))
def test_blocked_layout_small_shapes(shape, kind):
    if kind == "i8":
        x, f = int8_case(shape[-1] + 50, shape)
        want = exact_i8(x, f)
        xb, fb = torch.from_numpy(to_blocked(x, 32)).cuda(), torch.from_numpy(to_blocked(f, 32)).cuda()
        for variant in KERNELS:
            print(f"int8 blocked {shape} variant {variant}", flush=True)
            got = dconv.dconv_general_i8(xb, fb, variant=variant, blocked=True)
            np.testing.assert_array_equal(got.cpu().numpy().astype(np.int64), want)
        return
    xr, fr, xbits, fbits = rounded_case(950 + shape[-1], shape, kind)
    acc, mag, _ = oracle.general(xr, fr)
    as_t = lambda bits: torch.from_numpy(to_blocked(bits, 16).view(np.int16)).view(TORCH_TYPE[kind]).cuda()
    xb, fb = as_t(xbits), as_t(fbits)
    for variant in KERNELS:
        print(f"half {kind} blocked {shape} variant {variant}", flush=True)
        got = dconv.dconv_general_half(xb, fb, variant=variant, blocked=True)
        assert_within_bound(got.cpu().numpy(), acc, mag, f"half {kind} blocked {shape} variant {variant}")


@pytest.mark.parametrize("kind", ["bf16", "i8"])
def test_blocked_layout_G3_sampled(kind):
    w = wl.CONFIGS["G3"]
    if kind == "i8":
        x, f = int8_case(78, (w.N, w.C, w.H, w.W, w.K, w.F))
        out = dconv.dconv_general_i8(torch.from_numpy(to_blocked(x, 32)).cuda(),
                                     torch.from_numpy(to_blocked(f, 32)).cuda(), blocked=True)
        idx = wl.sample_indices(33, out.numel(), 4000)
        got = out.view(-1)[torch.from_numpy(idx).to("cuda")].cpu().numpy().astype(np.int64)
        acc, _ = oracle.general_at(x.astype(np.float32), f.astype(np.float32), idx)
        np.testing.assert_array_equal(got, acc.astype(np.int64))
        return
    x, f = wl.make_inputs(w)
    xr, xbits = wl.to_16bit(x.reshape(w.N, w.C, w.H, w.W), kind)
    fr, fbits = wl.to_16bit(f.reshape(w.K, w.C, w.F, w.F), kind)
    as_t = lambda bits: torch.from_numpy(to_blocked(bits, 16).view(np.int16)).view(TORCH_TYPE[kind]).cuda()
    out = dconv.dconv_general_half(as_t(xbits), as_t(fbits), blocked=True)
    torch.cuda.synchronize()
    idx = wl.sample_indices(34, out.numel(), 4000)
    got = out.view(-1)[torch.from_numpy(idx).to("cuda")].cpu().numpy()
    acc, mag = oracle.general_at(xr, fr, idx)
    assert_within_bound(got, acc, mag, f"half {kind} blocked G3 sampled")


def test_blocked_layout_needs_whole_channel_blocks():
    lib = dconv.load_library()
    x = torch.zeros(1, 8, 8, 24, dtype=torch.float16, device="cuda")      # 24 channels: not a multiple of 16
    f = torch.zeros(2, 3, 3, 24, dtype=torch.float16, device="cuda")
    out = torch.zeros(1, 2, 6, 6, dtype=torch.float32, device="cuda")
    rc = lib.dconv_general_lowp(x.data_ptr(), 1, 24, 8, 8, f.data_ptr(), 2, 3, out.data_ptr(),
                                dconv.DTYPE_F16, dconv.LAYOUT_CHANNEL_BLOCKED, 0, None)
    assert rc == dconv.STATUS_BAD_SHAPE


def test_half_large_image_sampled():
    """2.7 GB of output from one image: output planes more than 2 GiB apart."""
    N, C, H, W, K, F = 1, 16, 2048, 2100, 160, 3
    x, f = wl.random_case(995, N, C, H, W, K, F)
    xr, xb = wl.to_16bit(x, "bf16")
    fr, fb = wl.to_16bit(f, "bf16")
    for variant in (TILED, TILE_SMALL, TILE_LARGE_DIRECT):
        print(f"half bf16 large image variant {variant}", flush=True)
        out = dconv.dconv_general_half(dev16(xb, "bf16"), dev16(fb, "bf16"), variant=variant)
        torch.cuda.synchronize()
        total = out.numel()
        idx = np.unique(np.concatenate([wl.sample_indices(996, total, 20000), np.arange(0, 2048),
                                        np.arange(total - 2048, total),
                                        np.arange((1 << 29) - 1024, (1 << 29) + 1024)]))
        got = out.view(-1)[torch.from_numpy(idx).to("cuda")].cpu().numpy()
        acc, mag = oracle.general_at(xr, fr, idx)
        assert_within_bound(got, acc, mag, f"half bf16 large image variant {variant}")
        del out


# ---- filters beyond 11 x 11: one filter row of a block of channels per chunk ----------------

LARGE_FILTER_HALF_SHAPES = [(1, 16, 20, 40, 64, 13), (2, 32, 34, 36, 9, 32), (1, 48, 30, 30, 70, 21),
                            (1, 16, 26, 90, 130, 17), (3, 32, 14, 60, 33, 12), (1, 64, 40, 40, 16, 25)]


@pytest.mark.parametrize("kind", ["f16", "bf16", "i8"])
@pytest.mark.parametrize("shape", LARGE_FILTER_HALF_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_short_types_filters_of_12_to_32(shape, kind):
    """The matrix-core kernel of the short data types is compiled for every filter side up to 32.
    Integer inputs, so every kernel must give the oracle's sums bit for bit; a forced tile whose
    filter block does not fit in LDS refuses the shape, the small register-staged tile and the
    library's own choice never do."""
    N, C, H, W, K, F = shape
    if kind == "i8":
        C = (C + 31) // 32 * 32
        x, f = int8_case(40 + F, (N, C, H, W, K, F))
        want = exact_i8(x, f)
        run = lambda v: run_i8(x, f, v).astype(np.int64)
    else:
        xr, fr, xb, fb = rounded_case(40 + F, shape, kind, integer=True)
        want = oracle.general(xr, fr, want32=True)[2]
        run = lambda v: run_half(xb, fb, kind, v)
    ran = 0
    for variant in KERNELS:
        try:
            got = run(variant)
        except dconv.DconvError as e:
            assert e.status == dconv.STATUS_UNSUPPORTED and variant not in (TILED, SIMPLE, TILE_SMALL), variant
            continue
        np.testing.assert_array_equal(got, want)
        ran += 1
    assert ran >= 3
    np.testing.assert_array_equal(run(AUTO), want)
