"""dconv_general_noalloc: the general case for callers that cannot allocate device memory.

Called through the C ABI by ctypes with raw device pointers and compared with dconv_general_v
on the same inputs.  Both run the same kernels in the same launch configuration and add the
parts of a shared tile in a fixed order, so the outputs must agree bit for bit (which is within
the floating-point bar a fortiori); the first case is also checked against the CPU oracle.
The calls come in pairs on one GPU, the second with a smaller input: the static array keeps
what the first call left in it.
"""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_1705_10591_amd as dconv
from helpers import assert_within_bound

pytestmark = pytest.mark.gpu

SHARED = dconv.VARIANT_TILED_CFG0 + 2 * 3          # + tile shape: tiles cut over channels
SHARED7 = dconv.VARIANT_TILED_CFG0 + 3 * 3         # the same on a grid of seven workgroups


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


def call(entry, x, f, out, variant, stream=None):
    """One call through the C ABI: raw device pointers, sizes, variant, stream."""
    N, C, H, W = x.shape
    K, _, F, _ = f.shape
    st = torch.cuda.current_stream().cuda_stream if stream is None else stream.cuda_stream
    fn = getattr(dconv.load_library(), entry)
    rc = fn(ctypes.c_void_p(x.data_ptr()), N, C, H, W, ctypes.c_void_p(f.data_ptr()), K, F,
            ctypes.c_void_p(out.data_ptr()), int(variant), ctypes.c_void_p(st))
    assert rc == dconv.STATUS_OK, f"{entry}: {dconv.status_string(rc)}"


def both(x, f, variant, what):
    """dconv_general_noalloc and dconv_general_v on the same device inputs; returns both outputs."""
    N, C, H, W = x.shape
    K, _, F, _ = f.shape
    shape = (N, K, H - F + 1, W - F + 1)
    got = torch.full(shape, float("nan"), device="cuda")
    ref = torch.full(shape, float("nan"), device="cuda")
    print(f"{what}: N,C,H,W={tuple(x.shape)} K,F={K},{F} variant={variant:#x}", flush=True)
    call("dconv_general_noalloc", x, f, got, variant)
    torch.cuda.synchronize()
    call("dconv_general_v", x, f, ref, variant)
    torch.cuda.synchronize()
    return got, ref


def test_two_calls_in_a_row_the_second_smaller_match_the_allocating_entry_point():
    # the deep-layer benchmark shape: the automatic schedule shares its tiles between workgroups
    w = wl.G3
    x, f = wl.make_inputs(w)
    dx, df = dev(x), dev(f)
    got, ref = both(dx, df, dconv.VARIANT_AUTO, "first call")
    assert torch.equal(got, ref)
    # the same layer on a quarter of the batch: fewer tiles than workgroups, every tile shared
    dx2 = dx[:8].contiguous()
    got2, ref2 = both(dx2, df, dconv.VARIANT_AUTO, "second call, smaller")
    assert torch.equal(got2, ref2)
    # (another schedule than the first call's, so another order of additions: close, not equal)
    assert torch.allclose(got2, got[:8], rtol=0, atol=2e-5)
    # the first call against the oracle on sampled outputs
    idx = wl.sample_indices(77, w.out_elems, 20000)
    acc, mag = oracle.general_at(x, f, idx)
    assert_within_bound(got.cpu().numpy().reshape(-1)[idx], acc, mag, "G3 through dconv_general_noalloc")


# (N, C, H, W, K, F)
SMALL = [(3, 16, 28, 28, 130, 3), (2, 12, 40, 150, 33, 5), (7, 24, 9, 35, 96, 3), (2, 3, 37, 41, 64, 11)]


@pytest.mark.parametrize("tile", [0, 1, 2])
def test_forced_shared_schedules_large_then_small(tile):
    """Every tile shape with tiles shared over the whole grid and over seven workgroups; after
    each shape a smaller one (a crop of the same images and a subset of the filters)."""
    for i, (N, C, H, W, K, F) in enumerate(SMALL):
        x, f = wl.random_case(500 + i, N, C, H, W, K, F)
        acc, mag, _ = oracle.general(x, f)
        for variant in (SHARED + tile, SHARED7 + tile):
            got, ref = both(dev(x), dev(f), variant, "large")
            assert torch.equal(got, ref)
            assert_within_bound(got.cpu().numpy(), acc, mag, f"noalloc {SMALL[i]} variant {variant:#x}")
            xs = np.ascontiguousarray(x[: max(1, N - 1), :, : H - 2, : W - 3])
            fs = np.ascontiguousarray(f[: max(1, K - 5)])
            got, ref = both(dev(xs), dev(fs), variant, "smaller")
            assert torch.equal(got, ref)


def test_integer_inputs_are_exact_and_repeat():
    x, f = wl.integer_case(9, 3, 16, 28, 28, 130, 3)
    acc, _, _ = oracle.general(x, f)
    dx, df = dev(x), dev(f)
    for rep in range(3):
        got, _ = both(dx, df, SHARED7 + 1, f"integer inputs, repeat {rep}")
        assert np.array_equal(got.cpu().numpy().astype(np.float64), acc)


def test_variants_without_shared_tiles_and_errors():
    x, f = wl.random_case(610, 2, 3, 20, 23, 5, 3)
    for variant in (dconv.VARIANT_SIMPLE, dconv.VARIANT_TILED, dconv.VARIANT_SPECIAL_CASE):
        got, ref = both(dev(x), dev(f), variant, "no shared tiles")
        assert torch.equal(got, ref)
    lib = dconv.load_library()
    fake = ctypes.c_void_p(0x1000)          # never dereferenced: validation fails first
    assert lib.dconv_general_noalloc(None, 1, 2, 8, 8, fake, 2, 3, fake, 0, None) == dconv.STATUS_NULL_POINTER
    assert lib.dconv_general_noalloc(fake, 1, 2, 4, 8, fake, 2, 5, fake, 0, None) == dconv.STATUS_BAD_SHAPE
    assert lib.dconv_general_noalloc(fake, 1, 2, 8, 8, fake, 2, 3, fake, 99, None) == dconv.STATUS_UNSUPPORTED


def test_one_image_of_one_channel_that_the_general_kernel_runs():
    """One channel is the special case, but this shape runs on the general-case kernel (few tiles,
    shared between workgroups: the static array is in use), then a smaller one."""
    for i, (H, W, K, F) in enumerate(((64, 64, 128, 8), (50, 60, 96, 8))):
        assert dconv.tile_choice(False, 1, 1, H, W, K, F) >= 0
        x, f = wl.random_case(612 + i, 1, 1, H, W, K, F)
        acc, mag, _ = oracle.general(x, f)
        got, ref = both(dev(x), dev(f), dconv.VARIANT_AUTO, "one channel")
        assert torch.equal(got, ref)
        assert_within_bound(got.cpu().numpy(), acc, mag, f"noalloc one channel {(H, W, K, F)}")


def test_nothing_is_allocated_on_a_fresh_stream():
    """On a stream the library has never seen, dconv_general_v allocates its workspace (64 MiB on
    this chip); dconv_general_noalloc leaves the device's free memory as it is."""
    x, f = wl.random_case(611, 3, 16, 28, 28, 130, 3)
    dx, df = dev(x), dev(f)
    out = torch.empty(3, 130, 26, 26, device="cuda")
    ref = torch.empty_like(out)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    with torch.cuda.stream(s):
        call("dconv_general_noalloc", dx, df, out, SHARED + 1, stream=s)
    s.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free0 - free1 < (8 << 20), f"free device memory fell by {free0 - free1} bytes"
    with torch.cuda.stream(s):
        call("dconv_general_v", dx, df, ref, SHARED + 1, stream=s)
    s.synchronize()
    assert torch.equal(out, ref)
