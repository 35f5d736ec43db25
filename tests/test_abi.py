"""CPU-side checks of the C ABI: the library loads, exports what the header
declares, and validates arguments before touching the GPU."""
import ctypes
import re
from pathlib import Path

import pytest

import paper_1705_10591_amd as dconv

ROOT = Path(__file__).resolve().parent.parent


def _declared_functions():
    text = (ROOT / "include" / "dconv.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dconv_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    assert _declared_functions() == sorted(dconv.EXPORTS)


def test_library_exports_every_declared_symbol():
    lib = dconv.load_library()
    for name in _declared_functions():
        assert hasattr(lib, name), f"libdconv.so does not export {name}"


def test_version_and_status_strings():
    assert dconv.version() >= 1003
    seen = {dconv.status_string(s) for s in range(6)}
    assert len(seen) == 6 and all(seen)
    assert dconv.status_string(12345)


FAKE = ctypes.c_void_p(0x1000)   # never dereferenced: every call below fails validation


@pytest.mark.parametrize("variant", [0, 1, 2])
def test_null_pointers_are_rejected(variant):
    lib = dconv.load_library()
    assert lib.dconv_single_channel_v(None, 8, 8, FAKE, 2, 3, FAKE, variant, None) == dconv.STATUS_NULL_POINTER
    assert lib.dconv_single_channel_v(FAKE, 8, 8, None, 2, 3, FAKE, variant, None) == dconv.STATUS_NULL_POINTER
    assert lib.dconv_single_channel_v(FAKE, 8, 8, FAKE, 2, 3, None, variant, None) == dconv.STATUS_NULL_POINTER
    assert lib.dconv_general_v(None, 1, 2, 8, 8, FAKE, 2, 3, FAKE, variant, None) == dconv.STATUS_NULL_POINTER
    assert lib.dconv_general(FAKE, 1, 2, 8, 8, FAKE, 2, 3, None, None) == dconv.STATUS_NULL_POINTER
    assert lib.dconv_single_channel(FAKE, 8, 8, None, 2, 3, FAKE, None) == dconv.STATUS_NULL_POINTER


@pytest.mark.parametrize("dims", [
    (0, 1, 8, 8, 1, 3), (1, 0, 8, 8, 1, 3), (1, 1, 0, 8, 1, 3), (1, 1, 8, 0, 1, 3),
    (1, 1, 8, 8, 0, 3), (1, 1, 8, 8, 1, 0), (1, 1, 8, 8, 1, -3), (-1, 1, 8, 8, 1, 3),
    (1, 1, 4, 8, 1, 5),            # filter taller than the image
    (1, 1, 8, 4, 1, 5),            # filter wider than the image
    (64, 1024, 1024, 1024, 1, 3),  # input beyond 2^31-1 elements
    (1, 1, 40000, 40000, 4, 3),    # one image's output beyond 2^31-1 elements
    (1, 30000, 64, 64, 30000, 3),  # filter bank beyond 2^31-1 elements
])
def test_bad_shapes_are_rejected(dims):
    N, C, H, W, K, F = dims
    lib = dconv.load_library()
    assert lib.dconv_general(FAKE, N, C, H, W, FAKE, K, F, FAKE, None) == dconv.STATUS_BAD_SHAPE
    if N == 1 and C == 1:
        assert lib.dconv_single_channel(FAKE, H, W, FAKE, K, F, FAKE, None) == dconv.STATUS_BAD_SHAPE


def test_unknown_variant_and_unsupported_tiled_shape():
    lib = dconv.load_library()
    assert lib.dconv_general_v(FAKE, 1, 1, 8, 8, FAKE, 1, 3, FAKE, 99, None) == dconv.STATUS_UNSUPPORTED
    # filter side above the largest compiled tiled kernel
    assert lib.dconv_general_v(FAKE, 1, 1, 64, 64, FAKE, 1, 33, FAKE, dconv.VARIANT_TILED, None) \
        == dconv.STATUS_UNSUPPORTED
    assert lib.dconv_single_channel_v(FAKE, 32, 32, FAKE, 1, 13, FAKE, dconv.VARIANT_TILED, None) \
        == dconv.STATUS_UNSUPPORTED


def test_tile_configuration_variants_are_bounded():
    lib = dconv.load_library()
    for single in (0, 1):
        n = dconv.tile_config_count(bool(single))
        assert n >= 1
        beyond = dconv.VARIANT_TILED_CFG0 + n
        if single:
            assert lib.dconv_single_channel_v(FAKE, 32, 32, FAKE, 1, 3, FAKE, beyond, None) \
                == dconv.STATUS_UNSUPPORTED
        else:
            assert lib.dconv_general_v(FAKE, 1, 1, 32, 32, FAKE, 1, 3, FAKE, beyond, None) \
                == dconv.STATUS_UNSUPPORTED


def test_two_threads_in_the_dispatcher_at_once():
    """Host-side state (shape checks, tile choice, cached launch parameters) under two threads.
    Without a GPU every call that passes validation ends at the first HIP query with
    DCONV_LAUNCH_FAILED; what is checked is that concurrent calls neither crash nor disturb each
    other's validation results."""
    import threading
    import torch
    if torch.cuda.is_available():
        pytest.skip("with a GPU the calls would launch on fake pointers; see tests/test_threads_gpu.py")
    lib = dconv.load_library()
    shapes = [(4, 16, 28, 28, 130, 3), (2, 3, 64, 64, 32, 11), (8, 64, 14, 14, 64, 1), (1, 1, 200, 300, 16, 5)]
    seen = [set(), set()]

    def worker(t):
        for rep in range(200):
            N, C, H, W, K, F = shapes[(rep + t) % len(shapes)]
            seen[t].add(lib.dconv_general(FAKE, N, C, H, W, FAKE, K, F, FAKE, None))
            seen[t].add(10 + lib.dconv_general(FAKE, N, C, F - 1, W, FAKE, K, F, FAKE, None))
            seen[t].add(20 + lib.dconv_general_v(FAKE, N, C, 64, 64, FAKE, K, 33, FAKE, dconv.VARIANT_TILED, None))

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(2)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    for t in range(2):
        assert seen[t] == {dconv.STATUS_LAUNCH_FAILED, 10 + dconv.STATUS_BAD_SHAPE, 20 + dconv.STATUS_UNSUPPORTED}


def test_python_binding_refuses_cpu_tensors():
    import torch
    with pytest.raises(TypeError):
        dconv.dconv_general(torch.zeros(1, 1, 4, 4), torch.zeros(1, 1, 3, 3))
    with pytest.raises(TypeError):
        dconv.dconv_single_channel(torch.zeros(4, 4), torch.zeros(1, 3, 3))


def test_16_bit_entry_points_validate_before_launching():
    lib = dconv.load_library()
    ok_dims = (1, 16, 8, 8)
    for fn in (lib.dconv_general_f16, lib.dconv_general_bf16):
        assert fn(None, *ok_dims, FAKE, 2, 3, FAKE, None) == dconv.STATUS_NULL_POINTER
        assert fn(FAKE, *ok_dims, FAKE, 2, 3, None, None) == dconv.STATUS_NULL_POINTER
        assert fn(FAKE, 1, 16, 4, 8, FAKE, 2, 5, FAKE, None) == dconv.STATUS_BAD_SHAPE
        assert fn(FAKE, 1, 0, 8, 8, FAKE, 2, 3, FAKE, None) == dconv.STATUS_BAD_SHAPE
    odd = ctypes.c_void_p(0x1001)             # 16-bit data cannot start at an odd address
    assert lib.dconv_general_f16(odd, *ok_dims, FAKE, 2, 3, FAKE, None) == dconv.STATUS_BAD_SHAPE
    # unknown element type / a variant the 16-bit path does not have
    assert lib.dconv_general_half_v(FAKE, *ok_dims, FAKE, 2, 3, FAKE, 7, 0, None) == dconv.STATUS_UNSUPPORTED
    assert lib.dconv_general_half_v(FAKE, *ok_dims, FAKE, 2, 3, FAKE, 0, dconv.VARIANT_FEW_FILTERS, None) \
        == dconv.STATUS_UNSUPPORTED
    assert lib.dconv_general_half_v(FAKE, *ok_dims, FAKE, 2, 3, FAKE, dconv.DTYPE_I8, 0, None) \
        == dconv.STATUS_UNSUPPORTED          # int8 has entry points of its own (int32 output)
    assert lib.dconv_general_lowp(FAKE, *ok_dims, FAKE, 2, 3, FAKE, 0, 5, 0, None) == dconv.STATUS_UNSUPPORTED
    assert lib.dconv_general_lowp(FAKE, *ok_dims, FAKE, 2, 3, FAKE, 9, 0, 0, None) == dconv.STATUS_UNSUPPORTED
    assert lib.dconv_general_lowp(FAKE, 1, 24, 8, 8, FAKE, 2, 3, FAKE, 0, dconv.LAYOUT_CHANNEL_BLOCKED, 0, None) \
        == dconv.STATUS_BAD_SHAPE            # a blocked layout has whole blocks of channels only
    assert lib.dconv_general_lowp(None, *ok_dims, FAKE, 2, 3, FAKE, 0, 0, 0, None) == dconv.STATUS_NULL_POINTER
    assert lib.dconv_general_i8(None, *ok_dims, FAKE, 2, 3, FAKE, None) == dconv.STATUS_NULL_POINTER
    assert lib.dconv_general_i8(FAKE, 1, 32, 4, 8, FAKE, 2, 5, FAKE, None) == dconv.STATUS_BAD_SHAPE
    assert lib.dconv_general_i8_v(FAKE, *ok_dims, FAKE, 2, 3, FAKE, dconv.VARIANT_FEW_FILTERS, None) \
        == dconv.STATUS_UNSUPPORTED


@pytest.mark.gpu
def test_lds_width_microbenchmark_runs_and_narrow_units_lose_bandwidth():
    """The paper's bank-width experiment on the LDS: 2-byte units get about half of 4-byte ones."""
    import subprocess
    from paper_1705_10591_amd.build import LDS_BENCH
    if not LDS_BENCH.exists():
        pytest.skip("lds_width_bench is not built (python -m paper_1705_10591_amd.build)")
    r = subprocess.run([str(LDS_BENCH)], capture_output=True, text=True, timeout=60)
    assert r.returncode == 0, r.stderr
    rate = {(m.group(1), int(m.group(2))): float(m.group(3))
            for m in re.finditer(r"(read|write)\s+(\d+) B per lane:\s+[\d.]+ ms\s+([\d.]+) B/clk/CU", r.stdout)}
    assert len(rate) == 8, r.stdout
    assert rate[("read", 2)] < 0.6 * rate[("read", 4)]
    assert rate[("read", 4)] < 0.6 * rate[("read", 8)]
    assert rate[("read", 16)] > rate[("read", 8)]


@pytest.mark.gpu
def test_hardware_rate_microbenchmark_runs():
    """Straddled 128-byte runs are written much slower than aligned ones; vector-ALU work next to
    the matrix-core loop costs matrix-core time."""
    import subprocess
    from paper_1705_10591_amd.build import HW_BENCH
    if not HW_BENCH.exists():
        pytest.skip("hw_bench is not built (python -m paper_1705_10591_amd.build)")
    r = subprocess.run([str(HW_BENCH)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stderr
    val = {m.group(1).strip(): float(m.group(2))
           for m in re.finditer(r"^([^#\n][^:]*):\s+[\d.]+ ms\s+([\d.]+) (?:GB/s|TFLOP/s|TOP/s)", r.stdout, re.M)}
    assert len(val) == 18, r.stdout
    assert val["128 B runs, rows of 4092 floats"] < 0.8 * val["128 B runs, rows of 4096 floats"]
    assert val["+ 32 integer VALU per 4 MFMA"] < 0.8 * val["no other vector instructions"]
    # matrix-core waves and store waves on one SIMD take the sum of their times; a wave's own
    # stores between its own matrix-core instructions overlap
    m = re.search(r"^\s*0 idle clocks per 4 MFMA: matrix cores alone\s+([\d.]+) ms, stores alone\s+([\d.]+) ms, "
                  r"together\s+([\d.]+) ms", r.stdout, re.M)
    assert m and float(m.group(3)) > 0.85 * (float(m.group(1)) + float(m.group(2))), r.stdout
    # the 16-bit matrix-core loop is bound by power: the same instructions run faster on zeros
    assert val["bf16 loop, operands zeros"] > 1.1 * val["bf16 loop, operands random bits"], r.stdout
    m = re.search(r"^1 store per 4 MFMA:\s+matrix cores alone\s+([\d.]+) ms, stores alone\s+([\d.]+) ms, "
                  r"interleaved\s+([\d.]+) ms", r.stdout, re.M)
    assert m and float(m.group(3)) < 0.8 * (float(m.group(1)) + float(m.group(2))), r.stdout
