"""MI355X-native direct fp32 2D convolution (gfx950): Python binding of libdconv.so.

The functions here only marshal arguments: they take torch CUDA tensors
(device memory and the current stream come from PyTorch), pass raw device
pointers and sizes through the C ABI declared in include/dconv.h, and return
the output tensor.  Every step of the computation runs in the HIP kernels of
the library.  There is no CPU or PyTorch fallback: if the library has not
been built, importing the compute functions raises.
"""
from __future__ import annotations

import ctypes
from pathlib import Path

import torch

_PKG = Path(__file__).resolve().parent
LIB_PATH = _PKG / "libdconv.so"

VARIANT_AUTO, VARIANT_SIMPLE, VARIANT_TILED, VARIANT_FEW_FILTERS = 0, 1, 2, 3
VARIANT_TILED_CFG0 = 0x100     # + i: tiled kernel with tile configuration i forced
VARIANT_SPECIAL_CASE = 4       # dconv_general with one channel: the single-channel tiled kernel
VARIANT_SPECIAL_CASE_CFG0 = 0x200   # + i: the same with its tile configuration i forced
STATUS_OK, STATUS_NULL_POINTER, STATUS_BAD_SHAPE, STATUS_UNSUPPORTED, STATUS_LAUNCH_FAILED, \
    STATUS_SCRATCH_EXCEEDED = range(6)

EXPORTS = ("dconv_single_channel", "dconv_general", "dconv_single_channel_v",
           "dconv_general_v", "dconv_status_string", "dconv_version",
           "dconv_tile_config_count", "dconv_tile_choice", "dconv_release_workspace",
           "dconv_general_f16", "dconv_general_bf16", "dconv_general_half_v",
           "dconv_general_i8", "dconv_general_i8_v", "dconv_general_lowp", "dconv_general_noalloc")
DTYPE_F16, DTYPE_BF16, DTYPE_I8 = 0, 1, 2
LAYOUT_CHANNELS_LAST, LAYOUT_CHANNEL_BLOCKED = 0, 1

_lib = None


class DconvError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"dconv status {status}: {message}")
        self.status = status


def load_library() -> ctypes.CDLL:
    """Load libdconv.so from the package directory; raise if it was never built."""
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_1705_10591_amd.build` "
                "(there is no fallback path)")
        lib = ctypes.CDLL(str(LIB_PATH))
        p, i = ctypes.c_void_p, ctypes.c_int
        lib.dconv_single_channel.argtypes = [p, i, i, p, i, i, p, p]
        lib.dconv_single_channel_v.argtypes = [p, i, i, p, i, i, p, i, p]
        lib.dconv_general.argtypes = [p, i, i, i, i, p, i, i, p, p]
        lib.dconv_general_v.argtypes = [p, i, i, i, i, p, i, i, p, i, p]
        lib.dconv_general_noalloc.argtypes = [p, i, i, i, i, p, i, i, p, i, p]
        lib.dconv_general_f16.argtypes = [p, i, i, i, i, p, i, i, p, p]
        lib.dconv_general_bf16.argtypes = [p, i, i, i, i, p, i, i, p, p]
        lib.dconv_general_half_v.argtypes = [p, i, i, i, i, p, i, i, p, i, i, p]
        lib.dconv_general_i8.argtypes = [p, i, i, i, i, p, i, i, p, p]
        lib.dconv_general_i8_v.argtypes = [p, i, i, i, i, p, i, i, p, i, p]
        lib.dconv_general_lowp.argtypes = [p, i, i, i, i, p, i, i, p, i, i, i, p]
        for name in ("dconv_single_channel", "dconv_single_channel_v",
                     "dconv_general", "dconv_general_v", "dconv_general_noalloc", "dconv_version",
                     "dconv_release_workspace", "dconv_general_f16", "dconv_general_bf16",
                     "dconv_general_half_v", "dconv_general_i8", "dconv_general_i8_v",
                     "dconv_general_lowp"):
            getattr(lib, name).restype = i
        lib.dconv_tile_config_count.argtypes = [i]
        lib.dconv_tile_config_count.restype = i
        lib.dconv_tile_choice.argtypes = [i] * 7
        lib.dconv_tile_choice.restype = i
        lib.dconv_status_string.argtypes = [i]
        lib.dconv_status_string.restype = ctypes.c_char_p
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load_library().dconv_status_string(int(status)).decode()


def tile_config_count(single_channel: bool) -> int:
    """Number of tile configurations of the tiled kernel (see VARIANT_TILED_CFG0)."""
    return int(load_library().dconv_tile_config_count(1 if single_channel else 0))


CHOICE_FEW_FILTERS, CHOICE_SPECIAL_CASE, CHOICE_SIMPLE, CHOICE_INVALID, CHOICE_GENERAL_CASE = -1, -2, -3, -4, -5


def tile_choice(single_channel: bool, N: int, C: int, H: int, W: int, K: int, F: int) -> int:
    """What VARIANT_AUTO picks for a shape: a tile configuration (>= 0) or a CHOICE_* value.
    Host arithmetic only: works without a GPU."""
    return int(load_library().dconv_tile_choice(1 if single_channel else 0, N, C, H, W, K, F))


def release_workspace() -> None:
    """Free the device workspaces dconv_general keeps per (device, stream)."""
    torch.cuda.synchronize()
    load_library().dconv_release_workspace()


def version() -> int:
    return int(load_library().dconv_version())


def _check(t: torch.Tensor, ndim: int, what: str):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32
            and t.dim() == ndim and t.is_contiguous()):
        raise TypeError(f"{what} must be a contiguous float32 CUDA tensor with {ndim} dims")


def _raise(rc: int):
    if rc != STATUS_OK:
        raise DconvError(rc, status_string(rc))


def _stream_ptr(device) -> int:
    return torch.cuda.current_stream(device).cuda_stream


def dconv_single_channel(img: torch.Tensor, filt: torch.Tensor, out: torch.Tensor | None = None,
                         variant: int = VARIANT_AUTO) -> torch.Tensor:
    """out[k,y,x] = sum_{i,j} img[y+i,x+j] * filt[k,i,j]   (one input channel, K filters)."""
    _check(img, 2, "img")
    _check(filt, 3, "filt")
    H, W = img.shape
    K, F, F2 = filt.shape
    if F != F2:
        raise ValueError("filters must be square")
    if F > H or F > W:
        _raise(STATUS_BAD_SHAPE)
    if out is None:
        out = torch.empty((K, H - F + 1, W - F + 1), dtype=torch.float32, device=img.device)
    else:
        _check(out, 3, "out")
        if tuple(out.shape) != (K, H - F + 1, W - F + 1):
            raise ValueError("out has the wrong shape")
    with torch.cuda.device(img.device):
        rc = load_library().dconv_single_channel_v(
            img.data_ptr(), H, W, filt.data_ptr(), K, F, out.data_ptr(), int(variant),
            _stream_ptr(img.device))
    _raise(rc)
    return out


def dconv_general(x: torch.Tensor, filt: torch.Tensor, out: torch.Tensor | None = None,
                  variant: int = VARIANT_AUTO, noalloc: bool = False) -> torch.Tensor:
    """out[n,k,y,x] = sum_{c,i,j} x[n,c,y+i,x+j] * filt[k,c,i,j].

    noalloc: call dconv_general_noalloc (shared tiles meet in the library's static device array;
    the library allocates nothing; pass `out`, or torch allocates the result)."""
    _check(x, 4, "in")
    _check(filt, 4, "filt")
    N, C, H, W = x.shape
    K, C2, F, F2 = filt.shape
    if C2 != C or F != F2:
        raise ValueError("filter shape does not match the input")
    if F > H or F > W:
        _raise(STATUS_BAD_SHAPE)
    if out is None:
        out = torch.empty((N, K, H - F + 1, W - F + 1), dtype=torch.float32, device=x.device)
    else:
        _check(out, 4, "out")
        if tuple(out.shape) != (N, K, H - F + 1, W - F + 1):
            raise ValueError("out has the wrong shape")
    with torch.cuda.device(x.device):
        lib = load_library()
        rc = (lib.dconv_general_noalloc if noalloc else lib.dconv_general_v)(
            x.data_ptr(), N, C, H, W, filt.data_ptr(), K, F, out.data_ptr(), int(variant),
            _stream_ptr(x.device))
    _raise(rc)
    return out


def _lowp(x, filt, out, variant, blocked, types, out_type):
    for t, what in ((x, "in"), (filt, "filt")):
        if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dim() == (5 if blocked else 4)
                and t.is_contiguous() and t.dtype in types):
            raise TypeError(f"{what} must be a contiguous CUDA tensor of type {types} with "
                            f"{5 if blocked else 4} dims")
    if x.dtype != filt.dtype:
        raise TypeError("in and filt must have the same type")
    if blocked:
        N, CG, H, W, cb = x.shape
        K, CG2, F, F2, cb2 = filt.shape
        if cb * x.element_size() != 32 or (CG2, cb2) != (CG, cb):
            raise ValueError("channel blocks must be 32 bytes and match between in and filt")
        C = CG * cb
    else:
        N, H, W, C = x.shape
        K, F, F2, C2 = filt.shape
        if C2 != C:
            raise ValueError("filter shape does not match the input")
    if F != F2:
        raise ValueError("filters must be square")
    if F > H or F > W:
        _raise(STATUS_BAD_SHAPE)
    shape = (N, K, H - F + 1, W - F + 1)
    if out is None:
        out = torch.empty(shape, dtype=out_type, device=x.device)
    elif not (isinstance(out, torch.Tensor) and out.is_cuda and out.dtype == out_type
              and out.is_contiguous() and tuple(out.shape) == shape):
        raise TypeError(f"out must be a contiguous {out_type} CUDA tensor of shape {shape}")
    dtype = {torch.float16: DTYPE_F16, torch.bfloat16: DTYPE_BF16, torch.int8: DTYPE_I8}[x.dtype]
    with torch.cuda.device(x.device):
        rc = load_library().dconv_general_lowp(
            x.data_ptr(), N, C, H, W, filt.data_ptr(), K, F, out.data_ptr(), dtype,
            LAYOUT_CHANNEL_BLOCKED if blocked else LAYOUT_CHANNELS_LAST, int(variant), _stream_ptr(x.device))
    _raise(rc)
    return out


def dconv_general_half(x: torch.Tensor, filt: torch.Tensor, out: torch.Tensor | None = None,
                       variant: int = VARIANT_AUTO, blocked: bool = False) -> torch.Tensor:
    """16-bit inputs (both torch.float16 or both torch.bfloat16), fp32 accumulation and output:
    out[n,k,y,x] = sum_{i,j,c} in[n,y+i,x+j,c] * filt[k,i,j,c].
    Channels last: x [N,H,W,C], filt [K,F,F,C]; blocked: x [N,C/16,H,W,16], filt [K,C/16,F,F,16]."""
    return _lowp(x, filt, out, variant, blocked, (torch.float16, torch.bfloat16), torch.float32)


def dconv_general_i8(x: torch.Tensor, filt: torch.Tensor, out: torch.Tensor | None = None,
                     variant: int = VARIANT_AUTO, blocked: bool = False) -> torch.Tensor:
    """Signed 8-bit inputs, exact int32 sums and output.  Channels last: x [N,H,W,C],
    filt [K,F,F,C]; blocked: x [N,C/32,H,W,32], filt [K,C/32,F,F,32]."""
    return _lowp(x, filt, out, variant, blocked, (torch.int8,), torch.int32)
