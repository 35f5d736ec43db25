// Dispatch of the general case for short data types (fp16, bf16, int8): the matrix-core kernel where the shape allows it, the
// one-thread-per-output kernel otherwise.
#include "half_kernel.h"

namespace dconv {

namespace {

int launch_tiled(const void* in, const void* filt, float* out, const Shape& s, hipStream_t st,
                 int dtype, bool large_tile, bool blocked, bool dry)
{
    switch (s.F) {
    case 1: return half_launch_for_F<1>(in, filt, out, s, st, dtype, large_tile, blocked, dry);
    case 2: return half_launch_for_F<2>(in, filt, out, s, st, dtype, large_tile, blocked, dry);
    case 3: return half_launch_for_F<3>(in, filt, out, s, st, dtype, large_tile, blocked, dry);
    case 4: return half_launch_for_F<4>(in, filt, out, s, st, dtype, large_tile, blocked, dry);
    case 5: return half_launch_for_F<5>(in, filt, out, s, st, dtype, large_tile, blocked, dry);
    case 6: return half_launch_for_F<6>(in, filt, out, s, st, dtype, large_tile, blocked, dry);
    case 7: return half_launch_for_F<7>(in, filt, out, s, st, dtype, large_tile, blocked, dry);
    case 8: return half_launch_for_F<8>(in, filt, out, s, st, dtype, large_tile, blocked, dry);
    case 9: return half_launch_for_F<9>(in, filt, out, s, st, dtype, large_tile, blocked, dry);
    case 10: return half_launch_for_F<10>(in, filt, out, s, st, dtype, large_tile, blocked, dry);
    case 11: return half_launch_for_F<11>(in, filt, out, s, st, dtype, large_tile, blocked, dry);
    default: return DCONV_UNSUPPORTED;
    }
}

int launch_simple_half(const void* in, const void* filt, float* out, const Shape& s, hipStream_t st,
                       int dtype, bool blocked)
{
    const int64_t total = (int64_t)s.N * s.K * s.Ho * s.Wo;
    const int64_t blocks = (total + kThreads - 1) / kThreads;
    if (blocks > 2147483647LL) return DCONV_UNSUPPORTED;
    auto kern = dtype == kI8 ? simple_half_kernel<kI8>
              : dtype == kBF16 ? simple_half_kernel<kBF16> : simple_half_kernel<kF16>;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(kThreads), 0, st,
                       in, filt, out, s.N, s.C, s.H, s.W, s.K, s.F, s.Ho, s.Wo, blocked ? 1 : 0);
    return hipGetLastError() == hipSuccess ? DCONV_OK : DCONV_LAUNCH_FAILED;
}

// The large tile (128 filters x 512 pixels) where its filter tile is mostly full, there are
// enough tiles for most of the CUs (one workgroup each) and a tile has enough chunks to pay for
// its longer prologue and write-back; the small one otherwise.  (Measured on ten layer shapes:
// 10-25 % faster where chosen.)
bool large_tile_preferred(const Shape& s, int dtype)
{
    const int64_t tiles = (((int64_t)s.N * s.Ho * s.Wo + 511) / 512) * ((s.K + 127) / 128);
    const int rg = half_row_group(s.F);
    const int chunks = s.C / (kHalfChunkBytes / elem_bytes(dtype)) * ((s.F + rg - 1) / rg);
    return s.K >= 96 && tiles >= 128 && chunks >= 8;
}

}  // namespace

int launch_general_half(const void* in, const void* filt, float* out, const Shape& s, hipStream_t st,
                        int dtype, int layout, int variant)
{
    if (dtype != kF16 && dtype != kBF16 && dtype != kI8) return DCONV_UNSUPPORTED;
    if (layout != DCONV_LAYOUT_CHANNELS_LAST && layout != DCONV_LAYOUT_CHANNEL_BLOCKED) return DCONV_UNSUPPORTED;
    const bool blocked = layout == DCONV_LAYOUT_CHANNEL_BLOCKED;
    // a blocked layout exists only for whole blocks of channels
    if (blocked && s.C % (kHalfChunkBytes / elem_bytes(dtype)) != 0) return DCONV_BAD_SHAPE;
    if (variant == DCONV_VARIANT_SIMPLE) return launch_simple_half(in, filt, out, s, st, dtype, blocked);
    // the two tile shapes of the matrix-core kernel, forced (tests, tuning)
    if (variant == DCONV_VARIANT_TILED_CFG0 || variant == DCONV_VARIANT_TILED_CFG0 + 1)
        return launch_tiled(in, filt, out, s, st, dtype, variant == DCONV_VARIANT_TILED_CFG0 + 1, blocked, false);
    if (variant != DCONV_VARIANT_AUTO && variant != DCONV_VARIANT_TILED) return DCONV_UNSUPPORTED;
    int rc = DCONV_UNSUPPORTED;
    if (large_tile_preferred(s, dtype)) rc = launch_tiled(in, filt, out, s, st, dtype, true, blocked, false);
    if (rc == DCONV_UNSUPPORTED) rc = launch_tiled(in, filt, out, s, st, dtype, false, blocked, false);
    if (rc == DCONV_UNSUPPORTED && variant == DCONV_VARIANT_AUTO)
        return launch_simple_half(in, filt, out, s, st, dtype, blocked);
    return rc;
}

}  // namespace dconv
