// Dispatch of the general case for short data types (fp16, bf16, int8): the matrix-core kernel where the shape allows it, the
// one-thread-per-output kernel otherwise.
#include "half_kernel.h"

namespace dconv {

namespace {

int launch_tiled(const void* in, const void* filt, float* out, const Shape& s, hipStream_t st,
                 int dtype, int config, bool blocked, bool dry)
{
    switch (s.F) {
    case 1: return half_launch_for_F<1>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 2: return half_launch_for_F<2>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 3: return half_launch_for_F<3>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 4: return half_launch_for_F<4>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 5: return half_launch_for_F<5>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 6: return half_launch_for_F<6>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 7: return half_launch_for_F<7>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 8: return half_launch_for_F<8>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 9: return half_launch_for_F<9>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 10: return half_launch_for_F<10>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 11: return half_launch_for_F<11>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 12: return half_launch_for_F<12>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 13: return half_launch_for_F<13>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 14: return half_launch_for_F<14>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 15: return half_launch_for_F<15>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 16: return half_launch_for_F<16>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 17: return half_launch_for_F<17>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 18: return half_launch_for_F<18>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 19: return half_launch_for_F<19>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 20: return half_launch_for_F<20>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 21: return half_launch_for_F<21>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 22: return half_launch_for_F<22>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 23: return half_launch_for_F<23>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 24: return half_launch_for_F<24>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 25: return half_launch_for_F<25>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 26: return half_launch_for_F<26>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 27: return half_launch_for_F<27>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 28: return half_launch_for_F<28>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 29: return half_launch_for_F<29>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 30: return half_launch_for_F<30>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 31: return half_launch_for_F<31>(in, filt, out, s, st, dtype, config, blocked, dry);
    case 32: return half_launch_for_F<32>(in, filt, out, s, st, dtype, config, blocked, dry);
    default: return DCONV_UNSUPPORTED;
    }
}

int launch_simple_half(const void* in, const void* filt, float* out, const Shape& s, hipStream_t st,
                       int dtype, bool blocked)
{
    const int64_t total = (int64_t)s.N * s.K * s.Ho * s.Wo;
    int64_t blocks = (total + kThreads - 1) / kThreads;
    if (blocks > 256 * 64) blocks = 256 * 64;     // grid-stride beyond that
    auto kern = dtype == kI8 ? simple_half_kernel<kI8>
              : dtype == kBF16 ? simple_half_kernel<kBF16> : simple_half_kernel<kF16>;
    begin_launch();
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(kThreads), 0, st,
                       in, filt, out, s.N, s.C, s.H, s.W, s.K, s.F, s.Ho, s.Wo, blocked ? 1 : 0);
    return launch_status();
}

// Which tile configuration a shape gets.  The large tile (128 filters x 512 pixels, one workgroup
// per CU) does the work of four small ones (64 x 256, two workgroups per CU) in the time of
// about three (fewer operand reads and half the staging per matrix-core instruction; measured
// 2.5 to 3.4 over shapes and boxes), so it wins where its tiles fill the CUs in whole rounds:
// compare rounds x time per tile.  Its filter tile has to be mostly full and a tile long enough
// to pay for the longer prologue and write-back.
// Staging (see general_half_kernel): the small tile goes directly into LDS when a pixel's
// channel block is contiguous with its neighbours' (blocked layout) and through registers
// otherwise; the large tile goes directly in both layouts, except that with chunks of one or
// two steps (1x1 filters) the register path is faster on channels-last inputs and the small
// tile, whose two workgroups per CU hide the barrier after every chunk better, on blocked ones
// (measured: 12 and 20 %).
int preferred_config(const Shape& s, int dtype, bool blocked)
{
    const int small_cfg = blocked ? 2 : 0;
    const int rg = half_row_group(s.F);
    const int chunks = s.C / (kHalfChunkBytes / elem_bytes(dtype)) * ((s.F + rg - 1) / rg);
    const bool short_chunks = rg * s.F <= 2;
    if (s.K < 96 || chunks < 4 || (blocked && short_chunks)) return small_cfg;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        cus = 256;
    const int64_t px = (int64_t)s.N * s.Ho * s.Wo;
    const int64_t large = ((px + 511) / 512) * ((s.K + 127) / 128);
    const int64_t mid = ((px + 383) / 384) * ((s.K + 127) / 128);
    const int64_t small = ((px + 255) / 256) * ((s.K + 63) / 64);
    // rounds of tiles over the CUs x time per tile, in units of a small tile's time (measured over
    // the twelve shapes of the search table in both layouts).  The mid tile does three quarters of
    // the large one's work per chunk and has less to do before and after its chunks, which
    // counts for more the fewer chunks a tile has; the large tile needs eight chunks to pay.
    const double large_cost = chunks >= 8 ? (double)((large + cus - 1) / cus) * 2.95 : 1e30;
    // (with channels last its direct loads touch a line per lane, and a tile of four chunks does
    // not pay for them: 64 channels of 3x3, 16 x 16 .. 114 x 114 maps: 8-25 % slower than the small
    // tile staged through registers; in the blocked layout it wins there)
    const bool mid_ok = !short_chunks && (blocked || chunks >= 8);
    const double mid_cost = mid_ok ? (double)((mid + cus - 1) / cus) * (chunks >= 12 ? 2.45 : 2.1) : 1e30;
    const double small_cost = (double)((small + cus - 1) / cus);
    if (mid_cost < large_cost && mid_cost < small_cost) return 4;
    if (large_cost >= small_cost) return small_cfg;
    return short_chunks ? 1 : 3;
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
    // one tile configuration of the matrix-core kernel, forced (tests, tuning)
    if (variant >= DCONV_VARIANT_TILED_CFG0 && variant < DCONV_VARIANT_TILED_CFG0 + kHalfConfigs)
        return launch_tiled(in, filt, out, s, st, dtype, variant - DCONV_VARIANT_TILED_CFG0, blocked, false);
    if (variant != DCONV_VARIANT_AUTO && variant != DCONV_VARIANT_TILED) return DCONV_UNSUPPORTED;
    const int cfg = preferred_config(s, dtype, blocked);
    int rc = launch_tiled(in, filt, out, s, st, dtype, cfg, blocked, false);
    // (the small tiles hold every shape the large one does, and the register-staged one the most)
    if (rc == DCONV_UNSUPPORTED && cfg != 0) rc = launch_tiled(in, filt, out, s, st, dtype, 0, blocked, false);
    if (rc == DCONV_UNSUPPORTED && variant == DCONV_VARIANT_AUTO)
        return launch_simple_half(in, filt, out, s, st, dtype, blocked);
    return rc;
}

}  // namespace dconv
