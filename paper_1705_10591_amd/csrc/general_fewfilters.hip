// The few-filters kernel of the general case (general_few_kernel.h): when it runs.
#include "general_few_kernel.h"

#include <algorithm>

namespace dconv {

// Filter sides with a window that fits the register file comfortably, up to sixteen filters.
bool general_few_supports(const Shape& s)
{
    return s.F >= 1 && s.F <= 7 && s.K >= 1 && s.K <= 16;
}

// Worth it when its estimated time is below nine tenths of the matrix-core kernel's.  Estimates in
// microseconds, fitted to 460 measured layers (1 to 8 filters of 1x1 to 7x7, 2 to 256 channels,
// 14 x 14 to 512 x 640 maps, 1 to 512 images; this kernel's within 22 % rms, the other's 23 %):
//   this kernel: 8 us plus the largest of three bounds -- a barrier and a round of LDS latencies
//     per channel (0.55 us), input and output at 6 TB/s, and K x F x F multiply-adds per pixel
//     and channel (K rounded up to the filter counts it is compiled for, divided by the share
//     of its lanes that fall inside the map) at 62 TFLOP/s with one row per band, 64 with two,
//     70 with four (two thirds of that with one filter, whose weights go through scalar
//     registers), stretched when there are fewer than 384 tiles;
//   the matrix-core kernel: 12 us plus a 32-filter block at 90 TFLOP/s whatever the filter
//     count, or input and output at 2.5 TB/s.
// On those layers the choice is within 1.4 % of the faster kernel on average (14 of 460 are 15 %
// or more off); where this kernel is chosen it is up to 6 times faster (101 x 3 x 64 x 640, two
// 1x1 filters: 97 -> 16 us; 8 x 16 x 224 x 224, one 7x7 filter: 189 -> 25 us; 8 x 64 x 224 x 224,
// three 3x3 filters: 139 -> 51 us; eight: 139 -> 81 us).
// Nine to sixteen filters (compiled for twelve and sixteen, one row per band, one channel per
// barrier) pay off on layers of few channels, where the matrix-core kernel is bound by its
// write-back: the same estimate with 58 TFLOP/s stretched below 512 tiles, 1.5 us per channel and
// 4 TB/s, chosen where it is below the other's.  On 280 further measured layers of 9 to 16 filters
// that choice is within 2 % of the faster kernel on average (10 of 280 are 15 % or more off; 18 %
// with the matrix-core kernel alone), and up to 2.8 times faster (512 x 3 x 28 x 320, ten 1x1
// filters: 108 -> 38 us; 21 x 8 x 96 x 640, twelve 5x5: 174 -> 80 us).
bool general_few_preferred(const Shape& s)
{
    // (one image of one channel is the special case proper, which has its own few-filters kernel)
    if (!general_few_supports(s) || (s.C == 1 && s.N == 1)) return false;
    const GfTile t = gf_tile_for(s);
    const double tiles = (double)gf_tiles(s, t.lpr, t.rpw);
    static const int kCompiled[17] = {0, 1, 2, 3, 4, 6, 6, 8, 8, 12, 12, 12, 12, 16, 16, 16, 16};
    if (tiles < 32) {
        // A launch of a few tiles: both kernels take the time of one workgroup's chain of
        // latencies.  This kernel's grows with the channels it walks (a barrier, the staging of
        // the tile's rows and the tile's multiply-adds per channel); the matrix-core kernel
        // shares a tile's channels between workgroups and grows slowly.  Kernel times from
        // replayed graphs (1 to 16 images of 28^2 .. 224^2, 3 to 64 channels, 1 to 8 filters of
        // 1x1 .. 5x5; within 7 % and 17 % rms), microseconds: over the 319 measured layers with
        // fewer than 32 tiles the choice goes from 5.3 % above the faster kernel to 1.0 %
        // (1 x 3 x 112 x 112, one 5x5 filter: 7.9 -> 4.4 us).
        const int kc = kCompiled[s.K], ff = s.F * s.F;
        const double few = 3.1 + s.C * (0.32 + 0.036 * (s.F - 1) + 0.0081 * kc * ff + 0.025 * kc);
        const double tiled = 5.4 + 0.059 * s.C + 0.144 * ff + 0.0071 * s.C * ff;
        return few < 0.9 * tiled;
    }
    const double tw = 4.0 * t.lpr, tr = 4.0 * (kWave / t.lpr) * t.rpw;
    const double inside = (double)s.Wo * s.Ho /
                          ((double)((s.Wo + (int)tw - 1) / (int)tw) * tw * (double)((s.Ho + (int)tr - 1) / (int)tr) * tr);
    const double macs = (double)s.N * s.Ho * s.Wo * s.C * s.F * s.F;      // per filter
    const double bytes = 4.0 * ((double)s.N * s.C * s.H * s.W + (double)s.N * s.K * s.Ho * s.Wo);
    const double tiled = 12.0 + std::max(2.0 * macs * 32 / 90e6, bytes / 2.5e6);
    if (s.K > 8) {
        const double alu = 2.0 * macs * kCompiled[s.K] / inside / 58e6 * std::max(1.0, 512.0 / tiles);
        return 8.0 + std::max({1.5 * s.C, bytes / 4e6, alu}) < tiled;
    }
    const double rate = (t.rpw == 1 ? 62e6 : t.rpw == 2 ? 64e6 : 70e6) * (s.K == 1 ? 0.65 : 1.0);
    const double alu = 2.0 * macs * kCompiled[s.K] / inside / rate * std::max(1.0, 384.0 / tiles);
    const double few = 8.0 + std::max({0.55 * s.C, bytes / 6e6, alu});
    return few < 0.9 * tiled;
}

int launch_general_few(const float* in, const float* filt, float* out, const Shape& s, hipStream_t st)
{
    if (!general_few_supports(s)) return DCONV_UNSUPPORTED;
    switch (s.F) {
    case 1: return gf_launch_for_F<1>(in, filt, out, s, st);
    case 2: return gf_launch_for_F<2>(in, filt, out, s, st);
    case 3: return gf_launch_for_F<3>(in, filt, out, s, st);
    case 4: return gf_launch_for_F<4>(in, filt, out, s, st);
    case 5: return gf_launch_for_F<5>(in, filt, out, s, st);
    case 6: return gf_launch_for_F<6>(in, filt, out, s, st);
    case 7: return gf_launch_for_F<7>(in, filt, out, s, st);
    default: return DCONV_UNSUPPORTED;
    }
}

}  // namespace dconv
