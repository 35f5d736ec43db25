// The few-filters kernel of the general case (general_few_kernel.h): when it runs.
#include "general_few_kernel.h"

#include <algorithm>

namespace dconv {

// Filter sides with a window that fits the register file comfortably, up to sixteen filters.
bool general_few_supports(const Shape& s)
{
    return s.F >= 1 && s.F <= 7 && s.K >= 1 && s.K <= 16;
}

// Worth it when its estimated kernel time is below the matrix-core kernel's (below 95 % of it
// for launches of under 768 tiles).  Both estimates are fitted to the kernel times of 1015 layers
// measured from replayed graphs, so that launches of a few microseconds count as what they take
// on the GPU and not as what the host needs to issue them (1 to 16 filters of 1x1 to 7x7, 2 to
// 256 channels, 14 x 14 to 512 x 640 maps, 1 to 512 images, 3 us to 2 ms; this kernel's within
// 16 % rms, the other's 23 %), in microseconds:
//   this kernel: 3.4 plus the largest of three bounds --
//     the chain of one workgroup, C channels of a barrier and a round of LDS latencies (0.30,
//     shared by two channels where two go per barrier), the staging of the tile's rows (0.010
//     a row), the tile's multiply-adds (0.0105 x K x F x F x rows per band) and the filters'
//     weights (0.03 x K), K rounded up to the counts it is compiled for, times the rounds of
//     tiles over 430 workgroups;
//     input and output at 5.1 TB/s;
//     K x F x F multiply-adds per pixel and channel, divided by the share of its lanes that
//     fall inside the map, at 70 TFLOP/s;
//   the matrix-core kernel: 7.1 plus the largest of a chain of 0.055 + 0.009 x F x F per channel
//     (it shares a tile's channels between workgroups), a 32-filter block at 88 TFLOP/s whatever
//     the filter count, and input and output at 2.6 TB/s.
// With the halves of the layers swapped between fitting and checking the choice is 1.2 to 1.6 %
// above the faster kernel on the checked half; on all 1015 layers 1.3 % (35 are 15 % or more off),
// against 3.8 % for the rule this replaces, which was fitted to times that included the host's
// launch cost (4 x 16 x 224 x 224 with one 1x1 filter: 13.3 -> 5.1 us).  Where this kernel is
// chosen it is up to 6 times faster (101 x 3 x 64 x 640, two 1x1 filters: 97 -> 16 us; 8 x 16 x 224
// x 224, one 7x7 filter: 189 -> 23 us; 8 x 64 x 224 x 224, three 3x3 filters: 139 -> 49 us; eight:
// 139 -> 81 us; 21 x 8 x 96 x 640, twelve 5x5: 174 -> 80 us).
bool general_few_preferred(const Shape& s)
{
    // (one image of one channel is the special case proper, which has its own few-filters kernel)
    if (!general_few_supports(s) || (s.C == 1 && s.N == 1)) return false;
    static const int kCompiled[17] = {0, 1, 2, 3, 4, 6, 6, 8, 8, 12, 12, 12, 12, 16, 16, 16, 16};
    const GfTile t = gf_tile_for(s);
    const double tiles = (double)gf_tiles(s, t.lpr, t.rpw);
    const int kc = kCompiled[s.K], ff = s.F * s.F;
    const int tw = 4 * t.lpr, tr = 4 * (kWave / t.lpr) * t.rpw;
    const double inside = (double)s.Wo * s.Ho /
                          ((double)((s.Wo + tw - 1) / tw) * tw * (double)((s.Ho + tr - 1) / tr) * tr);
    const double macs = (double)s.N * s.Ho * s.Wo * s.C * ff;             // per filter
    const double bytes = 4.0 * ((double)s.N * s.C * s.H * s.W + (double)s.N * s.K * s.Ho * s.Wo);
    const int per_barrier = (t.rpw == 1 && kc <= 8) ? 2 : 1;              // channels (see launch_gf)
    const double chain = s.C * (0.30 / per_barrier + 0.010 * (tr + s.F - 1) + 0.0105 * kc * ff * t.rpw + 0.03 * kc);
    const double few = 3.4 + std::max({chain * std::max(1.0, tiles / 430.0), bytes / 5.1e6,
                                       2.0 * macs * kc / inside / 70e6});
    const double tiled = 7.1 + std::max({0.055 * s.C + 0.009 * s.C * ff, 2.0 * macs * 32 / 88e6, bytes / 2.6e6});
    return few < (tiles >= 768 ? 1.0 : 0.95) * tiled;
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
