// The few-filters kernel of the general case (general_few_kernel.h): when it runs.
#include "general_few_kernel.h"

#include <algorithm>

namespace dconv {

// Filter sides with a window that fits the register file comfortably, up to eight filters.
bool general_few_supports(const Shape& s)
{
    return s.F >= 1 && s.F <= 7 && s.K >= 1 && s.K <= 8;
}

// Worth it when its tiles cover the chip (200 or more) and its estimated time is below the
// matrix-core kernel's.  Estimates in microseconds, fitted to measurements on 8 x 64 x 224 x 224
// .. 128 x 64 x 56 x 56 layers with 1 to 8 filters of 1x1 to 7x7:
//   this kernel: the largest of three bounds -- a barrier and a round of LDS latencies per
//     channel (0.45 us), the input read at 3.5 TB/s, K x F x F multiply-adds per pixel and
//     channel at 40 TFLOP/s (K rounded up to the filter counts it is compiled for) -- times
//     1.3, plus 8 us;
//   the matrix-core kernel: a 32-filter block at 110 TFLOP/s whatever the filter count, or the
//     input read at 2.5 TB/s.
// Where it is chosen it is 1.2 to 7.7 times faster (8 x 16 x 224 x 224, one 7x7 filter: 189 -> 25 us;
// 8 x 64 x 224 x 224, three 3x3 filters: 139 -> 61 us; eight: 139 -> 121 us).
bool general_few_preferred(const Shape& s)
{
    if (!general_few_supports(s) || s.C < 2) return false;
    if (gf_auto_tiles(s) < 200) return false;
    static const int kCompiled[9] = {0, 1, 2, 3, 4, 6, 6, 8, 8};
    const double macs = (double)s.N * s.Ho * s.Wo * s.C * s.F * s.F;      // per filter
    const double in_bytes = 4.0 * s.N * s.C * s.H * s.W;
    const double few = 1.3 * std::max({0.45 * s.C, in_bytes / 3.5e6, 2.0 * macs * kCompiled[s.K] / 40e6}) + 8.0;
    const double tiled = std::max(2.0 * macs * 32 / 110e6, in_bytes / 2.5e6);
    return few < tiled;
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
