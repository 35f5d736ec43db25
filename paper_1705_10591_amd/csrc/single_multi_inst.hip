// Instantiations of the special-case kernel for a FEW input channels (DCONV_C of them, given on
// the compiler command line) and filters up to 5x5: shapes whose time is the output stream, as
// in the one-channel case, so that the line-aligned write-back of that kernel is what counts.
#include "single_kernel.h"

#ifndef DCONV_C
#error "compile with -DDCONV_C=<input channels>"
#endif

namespace dconv {

namespace {

constexpr int C = DCONV_C;

// the image tile of all channels and the four write-back strips: at most half the LDS of a CU,
// so that two workgroups share one
template <int F, int TW, int TR>
constexpr bool fits()
{
    constexpr int LS = TW + 32 + F - 1 + 32 + F - 1, ROWS = TR + F - 1;
    return (((C * ROWS + 1) * LS + 3) & ~3) + 4 * 8 * (32 * 5 + 32) <= 20 * 1024;
}

// Tile configurations, numbered as in the one-channel case: 0: 512 x 4, or 256 x 4 where that
// does not fit with all the channels; 3: 256 x 2; 4: 128 x 4; 5 and 6: 128 x 4 with passes of 64
// and of 32 pixels; cfg < 0 picks one by shape.
template <int F>
int launch_F(const float* img, const float* filt, float* out, const Shape& s, hipStream_t st, int cfg)
{
    // waves per SIMD the registers are budgeted for: the filter operands of all taps stay in
    // registers (one per pair of taps), with more than 48 taps that takes the larger budget
    constexpr int WPE = C * F * F > 48 ? 2 : 3;
    if (cfg < 0) {
        const int64_t fgroups = (((s.K + 31) / 32) + 3) / 4 * s.N;
        const int64_t t128 = (int64_t)((s.Wo + 127) / 128) * ((s.Ho + 3) / 4) * fgroups;
        cfg = (s.Wo >= 96 && s.Wo < 192) ? short_pass_config(s.Wo) : t128 < 1536 ? 4 : 0;
    }
    if (cfg == 0) {
        if constexpr (fits<F, 512, 4>()) return launch_cfg<F, 512, 4, 4, WPE, C>(img, filt, out, s, st);
        else if constexpr (fits<F, 256, 4>()) return launch_cfg<F, 256, 4, 4, WPE, C>(img, filt, out, s, st);
        cfg = 3;
    }
    if (cfg == 3) {
        if constexpr (fits<F, 256, 2>()) return launch_cfg<F, 256, 2, 4, WPE, C>(img, filt, out, s, st);
        return DCONV_UNSUPPORTED;
    }
    if (cfg == 4) {
        if constexpr (fits<F, 128, 4>()) return launch_cfg<F, 128, 4, 4, WPE, C>(img, filt, out, s, st);
        return DCONV_UNSUPPORTED;
    }
    if (cfg == 5) {           // the same tile with passes of 64 pixels (images 128 to 191 wide)
        if constexpr (fits<F, 128, 4>()) return launch_cfg<F, 128, 4, 2, WPE, C>(img, filt, out, s, st);
        return DCONV_UNSUPPORTED;
    }
    if (cfg == 6) {           // ... and of 32 pixels (images 96 to 127 wide)
        if constexpr (fits<F, 128, 4>()) return launch_cfg<F, 128, 4, 1, WPE, C>(img, filt, out, s, st);
        return DCONV_UNSUPPORTED;
    }
    return DCONV_UNSUPPORTED;
}

}  // namespace

template <>
int single_multi_launch_for_C<DCONV_C>(const float* img, const float* filt, float* out, const Shape& s,
                                       hipStream_t st, int cfg)
{
    switch (s.F) {
    case 1: return launch_F<1>(img, filt, out, s, st, cfg);
    case 2: return launch_F<2>(img, filt, out, s, st, cfg);
    case 3: return launch_F<3>(img, filt, out, s, st, cfg);
    case 4: return launch_F<4>(img, filt, out, s, st, cfg);
    case 5: return launch_F<5>(img, filt, out, s, st, cfg);
    default: return DCONV_UNSUPPORTED;
    }
}

}  // namespace dconv
