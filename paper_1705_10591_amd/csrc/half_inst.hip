// Instantiations of the 16-bit general-case kernel for ONE filter side (DCONV_F, given on the
// compiler command line): fp16, bf16 and int8.
#include "half_kernel.h"

#ifndef DCONV_F
#error "compile with -DDCONV_F=<filter side>"
#endif

namespace dconv {

namespace {
constexpr int F = DCONV_F;
constexpr int kRowGroup = half_row_group(F);

// (This helper depends on F without naming it in its template arguments: it must stay local to
// the translation unit, or the linker may keep one filter side's copy for all of them.)
template <class TL, bool DIRECT>
int launch_dtype(const void* in, const void* filt, float* out, const Shape& s, hipStream_t st,
                 int dtype, bool blocked, bool dry)
{
    switch (dtype) {
    case kF16: return half_try_launch<F, kRowGroup, kF16, TL, DIRECT>(in, filt, out, s, st, dry, blocked);
    case kBF16: return half_try_launch<F, kRowGroup, kBF16, TL, DIRECT>(in, filt, out, s, st, dry, blocked);
    case kI8: return half_try_launch<F, kRowGroup, kI8, TL, DIRECT>(in, filt, out, s, st, dry, blocked);
    default: return DCONV_UNSUPPORTED;
    }
}

}  // namespace

template <>
int half_launch_for_F<DCONV_F>(const void* in, const void* filt, float* out, const Shape& s,
                               hipStream_t st, int dtype, int config, bool blocked, bool dry)
{
    switch (config) {
    case 0: return launch_dtype<HalfTileSmall, false>(in, filt, out, s, st, dtype, blocked, dry);
    case 1: return launch_dtype<HalfTileLarge, false>(in, filt, out, s, st, dtype, blocked, dry);
    case 2: return launch_dtype<HalfTileSmall, true>(in, filt, out, s, st, dtype, blocked, dry);
    case 3: return launch_dtype<HalfTileLarge, true>(in, filt, out, s, st, dtype, blocked, dry);
    case 4: return launch_dtype<HalfTileMid, true>(in, filt, out, s, st, dtype, blocked, dry);
    default: return DCONV_UNSUPPORTED;
    }
}

}  // namespace dconv
