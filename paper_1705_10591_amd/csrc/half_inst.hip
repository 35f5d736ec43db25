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
}  // namespace

template <class TL>
int launch_dtype(const void* in, const void* filt, float* out, const Shape& s, hipStream_t st,
                 int dtype, bool blocked, bool dry)
{
    switch (dtype) {
    case kF16: return half_try_launch<F, kRowGroup, kF16, TL>(in, filt, out, s, st, dry, blocked);
    case kBF16: return half_try_launch<F, kRowGroup, kBF16, TL>(in, filt, out, s, st, dry, blocked);
    case kI8: return half_try_launch<F, kRowGroup, kI8, TL>(in, filt, out, s, st, dry, blocked);
    default: return DCONV_UNSUPPORTED;
    }
}

template <>
int half_launch_for_F<DCONV_F>(const void* in, const void* filt, float* out, const Shape& s,
                               hipStream_t st, int dtype, bool large_tile, bool blocked, bool dry)
{
    return large_tile ? launch_dtype<HalfTileLarge>(in, filt, out, s, st, dtype, blocked, dry)
                      : launch_dtype<HalfTileSmall>(in, filt, out, s, st, dtype, blocked, dry);
}

}  // namespace dconv
