// Instantiations of the 16-bit general-case kernel for ONE filter side (DCONV_F, given on the
// compiler command line): fp16, bf16 and int8.
#include "half_kernel.h"

#ifndef DCONV_F
#error "compile with -DDCONV_F=<filter side>"
#endif

namespace dconv {

namespace {
constexpr int F = DCONV_F;
// filter rows per chunk: 7 to 12 matrix-core steps per chunk where the filter allows it (a
// step is one tap of sixteen channels); the filter block of a chunk is 2 KiB per step
constexpr int kRowGroup = F <= 3 ? F : F <= 6 ? 2 : 1;
}  // namespace

template <>
int half_launch_for_F<DCONV_F>(const void* in, const void* filt, float* out, const Shape& s,
                               hipStream_t st, int dtype, bool dry)
{
    switch (dtype) {
    case kF16: return half_try_launch<F, kRowGroup, kF16>(in, filt, out, s, st, dry);
    case kBF16: return half_try_launch<F, kRowGroup, kBF16>(in, filt, out, s, st, dry);
    case kI8: return half_try_launch<F, kRowGroup, kI8>(in, filt, out, s, st, dry);
    default: return DCONV_UNSUPPORTED;
    }
}

}  // namespace dconv
