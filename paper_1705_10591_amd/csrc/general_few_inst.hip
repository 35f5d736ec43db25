// Instantiations of the few-filters kernel of the general case for ONE filter side (DCONV_F,
// given on the compiler command line), so that the filter sides compile in parallel.
#include "general_few_kernel.h"

#ifndef DCONV_F
#error "compile with -DDCONV_F=<filter side>"
#endif

namespace dconv {

template <>
int gf_launch_for_F<DCONV_F>(const float* in, const float* filt, float* out, const Shape& s, hipStream_t st)
{
    constexpr int F = DCONV_F;
    switch (s.K) {
    case 1: return launch_gf_K<F, 1>(in, filt, out, s, st);
    case 2: return launch_gf_K<F, 2>(in, filt, out, s, st);
    case 3: return launch_gf_K<F, 3>(in, filt, out, s, st);
    case 4: return launch_gf_K<F, 4>(in, filt, out, s, st);
    case 5: case 6: return launch_gf_K<F, 6>(in, filt, out, s, st);
    case 7: case 8: return launch_gf_K<F, 8>(in, filt, out, s, st);
    case 9: case 10: case 11: case 12: return launch_gf_K<F, 12>(in, filt, out, s, st);
    case 13: case 14: case 15: case 16: return launch_gf_K<F, 16>(in, filt, out, s, st);
    default: return DCONV_UNSUPPORTED;
    }
}

}  // namespace dconv
