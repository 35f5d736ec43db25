// C ABI of libdconv.so: argument validation and kernel dispatch.
#include "common.h"
#include "../../include/dconv.h"

using dconv::Shape;

namespace {

constexpr int64_t kMaxElems = 2147483647LL;

int validate(const void* in, const void* filt, const void* out,
             int N, int C, int H, int W, int K, int F, Shape* s)
{
    if (!in || !filt || !out) return DCONV_NULL_POINTER;
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || F <= 0) return DCONV_BAD_SHAPE;
    if (F > H || F > W) return DCONV_BAD_SHAPE;
    const int Ho = H - F + 1, Wo = W - F + 1;
    // sizes are checked in floating point first so the int64 products below cannot overflow
    const double in_elems = (double)N * C * H * W;
    const double filt_elems = (double)K * C * F * F;
    const double img_out = (double)K * Ho * Wo;
    if (in_elems > (double)kMaxElems || filt_elems > (double)kMaxElems ||
        img_out > (double)kMaxElems || (double)N * img_out > 9.0e18)
        return DCONV_BAD_SHAPE;
    *s = Shape{N, C, H, W, K, F, Ho, Wo};
    return DCONV_OK;
}

int dispatch(bool single, const float* in, const float* filt, float* out,
             const Shape& s, int variant, void* stream, bool static_ws = false)
{
    hipStream_t st = (hipStream_t)stream;
    const bool tiled_ok = single ? dconv::single_tiled_supports(s)
                                 : dconv::general_tiled_supports(s);
    auto tiled = [&](int cfg) {
        return single ? dconv::launch_single_tiled(in, filt, out, s, st, cfg)
                      : dconv::launch_general_tiled(in, filt, out, s, st, cfg, static_ws);
    };
    switch (variant) {
    case DCONV_VARIANT_AUTO:
        if (single && dconv::single_few_preferred(s)) return dconv::launch_single_few(in, filt, out, s, st);
        // (filters beyond the special case's 11 x 11: the general kernel takes one channel too;
        // so do narrow or short images and large filters, where it is the faster one)
        if (single && (!tiled_ok || dconv::single_general_preferred(s)) && dconv::general_tiled_supports(s))
            return dconv::launch_general_tiled(in, filt, out, s, st, -1, static_ws);
        return tiled_ok ? tiled(-1) : dconv::launch_simple(in, filt, out, s, st);
    case DCONV_VARIANT_FEW_FILTERS:
        if (!single) return dconv::launch_general_few(in, filt, out, s, st);   // (refuses what it cannot run)
        if (!dconv::single_few_supports(s)) return DCONV_UNSUPPORTED;
        return dconv::launch_single_few(in, filt, out, s, st);
    case DCONV_VARIANT_SIMPLE:
        return dconv::launch_simple(in, filt, out, s, st);
    case DCONV_VARIANT_TILED:
        return tiled_ok ? tiled(-1) : DCONV_UNSUPPORTED;
    default:
        break;
    }
    const int ncfg = single ? dconv::single_tile_configs() : dconv::general_tile_configs();
    if (variant >= DCONV_VARIANT_TILED_CFG0 && variant < DCONV_VARIANT_TILED_CFG0 + ncfg)
        return tiled_ok ? tiled(variant - DCONV_VARIANT_TILED_CFG0) : DCONV_UNSUPPORTED;
    return DCONV_UNSUPPORTED;
}

int general_entry(const float* in, int N, int C, int H, int W, const float* filt, int K, int F,
                  float* out, int variant, void* stream, bool static_ws)
{
    Shape s;
    const int rc = validate(in, filt, out, N, C, H, W, K, F, &s);
    if (rc != DCONV_OK) return rc;
    // one channel is the special case, layouts included (a batch of images: its kernel takes
    // the images as further work items)
    if (variant == DCONV_VARIANT_SPECIAL_CASE ||
        (variant >= DCONV_VARIANT_SPECIAL_CASE_CFG0 &&
         variant < DCONV_VARIANT_SPECIAL_CASE_CFG0 + dconv::single_tile_configs())) {
        if (!dconv::single_tiled_supports(s)) return DCONV_UNSUPPORTED;
        return dispatch(true, in, filt, out, s,
                        variant == DCONV_VARIANT_SPECIAL_CASE
                            ? DCONV_VARIANT_TILED
                            : variant - DCONV_VARIANT_SPECIAL_CASE_CFG0 + DCONV_VARIANT_TILED_CFG0,
                        stream);
    }
    // (the same kernel takes two to four channels with small filters: such shapes are bound by
    // the output stream like the one-channel case)
    // (with up to sixteen filters the vector-ALU kernel of the general case goes first: up to
    // eight it is 2 to 10 times faster than a mostly padded matrix-core block of either kernel,
    // from nine on up to 2.8 times on layers of few channels)
    if (variant == DCONV_VARIANT_AUTO && !(N == 1 && C == 1) && dconv::general_few_preferred(s))
        return dconv::launch_general_few(in, filt, out, s, (hipStream_t)stream);
    if (variant == DCONV_VARIANT_AUTO &&
        ((N == 1 && C == 1) || dconv::single_batch_preferred(s) ||
         (dconv::single_tiled_supports(s) && !dconv::general_tiled_supports(s))))
        return dispatch(true, in, filt, out, s, variant, stream);
    return dispatch(false, in, filt, out, s, variant, stream, static_ws);
}

}  // namespace

extern "C" {

int dconv_single_channel_v(const float* img, int H, int W, const float* filt, int K, int F,
                           float* out, int variant, void* stream)
{
    Shape s;
    const int rc = validate(img, filt, out, 1, 1, H, W, K, F, &s);
    if (rc != DCONV_OK) return rc;
    return dispatch(true, img, filt, out, s, variant, stream);
}

int dconv_general_v(const float* in, int N, int C, int H, int W, const float* filt, int K, int F,
                    float* out, int variant, void* stream)
{
    return general_entry(in, N, C, H, W, filt, K, F, out, variant, stream, false);
}

int dconv_general_noalloc(const float* in, int N, int C, int H, int W, const float* filt, int K, int F,
                          float* out, int variant, void* stream)
{
    return general_entry(in, N, C, H, W, filt, K, F, out, variant, stream, true);
}

int dconv_single_channel(const float* img, int H, int W, const float* filt, int K, int F,
                         float* out, void* stream)
{
    return dconv_single_channel_v(img, H, W, filt, K, F, out, DCONV_VARIANT_AUTO, stream);
}

int dconv_general(const float* in, int N, int C, int H, int W, const float* filt, int K, int F,
                  float* out, void* stream)
{
    return dconv_general_v(in, N, C, H, W, filt, K, F, out, DCONV_VARIANT_AUTO, stream);
}

int dconv_general_half_v(const void* in, int N, int C, int H, int W, const void* filt, int K, int F,
                         float* out, int dtype, int variant, void* stream)
{
    Shape s;
    const int rc = validate(in, filt, out, N, C, H, W, K, F, &s);
    if (rc != DCONV_OK) return rc;
    if (dtype != DCONV_DTYPE_F16 && dtype != DCONV_DTYPE_BF16) return DCONV_UNSUPPORTED;
    if ((((uintptr_t)in) & 1) != 0 || (((uintptr_t)filt) & 1) != 0) return DCONV_BAD_SHAPE;
    return dconv::launch_general_half(in, filt, out, s, (hipStream_t)stream, dtype,
                                      DCONV_LAYOUT_CHANNELS_LAST, variant);
}

int dconv_general_lowp(const void* in, int N, int C, int H, int W, const void* filt, int K, int F,
                       void* out, int dtype, int layout, int variant, void* stream)
{
    Shape s;
    const int rc = validate(in, filt, out, N, C, H, W, K, F, &s);
    if (rc != DCONV_OK) return rc;
    if (dtype != DCONV_DTYPE_I8 && ((((uintptr_t)in) & 1) != 0 || (((uintptr_t)filt) & 1) != 0))
        return DCONV_BAD_SHAPE;
    return dconv::launch_general_half(in, filt, (float*)out, s, (hipStream_t)stream, dtype, layout, variant);
}

int dconv_general_i8_v(const void* in, int N, int C, int H, int W, const void* filt, int K, int F,
                       int* out, int variant, void* stream)
{
    Shape s;
    const int rc = validate(in, filt, out, N, C, H, W, K, F, &s);
    if (rc != DCONV_OK) return rc;
    return dconv::launch_general_half(in, filt, (float*)out, s, (hipStream_t)stream, DCONV_DTYPE_I8,
                                      DCONV_LAYOUT_CHANNELS_LAST, variant);
}

int dconv_general_i8(const void* in, int N, int C, int H, int W, const void* filt, int K, int F,
                     int* out, void* stream)
{
    return dconv_general_i8_v(in, N, C, H, W, filt, K, F, out, DCONV_VARIANT_AUTO, stream);
}

int dconv_general_f16(const void* in, int N, int C, int H, int W, const void* filt, int K, int F,
                      float* out, void* stream)
{
    return dconv_general_half_v(in, N, C, H, W, filt, K, F, out, DCONV_DTYPE_F16, DCONV_VARIANT_AUTO, stream);
}

int dconv_general_bf16(const void* in, int N, int C, int H, int W, const void* filt, int K, int F,
                       float* out, void* stream)
{
    return dconv_general_half_v(in, N, C, H, W, filt, K, F, out, DCONV_DTYPE_BF16, DCONV_VARIANT_AUTO, stream);
}

const char* dconv_status_string(int status)
{
    switch (status) {
    case DCONV_OK: return "ok";
    case DCONV_NULL_POINTER: return "null pointer argument";
    case DCONV_BAD_SHAPE: return "bad shape";
    case DCONV_UNSUPPORTED: return "variant does not support this shape";
    case DCONV_LAUNCH_FAILED: return "kernel launch failed";
    case DCONV_SCRATCH_EXCEEDED: return "shape needs more scratch memory than the static device array holds";
    default: return "unknown status";
    }
}

int dconv_tile_config_count(int single_channel)
{
    return single_channel ? dconv::single_tile_configs() : dconv::general_tile_configs();
}

int dconv_tile_choice(int single_channel, int N, int C, int H, int W, int K, int F)
{
    Shape s;
    const int dummy = 0;       // (validate only tests its pointers against null)
    if (validate(&dummy, &dummy, &dummy, N, C, H, W, K, F, &s) != DCONV_OK ||
        (single_channel && (N != 1 || C != 1)))
        return DCONV_CHOICE_INVALID;
    // the routing of general_entry and dispatch for DCONV_VARIANT_AUTO
    if (!single_channel && !(N == 1 && C == 1) && dconv::general_few_preferred(s)) return DCONV_CHOICE_FEW_FILTERS;
    const bool special = single_channel || (N == 1 && C == 1) || dconv::single_batch_preferred(s) ||
                         (dconv::single_tiled_supports(s) && !dconv::general_tiled_supports(s));
    if (special) {
        if (dconv::single_few_preferred(s)) return DCONV_CHOICE_FEW_FILTERS;
        if (!dconv::general_tiled_supports(s) && !dconv::single_tiled_supports(s)) return DCONV_CHOICE_SIMPLE;
        // (one channel on the general-case kernel: dconv_general names the tile shape it runs with)
        if (dconv::general_tiled_supports(s) &&
            (!dconv::single_tiled_supports(s) || dconv::single_general_preferred(s)))
            return single_channel ? DCONV_CHOICE_GENERAL_CASE : dconv::general_auto_shape(s);
        if (!single_channel) return DCONV_CHOICE_SPECIAL_CASE;
        return dconv::single_auto_config(s);
    }
    if (!dconv::general_tiled_supports(s)) return DCONV_CHOICE_SIMPLE;
    return dconv::general_auto_shape(s);
}

int dconv_release_workspace(void)
{
    dconv::release_general_workspaces();
    return DCONV_OK;
}

int dconv_version(void) { return 1014; }

}  // extern "C"
