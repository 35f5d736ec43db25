// Instantiations of the general-case kernel for ONE filter side (DCONV_F, given on the
// compiler command line), so that the filter sides compile in parallel.
//
// Channel chunk per filter side: 16-36 reduction indices per chunk for small filters (short
// enough that three chunks of a tile fit in LDS with two or three workgroups per CU), one
// channel per chunk from 5x5 on.  The chunk has to divide the channel count; smaller chunks
// (down to one channel) are there for the counts it does not.
#include "general_kernel.h"

#ifndef DCONV_F
#error "compile with -DDCONV_F=<filter side>"
#endif

namespace dconv {

namespace {

constexpr int F = DCONV_F;
constexpr int kChunkBig = F == 1 ? 16 : F == 2 ? 8 : F == 3 ? 4 : F == 4 ? 2 : 1;
constexpr int kChunkSmall = F == 1 ? 4 : F == 2 ? 2 : F == 3 ? 3 : 1;   // 3: RGB inputs
// filter rows per chunk: whole filters up to 5x5, groups of rows above (see GenGeom)
constexpr int kRowGroup = F <= 5 ? F : F == 6 ? 3 : F == 9 ? 3 : F == 10 ? 5 : F <= 12 ? 4 : F <= 16 ? 3 : F <= 24 ? 2 : 1;
// image words a thread stages per chunk: eight cover a 256-pixel tile of the widest column
// strips with its halo rows; 1x1 filters (sixteen channels per chunk) take sixteen, and the
// larger filters have a second set of kernels with sixteen for shapes (tiny maps, where a
// tile spans many images) whose image block does not fit in eight
constexpr int kImaxF = F == 1 ? 16 : 8;
// (3x3 and 4x4 filters: for few channels only, see launch_tile)
constexpr bool kSecondImax = F >= 3;

// Three LDS slots when three chunks with the largest image block fit twice on a CU (or at
// least once, for chunks with enough steps); two otherwise.
template <int CSH, int MT, int IMAX>
constexpr int nbuf_for()
{
    constexpr int RG = CSH == 1 ? kRowGroup : F, NG = (F + RG - 1) / RG, RGL = F - (NG - 1) * RG;
    constexpr int T = CSH * RG * F, TP = T + (T & 1), S = (CSH * RGL * F + 1) / 2;
    constexpr long slot = 4L * ((long)(TP + 16) * (MT + 1) + IMAX * kThreads + 8);   // rows: see TROWS
    return (S >= 4 && 3 * slot <= kGenLdsLimit) ? 3 : 2;
}

template <int CSH, int IMAX>
int launch_tile_imax(const float* in, const float* filt, float* out, const Shape& s, hipStream_t st,
                     int tile_cfg, const GenSched& sched, bool dry)
{
    // Four waves side by side in every tile, each with all the filters of its pixels.
    // tile 0: 64 filters x 128 pixels, 2 x 1 blocks per wave (light on registers: three
    // workgroups per CU); tile 1: 64 filters x 256 pixels, 2 x 2 blocks per wave (four
    // matrix-core instructions per pair of operand loads); tile 2: 32 filters x 256 pixels,
    // 1 x 2 blocks per wave.  (A 128 x 128 tile of 2 x 2 waves was never the fastest of the
    // four on any of twenty layer shapes and is no longer compiled.)
    constexpr int RG = CSH == 1 ? kRowGroup : F;
    if (tile_cfg == 1)
        return gen_try_launch<F, CSH, RG, 2, 2, 1, 4, IMAX, nbuf_for<CSH, 64, IMAX>(), 2>(in, filt, out, s, st, sched, dry);
    if (tile_cfg == 2)
        return gen_try_launch<F, CSH, RG, 1, 2, 1, 4, IMAX, nbuf_for<CSH, 32, IMAX>(), 3>(in, filt, out, s, st, sched, dry);
    return gen_try_launch<F, CSH, RG, 2, 1, 1, 4, IMAX, nbuf_for<CSH, 64, IMAX>(), 3>(in, filt, out, s, st, sched, dry);
}

// The kernels with the small image block first, as long as they can keep the widest column
// strips; then the large one; then the small one with narrower strips.
template <int CSH>
int launch_tile(const float* in, const float* filt, float* out, const Shape& s, hipStream_t st,
                int tile_cfg, const GenSched& sched, bool dry)
{
    if (!kSecondImax) return launch_tile_imax<CSH, kImaxF>(in, filt, out, s, st, tile_cfg, sched, dry);
    // 3x3 and 4x4 filters with few channels.  With eight words per thread the image block of a
    // chunk holds narrow column strips only (four channels of 3x3 on 222-wide maps: four strips
    // of 56 columns under a 128-pixel tile, and a 256-pixel tile cannot even keep a 110-wide map
    // whole), and every strip row is a run of its own in the output.  With up to 160
    // multiply-adds per output element the stores bound such shapes and the wide strips of the
    // large image block pay, most of all under the 64 x 256 tile (256 images of 112 x 112, 8
    // channels, 64 filters: 0.42 -> 0.35 ms; 64 of 224 x 224: 0.49 -> 0.37 ms; 16 channels:
    // 0.63 -> 0.58 ms); with more channels its LDS costs a workgroup per CU and more than it saves.
    if (F < 5 && s.C * F * F > 160) return launch_tile_imax<CSH, kImaxF>(in, filt, out, s, st, tile_cfg, sched, dry);
    GenSched widest = sched;
    widest.widest_only = true;
    int rc = launch_tile_imax<CSH, kImaxF>(in, filt, out, s, st, tile_cfg, widest, dry);
    if (rc != DCONV_UNSUPPORTED) return rc;
    rc = launch_tile_imax<CSH, kSecondImax ? 16 : kImaxF>(in, filt, out, s, st, tile_cfg, sched, dry);
    if (rc != DCONV_UNSUPPORTED) return rc;
    return launch_tile_imax<CSH, kImaxF>(in, filt, out, s, st, tile_cfg, sched, dry);
}

}  // namespace

template <>
int gen_launch_for_F<DCONV_F>(const float* in, const float* filt, float* out, const Shape& s,
                              hipStream_t st, int tile_cfg, const GenSched& sched, bool dry)
{
    int rc = DCONV_UNSUPPORTED;
    // 2x2 filters with few channels: the stores bound the time, and an image block of eight
    // channels holds narrow column strips only (223-wide maps under the 128-pixel tile: strips
    // of 28 columns, every strip row a run of 112 bytes in the output).  The chunk that keeps
    // the widest strips goes first there (94 images of 224 x 224, 8 channels, 64 filters, 128-pixel
    // tile: 1.10 -> 0.58 ms with chunks of two channels).
    if (F == 2 && s.C * F * F <= 160 && !sched.widest_only) {
        GenSched widest = sched;
        widest.widest_only = true;
        rc = gen_launch_for_F<DCONV_F>(in, filt, out, s, st, tile_cfg, widest, dry);
        if (rc != DCONV_UNSUPPORTED) return rc;
    }
    // the largest compiled chunk that divides the channel count (one channel always does)
    if (s.C % kChunkBig == 0) {
        rc = launch_tile<kChunkBig>(in, filt, out, s, st, tile_cfg, sched, dry);
        if (rc != DCONV_UNSUPPORTED) return rc;
    }
    if (kChunkSmall != kChunkBig && s.C % kChunkSmall == 0) {
        rc = launch_tile<kChunkSmall>(in, filt, out, s, st, tile_cfg, sched, dry);
        if (rc != DCONV_UNSUPPORTED) return rc;
    }
    if (kChunkSmall != 1) rc = launch_tile<1>(in, filt, out, s, st, tile_cfg, sched, dry);
    return rc;
}

}  // namespace dconv
