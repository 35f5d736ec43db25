// Dispatch of the special case (one input channel, paper Sec. 3): tile configurations of the
// kernel in single_kernel.h and the rules that pick one.
#include "single_kernel.h"

#include <algorithm>
#include <cmath>

namespace dconv {

namespace {

// Tile configurations compiled for every filter side, and the rule that picks one.  Measured
// on 4096 x 4096 images with 64 filters: the output stream bounds the time up to 5x5 and wide
// tiles (fewer first-of-row passes, which cannot take over a block) win; from 7x7 on the matrix
// cores bound it and, for the largest filters, taller tiles (fewer halo rows staged per output
// row) win.  Small images get small tiles so that the launch still covers the chip; with up to
// 32 filters (one filter block, rows dealt to the waves) the smallest, 128 x 4.  Configuration 5
// is that tile with passes of 64 instead of 128 pixels, for images 128 to 199 pixels wide, and
// configuration 6 with passes of 32 pixels, for images 96 to 127 wide.
// Configuration 7 is configuration 0 with a unit of one word instead of four on the way out (strip
// reads and stores): the width-matching ablation, never chosen by shape.  Configuration 8 is a
// 64 x 4 tile with passes of 32 pixels, for images so small that 128-pixel tiles would leave
// CUs without a workgroup: every wave then has half the passes in its chain of latencies.
// Configurations 9 and 10 compute with matrix-core blocks of 16 filters (v_mfma_f32_16x16x4_f32)
// instead of 32, on 512 x 4 tiles and on 128 x 4 tiles with passes of 32 pixels: for up to 16
// filters (single_blocks16_preferred below).
constexpr int kSingleConfigs = 11;

// Imbalance of a tile shape: the workgroups of the fullest CU over the mean per CU, tiles
// counted by their passes (the last tile column may hold fewer than the others).  The
// hardware deals workgroups evenly, so a launch of 534 wide tiles takes as long as one of
// 768 (a handful of tiles beyond a multiple of the CUs is not counted as a round: those
// run on CUs that have little else left).  `round_up` says how much of the last,
// partly filled round counts: all of it for the wide tiles, less for the small ones,
// which are dealt as slots fall free.  For filters bound by the matrix cores this factor
// predicts the measured time per pixel of 512-pixel tiles on 720 x 1280 .. 3000 x 3000
// images within a few per cent.
double tile_imbalance(const Shape& s, int tw, int tr, int pass, double round_up)
{
    constexpr double kCUs = 256;
    // (work items of all images count: a batch of small images fills the chip like one
    // large image)
    const int64_t fgroups = (((s.K + 31) / 32) + 3) / 4 * s.N;
    const int64_t cols = (s.Wo + tw - 1) / tw, rows = (s.Ho + tr - 1) / tr;
    const int64_t per_tile = tw / pass;
    const int64_t last = (s.Wo - tw * (cols - 1) + pass - 1) / pass;
    const double mean = (double)(rows * fgroups * (per_tile * (cols - 1) + last)) /
                        ((double)per_tile * kCUs);
    const double per_cu = std::max(1.0, (double)(cols * rows * fgroups) / kCUs);
    const double full = std::max(1.0, std::ceil(per_cu - 0.05));
    return (full > per_cu ? per_cu + round_up * (full - per_cu) : full) / mean;
}

// The configuration by shape (what launch_F runs when none is forced).
int auto_config(const Shape& s)
{
    int cfg;
    // (work items of all images count: a batch of small images fills the chip like one
    // large image)
    const int64_t fgroups = (((s.K + 31) / 32) + 3) / 4 * s.N;
    auto items = [&](int tw, int tr) {
        return (int64_t)((s.Wo + tw - 1) / tw) * ((s.Ho + tr - 1) / tr) * fgroups;
    };
    auto imbalance = [&](int tw, int tr, int pass, double round_up) {
        return tile_imbalance(s, tw, tr, pass, round_up);
    };
    // (128 x 4 with passes of 32 pixels, or 256 x 2: whichever divides the image more evenly)
    auto small_tile = [&](double bias) {
        return imbalance(128, 4, 32, 0.0) < bias * imbalance(256, 2, 128, 0.75) ? 6 : 3;
    };
    // measured with the tile search (paper_1705_10591_amd.tune) on 256^2 .. 4096^2 images
    const int64_t t128 = (int64_t)((s.Wo + 127) / 128) * ((s.Ho + 3) / 4) * s.N;
    if (single_blocks16_preferred(s)) {
        // (the small tile with short passes for 3x3 on mid-sized images, as for 32-filter
        // blocks, where 512-pixel tile columns would overhang the image by 15 % or more, and
        // where there are too few wide tiles for the CUs: 600 x 1000, 5x5: 20 -> 17 us)
        const bool overhang = (int64_t)((s.Wo + 511) / 512) * 512 * 100 >= (int64_t)s.Wo * 115;
        const bool uneven = imbalance(512, 4, 128, 1.0) > 1.5;
        cfg = ((s.F == 3 && (int64_t)s.Ho * s.Wo < 3000000) || overhang || uneven) ? 10 : 9;
    } else if (items(128, 4) <= 320 && items(64, 4) > items(128, 4)) {
        // so few 128-pixel tiles that CUs would stay without a workgroup (up to about 384 x 384
        // with one filter group): 64-pixel tiles, twice the workgroups, half the passes per wave
        // (256 x 256, 16 filters of 3 x 3: 7.1 -> 5.8 us per launch replayed from a graph)
        cfg = 8;
    } else if (s.Wo >= 96 && s.Wo < 200) {
        // rows too short for a 160-pixel pass to complete their ends across rows: passes of
        // 64 pixels (from 128 pixels of width on) or of 32, whichever computes fewer blocks
        // per row (1.2 to 1.7 times faster than the wider passes there)
        cfg = short_pass_config(s.Wo);
    } else if (s.K <= 32 && t128 < ((s.F <= 4 && s.K > 16) ? 8192 : 1536)) {
        // one filter block: the four waves of a workgroup take one row each, and on images up
        // to about 768^2 (1080p for a full block of small filters) the smallest tile is the
        // shortest chain of latencies; with passes of 64 pixels the stores of a wave begin
        // earlier still (5 to 16 % over passes of 128); with up to 16 filters or from 5x5 on,
        // passes of 32 pixels are a few per cent faster again
        cfg = (s.K <= 16 || s.F >= 5) ? 6 : 5;
    } else if (s.K <= 32 && s.F < 8 && s.Wo < 3072) {
        cfg = (s.F >= 5 && imbalance(512, 4, 128, 1.0) > 1.25) ? 6 : 0;
    } else if (s.F <= 4) {
        // (mid-sized problems: 256 x 2, or with up to 64 filters 128 x 4 with short passes)
        cfg = items(512, 4) < 1280 ? (s.K <= 64 ? 5 : 3) : 0;
    } else if (items(512, 4) < 384) {
        cfg = small_tile(1.0);
    } else if (s.F >= 8) {
        // bound by the matrix cores: the time of a tile shape is its cost per pixel (relative
        // to 512 x 4, measured on 3000 x 3000 images) times its imbalance.  The taller tile
        // pays only with several workgroups per CU and, with more than one filter block, must
        // win by a margin: its model is the least exact there.
        const double wide = imbalance(512, 4, 128, 1.0);
        const bool one_block = s.K <= 32;  // (each wave then takes whole rows of the tile)
        double tall = 1e9, small;
        if (one_block) {
            if (items(512, 8) >= 380) tall = 0.95 * imbalance(512, 8, 128, 1.0);
            small = s.F == 8 ? 1.40 : s.F >= 11 ? 1.30 : 1.25;
        } else {
            if (items(512, 8) >= 920)
                tall = 1.05 * (s.F == 8 ? 0.99 : 0.95) * imbalance(512, 8, 128, 1.0);
            small = s.F == 8 ? 1.30 : s.F >= 11 ? 1.25 : 1.20;
        }
        if (small < wide && small < tall) cfg = s.F >= 11 ? 5 : 6;
        else cfg = tall < wide ? 2 : 0;
    } else {
        // 5x5 .. 7x7: a small tile where the wide one would leave CUs idle (7x7 is bound by
        // the matrix cores and tolerates a little more)
        const int64_t it = items(512, 4);
        const bool mid = it >= 520 && it < (s.F == 7 ? 4200 : 2000);
        cfg = (mid && imbalance(512, 4, 128, 1.0) > (s.F == 7 ? 1.25 : 1.20)) ? small_tile(0.95) : 0;
    }
    return cfg;
}

template <int F>
int launch_F(const float* img, const float* filt, float* out, const Shape& s, hipStream_t st,
             int cfg)
{
    if (cfg >= kSingleConfigs) return DCONV_UNSUPPORTED;
    if (cfg < 0) cfg = auto_config(s);
    // (the small tiles keep three waves per SIMD in registers up to 8x8; beyond, the filter
    // operands of all taps would spill)
    constexpr int WS = F >= 9 ? 2 : 3;
    switch (cfg) {
    case 1: return launch_cfg<F, 1024, 4, 4, 2>(img, filt, out, s, st);
    case 2: return launch_cfg<F, 512, 8, 4, 3>(img, filt, out, s, st);
    case 3: return launch_cfg<F, 256, 2, 4, WS>(img, filt, out, s, st);
    case 4: return launch_cfg<F, 128, 4, 4, WS>(img, filt, out, s, st);
    case 5: return launch_cfg<F, 128, 4, 2, WS>(img, filt, out, s, st);
    case 6: return launch_cfg<F, 128, 4, 1, WS>(img, filt, out, s, st);
    case 7: return launch_cfg<F, 512, 4, 4, 3, 1, 1>(img, filt, out, s, st);
    case 8: return launch_cfg<F, 64, 4, 1, WS>(img, filt, out, s, st);
    case 9: return launch_cfg<F, 512, 4, 4, 3, 1, 4, 16>(img, filt, out, s, st);
    case 10: return launch_cfg<F, 128, 4, 1, 3, 1, 4, 16>(img, filt, out, s, st);
    default: return launch_cfg<F, 512, 4, 4, 3>(img, filt, out, s, st);
    }
}

}  // namespace

// Five to sixteen filters on one image (paper Sec. 5.1: few filters are the method's weak spot).
// A 32-filter matrix-core block would be half padding or more; configurations 9 and 10 compute
// with 16-filter blocks and are 5-30 % faster than the 32-filter blocks from 3x3 on (720 x 1280 ..
// 4096 x 4096 images; 4096 x 4096, 16 filters of 5x5: 0.31 -> 0.26 ms).  Where the vector-ALU
// kernel is faster still is its own rule (single_few_preferred in single_fewfilters.hip).
bool single_blocks16_preferred(const Shape& s)
{
    if (s.C != 1 || s.N != 1 || s.K > 16 || s.K < 5 || s.F < 3 || s.F > 11 || s.Wo < 256) return false;
    const int64_t px = (int64_t)s.Ho * s.Wo;
    // (from about 560 x 560 on for 5x5 and larger: 5 to 20 % there; smaller launches are all
    // latency)
    if (px < (s.F >= 5 ? 300000 : 500000) || px >= (1LL << 29)) return false;
    return !single_few_preferred(s);
}

bool single_tiled_supports(const Shape& s)
{
    // lane offsets of the write-back are 32-bit: one output plane plus a row must fit
    if (s.N < 1 || s.F < 1 || (int64_t)s.Ho * s.Wo >= (1LL << 29)) return false;
    if (s.C == 1) return s.F <= 11;
    // a few channels with small filters (single_multi_inst.hip)
    return s.C <= kSingleMultiMaxC && s.F <= kSingleMultiMaxF &&
           (int64_t)s.N * s.C * s.H * s.W < (1LL << 31);
}

// A batch of one-channel images (dconv_general with C = 1, N > 1): this kernel takes the images as
// further work items.  It is the better choice where its line-aligned output stream pays: large
// output volumes (beyond what the memory-side cache absorbs) of images wide enough for its
// 128-pixel passes, with filters small enough for the output stream to bound the time.  Measured
// against the general kernel on 128^2 .. 1024^2 images, 32 and 64 filters, 3x3 .. 11x11, 40 M to
// 320 M outputs: 1.4 to 2.2 times faster where chosen, the general kernel up to 1.9 times
// faster elsewhere (it numbers its pixels across rows and images and wastes nothing on narrow
// ones).
// With two to four channels the same holds for filters up to 3x3 (5x5 with two channels on wide
// images): beyond that the shapes are no longer bound by the output stream, and the general
// kernel makes better use of the matrix cores.  Measured on 64^2 .. 1024^2 images, 32 to 128
// filters, 40 M and 200 M outputs: 1.1 to 2.2 times faster where chosen.
bool single_batch_preferred(const Shape& s)
{
    if (!single_tiled_supports(s)) return false;
    const int64_t outputs = (int64_t)s.N * s.K * s.Ho * s.Wo;
    if (outputs < 100000000LL) return false;
    if (s.C == 1) return (s.F <= 5 && s.Wo >= 96) || (s.F <= 8 && s.Wo >= 256);
    return (s.F == 1 && s.Wo >= 96) || (s.F <= 3 && s.Wo >= 104) || (s.C == 2 && s.Wo >= 400);
}

// One image of one channel on the GENERAL-case kernel (Sec. 4 with C = 1): the special case's
// kernel spends its store time and its matrix-core time one after the other and cuts the image
// into row strips, which suits large images with small filters (the paper's sweep: output-bound,
// whole rows per strip); the general kernel overlaps the two and tiles the flattened pixels, which
// suits everything narrow, short or heavy in arithmetic.  A linear rule in the filter side and the
// logarithms of the sizes, with three flags: fewer than 32 filters (the special case's 16-filter
// blocks and small tiles are hard to beat), filter blocks left over beyond groups of four that
// do not get a launch of their own (single_split_filters below: a leftover group of one or two
// blocks runs with the tile shape chosen for the full groups, which suits it badly), and a large
// image that the special case's wide tiles divide evenly over the CUs (there it is at its best:
// 1024^2, 2048^2 and 3000^2 with 64 filters of 9x9 .. 11x11 are 6-8 % faster on it).  Fitted to
// 960 measured shapes (64^2 .. 4096^2, 9 to 512 filters of 1x1 .. 11x11; fitted on two thirds and
// checked on the third, in turn): within 2-2.5 % of the faster kernel on average, against 26 %
// with the special case's kernels alone and 17 % with the general one alone (64 x 64 with 128
// 8x8 filters: 32 -> 11 us; 384 x 384, 192 11x11: 140 -> 75 us; 768 x 768, 192 8x8: 247 -> 166 us;
// 1536 x 1280, 96 11x11: 643 -> 471 us).  The 4096 x 4096 shapes of the paper's sweep stay on the
// special case's kernel for every filter side.
bool single_general_preferred(const Shape& s)
{
    if (s.N != 1 || s.C != 1) return false;
    // (fewer than nine filters: only small images with large filters, where both kernels take the
    // time of their chains of latencies and the general one's is the shorter -- kernel times from
    // replayed graphs, 96^2 .. 2048^2, 2 to 8 filters: 224 x 320, eight 10x10 filters 15.3 -> 11.4 us;
    // from 512 x 512 on the special case's 16-filter blocks win, up to 1.8 times)
    if (s.K < 9) return s.F >= 6 && (int64_t)s.Ho * s.Wo <= 200000;
    const int blocks = (s.K + 31) / 32;
    const bool leftover = blocks > 2 && blocks % 4 != 0 && single_split_filters(s) == 0;
    const bool even = s.Wo >= 900 && tile_imbalance(s, 512, 4, 128, 1.0) <= 1.06;
    const double score = 0.63 * s.F - 0.20 * std::log2((double)s.K) - 0.70 * std::log2((double)s.Ho) -
                         1.12 * std::log2((double)s.Wo) - (s.K < 32 ? 2.62 : 0.0) +
                         (leftover ? 1.17 : 0.0) - (even ? 1.57 : 0.0) + 15.06;
    return score > 0.0;
}

int single_tile_configs() { return kSingleConfigs; }

int single_auto_config(const Shape& s) { return auto_config(s); }

// Filter blocks left over beyond groups of four, run as a launch of their own: a leftover group
// inside one launch works with the tile shape chosen for the full groups, which suits it badly
// where the matrix cores set the pace (160 filters of 9x9 on 2048 x 2048: 1532 us, against
// 788 us for 128 filters plus 217 us for 32: 1029 us in two launches; 96 filters of 11x11 on
// 3000 x 3000: 2436 -> 1929 us as 64 + 32).  Worth it from 5x5 on with one block left over
// (or three blocks in all: 64 + 32), from 7x7 with two, from 9x9 with three after full groups
// (128 + 64 + 32); with small filters the output stream sets the pace and one launch is as good
// (measured on 1024^2 .. 3000^2 images, 96 to 224 filters of 1x1 .. 11x11).  Returns the filters
// of the first launch, 0 for one launch.
int single_split_filters(const Shape& s)
{
    if (s.N != 1 || s.C != 1) return 0;
    const int blocks = (s.K + 31) / 32, full = blocks / 4, rem = blocks % 4;
    if (blocks <= 2 || rem == 0) return 0;
    const int fmin = (rem == 1 || full == 0) ? 5 : rem == 2 ? 7 : 9;
    if (s.F < fmin) return 0;
    return full > 0 ? 128 * full : 64;
}

int launch_single_tiled(const float* img, const float* filt, float* out, const Shape& s,
                        hipStream_t st, int cfg)
{
    if (!single_tiled_supports(s)) return DCONV_UNSUPPORTED;
    if (cfg < 0) {
        // (each part with the configuration of its own shape; a forced configuration runs the
        // whole layer in one launch)
        if (const int first = single_split_filters(s)) {
            Shape a = s, b = s;
            a.K = first;
            b.K = s.K - first;
            const int rc = launch_single_tiled(img, filt, out, a, st, -1);
            if (rc != DCONV_OK) return rc;
            return launch_single_tiled(img, filt + (int64_t)first * s.F * s.F,
                                       out + (int64_t)first * s.Ho * s.Wo, b, st, -1);
        }
    }
    switch (s.C) {
    case 1: break;
    case 2: return single_multi_launch_for_C<2>(img, filt, out, s, st, cfg);
    case 3: return single_multi_launch_for_C<3>(img, filt, out, s, st, cfg);
    case 4: return single_multi_launch_for_C<4>(img, filt, out, s, st, cfg);
    default: return DCONV_UNSUPPORTED;
    }
    switch (s.F) {
    case 1: return launch_F<1>(img, filt, out, s, st, cfg);
    case 2: return launch_F<2>(img, filt, out, s, st, cfg);
    case 3: return launch_F<3>(img, filt, out, s, st, cfg);
    case 4: return launch_F<4>(img, filt, out, s, st, cfg);
    case 5: return launch_F<5>(img, filt, out, s, st, cfg);
    case 6: return launch_F<6>(img, filt, out, s, st, cfg);
    case 7: return launch_F<7>(img, filt, out, s, st, cfg);
    case 8: return launch_F<8>(img, filt, out, s, st, cfg);
    case 9: return launch_F<9>(img, filt, out, s, st, cfg);
    case 10: return launch_F<10>(img, filt, out, s, st, cfg);
    case 11: return launch_F<11>(img, filt, out, s, st, cfg);
    default: return DCONV_UNSUPPORTED;
    }
}

}  // namespace dconv
