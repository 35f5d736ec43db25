// General-case direct convolution for VERY FEW filters (paper Sec. 4, Algorithm 2), gfx950.
//
// With up to sixteen filters the matrix-core kernel of general_kernel.h computes a 32-filter block
// that is half padding or more, and with a few filters the layer is bound by reading its input.  This
// kernel is the paper's general-case scheme taken almost literally, on the vector ALU, with the
// thread's filter tile F_T = all K filters:
//  * the output is cut into tiles of one image (256 x 4 to 64 x 32 outputs, by map size and
//    batch); a workgroup walks the channels, staging the tile of one channel (two, where a
//    channel is little work), plus the F-1 halo columns and rows, in LDS while it computes the
//    previous one (two LDS buffers: the paper's prefetch of the next chunk, Sec. 4.2, here done
//    by loads that write LDS directly and need no registers);
//  * a lane owns four consecutive output columns of a band of rows (W_T = 4) and keeps their
//    sums for every filter in registers across the whole channel loop: RPW x K x 4 accumulators;
//  * per channel it reads the image rows of its band from LDS once (16 bytes per lane and
//    instruction) and runs filter after filter over them, every pixel of the window used F
//    times per filter row: the paper's register reuse, Sec. 4.3 (6x6 and 7x7 filters keep a
//    ring of F rows per filter instead: the band's rows do not fit the registers);
//  * the filters are wave-uniform.  From two filters on, the F x F weights of every (filter,
//    channel) pair of a trip are staged in LDS like the tile (one 64-word load each) and a
//    multiply-add takes its weight from a register that all lanes read from the same LDS address:
//    the counterpart of the paper's constant-cache broadcast.  With one filter they arrive with
//    one vector load (lane t takes weight t) and move to scalar registers tap by tap; that is
//    5-15 % faster for one filter and 7-32 % slower for three to eight, where the moves take a
//    quarter of the vector instructions (scalar loads of the weights: 10-40 % slower, their
//    latency is in the way of every filter);
//  * after the last channel a lane stores its four outputs per row and filter as 16 bytes.
// Every input pixel is read from HBM once per tile (halo aside) whatever the filter count, and
// the arithmetic is K x F x F multiply-adds per pixel and channel with no padding.
#pragma once
#include "common.h"
#include "../../include/dconv.h"

namespace dconv {

struct GenFewParams {
    const float* in;
    const float* filt;
    float* out;
    int N, C, H, W, K, Ho, Wo;
    int tiles_x, tiles_y;
    int tiles;       // all tiles: N * tiles_y * tiles_x
    int per_xcd;     // tiles per XCD (the grid has 8 * per_xcd workgroups)
};

// KT:  filters a lane sums at once (K rounded up to 1, 2, 3, 4, 6, 8, 12 or 16; filters beyond K
//      have zero weights and are not stored).
// LPR: lanes side by side in a row of the tile (64, 32 or 16: tiles 256, 128 or 64 columns wide);
//      a wave holds 64 / LPR bands of rows, one below the other.
// RPW: output rows per band.  A tile is 4 * LPR columns x 4 * (64 / LPR) * RPW rows.
template <int F, int KT, int RPW, int LPR, int CC>
__global__ void __launch_bounds__(kThreads)
general_few_kernel(GenFewParams p)
{
    constexpr int BANDS = kWave / LPR;             // bands per wave
    constexpr int TW = 4 * LPR, TR = 4 * BANDS * RPW;
    constexpr int FF = F * F;
    constexpr int WIN = 4 + F - 1;                 // window columns of a lane
    constexpr int NV = (WIN + 3) / 4;              // 16-byte LDS reads per window row
    constexpr int SEGS = (TW + 4 * NV - 4 + kWave - 1) / kWave;   // 64-word pieces of a row
    constexpr int LS = SEGS * kWave;               // LDS row stride: the last lane's reads stay in the row
    constexpr int ROWS = TR + F - 1;
    constexpr bool kWholeWindow = (RPW + F - 1) * 4 * NV <= 64;   // registers for a band's image rows
    static_assert(LS % 4 == 0, "16-byte aligned rows");
    static_assert(2 * (CC * ROWS * LS + (KT >= 2 ? CC * KT * kWave : 4)) * 4 <= 64 * 1024,
                  "two sets of tiles and weights fit static LDS");
    static_assert(FF <= kWave, "one lane per weight");

    __shared__ __attribute__((aligned(16))) float sh[2][CC * ROWS * LS];
    // From two filters on the weights go through LDS too (64 words per filter and channel) and a
    // multiply-add takes its weight from a register that every lane read from the same LDS
    // address; with one filter they go through scalar registers (moved there lane by lane), which
    // is 5-15 % faster for one filter and 7-32 % slower for three to eight.
    constexpr bool kLdsWeights = KT >= 2;
    __shared__ __attribute__((aligned(16))) float wsh[2][kLdsWeights ? CC * KT * kWave : 4];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Workgroups go to the eight XCDs round-robin; each XCD gets a contiguous run of tiles.
    const int tile = (int)(blockIdx.x % 8) * p.per_xcd + (int)(blockIdx.x / 8);
    if (tile >= p.tiles) return;                   // uniform: before any barrier
    const int per_image = p.tiles_x * p.tiles_y;
    const int n = tile / per_image, t2 = tile - n * per_image;
    const int ty = t2 / p.tiles_x, tx = t2 - ty * p.tiles_x;
    const int x0 = tx * TW, y0 = ty * TR;

    // ---- staging: the waves take the rows of a channel's tile in turn, 64 words per
    // instruction, straight into LDS.  A row's descriptor starts at the row's first pixel in
    // the tile and ends with the input: lanes beyond that write zeros; lanes beyond the row's
    // end (or rows below the image) but inside the input bring pixels of the next row, channel
    // or image, which only outputs beyond the row's or the map's end would use, and those are
    // not stored.
    typedef __attribute__((address_space(3))) void* lds_ptr;
    constexpr int kRsrcFlags = 0x00020000;         // raw buffer of 32-bit words
    const int64_t in_words = (int64_t)p.N * p.C * p.H * p.W;
    int voff[SEGS];
#pragma unroll
    for (int j = 0; j < SEGS; ++j) voff[j] = 4 * (lane + kWave * j);
    auto stage = [&](int c, float* buf) __attribute__((always_inline)) {
        const int64_t chan = ((int64_t)n * p.C + c) * p.H;
        for (int r = wave; r < ROWS; r += 4) {     // (uniform)
            const int64_t first = (chan + y0 + r) * p.W + x0;
            const int64_t left = (in_words - first) * 4;
            const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
                (void*)(p.in + first), 0, (int)(left < 0 ? 0 : left > 0x7FFFFFFF ? 0x7FFFFFFF : left), kRsrcFlags);
#pragma unroll
            for (int j = 0; j < SEGS; ++j)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_ptr)(buf + r * LS + kWave * j), 4, voff[j], 0, 0, 0);
        }
    };
    // the weights of filters 0..KT-1 for channel c: lane t holds weight t of each
    const int64_t CFF = (int64_t)p.C * FF;
    auto load_weights = [&](int c, float (&w)[KT]) __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < KT; ++k)
            w[k] = (lane < FF && k < p.K && c < p.C) ? p.filt[k * CFF + (int64_t)c * FF + lane] : 0.f;
    };

    // the weights of (filter k, channel c) straight into LDS, 64 words per instruction (the F x F
    // weights and whatever follows them; a filter or channel beyond the last reads as zeros)
    const int64_t filt_words = (int64_t)p.K * CFF;
    auto stage_weights = [&](int c, int cc, float* wbuf) __attribute__((always_inline)) {
        for (int k = wave; k < KT; k += 4) {       // (uniform)
            const int64_t first = k * CFF + (int64_t)c * FF;
            const int64_t left = (k < p.K && c < p.C) ? (filt_words - first) * 4 : 0;
            const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
                (void*)(p.filt + (left > 0 ? first : 0)), 0, (int)(left > 0x7FFFFFFF ? 0x7FFFFFFF : left), kRsrcFlags);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_ptr)(wbuf + (cc * KT + k) * kWave), 4, voff[0], 0, 0, 0);
        }
    };
    const int lx = lane % LPR;
    const int r0 = (wave * BANDS + lane / LPR) * RPW;   // first output row of this lane's band
    const int xo = x0 + 4 * lx;                    // first output column of this lane

    float acc[RPW][KT][4];
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr)
#pragma unroll
        for (int k = 0; k < KT; ++k)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[rr][k][e] = 0.f;

    // CC channels per trip: one barrier and one round of LDS latencies for all of them
    float wcur[CC][KT], wnext[CC][KT];
#pragma unroll
    for (int cc = 0; cc < CC; ++cc) {
        if (cc < p.C) stage(cc, sh[0] + cc * (ROWS * LS));
        if constexpr (kLdsWeights) stage_weights(cc, cc, wsh[0]);
        else load_weights(cc, wcur[cc]);
    }
    for (int c0 = 0; c0 < p.C; c0 += CC) {         // uniform loop
        // this wave's pieces of these channels are in LDS (and the weights in registers); after
        // the barrier so are everyone's, and everyone has left the other buffer
        __builtin_amdgcn_s_waitcnt(0x0F70);        // vmcnt(0)
        __syncthreads();
        const int cur = (c0 / CC) & 1;
#pragma unroll
        for (int cc = 0; cc < CC; ++cc) {
            if (c0 + CC + cc < p.C) stage(c0 + CC + cc, sh[cur ^ 1] + cc * (ROWS * LS));
            if constexpr (kLdsWeights) stage_weights(c0 + CC + cc, cc, wsh[cur ^ 1]);
            else load_weights(c0 + CC + cc, wnext[cc]);
        }
#pragma unroll
        for (int cc = 0; cc < CC; ++cc) {
            // (a channel beyond the last has zero weights, but its place in LDS holds pixels of
            // the next image: not multiplied at all, so that a NaN there stays where it belongs)
            if (c0 + cc >= p.C) break;             // uniform
            const float* wrow = sh[cur] + cc * (ROWS * LS) + r0 * LS + 4 * lx;
            auto load_row = [&](int rr, float (&w)[4 * NV]) __attribute__((always_inline)) {
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    const v4f q = *reinterpret_cast<const v4f*>(wrow + rr * LS + 4 * v);
#pragma unroll
                    for (int e = 0; e < 4; ++e) w[4 * v + e] = q[e];
                }
            };
            if constexpr (kWholeWindow) {
                // all image rows of the band at once, then filter after filter over them: one
                // LDS read per pixel and channel whatever the filter count
                float win[RPW + F - 1][4 * NV];
#pragma unroll
                for (int i = 0; i < RPW + F - 1; ++i) load_row(i, win[i]);
#pragma unroll
                for (int k = 0; k < KT; ++k) {
                    float wgt[FF];
#pragma unroll
                    for (int t = 0; t < FF; ++t) {
                        if constexpr (kLdsWeights) wgt[t] = wsh[cur][(cc * KT + k) * kWave + t];
                        else wgt[t] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wcur[cc][k]), t));
                    }
#pragma unroll
                    for (int rr = 0; rr < RPW; ++rr)
#pragma unroll
                        for (int i = 0; i < F; ++i)
#pragma unroll
                            for (int j = 0; j < F; ++j)
#pragma unroll
                                for (int e = 0; e < 4; ++e)
                                    acc[rr][k][e] = __builtin_fmaf(win[rr + i][j + e], wgt[i * F + j], acc[rr][k][e]);
                }
            } else {
                // (6x6 and 7x7: the band's rows do not fit the registers; a ring of F rows per
                // filter, whose 36 or 49 multiply-adds per pixel dwarf the reads anyway)
#pragma unroll
                for (int k = 0; k < KT; ++k) {
                    float wgt[FF];
#pragma unroll
                    for (int t = 0; t < FF; ++t) {
                        if constexpr (kLdsWeights) wgt[t] = wsh[cur][(cc * KT + k) * kWave + t];
                        else wgt[t] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wcur[cc][k]), t));
                    }
                    // window row of band row rr lives in win[rr % F]
                    float win[F][4 * NV];
#pragma unroll
                    for (int i = 0; i < F - 1; ++i) load_row(i, win[i]);
#pragma unroll
                    for (int rr = 0; rr < RPW; ++rr) {
                        load_row(rr + F - 1, win[(rr + F - 1) % F]);
#pragma unroll
                        for (int i = 0; i < F; ++i)
#pragma unroll
                            for (int j = 0; j < F; ++j)
#pragma unroll
                                for (int e = 0; e < 4; ++e)
                                    acc[rr][k][e] = __builtin_fmaf(win[(rr + i) % F][j + e], wgt[i * F + j], acc[rr][k][e]);
                    }
                }
            }
        }
#pragma unroll
        for (int cc = 0; cc < CC; ++cc)
#pragma unroll
            for (int k = 0; k < KT; ++k) wcur[cc][k] = wnext[cc][k];
    }

    const int64_t plane = (int64_t)p.Ho * p.Wo;
    typedef float v4f_a4 __attribute__((ext_vector_type(4), aligned(4)));
#pragma unroll
    for (int k = 0; k < KT; ++k) {
        // (a uniform branch per filter, not a loop exit: with an early exit the compiler leaves
        // loops of more than eight trips rolled, and the sums would live in scratch memory)
        if (k < p.K) {
            float* plane_k = p.out + ((int64_t)n * p.K + k) * plane;
#pragma unroll
            for (int rr = 0; rr < RPW; ++rr) {
                const int y = y0 + r0 + rr;
                if (y < p.Ho) {
                    float* dst = plane_k + (int64_t)y * p.Wo + xo;
                    // 16 bytes at once where they fit (rows start at any 4-byte offset: the store
                    // is declared 4-byte aligned), single words at the row end
                    if (xo + 3 < p.Wo) {
                        *reinterpret_cast<v4f_a4*>(dst) = (v4f_a4){acc[rr][k][0], acc[rr][k][1], acc[rr][k][2], acc[rr][k][3]};
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (xo + e < p.Wo) dst[e] = acc[rr][k][e];
                    }
                }
            }
        }
    }
}

// Tile shape by map and batch: the width that wastes the fewest lanes on columns beyond the
// map (the widest such: fewer halo columns), then the tallest bands that still give every CU
// three workgroups (shorter bands re-read more halo rows).
struct GfTile { int lpr, rpw; };
inline int64_t gf_tiles(const Shape& s, int lpr, int rpw)
{
    const int tw = 4 * lpr, tr = 4 * (kWave / lpr) * rpw;
    return (int64_t)s.N * ((s.Wo + tw - 1) / tw) * ((s.Ho + tr - 1) / tr);
}
inline GfTile gf_tile_for(const Shape& s)
{
    int lpr = 64;
    int64_t best = (int64_t)((s.Wo + 255) / 256) * 256;
    for (int l : {32, 16}) {
        const int64_t padded = (int64_t)((s.Wo + 4 * l - 1) / (4 * l)) * (4 * l);
        if (padded * 10 < best * 9) { best = padded; lpr = l; }
    }
    // (nine to sixteen filters: two rows per band only for 1x1 filters, 10-20 % faster there;
    // with larger filters the registers of two rows cost more waves per SIMD than the rows save:
    // measured 15-30 % slower from 2x2 on)
    const int rmax = s.K > 8 ? (s.F == 1 ? 2 : 1) : s.K > 4 ? 2 : lpr == 64 ? 4 : 2;
    int rpw = rmax;
    while (rpw > 1 && gf_tiles(s, lpr, rpw) < 768) rpw /= 2;
    return {lpr, rpw};
}

template <int F, int KT, int RPW, int LPR>
int launch_gf(const float* in, const float* filt, float* out, const Shape& s, hipStream_t st)
{
    constexpr int TW = 4 * LPR, TR = 4 * (kWave / LPR) * RPW;
    GenFewParams p{in, filt, out, s.N, s.C, s.H, s.W, s.K, s.Ho, s.Wo,
                   (s.Wo + TW - 1) / TW, (s.Ho + TR - 1) / TR, 0, 0};
    const int64_t tiles = (int64_t)s.N * p.tiles_x * p.tiles_y;
    if (tiles > 2000000000LL) return DCONV_UNSUPPORTED;
    p.tiles = (int)tiles;
    p.per_xcd = (int)((tiles + 7) / 8);
    begin_launch();
    // (one row per band is so little work per channel that two channels share a barrier:
    // 8 x 64 x 224 x 224, 1x1 filters: 29 -> 23 us; not with twelve or sixteen filters, which
    // are work enough and whose weights take the LDS a second channel would need)
    constexpr int CC = (RPW == 1 && KT <= 8) ? 2 : 1;
    hipLaunchKernelGGL((general_few_kernel<F, KT, RPW, LPR, CC>), dim3((unsigned)(p.per_xcd * 8)), dim3(kThreads), 0, st, p);
    return launch_status();
}

template <int F, int KT>
int launch_gf_K(const float* in, const float* filt, float* out, const Shape& s, hipStream_t st)
{
    const GfTile t = gf_tile_for(s);
    // (six and eight filters: at most two rows per band, so that the sums and a 7x7 window fit
    // the registers of two waves per SIMD; twelve and sixteen: one row, two for 1x1 filters)
    if constexpr (KT > 8) {
        constexpr int R2 = F == 1 ? 2 : 1;
        if (t.lpr == 64) return t.rpw >= 2 ? launch_gf<F, KT, R2, 64>(in, filt, out, s, st) : launch_gf<F, KT, 1, 64>(in, filt, out, s, st);
        if (t.lpr == 32) return t.rpw >= 2 ? launch_gf<F, KT, R2, 32>(in, filt, out, s, st) : launch_gf<F, KT, 1, 32>(in, filt, out, s, st);
        return t.rpw >= 2 ? launch_gf<F, KT, R2, 16>(in, filt, out, s, st) : launch_gf<F, KT, 1, 16>(in, filt, out, s, st);
    } else {
        if (t.lpr == 64) {
            if (KT <= 4 && t.rpw == 4) return launch_gf<F, KT, (KT <= 4 ? 4 : 2), 64>(in, filt, out, s, st);
            if (t.rpw >= 2) return launch_gf<F, KT, 2, 64>(in, filt, out, s, st);
            return launch_gf<F, KT, 1, 64>(in, filt, out, s, st);
        }
        if (t.lpr == 32) {
            if (t.rpw >= 2) return launch_gf<F, KT, 2, 32>(in, filt, out, s, st);
            return launch_gf<F, KT, 1, 32>(in, filt, out, s, st);
        }
        if (t.rpw >= 2) return launch_gf<F, KT, 2, 16>(in, filt, out, s, st);
        return launch_gf<F, KT, 1, 16>(in, filt, out, s, st);
    }
}

// Implemented once per filter side, each in its own translation unit.
template <int F>
int gf_launch_for_F(const float* in, const float* filt, float* out, const Shape& s, hipStream_t st);

// the tile count of the shape's own tile choice (for the dispatcher's rule)
inline int64_t gf_auto_tiles(const Shape& s)
{
    const GfTile t = gf_tile_for(s);
    return gf_tiles(s, t.lpr, t.rpw);
}

}  // namespace dconv
