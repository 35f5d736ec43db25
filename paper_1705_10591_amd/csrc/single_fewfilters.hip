// Special-case direct convolution for VERY FEW filters (paper Sec. 3, Algorithm 1), gfx950.
//
// With a handful of filters the single-channel case is pure communication: the
// matrix-core kernel of single.hip would fill a 32-filter block with one or two
// filters.  This kernel is the paper's scheme taken almost literally, on the
// vector ALU:
//  * the image is cut into tiles, a workgroup stages its tile plus the F-1 halo
//    columns and rows right and below in LDS, so every pixel is read from HBM
//    once (halo aside);
//  * a lane owns four consecutive output columns and sweeps a band of rows
//    downwards with a window of F image rows in registers: every step reads ONE
//    new image row segment from LDS (16 bytes per lane and instruction) and
//    reuses the other F-1 rows, which is the paper's sliding register window;
//  * the filters are wave-uniform: the weights of one filter at a time sit in
//    scalar registers (the counterpart of the constant-cache broadcast), so each
//    multiply-add takes its weight from a scalar operand and its pixel from the
//    window;
//  * the four outputs of a lane are stored as 16 bytes, a wave writes 1 KiB of
//    consecutive pixels per filter and row.
// What differs: no rolling one-row prefetch from global memory (several
// workgroups share a CU and overlap each other's loads); the window does not
// shift, the row loop is unrolled so that the ring index is a compile-time
// constant; the filters are the outer loop, so a filter's weights are fetched
// once per wave and tile (one load, issued a filter ahead).  The tile goes from
// global memory straight into LDS (buffer loads with the LDS bit, 64 words per
// wave instruction, a row's five instructions with a scalar base and no
// vector-ALU work): all of a wave's loads are in flight at once, where a loop of
// load, wait, LDS store per word paid one memory latency per trip and, with one
// filter, took longer than the arithmetic.
#include <type_traits>
#include "common.h"
#include "../../include/dconv.h"

namespace dconv {

namespace {

struct FewParams {
    const float* img;
    const float* filt;
    float* out;
    int H, W, K, Ho, Wo;
    int tiles_x;
    int tiles;       // all tiles
    int per_xcd;     // tiles per XCD (the grid has 8 * per_xcd workgroups)
};

constexpr int kFewTW = 256;          // tile width: 64 lanes x 4 columns
// Output rows per wave (RPW; a tile has four bands of that many rows, one per wave).  Short bands
// mean more halo rows per output row but smaller tiles, so more workgroups share a CU and more
// loads are in flight: measured on 4096 x 4096 images, four rows win for filters up to 3x3
// (12-16 % over eight) and for one or two filters up to 5x5, eight rows from there on.
constexpr int few_rpw(int F, int K) { return (F <= 3 || (F <= 5 && K <= 2)) ? 4 : 8; }


template <int F, int RPW>
__global__ void __launch_bounds__(kThreads)
single_few_kernel(FewParams p)
{
    constexpr int kFewRPW = RPW, kFewTR = 4 * RPW;
    constexpr int FF = F * F;
    constexpr int WIN = 4 + F - 1;                 // window columns of a lane
    constexpr int NV = (WIN + 3) / 4;              // 16-byte LDS reads per window row
    constexpr int SEGS = (kFewTW + 4 * NV - 4 + kWave - 1) / kWave;   // 64-word pieces of a row
    constexpr int LS = SEGS * kWave;               // LDS row stride: the last lane's reads stay in the row
    constexpr int ROWS = kFewTR + F - 1;
    static_assert(LS % 4 == 0, "16-byte aligned rows");
    static_assert(ROWS * LS * 4 <= 64 * 1024, "the tile fits a static LDS array");

    __shared__ __attribute__((aligned(16))) float sh[ROWS * LS];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Workgroups go to the eight XCDs round-robin; each XCD gets a contiguous run of tiles, so
    // that the 128-byte output lines two neighbouring tiles share meet in one L2 and leave it whole.
    const int tile = (int)(blockIdx.x % 8) * p.per_xcd + (int)(blockIdx.x / 8);
    if (tile >= p.tiles) return;                   // uniform: before any barrier
    const int ty = tile / p.tiles_x, tx = tile - ty * p.tiles_x;
    const int x0 = tx * kFewTW, y0 = ty * kFewTR;

    // ---- stage the tile: the waves take rows in turn, 64 words per instruction, straight into
    // LDS.  A row's descriptor starts at the row's first pixel in the tile and ends with the
    // image: lanes beyond that write zeros (rows below the image), lanes beyond the row's end
    // but inside the image bring pixels of the next row, which only outputs beyond the row's end
    // would use, and those are not stored.
    {
        typedef __attribute__((address_space(3))) void* lds_ptr;
        constexpr int kRsrcFlags = 0x00020000;     // raw buffer of 32-bit words
        const int64_t img_words = (int64_t)p.H * p.W;
        int voff[SEGS];
#pragma unroll
        for (int j = 0; j < SEGS; ++j) voff[j] = 4 * (lane + kWave * j);
        for (int r = wave; r < ROWS; r += 4) {     // (uniform)
            const int64_t first = (int64_t)(y0 + r) * p.W + x0;
            const int64_t left = (img_words - first) * 4;
            const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
                (void*)(p.img + first), 0, (int)(left < 0 ? 0 : left > 0x7FFFFFFF ? 0x7FFFFFFF : left), kRsrcFlags);
#pragma unroll
            for (int j = 0; j < SEGS; ++j)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_ptr)(sh + r * LS + kWave * j), 4, voff[j], 0, 0, 0);
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);        // vmcnt(0): this wave's pieces are in LDS
    }
    __syncthreads();

    const int r0 = wave * kFewRPW;                 // first output row of this wave's band
    const int xo = x0 + 4 * lane;                  // first output column of this lane
    if (y0 + r0 >= p.Ho) return;                   // uniform per wave; no barrier follows
    const int64_t plane = (int64_t)p.Ho * p.Wo;
    const float* wrow = sh + 4 * lane;

    // window row of image row (r0 + rr) lives in win[(rr) % F]
    auto load_row = [&](int rr, float (&w)[4 * NV]) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const v4f q = *reinterpret_cast<const v4f*>(wrow + (r0 + rr) * LS + 4 * v);
#pragma unroll
            for (int e = 0; e < 4; ++e) w[4 * v + e] = q[e];
        }
    };

    // One filter at a time (more at once cost registers, hence occupancy, and were slower for
    // every filter count measured).  Its F*F weights arrive with ONE load, lane t taking weight
    // t, issued while the previous filter is being computed, and are moved to scalar registers
    // (the counterpart of the constant-cache broadcast) tap by tap.
    static_assert(FF <= kWave, "one lane per weight");
    auto load_weights = [&](int k) {
        return (lane < FF && k < p.K) ? p.filt[(int64_t)k * FF + lane] : 0.f;
    };
    float wnext = load_weights(0);
    for (int k = 0; k < p.K; ++k) {                // uniform loop
        const float wv = wnext;
        wnext = load_weights(k + 1);
        float wgt[FF];
#pragma unroll
        for (int t = 0; t < FF; ++t)
            wgt[t] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wv), t));

        float win[F][4 * NV];
#pragma unroll
        for (int i = 0; i < F - 1; ++i) load_row(i, win[i]);
        float* plane_k = p.out + (int64_t)k * plane;
#pragma unroll
        for (int rr = 0; rr < kFewRPW; ++rr) {
            load_row(rr + F - 1, win[(rr + F - 1) % F]);
            float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < F; ++i)
#pragma unroll
                for (int j = 0; j < F; ++j)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        acc[e] = __builtin_fmaf(win[(rr + i) % F][j + e], wgt[i * F + j], acc[e]);
            const int y = y0 + r0 + rr;
            if (y < p.Ho) {
                float* dst = plane_k + (int64_t)y * p.Wo + xo;
                // 16 bytes at once where they fit (rows start at any 4-byte offset: the store
                // is declared 4-byte aligned), single words at the row end
                typedef float v4f_a4 __attribute__((ext_vector_type(4), aligned(4)));
                if (xo + 3 < p.Wo) {
                    *reinterpret_cast<v4f_a4*>(dst) = (v4f_a4){acc[0], acc[1], acc[2], acc[3]};
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (xo + e < p.Wo) dst[e] = acc[e];
                }
            }
        }
    }
}

template <int F, int RPW>
int launch_few_rows(const float* img, const float* filt, float* out, const Shape& s, hipStream_t st)
{
    FewParams p{img, filt, out, s.H, s.W, s.K, s.Ho, s.Wo, (s.Wo + kFewTW - 1) / kFewTW, 0, 0};
    const int64_t tiles = (int64_t)p.tiles_x * ((s.Ho + 4 * RPW - 1) / (4 * RPW));
    if (tiles > 2000000000LL) return DCONV_UNSUPPORTED;
    p.tiles = (int)tiles;
    p.per_xcd = (int)((tiles + 7) / 8);
    begin_launch();
    hipLaunchKernelGGL((single_few_kernel<F, RPW>), dim3((unsigned)(p.per_xcd * 8)), dim3(kThreads), 0, st, p);
    return launch_status();
}

template <int F>
int launch_few_F(const float* img, const float* filt, float* out, const Shape& s, hipStream_t st)
{
    if (F <= 5 && few_rpw(F, s.K) == 4) return launch_few_rows<F, (F <= 5 ? 4 : 8)>(img, filt, out, s, st);
    return launch_few_rows<F, 8>(img, filt, out, s, st);
}

}  // namespace

// Filter sides with a window that fits the register file comfortably; any filter count (the
// groups are looped over), though it only pays for few.
bool single_few_supports(const Shape& s)
{
    return s.N == 1 && s.C == 1 && s.F >= 1 && s.F <= 7;
}

// Worth it (measured against the matrix-core kernel with blocks of 32 and of 16 filters on
// 128^2 .. 4096^2 images, 1 to 20 filters, 1x1 .. 7x7).  Its time grows with K * F * F, the
// matrix-core kernel's hardly at all up to a block's filters, so there is a filter count up to
// which it wins; that count is lower where its tiles (256 x 16 or 256 x 32 pixels, one per
// workgroup) do not cover the chip, because a launch then takes as long as one tile:
//  * fewer than 100 tiles (kernel time from replayed graphs, 2.5 to 20 us): both kernels take
//    the time of their chains of latencies, this one's grows with K * F * F, the other's with
//    the image: one to three 1x1 filters or one or two filters up to 5x5 on the smallest images
//    (under 120 k outputs per filter; 256 x 256, one 3x3 filter: 4.5 -> 3.2 us), four filters
//    up to 3x3 and two beyond up to 350 k, four from there on (640 x 640, one 7x7 filter:
//    22 -> 7 us);
//  * up to four filters: always from 100 tiles on;
//  * up to 3x3: as long as the output fits the memory-side cache (under 110 M outputs; under
//    70 M for 1x1 and 2x2, which have no arithmetic to hide behind: beyond, its rows, written
//    at any alignment, cost, and the matrix-core kernel's whole lines win; 3000 x 3000, twelve
//    2x2 filters: 121 -> 90 us) and the image is not too small for the filter count (20 filters
//    per million pixels);
//  * from 4x4 on: up to 6 filters with fewer than 200 tiles, 8 with fewer than 400, else 10
//    filters of 4x4 (16 while the output fits the memory-side cache) and 13 of 5x5 and
//    larger; 17 to 20 filters (two 16-filter blocks or a 32-filter block with padding) from
//    5x5 on images of at least 512 tiles.
bool single_few_preferred(const Shape& s)
{
    if (!single_few_supports(s) || s.K > 20) return false;
    const int tr = 4 * few_rpw(s.F, s.K);
    const int64_t tiles = (int64_t)((s.Wo + kFewTW - 1) / kFewTW) * ((s.Ho + tr - 1) / tr);
    if (tiles < 100) {
        const int64_t px = (int64_t)s.Ho * s.Wo;
        const int kmax = px < 120000 ? (s.F == 1 ? 3 : s.F <= 5 ? 2 : 0) : px < 350000 ? (s.F <= 3 ? 4 : 2) : 4;
        return s.K <= kmax;
    }
    if (s.K <= 4) return true;
    const int64_t outputs = (int64_t)s.K * s.Ho * s.Wo;
    // (up to 3x3: its time grows with the filter count while the matrix-core kernel on a small
    // image takes the time of its latencies whatever the count: 768 x 768, 16 filters of 3x3:
    // 19 against 14 us; about 20 filters per million output pixels is where they meet)
    if (s.F <= 3)
        return outputs < (s.F == 3 ? 110000000LL : 70000000LL) &&
               (int64_t)s.K * 1000000 <= 20 * (int64_t)s.Ho * s.Wo;
    if (s.K > 16) return s.F >= 5 && tiles >= 512;
    const int kmax = tiles < 200 ? 6 : tiles < 400 ? 8 : s.F > 4 ? 13 : outputs < 70000000LL ? 16 : 10;
    return s.K <= kmax;
}

int launch_single_few(const float* img, const float* filt, float* out, const Shape& s, hipStream_t st)
{
    switch (s.F) {
    case 1: return launch_few_F<1>(img, filt, out, s, st);
    case 2: return launch_few_F<2>(img, filt, out, s, st);
    case 3: return launch_few_F<3>(img, filt, out, s, st);
    case 4: return launch_few_F<4>(img, filt, out, s, st);
    case 5: return launch_few_F<5>(img, filt, out, s, st);
    case 6: return launch_few_F<6>(img, filt, out, s, st);
    case 7: return launch_few_F<7>(img, filt, out, s, st);
    default: return DCONV_UNSUPPORTED;
    }
}

}  // namespace dconv
