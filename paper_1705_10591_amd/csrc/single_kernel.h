// Special-case direct convolution, one input channel (paper Sec. 3, Algorithm 1), gfx950.
//
// What is kept from the paper's scheme: the image is cut into tiles; a
// workgroup stages its tile plus the F-1 halo columns/rows right and below in
// LDS once, so every pixel is read from HBM once (halo pixels aside); the
// waves then sweep the tile row by row and, for each row, produce the outputs
// of ALL filters before moving on, so the output -- K times larger than the
// input and the whole cost of this case -- streams out in long row segments;
// the filter bank is small, lives in registers for the whole kernel and is
// addressed uniformly.
//
// What differs (CDNA4 instead of Kepler): the per-thread register window and
// constant-memory broadcast become a matrix-core product.  For 32 consecutive
// pixels of an output row and 32 filters, out[k][x] = sum_t filt[k][t] *
// img[y + i_t][x + j_t] is a 32 x 32 x F*F contraction; one
// v_mfma_f32_32x32x2_f32 consumes two taps.  The filter operand of every step
// is loaded into registers once per wave; the pixel operand is one LDS word
// per lane, read at the tap's shifted address.  With plain (unpacked) fp32
// vector FMAs the 5x5 case would already be ALU-bound on this chip; on the
// matrix cores it stays bound by the output stream up to 5x5.
// Instead of the rolling one-row prefetch, the whole tile is staged up front:
// several workgroups share a CU, so one group's loads overlap the others'
// arithmetic and stores.
//
// Write-back.  The output is the whole cost of this case, and HBM only runs
// at full rate when whole, aligned 128-byte lines are stored: a line written
// in two pieces by different workgroups costs many times a whole one.  But
// rows of Wo floats start at arbitrary 4-byte offsets and every output plane
// has its own offset.  So a wave does not store its accumulators directly.
// It computes 32 more columns than it writes (NBW + 1 blocks of 32 pixels per
// pass), parks 8 filters at a time in a private LDS strip, each filter row
// shifted by its own misalignment s_k in [0,31], and then streams out, per
// filter, the window of 32*NBW pixels that begins on a line boundary of the
// global address, 16 bytes per lane.  Successive passes along a row use the
// same shift, so their windows tile the row exactly.  Rows follow each other
// without a gap in memory, so the line that holds the end of row y also holds
// the first pixels of row y+1: on wide images the last pass of a row computes
// those pixels too (its lanes beyond Wo wrap to the next row, whose first
// columns are staged beside the tile) and stores the shared line whole.  Only
// the very first and last line of a plane, and narrow images, are written
// piecemeal.
#pragma once
#include <type_traits>
#include "common.h"
#include "../../include/dconv.h"

namespace dconv {

struct SingleParams {
    const float* img;
    const float* filt;
    float* out;
    int N;           // images (each convolved with the same filters); img and out are dense over n
    int H, W, K, Ho, Wo;
    int tiles_x, tiles_y;
    int nfull;       // filter groups of four 32-filter blocks (one block per wave, every tile row)
    int rem;         // blocks left over (0..3): a group of two (two waves per block, every other
                     // row each) and / or a group of one (the four waves share its rows)
    int fgroups;     // filter groups: nfull + (rem == 3 ? 2 : rem ? 1 : 0); work items = N * tiles * fgroups
    int per_xcd;     // work items per XCD (the chip has 8), see the mapping in the kernel
    int wrap;        // 1: row ends are completed with the head of the next row (wide images)
};

// Kinds of pass, by how its windows may be stored.
enum : int { kPlain = 0, kTail = 1, kEdge = 2 };

// TW: nominal tile width in pixels, TR: tile rows, NBW: 32-pixel blocks written per pass,
// WPE: waves per SIMD the register budget is cut for.
// C: input channels.  One is the paper's special case.  A few channels with small filters
// (img [N][C][H][W], filt [K][C][F][F]; C*F*F taps instead of F*F, the tile staged per channel)
// are the same kernel: such shapes are bound by the output stream just the same, and the
// general-case kernel does not write whole lines.
// UNIT: words a lane moves per instruction on the way out (strip read and store): 4 (16 bytes),
// or 1 for the ablation of the paper's width-matching experiment (Sec. 5.1: the unit a thread
// reads from on-chip memory against the width the hardware serves best).
// FB: filters of a matrix-core block.  32: v_mfma_f32_32x32x2_f32, 32 filters x 32 pixels, two
// taps per instruction.  16: v_mfma_f32_16x16x4_f32, 16 filters x 16 pixels, four taps per
// instruction: with up to 16 filters (the paper's weak spot, Sec. 5.1) half of a 32-filter block
// would be padding, and from 5x5 filters on that padding bounds the time.
template <int F, int TW, int TR, int NBW, int WPE, int C = 1, int UNIT = 4, int FB = 32>
__global__ void __launch_bounds__(kThreads, WPE)
single_tiled_kernel(SingleParams p)
{
    static_assert(FB == 32 || (FB == 16 && UNIT == 4), "filter blocks of 32 or 16");
    constexpr int FF = F * F;
    constexpr int T = C * FF;                   // taps: (channel, filter row, filter column)
    constexpr int TPM = FB == 32 ? 2 : 4;       // taps per matrix-core instruction
    constexpr int S = (T + TPM - 1) / TPM;      // matrix-core steps per block
    constexpr int BW = FB == 32 ? 32 : 16;      // pixels of a block
    constexpr int PC0 = TW + 32 + F - 1;        // first column of the next-row patch
    constexpr int PW = 32 + F - 1;              // its width: the head of the next row
    constexpr int LS = PC0 + PW;                // LDS row stride of the image tile
    constexpr int ROWS = TR + F - 1;            // staged image rows per channel; after the last
                                                // channel one more row, of zeros, follows
    constexpr int CHS = ROWS * LS;              // LDS words of one channel of the tile
    constexpr int NBP = NBW + 1;                // 32-pixel columns computed per pass
    constexpr int NB = 32 * NBP / BW;           // blocks computed per pass
    constexpr int CB = 32 / BW;                 // blocks a pass takes over from the one before
    using acc_t = typename std::conditional<FB == 32, v16f, v4f>::type;
    constexpr int PASS = 32 * NBW;              // pixels written per pass
    constexpr int CHUNKS = TW / PASS;
    constexpr int SW = 32 * NBP + 32;           // row stride of the write-back strip
    constexpr int LPR = PASS / 4;               // lanes that cover one filter's window, 16 B each
    constexpr int RPI = kWave / LPR;            // filter rows stored per instruction
    constexpr int ITS = 8 / RPI;                // store instructions per group of 8 filters
    constexpr int TOTAL = (C * ROWS + 1) * LS;
    constexpr int IMG_WORDS = (TOTAL + 3) & ~3;
    static_assert(TW % PASS == 0 && (NBW == 1 || NBW == 2 || NBW == 4 || NBW == 8), "tile shape");
    static_assert((IMG_WORDS + 4 * 8 * SW) * 4 <= 160 * 1024, "tile and strips must fit the LDS of a CU");

    __shared__ __attribute__((aligned(16))) float sh[IMG_WORDS + 4 * 8 * SW];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    // uniform: lets wave-level index math run on the scalar unit
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // 32-filter blocks: lane half h takes the odd tap of a pair, lane l32 one filter / pixel.
    // 16-filter blocks: lane quarter q4 takes one tap of four, lane l16 one filter / pixel; of
    // its quarter's four filters, hh says whether they are the lower or upper four of a group
    // of eight.  (The write-back below is written once, in terms of hh and lp.)
    const int h = lane >> 5, l32 = lane & 31;
    const int q4 = lane >> 4, l16 = lane & 15;
    const int hh = FB == 32 ? h : (q4 & 1), lp = FB == 32 ? l32 : l16;
    float* stg = sh + IMG_WORDS + wave * (8 * SW);

    // Workgroups are handed to the 8 XCDs round-robin by their linear id.  Give each XCD one
    // contiguous range of work items (a band of the image), walked along x, so that its L2
    // sees neighbouring tiles and every XCD gets the same mix of edge and interior tiles.
    const int item_all = (blockIdx.x % 8) * p.per_xcd + blockIdx.x / 8;
    const int ntiles = p.tiles_x * p.tiles_y;
    const int per_image = ntiles * p.fgroups;
    const int n = item_all / per_image, item = item_all - n * per_image;
    if (n >= p.N) return;                                  // uniform: before any barrier
    const float* img = p.img + (int64_t)n * C * p.H * p.W;
    float* out = p.out + (int64_t)n * p.K * p.Ho * p.Wo;
    // (the filter groups of a tile are neighbours in the order of work items: every XCD gets
    // the same mix of full and leftover groups, and its L2 serves a tile's pixels to all of them)
    const int tile = item / p.fgroups, fgroup = item - tile * p.fgroups;
    const int ty = tile / p.tiles_x, tx = tile - ty * p.tiles_x;
    const int x0 = tx * TW, y0 = ty * TR;
    // this group's blocks: four, or what is left over as two and / or one (no wave works on a
    // block of padding: 160 filters are a group of four blocks and a group of one)
    int fbw = 4, fb0 = 4 * fgroup;
    if (fgroup >= p.nfull) {
        const bool second = fgroup > p.nfull;              // (only with three blocks left over)
        fbw = p.rem == 3 ? (second ? 1 : 2) : p.rem;
        fb0 = 4 * p.nfull + (second ? 2 : 0);
    }
    const int fb = fb0 + wave % fbw;                       // this wave's 32-filter block
    const int row_start = wave / fbw, row_step = 4 / fbw;  // its share of the tile rows
    const bool wrap_tile = p.wrap && tx == p.tiles_x - 1;

    // ---- this wave's filter operands: a[s] = filt[k][tap 2s + h], zero beyond K / F*F --
    float a[S];
    {
        const int k = fb * FB + lp;
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const int t = FB == 32 ? 2 * s + h : 4 * s + q4;
            a[s] = (k < p.K && t < T) ? p.filt[(int64_t)k * T + t] : 0.f;
        }
    }
    // ---- stage the tile (zeros outside the image), coalesced along rows.  LDS row ch*ROWS + r
    // holds row y0+r of channel ch in columns [0, PC0) and, in the last tile column of a wide
    // image, the first PW pixels of its row y0+r+1 in columns [PC0, LS).
    {
        const int cols = min(PC0, p.W - x0);
        const int rows_ok = min(ROWS, p.H - y0);
        const int prow_ok = wrap_tile ? min(ROWS, p.H - y0 - 1) : 0;
        const float* src = img + (int64_t)y0 * p.W + x0;
        const float* psrc = img + (int64_t)(y0 + 1) * p.W - PC0;
        // all loads are issued before the first LDS store: one trip to HBM, not one per batch
        constexpr int UN = (TOTAL + kThreads - 1) / kThreads;
        float v[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int e = tid + u * kThreads;
            const int lr = e / LS, c = e - lr * LS;
            const int ch = lr / ROWS, r = lr - ch * ROWS;      // ch == C: the row of zeros
            float val = 0.f;
            if (e < TOTAL && ch < C) {
                const int64_t chofs = (int64_t)ch * p.H * p.W;
                if (c < PC0) { if (r < rows_ok && c < cols) val = src[chofs + (int64_t)r * p.W + c]; }
                else if (r < prow_ok) val = psrc[chofs + (int64_t)r * p.W + c];
            }
            v[u] = val;
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int e = tid + u * kThreads;
            if (e < TOTAL) sh[e] = v[u];
        }
    }
    __syncthreads();

    const int64_t plane = (int64_t)p.Ho * p.Wo;
    const int pm = (int)(plane & 31);
    const int a0 = (int)(((uintptr_t)out >> 2) & 31);     // misalignment of this image's output
    const int rows_here = min(TR, p.Ho - y0);
    const int dY = h * (LS - (F - 1));          // second tap of a pair sits on the next row
    const int dZ = h * (CHS - (F - 1) * LS - (F - 1));    // ... or is the first tap of the next channel
    const int kb = fb * FB;
    // (The write-back goes by groups of eight filters and skips the groups beyond K; in a last
    // group that is not full, the lanes of the missing filters store nothing.)
    const int rrow = lane / LPR, c4 = lane % LPR;          // read phase: strip row and 16 B column
    const int rdofs = rrow * SW + 32 + 4 * c4;
    // The shift of filter k in output row y is s = -(k*pm + c0(y)) mod 32.  k*pm is split into
    // a per-lane part (one register) and a wave-uniform part per accumulator register / store.
    const int wl = 4 * hh * SW + 32 + lp;                  // strip word of (q % 4 == 0, block 0, s = 0)
    const int tw_lane = (kb + 4 * hh) * pm;
    const unsigned gl = (unsigned)(rrow * (int)plane + 4 * c4);
    const int tr_lane = (kb + rrow) * pm;

    // sixteen-filter blocks: where tap 4s + q4 lies in the tile, from the lane's pixel
    int toff[FB == 16 ? S : 1];
    if (FB == 16) {
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const int t = min(4 * s + q4, T - 1);
            const int tc = t / FF, i = (t % FF) / F, j = t % F;
            toff[s] = tc * CHS + i * LS + j;
        }
    }
    bool contiguous = true;                // (per pass) the pass's pixels lie side by side in LDS

    // ---- the write-back of one pass ---------------------------------------------------------
    // Per group g of eight filters: park one accumulator register of every block in the strip
    // (4 pieces), read 16 B columns back (ITS pieces), store them (ITS pieces).  The stores are
    // nontemporal: the output is written once and not read again.
    struct PassOut {
        int tw, tr, trn;       // per-lane shift seeds of the pass's output row and of the next row
        float* orow;           // out[kb][y][X], wave-uniform
        int c0, c0n;           // the same seeds without their per-lane parts (uniform)
        int X;                 // first output column of the pass
        int kind;              // kPlain, kTail or kEdge
        bool head;             // kEdge only: also write the pixels before the first boundary
    };
    auto store4 = [&](float* dst, const v4f& v) {
        __builtin_nontemporal_store(v, reinterpret_cast<v4f*>(dst));
    };
    auto write_back = [&](const acc_t (&A)[NB], const PassOut& pd) {
#pragma unroll
        for (int g = 0; g < FB / 8; ++g) {
            if (kb + 8 * g >= p.K) break;        // (uniform) no filter of this group exists
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // the accumulator register that holds filter 8g + 4hh + j of the block: with
                // 32-filter blocks in every lane, with 16-filter blocks in lane half g
                const int q = FB == 32 ? 4 * g + j : j;
                const int sk = (-(pd.tw + (8 * g + j) * pm)) & 31;
                // the strip word as one opaque register: the stores then pair up with offsets of
                // 0..4 blocks and need no further address arithmetic on the vector ALU
                int word = (int)(stg - sh) + (wl - sk) + j * SW;
                asm volatile("" : "+v"(word));
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    if (FB == 32 || h == g) sh[word + nb * BW] = A[nb][q];
            }
            if constexpr (UNIT == 1) {
                // One word per lane: a wave instruction reads 64 pixels of one filter row from the
                // strip and stores them, four times the instructions of the 16-byte unit.
                static_assert(PASS % 64 == 0, "the one-word unit is compiled for passes of whole waves");
#pragma unroll
                for (int r8 = 0; r8 < 8; ++r8) {
                    const int kofs = (kb + 8 * g + r8) * pm;
                    const int sk = (-(pd.c0 + kofs)) & 31;
                    const int skn = (-(pd.c0n + kofs)) & 31;
                    float* ub = pd.orow + (8 * g + r8) * plane;     // out[kb + 8g + r8][y][X]
                    const bool kvalid = kb + 8 * g + r8 < p.K;
#pragma unroll
                    for (int ip = 0; ip < PASS / 64; ++ip) {
                        const int col = 64 * ip + lane;
                        const float v = stg[r8 * SW + 32 + col];
                        const int px = pd.X + sk + col;
                        float* dst = ub + (sk + col);
                        if (pd.kind == kPlain) { if (kvalid) __builtin_nontemporal_store(v, dst); }
                        else if (pd.kind == kTail) { if (kvalid && px < p.Wo + skn) __builtin_nontemporal_store(v, dst); }
                        else if (kvalid && px < p.Wo) *dst = v;
                    }
                    if (pd.kind == kEdge && pd.head && kvalid && lane < sk && lane < p.Wo)
                        (ub - pd.X)[lane] = stg[r8 * SW + 32 - sk + lane];
                }
                continue;
            }
            v4f held[ITS];
#pragma unroll
            for (int it = 0; it < ITS; ++it)
                held[it] = *reinterpret_cast<const v4f*>(stg + rdofs + it * RPI * SW);
            const int rows_left = p.K - kb - 8 * g;            // (uniform) filters of this group and beyond
#pragma unroll
            for (int it = 0; it < ITS; ++it) {
                const bool row_ok = rows_left >= 8 || it * RPI + rrow < rows_left;
                const int kofs = (8 * g + it * RPI) * pm;
                const int sk = (-(pd.tr + kofs)) & 31;
                float* ub = pd.orow + (8 * g + it * RPI) * plane;     // out[kb + 8g + it*RPI][y][X]
                float* dst = ub + (gl + (unsigned)sk);                // this lane's four pixels
                const int px = pd.X + sk + 4 * c4;
                if (pd.kind == kPlain) {
                    if (row_ok) store4(dst, held[it]);
                } else if (pd.kind == kTail) {
                    // The window runs over the end of the row into the head of the next one; it
                    // stops at the first line boundary of the next row, where that row's own
                    // passes begin.  Both limits are multiples of 16 B away from px.
                    const int skn = (-(pd.trn + kofs)) & 31;
                    if (row_ok && px < p.Wo + skn) store4(dst, held[it]);
                } else if (row_ok) {
                    // Same window, clipped to the row; whole 16 B pieces wherever they fit.
                    if (px + 3 < p.Wo) {
                        store4(dst, held[it]);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (px + e < p.Wo) dst[e] = held[it][e];
                    }
                    // The sk pixels before the first line boundary of the row.
                    if (pd.head && c4 < 8) {
                        const float* row = stg + (it * RPI + rrow) * SW + 32 - sk;
                        float* hd = ub + rrow * plane - pd.X;         // out[k][y][0]
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int hx = 4 * c4 + e;
                            if (hx < sk && hx < p.Wo) hd[hx] = row[hx];
                        }
                    }
                }
            }
        }
    };

    // ---- the matrix-core steps of one pass ---------------------------------------------------
    // Block 0 of a pass covers the same 32 pixels as block NB-1 of the pass before it on the
    // same row; when CARRY is set those sums are taken over instead of being formed again.
    auto compute = [&](auto carry_tag, acc_t (&A)[NB], const int (&base)[NB]) {
        constexpr bool CARRY = decltype(carry_tag)::value;
        constexpr int NB0 = CARRY ? CB : 0;
        if (CARRY) {
#pragma unroll
            for (int nb = 0; nb < CB; ++nb) A[nb] = A[NB - CB + nb];
        }
        if constexpr (FB == 16) {
            // Sixteen-filter blocks: lane quarter q4 brings tap 4s + q4 of step s, whose place in
            // the tile (toff) differs from lane to lane, so it cannot be an immediate; where the
            // pass's pixels are contiguous in LDS (every pass but the one that runs over the row
            // end into the next row's head), one addition per step gives the address of block 0
            // and the other blocks follow at immediate offsets.  A pad tap (beyond the last
            // one) reads the row of zeros; its weight is zero as well.
            auto load_b = [&](int s, float (&b)[NB]) {
                const bool pad = 4 * s + q4 >= T;                    // (only in the last step)
                if (contiguous) {
                    int addr = base[0] + toff[s];
                    if (4 * s + 3 >= T) addr = pad ? C * ROWS * LS + l16 : addr;
#pragma unroll
                    for (int nb = NB0; nb < NB; ++nb) b[nb] = sh[addr + nb * 16];
                } else {
#pragma unroll
                    for (int nb = NB0; nb < NB; ++nb) {
                        int addr = base[nb] + toff[s];
                        if (4 * s + 3 >= T) addr = pad ? C * ROWS * LS + l16 : addr;
                        b[nb] = sh[addr];
                    }
                }
            };
            float b0[NB], b1[NB];
            load_b(0, b0);
#pragma unroll
            for (int s = 0; s < S; ++s) {
                float (&b)[NB] = (s & 1) ? b1 : b0;
                if (s + 1 < S) load_b(s + 1, (s & 1) ? b0 : b1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int nb = NB0; nb < NB; ++nb)
                    A[nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[s], b[nb], s == 0 ? v4f{} : A[nb], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            return;
        }
        // (the other blocks start from a zero accumulator operand in step 0: no clearing)
        // pixel operands of step s; those of step s+1 are requested before the matrix-core
        // instructions of step s are issued, so the wave does not wait for LDS with the
        // matrix pipe idle
        auto load_b = [&](int s, float (&b)[NB]) {
            const int t0 = 2 * s, t1 = 2 * s + 1;
            const int tc = t0 / FF, i = (t0 % FF) / F, j = t0 % F;
            const int off = tc * CHS + i * LS + j;            // the first tap of the pair
#pragma unroll
            for (int nb = NB0; nb < NB; ++nb) {
                int addr;
                if (t1 >= T)             // pad tap: the zero row (any column of it)
                    addr = h ? (C * ROWS * LS + l32) : base[nb] + off;
                else if (t1 / FF != tc)      addr = base[nb] + dZ + off;   // next channel
                else if ((t1 % FF) / F != i) addr = base[nb] + dY + off;   // next row
                else                         addr = base[nb] + h + off;    // next column
                b[nb] = sh[addr];
            }
        };
        float b0[NB], b1[NB];
        load_b(0, b0);
#pragma unroll
        for (int s = 0; s < S; ++s) {
            float (&b)[NB] = (s & 1) ? b1 : b0;
            if (s + 1 < S) load_b(s + 1, (s & 1) ? b0 : b1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int nb = NB0; nb < NB; ++nb) {
                if constexpr (FB == 32) A[nb] = mfma_32x32x2(a[s], b[nb], s == 0 ? v16f{} : A[nb]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- the passes of this wave: along each of its rows, then on to its next row ------------
    const int ch_mine = min(CHUNKS, (p.Wo - x0 + PASS - 1) / PASS);      // passes per row here
    const int rows_mine = rows_here > row_start ? (rows_here - row_start + row_step - 1) / row_step : 0;
    const int npass = rows_mine * ch_mine;

    acc_t acc[NB];
    int ri = 0, ci = 0;                    // row and chunk counters of the next pass
#pragma unroll 1
    for (int q = 0; q < npass; ++q) {
        const int r = row_start + ri * row_step;
        const int ch = ci;
        if (++ci == ch_mine) { ci = 0; ++ri; }
        const int y = y0 + r;
        const int64_t rowoff = (int64_t)y * p.Wo;
        // alignment (in floats, mod 32) of out[k][y][X] is (k*pm + c0) mod 32 for every pass
        // of a row, because passes start at multiples of 32
        const int c0 = (int)((rowoff + a0) & 31);
        const int c0n = (int)((rowoff + p.Wo + a0) & 31);
        const int X = x0 + ch * PASS;                  // first output column of this pass
        int base[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int x = X + nb * BW + lp;
            // lanes beyond the row end compute the head of the next row from the patch
            base[nb] = r * LS + ((wrap_tile && x >= p.Wo) ? PC0 + min(x - p.Wo, 31) : x - x0);
        }
        const bool reaches_end = X + 32 + PASS > p.Wo;                // a window may cross Wo
        contiguous = !(wrap_tile && reaches_end);                     // no lane reads the next row's head
        const bool needs_head = X == 0 && (y == 0 || !p.wrap);
        int kind = kPlain;
        if (needs_head) kind = kEdge;
        else if (reaches_end) kind = (p.wrap && y < p.Ho - 1) ? kTail : kEdge;
        // every pass but the first of a row continues the previous pass of this wave
        if (ch > 0) compute(std::true_type{}, acc, base);
        else compute(std::false_type{}, acc, base);
        const PassOut pd{tw_lane + c0, tr_lane + c0, tr_lane + c0n,
                         out + kb * plane + rowoff + X, c0, c0n, X, kind, needs_head};
        write_back(acc, pd);
    }
}

template <int F, int TW, int TR, int NBW, int WPE, int C = 1, int UNIT = 4, int FB = 32>
int launch_cfg(const float* img, const float* filt, float* out, const Shape& s, hipStream_t st)
{
    if (s.C != C) return DCONV_UNSUPPORTED;
    SingleParams p;
    p.img = img; p.filt = filt; p.out = out;
    p.N = s.N;
    p.H = s.H; p.W = s.W; p.K = s.K; p.Ho = s.Ho; p.Wo = s.Wo;
    p.tiles_x = (s.Wo + TW - 1) / TW;
    p.tiles_y = (s.Ho + TR - 1) / TR;
    const int fblocks = (s.K + FB - 1) / FB;
    p.nfull = fblocks / 4;
    p.rem = fblocks % 4;
    p.fgroups = p.nfull + (p.rem == 3 ? 2 : p.rem ? 1 : 0);
    // Completing row ends with the next row's head needs a pass to span at most one row end,
    // and every pass that reaches the row end to lie in the last tile column.
    // (a pass computes 32 * NBW + 32 pixels from a multiple of 32 * NBW on: it crosses one row
    // end at most as soon as a row is that long)
    p.wrap = (s.Wo >= 32 * NBW + 64 && (p.tiles_x - 1) * TW + 32 <= s.Wo) ? 1 : 0;
    const int64_t items = (int64_t)p.tiles_x * p.tiles_y * p.fgroups * s.N;
    if (items > 2000000000LL) return DCONV_UNSUPPORTED;
    p.per_xcd = (int)((items + 7) / 8);
    begin_launch();
    hipLaunchKernelGGL((single_tiled_kernel<F, TW, TR, NBW, WPE, C, UNIT, FB>),
                       dim3((unsigned)(p.per_xcd * 8)), dim3(kThreads), 0, st, p);
    return launch_status();
}

// Images 96 to 199 pixels wide: configuration 5 (128 x 4 tile, passes of 64 pixels) or 6 (passes
// of 32).  A row of Wo pixels takes ceil(Wo / 64) passes of two new blocks or ceil(Wo / 32) of
// one (plus the block every pass takes over from the one before); the fewer blocks win, ties go
// to the wider pass.
inline int short_pass_config(int Wo)
{
    if (Wo < 128) return 6;
    return 2 * ((Wo + 63) / 64) <= (Wo + 31) / 32 ? 5 : 6;
}

// The same kernel for a few input channels, implemented once per channel count, each in its own
// translation unit (single_multi_inst.hip).
constexpr int kSingleMultiMaxC = 4, kSingleMultiMaxF = 5;
template <int C>
int single_multi_launch_for_C(const float* img, const float* filt, float* out, const Shape& s,
                              hipStream_t st, int cfg);

}  // namespace dconv
