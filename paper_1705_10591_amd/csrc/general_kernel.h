// General-case direct convolution (paper Sec. 4, Algorithm 2) for gfx950: the kernel.
//
// What is kept from the paper's scheme: a workgroup owns a block of filters
// times a block of output pixels; channels are consumed in chunks of CSH;
// each chunk's image block (with its halo) goes to LDS untransposed and the
// matching filter block goes to LDS transposed, with a padded row stride, so
// that both are read conflict-free; the next chunks are prefetched from HBM
// into registers while the current one is consumed; the image block is read
// at shifted addresses for the F*F taps instead of being unrolled in memory,
// so an input pixel is fetched once per tile and reused F*F*K times on chip.
//
// What differs (CDNA4 instead of Kepler):
//  * The multiply-accumulate runs on the matrix cores.  One
//    v_mfma_f32_32x32x2_f32 forms a 32-filter x 32-pixel block of partial
//    sums for two reduction indices at once; it is the only route to the
//    chip's fp32 peak, and it makes the per-lane register tile of the paper
//    (F_T x W_T) a per-wave tile of MW x NW such blocks.  The two reduction
//    indices of one instruction are two consecutive entries of the flattened
//    (channel, filter row, filter column) list of the chunk, so the image
//    operand of lane l is the LDS word of pixel (l % 32) at the tap chosen
//    by (l / 32).
//  * Output pixels are numbered along (image, row, column) of a column
//    strip, so a 32-pixel block may wrap over rows and images and no lanes
//    are wasted on narrow maps (Wo = 26, 54).
//  * LDS holds NBUF chunks (3 where they fit).  While chunk u is consumed,
//    chunk u+1 moves from registers to the next LDS slot and chunk u+2 is
//    requested from HBM: every staging register is written to LDS and
//    re-loaded in the same breath, one or two registers per matrix-core
//    step, so each load has a whole chunk period to arrive, the demand on
//    L2 is even, and there is no phase in which a workgroup only copies.
//    With three slots the one barrier per chunk sits two steps before the
//    chunk's end and the first operands of the next chunk are requested
//    across it, so the matrix pipe does not drain between chunks.
//  * The launch is persistent: a fixed number of workgroups (what fits on
//    the chip at once) each walk a contiguous range of (tile, chunk) units.
//    Prefetching runs across tile boundaries.  When the number of tiles does
//    not divide evenly over the chip, the range boundaries fall inside tiles:
//    a tile is then summed over channels by two or more workgroups, each of
//    which leaves its partial sums in a workspace and counts itself in; the
//    one that arrives last adds the partial sums in a fixed order and writes
//    the tile.  Nobody waits for anybody, so every workgroup always exits, and
//    the result does not depend on the order of arrival.
#pragma once
#include <algorithm>
#include "common.h"
#include "../../include/dconv.h"

namespace dconv {

// Division of a non-negative int below 2^31 by a fixed positive divisor d, as one multiply-high
// and a shift: with l = ceil(log2 d) and m = ceil(2^(31+l) / d) < 2^32, floor(n / d) equals
// (n * m) >> (31 + l).  d = 1 is flagged by m = 0.  The setup of a tile divides a dozen times.
struct FastDiv {
    uint32_t m;
    int sh;          // l - 1
    int d;
};
inline FastDiv make_fastdiv(int d)
{
    FastDiv f{0u, 0, d};
    if (d <= 1) return f;
    int l = 0;
    while ((1LL << l) < d) ++l;
    f.m = (uint32_t)(((1ULL << (31 + l)) + (uint64_t)d - 1) / (uint64_t)d);
    f.sh = l - 1;
    return f;
}
__device__ __forceinline__ int fdiv(int n, FastDiv f) {
    return f.m ? (int)(__umulhi((uint32_t)n, f.m) >> f.sh) : n;
}

struct GenParams {
    const float* in;
    const float* filt;
    float* out;
    float* part;     // workspace: partial tiles, [workgroup][2][MT * NT]
    int* cnt;        // workspace: arrivals per split tile, indexed by its first workgroup; all 0
    int N, C, H, W, K, Ho, Wo;
    int bw;          // width of a column strip of the output (the last strip may be narrower)
    int nstrips;
    int LS;          // LDS row stride of the image block: bw + F - 1, rounded up to a multiple of 4
    int RS;          // rows of the image block per channel
    int pt_full;     // pixel tiles in a full-width strip
    int KB;          // filter tiles
    int nch;         // channel chunks per tile
    int tiles;       // all tiles: ((nstrips - 1) * pt_full + pt_last) * KB
    int G;           // workgroups launched
    int split;       // 1: ranges are cut in units (tiles may be shared), 0: in whole tiles
    int aligned;     // 1: tiles are written back through LDS in whole 128-byte lines
    int pad_words;   // LDS words added to every slot so that it can hold a tile on its way out
    FastDiv d_strip; // by pt_full * KB
    FastDiv d_kb;    // by KB
    FastDiv d_wsf;   // by bw, the width of a full strip
    FastDiv d_wsl;   // by the width of the last strip
    FastDiv d_ho;    // by Ho
    FastDiv d_hc;    // by Hc
    FastDiv d_nch;   // by nch
    int Hc;          // image-block rows set aside per image: Ho + RG - 1
};

// Reduction index t of a chunk <-> (channel in chunk, filter row within the chunk's row group,
// filter column).  A chunk holds RG of the F filter rows of CSH channels.
template <int F, int RG> __device__ __forceinline__ constexpr int tap_c(int t) { return t / (RG * F); }
template <int F, int RG> __device__ __forceinline__ constexpr int tap_i(int t) { return (t % (RG * F)) / F; }
template <int F, int RG> __device__ __forceinline__ constexpr int tap_j(int t) { return t % F; }

// First unit of workgroup j's range and the workgroup that owns unit v, for U units cut
// evenly over G workgroups: range(j) = [j*U/G, (j+1)*U/G).
__device__ __forceinline__ int range_start(int j, int U, int G) {
    return (int)(((int64_t)j * U) / G);
}
__device__ __forceinline__ int unit_owner(int v, int U, int G) {
    return (int)((((int64_t)v + 1) * G - 1) / U);
}

// Compile-time geometry of one instantiation, shared by the kernel and its launcher.
//   RG:   filter rows per chunk; RG < F (large filters, one channel per chunk) cuts a channel
//         into row groups so that the filter block of a chunk stays small; the last group
//         may have fewer rows, its chunk then ends after fewer steps
//   IMAX: image words a thread stages per chunk, at most (a multiple of four: the image block
//         moves in 16-byte pieces)
//   NBUF: chunks held in LDS
//   OCC:  workgroups per CU the register budget is cut for
template <int F, int CSH, int RG, int MW, int NW, int WM, int WN, int IMAX, int NBUF, int OCC>
struct GenGeom {
    static_assert(RG >= 1 && RG <= F && (RG == F || CSH == 1), "row groups need one channel per chunk");
    static constexpr int NG = (F + RG - 1) / RG;     // row groups per channel
    static constexpr int RGL = F - (NG - 1) * RG;    // filter rows in the last group
    static constexpr int MT = 32 * MW * WM;          // filters per tile
    static constexpr int NT = 32 * NW * WN;          // output pixels per tile
    static constexpr int FF = F * F;
    static constexpr int T = CSH * RG * F;           // reduction indices per chunk
    static constexpr int TP = T + (T & 1);           // padded to a whole number of pairs
    static constexpr int S = TP / 2;                 // matrix-core steps per chunk
    static constexpr int TL = CSH * RGL * F;         // the same for the chunk of a last row group
    static constexpr int SL = (TL + 1) / 2;
    static constexpr int LDK = MT + 1;               // odd row stride: transposing writes hit 32 banks
    static constexpr int TPF = kThreads / MT;        // threads that share one filter when staging
    static constexpr int EPT = (T + TPF - 1) / TPF;  // reduction indices per thread
    static constexpr int NFI = (EPT + 3) / 4;        // 16-byte filter loads per thread per chunk
    // rows of the filter block in LDS: every thread's run is written whole (rows beyond T are
    // never read), so the write addresses need no test
    static constexpr int TROWS = TPF * EPT > TP ? TPF * EPT : TP;
    static_assert(IMAX % 4 == 0, "16-byte image pieces");
    static constexpr int NII = IMAX / 4;             // image loads per thread per chunk
    static constexpr int NI = NII + NFI;             // staging items per thread per chunk
    static constexpr int IOFF = (TROWS * LDK + 3) & ~3;   // first word of the image block in a slot
    static_assert(NBUF == 2 || (NBUF == 3 && SL >= 4), "three LDS slots need at least four steps");
    // steps that carry staging items (every chunk has them); with three slots the barrier sits
    // two steps before the chunk's end
    static constexpr int NS = NBUF == 3 ? SL - 2 : SL;
    static constexpr int IPS = (NI + NS - 1) / NS;   // items per step
};

template <int F, int CSH, int RG, int MW, int NW, int WM, int WN, int IMAX, int NBUF, int OCC>
__global__ void __launch_bounds__(kThreads, OCC)
general_tiled_kernel(GenParams p)
{
    static_assert(WM * WN * kWave == kThreads, "four waves per workgroup");
    using Gm = GenGeom<F, CSH, RG, MW, NW, WM, WN, IMAX, NBUF, OCC>;
    constexpr int NG = Gm::NG, RGL = Gm::RGL, TL = Gm::TL, SL = Gm::SL;
    constexpr int MT = Gm::MT, NT = Gm::NT, FF = Gm::FF, T = Gm::T, TP = Gm::TP, S = Gm::S;
    constexpr int LDK = Gm::LDK, TPF = Gm::TPF, EPT = Gm::EPT, NFI = Gm::NFI, NI = Gm::NI;
    constexpr int NS = Gm::NS, IPS = Gm::IPS, TROWS = Gm::TROWS, NII = Gm::NII, IOFF = Gm::IOFF;

    extern __shared__ __attribute__((aligned(16))) float lds[];
    __shared__ int s_old;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: index math on the scalar unit
    const int h = lane >> 5, l32 = lane & 31;
    const int wm = wave / WN, wn = wave % WN;

    const int LS = p.LS, PL = p.RS * p.LS;
    const int img_words = CSH * PL;             // a multiple of four: LS is
    // one LDS slot: filter block [TROWS][LDK], image block [CSH][RS][LS] on a 16-byte boundary,
    // a zero word (and three spare ones), four trash words
    const int zero_word = IOFF + img_words + p.pad_words;
    const int trash_word = zero_word + 4;
    const int BUF = zero_word + 8;

    // Workgroups are handed to the 8 XCDs round-robin by their id; give each XCD one contiguous
    // stretch of the unit list so that neighbouring tiles share its L2.
    const int G = p.G;
    const int j = (G % 8 == 0) ? (int)(blockIdx.x % 8) * (G / 8) + (int)(blockIdx.x / 8)
                               : (int)blockIdx.x;
    const int nch = p.nch;
    const int U = p.split ? p.tiles * nch : p.tiles;
    const int unit_scale = p.split ? 1 : nch;
    const int u0 = range_start(j, U, G) * unit_scale;
    const int u1 = range_start(j + 1, U, G) * unit_scale;
    if (u0 >= u1) return;                                   // uniform: before any barrier

    const int HW = p.H * p.W;
    const int64_t plane = (int64_t)p.Ho * p.Wo;
    const int CFF = p.C * FF;
    const int per_strip = p.pt_full * p.KB;

    // ---- the staging side ------------------------------------------------------------------------
    // HBM is read through buffer descriptors: a wave-uniform base and extent (scalar registers)
    // plus a 32-bit byte offset per lane, range-checked by the hardware.  A lane with nothing
    // to bring uses an offset beyond the extent and receives zero, so every load is issued
    // unconditionally and its value goes to LDS as it is: no compare or select on the vector
    // ALU, whose every instruction takes time from the matrix cores.  The host has checked
    // that the offsets of one tile stay below 2 GiB.  The state of the unit being requested
    // (suffix _f) and of the unit on its way from registers to LDS (suffix _c) is kept apart,
    // because the two may belong to different tiles.
    constexpr uint32_t kNowhere = 0xC0000000u;  // beyond every extent (extents are at most 2^31)
    constexpr int kRsrcFlags = 0x00020000;      // raw buffer of 32-bit words
    uint32_t ig[NII];        // image: byte offset of a 4-word piece from in[n_first][c0][0][0], or kNowhere
    const int wkl = tid / TPF, we0 = (tid % TPF) * EPT;
    const uint32_t wofs = (uint32_t)(wkl * CFF + we0) * 4u;   // filter: byte offset from filt[k0][c0][0][0]
    const char* ibase = (const char*)p.in;      // in[n_first][0][0][0] of the tile being requested
    int64_t ileft = 0;                          // bytes from there to the end of the input
    int64_t wfirst = 0;                         // first filter word of the tile being requested
    const int64_t in_bytes = (int64_t)p.N * p.C * HW * 4, filt_words = (int64_t)p.K * CFF;
    __amdgpu_buffer_rsrc_t irs = __builtin_amdgcn_make_buffer_rsrc((void*)p.in, 0, 0, kRsrcFlags);
    __amdgpu_buffer_rsrc_t wrs = __builtin_amdgcn_make_buffer_rsrc((void*)p.filt, 0, 0, kRsrcFlags);
    auto setup_fetch = [&](int tile) __attribute__((always_inline)) {
        const int strip = min(fdiv(tile, p.d_strip), p.nstrips - 1);
        const int rem = tile - strip * per_strip;
        const int ptile = fdiv(rem, p.d_kb), kb = rem - ptile * p.KB;
        const int x0 = strip * p.bw;
        const int ws = min(p.bw, p.Wo - x0);
        const bool last_strip = strip == p.nstrips - 1;
        const FastDiv d_ws{last_strip ? p.d_wsl.m : p.d_wsf.m, last_strip ? p.d_wsl.sh : p.d_wsf.sh, ws};
        const int total_p = p.N * p.Ho * ws;
        const int p0 = ptile * NT;
        // The image block of a chunk holds, for every output row of the tile, the RG input rows
        // of the chunk's filter rows: block row (n - n_first)*Hc + (y - y_first) + i for output
        // row y of image n and filter row i of the group, with Hc = Ho + RG - 1 rows set
        // aside per image.  Which input row that is depends on the group only through a shift
        // of RG*W words per group, which goes into the chunk's buffer base (set_chunk).
        const int Q0 = fdiv(p0, d_ws);
        const int n_first = fdiv(Q0, p.d_ho);
        const int y_first = Q0 - n_first * p.Ho;
        const int Ql = fdiv(min(p0 + NT, total_p) - 1, d_ws);
        const int nl = fdiv(Ql, p.d_ho);
        const int nslots = (nl - n_first) * p.Hc + (Ql - nl * p.Ho) - y_first + RG;
#pragma unroll
        for (int it = 0; it < NII; ++it) {
            const int e = 4 * (tid + it * kThreads);           // LS is a multiple of four: one row
            uint32_t g = kNowhere;
            if (e < img_words) {
                const int cc = e / PL, r2 = e - cc * PL;
                const int slot = r2 / LS, col = r2 - slot * LS;
                const int dn = fdiv(y_first + slot, p.d_hc);         // images past the first one
                const int yy = y_first + slot - dn * p.Hc;           // input row, for the first group
                if (slot < nslots && n_first + dn < p.N && x0 + col < p.W)
                    g = (uint32_t)(((dn * p.C + cc) * p.H + yy) * p.W + x0 + col) * 4u;
            }
            ig[it] = g;
        }
        const int64_t ifirst = (int64_t)n_first * p.C * HW * 4;
        ibase = (const char*)p.in + ifirst;
        ileft = in_bytes - ifirst;
        wfirst = (int64_t)kb * MT * CFF;
    };
    auto set_chunk = [&](int chunk) __attribute__((always_inline)) {
        const int cidx = chunk / NG, g = chunk - cidx * NG;
        const int c0 = cidx * CSH;
        const int64_t ioff = ((int64_t)c0 * HW + (int64_t)g * (RG * p.W)) * 4;
        const int64_t ibytes = ileft - ioff;
        irs = __builtin_amdgcn_make_buffer_rsrc((void*)(ibase + ioff), 0,
                                                (int)min(ibytes, (int64_t)0x7FFFFFFF), kRsrcFlags);
        const int64_t w0 = wfirst + (int64_t)c0 * FF + g * (RG * F);
        const int64_t wbytes = (filt_words - w0) * 4;
        wrs = __builtin_amdgcn_make_buffer_rsrc((void*)(p.filt + w0), 0,
                                                (int)min(wbytes, (int64_t)0x7FFFFFFF), kRsrcFlags);
    };

    float ireg[IMAX];
    float wreg[4 * NFI];     // (the last load may bring words of the next thread's run: not committed)
    int wrow[4];             // LDS word of this thread's filter run, one base per word of a 16-byte load
#pragma unroll
    for (int e = 0; e < 4; ++e) wrow[e] = we0 * LDK + wkl + e * LDK;
    // Staging item w < NII is a piece of four image words, item NII + q a filter load (one word,
    // or four).  Image pieces start at any 4-byte boundary of HBM; the words of a piece that lie
    // beyond the end of the input read as zero one by one, those beyond the end of an image row
    // are the head of the next row and land in columns that no valid pixel reads.
    // A thread whose filter lies beyond K has offsets beyond the end of the filter bank.  A
    // run may reach past the chunk's reduction indices (into the next row group, channel or
    // filter): those words land in rows of the filter block that no step reads.
    auto fetch_item = [&](int w) __attribute__((always_inline)) {
        if (w < NII) {
            // (the whole 16 bytes are reinterpreted at once: converting the builtin's result
            // element by element through another vector type drops all but the first word)
            const v4f v = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(irs, ig[w], 0, 0));
#pragma unroll
            for (int e = 0; e < 4; ++e) ireg[4 * w + e] = v[e];
        } else {
            const int q = w - NII;
            const v4f v = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(wrs, wofs + 16u * q, 0, 0));
#pragma unroll
            for (int e = 0; e < 4; ++e) wreg[4 * q + e] = v[e];
        }
    };
    auto commit_item = [&](int w, float* slot) __attribute__((always_inline)) {
        if (w < NII) {
            const int e = 4 * (tid + w * kThreads);
            *reinterpret_cast<v4f*>(slot + (e < img_words ? IOFF + e : trash_word)) =
                (v4f){ireg[4 * w], ireg[4 * w + 1], ireg[4 * w + 2], ireg[4 * w + 3]};
        } else {
            const int q = w - NII;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (4 * q + e < EPT) slot[wrow[e] + 4 * q * LDK] = wreg[4 * q + e];
        }
    };

    // ---- the compute side: where this lane's pixels sit in LDS and in the output --------------
    int base[NW];            // LDS word (within a slot) of tap (0,0,0) of the lane's pixel
    uint32_t oofs[NW];       // byte offset of out[n][k0 + 32*wm*MW + 4*h][y][x] from out[n_first][k0][0][0]
    bool valid[NW];
    int kleft = 0;           // filters from k0 + 32*wm*MW + 4*h to K
    float* obase_t = p.out;  // out[n_first][k0][0][0]
    auto setup_compute = [&](int tile) __attribute__((always_inline)) {
        const int strip = min(fdiv(tile, p.d_strip), p.nstrips - 1);
        const int rem = tile - strip * per_strip;
        const int ptile = fdiv(rem, p.d_kb), kb = rem - ptile * p.KB;
        const int x0 = strip * p.bw;
        const int ws = min(p.bw, p.Wo - x0);
        const bool last_strip = strip == p.nstrips - 1;
        const FastDiv d_ws{last_strip ? p.d_wsl.m : p.d_wsf.m, last_strip ? p.d_wsl.sh : p.d_wsf.sh, ws};
        const int total_p = p.N * p.Ho * ws;
        const int p0 = ptile * NT;
        const int Q0 = fdiv(p0, d_ws);
        const int n_first = fdiv(Q0, p.d_ho);
        const int y_first = Q0 - n_first * p.Ho;
        const int k0 = kb * MT;
        kleft = p.K - k0 - 32 * wm * MW - 4 * h;
        obase_t = p.out + ((int64_t)n_first * p.K + k0) * plane;
        // one image of the output, in words.  The host checks that everything a lane adds to its
        // tile's base fits 32 bits; where a tile cannot reach a second image this product may
        // not fit and is multiplied by zero.
        const uint32_t kplane = (uint32_t)p.K * (uint32_t)plane;
#pragma unroll
        for (int nt = 0; nt < NW; ++nt) {
            const int pp = p0 + (wn * NW + nt) * 32 + l32;
            valid[nt] = pp < total_p;
            const int pc = valid[nt] ? pp : total_p - 1;
            const int Q = fdiv(pc, d_ws), xl = pc - Q * ws;
            const int n = fdiv(Q, p.d_ho), y = Q - n * p.Ho;
            base[nt] = IOFF + ((n - n_first) * p.Hc + y - y_first) * LS + xl;
            oofs[nt] = ((uint32_t)(n - n_first) * kplane +
                        (uint32_t)((32 * wm * MW + 4 * h) * (int)plane + y * p.Wo + x0 + xl)) * 4u;
        }
    };
    // Offsets of the second tap of a pair relative to the first, by kind of pair.
    const int dX = h;                                         // next column, same row
    const int dY = h * (LS - (F - 1));                        // first column of the next row
    const int dZ = h * (PL - (RG - 1) * LS - (F - 1));        // first tap of the next channel
    // One LDS base per filter block of the wave and (below) per word of a 16-byte filter run,
    // each made opaque to the compiler once per chunk: reads and writes that share a base get
    // paired into two-address LDS instructions whose short offset fields then need a vector
    // add per pair; with a base of their own they keep full-range immediate offsets.
    int wb[MW];
#pragma unroll
    for (int mt = 0; mt < MW; ++mt) wb[mt] = h * LDK + wm * (MW * 32) + l32 + mt * 32;
    // operands of step s of the chunk in `slot`; bb: the lane's pixels at the group's first row;
    // shortg: the chunk is a last row group with fewer rows (its odd tap count is padded here)
    auto load_ops = [&](int s, const float* slot, const int (&bb)[NW], bool shortg, float (&a)[MW],
                        float (&b)[NW]) __attribute__((always_inline)) {
        const int t0 = 2 * s, t1 = 2 * s + 1;
        const int c = tap_c<F, RG>(t0), i = tap_i<F, RG>(t0), jj = tap_j<F, RG>(t0);
        const int rowoff = c * PL + i * LS;
#pragma unroll
        for (int nt = 0; nt < NW; ++nt) {
            int addr;
            if (t1 >= T)                                              // pad: second tap reads 0
                addr = h ? zero_word : bb[nt] + rowoff + jj;
            else if (tap_c<F, RG>(t1) != c) addr = bb[nt] + dZ + rowoff + jj;
            else if (tap_i<F, RG>(t1) != i) addr = bb[nt] + dY + rowoff + jj;
            else                            addr = bb[nt] + dX + rowoff + jj;
            if (TL != T && (TL & 1) && t1 == TL) addr = (shortg && h) ? zero_word : addr;
            b[nt] = slot[addr];
        }
        // the second tap of a padded pair takes a zero weight as well as a zero pixel: whatever
        // follows the chunk's last weight (another filter's, possibly not finite) stays out
        const bool pad = t1 >= T;
        const bool pad_short = TL != T && (TL & 1) && t1 == TL;
#pragma unroll
        for (int mt = 0; mt < MW; ++mt) {
            int addr = wb[mt] + t0 * LDK;
            if (pad) addr = h ? zero_word : addr;
            if (pad_short) addr = (shortg && h) ? zero_word : addr;
            a[mt] = slot[addr];
        }
    };

    v16f acc[MW][NW];
    auto zero_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int mt = 0; mt < MW; ++mt)
#pragma unroll
            for (int nt = 0; nt < NW; ++nt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0.f;
    };
    // 32 lanes hold 32 consecutive pixels of one output map
    auto store_out = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int mt = 0; mt < MW; ++mt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int kk = mt * 32 + mfma_row(r, 0);          // filter, from this lane's first one
                char* ob = (char*)(obase_t + kk * plane);          // uniform
#pragma unroll
                for (int nt = 0; nt < NW; ++nt)
                    if (valid[nt] && kk < kleft)
                        *reinterpret_cast<float*>(ob + oofs[nt]) = acc[mt][nt][r];
            }
        }
    };
    // Line-aligned write-back (the reorganisation through on-chip memory that the paper leaves
    // open for this kernel, Sec. 4.2).  HBM runs at full rate only when every 128-byte line is
    // written whole by one store instruction; straight from the accumulators, 32 lanes write 32
    // consecutive pixels of one map, which start anywhere in a line.  Here the tile goes through
    // LDS, GR filters at a time: every wave parks the accumulator registers of those filters
    // (rows of NT pixels, one row per filter), and after a barrier every half-wave takes its
    // share of the rows and stores them line by line: lane l of a half-wave always writes word
    // l of a line.  A tile's pixels are contiguous in memory only within a segment (one image
    // when the strip is the whole row, one row of the strip otherwise); each segment of each
    // filter has its own offset within a line, so only its first and last line may be partial.
    // Two regions alternate, one barrier per group: `r0` is the LDS slot of the chunk consumed
    // last and `r1` the slot that the chunk after next will go to (with two slots: the second
    // half of r0); nobody refills either before the next chunk's barrier.
    constexpr int kWbRows = NBUF == 3 ? (NT == 128 ? 32 : 16) : 8;     // GR
    constexpr int kWbStride = NT + 8;          // row stride: the two halves of a wave on different banks
    auto store_out_aligned = [&](int tile, float* r0, float* r1) __attribute__((always_inline)) {
        static_assert(WM == 1, "every wave holds all the tile's filters");
        constexpr int GR = kWbRows, RSW = kWbStride;
        constexpr int NGRP = MT / GR, RPH = GR / 8;  // groups per tile, rows per half-wave and group
        const int strip = min(fdiv(tile, p.d_strip), p.nstrips - 1);
        const int rem = tile - strip * per_strip;
        const int ptile = fdiv(rem, p.d_kb), kb = rem - ptile * p.KB;
        const int x0 = strip * p.bw;
        const int ws = min(p.bw, p.Wo - x0);
        const bool last_strip = strip == p.nstrips - 1;
        const FastDiv d_ws{last_strip ? p.d_wsl.m : p.d_wsf.m, last_strip ? p.d_wsl.sh : p.d_wsf.sh, ws};
        const int total_p = p.N * p.Ho * ws;
        const int p0 = ptile * NT;
        const int ntv = min(NT, total_p - p0);       // valid pixels of the tile
        const int n_first = fdiv(fdiv(p0, d_ws), p.d_ho);
        const int k0 = kb * MT;
        const uint32_t kplane = (uint32_t)p.K * (uint32_t)plane;
        // (tiny maps would cut the tile into many short segments: not worth the detour)
        if ((p.nstrips == 1 ? p.Ho * ws : ws) < 32) { store_out(); return; }       // uniform
        const int pm = (int)(plane & 31);
        const int abase = (int)(((uintptr_t)obase_t >> 2) & 31);
        const int hw = 2 * wave + h;                 // this half-wave's first filter row within a group
        auto park = [&](int g) __attribute__((always_inline)) {
            float* rg = (g & 1) ? r1 : r0;
#pragma unroll
            for (int q8 = 0; q8 < GR / 8; ++q8) {    // blocks of eight filters: one register quad each
                const int f8 = g * (GR / 8) + q8, mt = f8 / 4, gq = f8 % 4;
#pragma unroll
                for (int jq = 0; jq < 4; ++jq)
#pragma unroll
                    for (int nt = 0; nt < NW; ++nt)
                        rg[(8 * q8 + 4 * h + jq) * RSW + (wn * NW + nt) * 32 + l32] = acc[mt][nt][4 * gq + jq];
            }
        };
        __syncthreads();                             // everyone has consumed the slots' chunks
        park(0);
        // (one copy of the store code: the groups are a run-time loop, and only the parking,
        // which names accumulator registers, is selected group by group)
#pragma unroll 1
        for (int g = 0; g < NGRP; ++g) {
            __syncthreads();                         // group g is parked; group g-1 has been read
#pragma unroll
            for (int c = 1; c < NGRP; ++c)
                if (g + 1 == c) park(c);             // uniform
            const float* rg = (g & 1) ? r1 : r0;
#pragma unroll 1
            for (int rr = 0; rr < RPH; ++rr) {
                const int rowi = hw + 8 * rr;
                const int kk = GR * g + rowi;        // filter, from the tile's first
                const bool kvalid = k0 + kk < p.K;
                float* ob = obase_t + (int64_t)kk * plane;
                const int ak = abase + kk * pm;
                const float* row = rg + rowi * RSW;
                int pix = 0;                         // first pixel of the segment, from p0
                while (pix < ntv) {                  // uniform
                    const int pp = p0 + pix;
                    const int Q = fdiv(pp, d_ws), xl = pp - Q * ws;
                    const int n = fdiv(Q, p.d_ho), y = Q - n * p.Ho;
                    const int seg_end = p.nstrips == 1 ? (n + 1) * p.Ho * ws : (Q + 1) * ws;
                    const int len = min(seg_end, p0 + ntv) - pp;
                    // word offset of the segment's start from out[n_first][k][0][0]
                    const uint32_t oseg = (uint32_t)(n - n_first) * kplane + (uint32_t)(y * p.Wo + x0 + xl);
                    const int shift = (ak + (int)(oseg & 31u)) & 31;   // of that start within a line
                    const int t0 = l32 - shift;      // lane l writes word l of each line
                    float* dst = ob + oseg + t0;
                    const float* src = row + pix + t0;
                    const int nlines = (len + 62) >> 5;       // at most: a start at word 31 of a line
#pragma unroll
                    for (int q = 0; q <= NT / 32; ++q) {
                        if (q >= nlines) break;      // uniform
                        const int t = t0 + 32 * q;
                        if (kvalid && (unsigned)t < (unsigned)len) dst[32 * q] = src[32 * q];
                    }
                    pix += len;
                }
            }
        }
        if (NBUF == 2) __syncthreads();              // the slot is refilled right away
    };

    // A partial tile in the workspace: per wave, per block, per accumulator register, one word
    // per lane, so that every store and load is 256 B contiguous per wave.  The words are
    // written and read with device-scope accesses, which pass through the per-XCD L2 to the
    // memory side where all XCDs meet; no cache has to be flushed or invalidated as a whole.
    auto part_ptr = [&](int wg, int which) __attribute__((always_inline)) {
        char* b = (char*)(p.part + ((int64_t)(2 * wg + which)) * (MT * NT) +
                          wave * (MW * NW * 16 * kWave));              // uniform
        return reinterpret_cast<float*>(b + (uint32_t)lane * 4u);
    };
    // The tile whose chunks [.., last] this workgroup has just summed is complete if the
    // workgroup also summed its first chunk; otherwise it is shared with its neighbours.
    auto finish_tile = [&](int tile, bool whole, float* r0, float* r1) __attribute__((always_inline)) {
        auto emit = [&]() __attribute__((always_inline)) {
            if (p.aligned) store_out_aligned(tile, r0, r1);
            else store_out();
        };
        if (whole) { emit(); return; }
        const int t0u = tile * nch;
        const int first = unit_owner(t0u, U, G), last = unit_owner(t0u + nch - 1, U, G);
        const int m = last - first + 1;
        float* mine = part_ptr(j, u0 >= t0u ? 0 : 1);
#pragma unroll
        for (int mt = 0; mt < MW; ++mt)
#pragma unroll
            for (int nt = 0; nt < NW; ++nt)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    __hip_atomic_store(mine + ((mt * NW + nt) * 16 + r) * kWave, acc[mt][nt][r],
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // Every store of this workgroup has to be acknowledged (performed at device scope)
        // before its arrival is counted.  A workgroup-scope fence does not wait for that and a
        // device-scope one would write back the whole L2: each wave waits for its own stores
        // (s_waitcnt vmcnt(0), all other counters left alone), then the workgroup meets.
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();
        if (tid == 0)
            s_old = __hip_atomic_fetch_add(&p.cnt[first], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        const int old = s_old;
        if (old != m - 1) return;            // somebody else arrives later and writes the tile
        if (tid == 0)                        // ready for the next launch
            __hip_atomic_store(&p.cnt[first], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // Sum in the order of the workgroups, whoever does it.  With two parts the sum of this
        // workgroup's registers and the other part is that sum already (addition commutes).
        if (m > 2) zero_acc();
        for (int i = first; i <= last; ++i) {
            if (m == 2 && i == j) continue;
            const float* src = part_ptr(i, range_start(i, U, G) >= t0u ? 0 : 1);
#pragma unroll
            for (int mt = 0; mt < MW; ++mt)
#pragma unroll
                for (int nt = 0; nt < NW; ++nt) {
                    float v[16];
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        v[r] = __hip_atomic_load(src + ((mt * NW + nt) * 16 + r) * kWave,
                                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[mt][nt][r] += v[r];
                    __builtin_amdgcn_sched_barrier(0);   // one block's loads in flight at a time
                }
        }
        emit();
    };

    // ---- prologue: constant LDS words, first unit into slot 0, second unit into registers ------
    for (int b = 0; b < NBUF; ++b)
        if (tid == 0) lds[b * BUF + zero_word] = 0.f;
    int ftile = fdiv(u0, p.d_nch), fchunk = u0 - ftile * nch;   // the unit being requested
    const int ftile_first = ftile;
    setup_fetch(ftile);
    set_chunk(fchunk);
#pragma unroll
    for (int w = 0; w < NI; ++w) fetch_item(w);
    // (the compute-side setup runs while the first loads are on their way)
    int tile = ftile_first, chunk = u0 - tile * nch;       // the unit being consumed
    bool from_first = chunk == 0;                          // this workgroup summed the tile's chunk 0
    setup_compute(tile);
    zero_acc();
#pragma unroll
    for (int w = 0; w < NI; ++w) commit_item(w, lds);
    auto advance_fetch = [&]() __attribute__((always_inline)) {
        if (++fchunk == nch) { fchunk = 0; ++ftile; setup_fetch(ftile); }
        set_chunk(fchunk);
    };
    if (u0 + 1 < u1) advance_fetch();
#pragma unroll
    for (int w = 0; w < NI; ++w) fetch_item(w);           // unit u0+1 (or u0 again: never used)
    __syncthreads();

    auto is_short = [&](int ch) __attribute__((always_inline)) { return TL != T && ch % NG == NG - 1; };
    float a0[MW], b0[NW], a1[MW], b1[NW];
    load_ops(0, lds, base, is_short(chunk), a0, b0);
    int bi = 0;                                            // LDS slot of the unit being consumed

    // ---- main loop: one (tile, chunk) unit per trip --------------------------------------------
    for (int u = u0; u < u1; ++u) {
        const int bn = bi + 1 == NBUF ? 0 : bi + 1;
        const float* cur = lds + bi * BUF;
        float* nxt = lds + bn * BUF;
        const bool has1 = u + 1 < u1, has2 = u + 2 < u1;
        const bool tile_ends = chunk == nch - 1 || !has1;
        // the unit in the registers moves to LDS during this trip; the next one is requested
        if (has2) advance_fetch();
        const bool shortg = is_short(chunk);         // this chunk ends after SL steps
        // keep the tap addresses from being expanded into one register each outside the loop
#pragma unroll
        for (int nt = 0; nt < NW; ++nt) asm volatile("" : "+v"(base[nt]));
#pragma unroll
        for (int mt = 0; mt < MW; ++mt) asm volatile("" : "+v"(wb[mt]));
#pragma unroll
        for (int e = 0; e < 4; ++e) asm volatile("" : "+v"(wrow[e]));
#pragma unroll
        for (int s = 0; s < S; ++s) {
            if (s >= SL && shortg) continue;                 // uniform; compiled away when SL == S
            float (&a)[MW] = (s & 1) ? a1 : a0;
            float (&b)[NW] = (s & 1) ? b1 : b0;
            const bool last_step = s == S - 1 || (s == SL - 1 && shortg);
            // Operands of step s+1 are requested from LDS before the matrix-core instructions
            // of step s are issued, so a wave never waits for LDS with the matrix pipe idle.
            if (!last_step) load_ops(s + 1, cur, base, shortg, (s & 1) ? a0 : a1, (s & 1) ? b0 : b1);
            else if (NBUF == 3 && !tile_ends)
                load_ops(0, nxt, base, is_short(chunk + 1), (s & 1) ? a0 : a1, (s & 1) ? b0 : b1);
            if (s < NS) {
#pragma unroll
                for (int q = 0; q < IPS; ++q)
                    if (s * IPS + q < NI) {
                        commit_item(s * IPS + q, nxt);
                        fetch_item(s * IPS + q);
                    }
            }
            // unit u+1 is complete in LDS two steps before the chunk's end
            if (NBUF == 3 && (s == S - 2 || s == SL - 2) && (s == S - 2) != shortg) __syncthreads();
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mt = 0; mt < MW; ++mt)
#pragma unroll
                for (int nt = 0; nt < NW; ++nt)
                    acc[mt][nt] = mfma_32x32x2(a[mt], b[nt], acc[mt][nt]);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (NBUF == 2) __syncthreads();      // unit u+1 is in LDS; everyone is done with unit u

        if (tile_ends) {
            finish_tile(tile, from_first && chunk == nch - 1, lds + bi * BUF,
                        NBUF == 3 ? lds + (bi == 0 ? 2 : bi - 1) * BUF : lds + bi * BUF + kWbRows * kWbStride);
            if (has1) {
                ++tile; chunk = 0; from_first = true;
                setup_compute(tile);
                zero_acc();
                load_ops(0, nxt, base, is_short(0), a0, b0);
            }
        } else {
            ++chunk;
            if (NBUF == 2) load_ops(0, nxt, base, is_short(chunk), a0, b0);
            else if (((shortg ? SL : S) & 1) != 0) {   // the operands requested across the chunk end
#pragma unroll
                for (int mt = 0; mt < MW; ++mt) a0[mt] = a1[mt];
#pragma unroll
                for (int nt = 0; nt < NW; ++nt) b0[nt] = b1[nt];
            }
        }
        bi = bn;
    }
}

// ---- host side: one instantiation -------------------------------------------------------------

struct GenPlan {
    int bw, nstrips, LS, RS, pt_full, pt_last;
    bool ok;
};

// Column strips and LDS image-block geometry for tiles of NT pixels: the widest strips (at
// most 128 columns) whose image block of CSH channels a workgroup can stage with `imax`
// words per thread (with `widest_only`, the widest strips or nothing).
inline GenPlan make_gen_plan(const Shape& s, int NT, int CSH, int imax, int rg, bool widest_only)
{
    GenPlan pl{};
    const int first = (s.Wo + 127) / 128;
    for (int nstrips = first; nstrips <= (widest_only ? first : s.Wo); ++nstrips) {
        pl.bw = (s.Wo + nstrips - 1) / nstrips;
        pl.nstrips = (s.Wo + pl.bw - 1) / pl.bw;
        pl.LS = (pl.bw + s.F - 1 + 3) & ~3;      // whole 16-byte pieces per row
        // A run of NT consecutive strip pixels touches at most this many output rows, taken
        // over every strip width from the narrowest (the last strip) to bw ...
        const int wmin = s.Wo - (pl.nstrips - 1) * pl.bw;
        const int64_t all_rows = (int64_t)s.N * s.Ho;          // (there are no more than these)
        const int rows = (int)std::min<int64_t>(NT >= 2 ? (NT - 2) / wmin + 2 : 1, all_rows);
        // ... and crosses at most this many image boundaries; every image it touches adds the
        // rg-1 further input rows that a group of rg filter rows reaches below an output row.
        const int cross = std::min(rows >= 2 ? (rows - 2) / s.Ho + 1 : 0, s.N - 1);
        pl.RS = rows + (rg - 1) * (cross + 1);
        pl.pt_full = (int)(((int64_t)s.N * s.Ho * pl.bw + NT - 1) / NT);
        pl.pt_last = (int)(((int64_t)s.N * s.Ho * wmin + NT - 1) / NT);
        if ((int64_t)CSH * pl.RS * pl.LS <= (int64_t)imax * kThreads) { pl.ok = true; return pl; }
    }
    pl.ok = false;
    return pl;
}

// How a launch cuts the work; filled in by the dispatcher.
struct GenSched {
    int mode;          // 0: decide by shape, 1: whole tiles only, 2: cut inside tiles
    int force_G;       // > 0: this many workgroups (tests), 0: what the chip holds
    bool widest_only;  // refuse shapes whose image block needs narrower column strips
    bool static_ws;    // shared tiles meet in the library's static device array: nothing is allocated
    int wb;            // write-back: 0 by shape, 1 straight from the accumulators, 2 in whole lines through LDS
};

// Workspace of one (device, stream): grown on demand by the dispatcher.
struct GenWorkspace {
    float* part;
    int* cnt;
};
// Returns a workspace with room for `part_floats` floats of partial sums and `ncnt` counters,
// or nullptr members on allocation failure.
GenWorkspace gen_workspace(hipStream_t st, size_t part_floats, size_t ncnt);
// The same room inside the static device array of the current device, its counters cleared on
// `st` by a small kernel.  Allocates nothing.  Returns a dconv_status: DCONV_SCRATCH_EXCEEDED if
// the array is too small for the request.
int gen_static_workspace(hipStream_t st, size_t part_floats, size_t ncnt, GenWorkspace* ws);

constexpr int kGenLdsLimit = 160 * 1024 - 256;     // dynamic LDS; the rest is for the static word

template <int F, int CSH, int RG, int MW, int NW, int WM, int WN, int IMAX, int NBUF, int OCC>
int gen_try_launch(const float* in, const float* filt, float* out, const Shape& s, hipStream_t st,
                   const GenSched& sched, bool dry)
{
    using Gm = GenGeom<F, CSH, RG, MW, NW, WM, WN, IMAX, NBUF, OCC>;
    constexpr int MT = Gm::MT, NT = Gm::NT, TP = Gm::TP, LDK = Gm::LDK;
    const GenPlan pl = make_gen_plan(s, NT, CSH, IMAX, RG, sched.widest_only);
    if (!pl.ok) return DCONV_UNSUPPORTED;
    const int64_t img_words = (int64_t)CSH * pl.RS * pl.LS;
    // The line-aligned write-back parks a tile in the LDS slots that are free when a tile ends,
    // some filter rows of NT + 8 words at a time in two alternating regions; a slot too small
    // for a region (for both, where there are only two slots) is padded.  It runs only when asked
    // for: measured, it never beats the stores straight from the accumulators (see the
    // dispatcher).
    const bool want_aligned = sched.wb == 2;
    constexpr int kWbWords = (NBUF == 3 ? (NT == 128 ? 32 : 16) : 16) * (NT + 8);   // see store_out_aligned
    int64_t pad_words = want_aligned ? std::max<int64_t>(0, kWbWords - (Gm::IOFF + img_words)) : 0;
    pad_words = (pad_words + 3) & ~(int64_t)3;
    if (NBUF * 4 * (Gm::IOFF + img_words + pad_words + 8) > kGenLdsLimit) {
        if (sched.wb == 2 && NBUF * 4 * (Gm::IOFF + img_words + 8) <= kGenLdsLimit) return DCONV_UNSUPPORTED;
        pad_words = 0;
    }
    const int aligned = want_aligned && kWbWords <= Gm::IOFF + img_words + pad_words ? 1 : 0;
    const int64_t buf_words = Gm::IOFF + img_words + pad_words + 8;
    const int64_t lds_bytes = NBUF * 4 * buf_words;
    if (lds_bytes > kGenLdsLimit) return DCONV_UNSUPPORTED;
    const int KB = (s.K + MT - 1) / MT;
    if (s.C % CSH != 0) return DCONV_UNSUPPORTED;
    const int nch = s.C / CSH * Gm::NG;
    const int64_t tiles = ((int64_t)(pl.nstrips - 1) * pl.pt_full + pl.pt_last) * KB;
    if (tiles * nch > 2147483647LL || (int64_t)s.N * s.Ho * s.Wo > 2147483647LL)
        return DCONV_UNSUPPORTED;
    // Lanes address HBM with 32-bit byte offsets from per-tile bases (the first image of the
    // tile, the chunk's first channel, the tile's first filter; the filter a store belongs to is
    // in its uniform base): what a lane adds to them must stay below 2 GiB.  A tile of NT pixels
    // reaches into at most `span` images.
    {
        const int wmin = s.Wo - (pl.nstrips - 1) * pl.bw;
        const int64_t span = std::min<int64_t>(NT / ((int64_t)s.Ho * wmin) + 2, s.N);
        const int64_t plane = (int64_t)s.Ho * s.Wo;
        const int64_t lim = 1LL << 29;                                // floats: 2 GiB
        if (((span - 1) * s.C + CSH + 1) * s.H * s.W >= lim ||
            (span - 1) * s.K * plane + (32 * (WM - 1) * MW + 6) * plane >= lim ||
            (int64_t)MT * s.C * F * F >= lim)
            return DCONV_UNSUPPORTED;
    }
    if (dry) return DCONV_OK;

    auto kern = general_tiled_kernel<F, CSH, RG, MW, NW, WM, WN, IMAX, NBUF, OCC>;
    // Workgroups the chip holds at once for this LDS size (at most OCC per CU are used): cached
    // per instantiation for the last (device, LDS size) seen, key and count in one atomic word,
    // so that threads calling with different shapes can only repeat the query.
    static std::atomic<uint64_t> lds_limit_raised{0};
    static std::atomic<uint64_t> cached{0};        // device + 1 (8 bits) | LDS bytes (24) | per CU (8) | count (24)
    if (!raise_lds_limit((const void*)kern, kGenLdsLimit, lds_limit_raised)) return DCONV_LAUNCH_FAILED;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return DCONV_LAUNCH_FAILED;
    const uint64_t key = ((uint64_t)((dev & 0xFF) + 1) << 56) | ((uint64_t)lds_bytes << 32);
    uint64_t seen = cached.load(std::memory_order_relaxed);
    if ((seen & ~0xFFFFFFFFull) != key) {
        int cus = 0, per_cu = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)kern, kThreads,
                                                         (size_t)lds_bytes) != hipSuccess ||
            cus <= 0 || per_cu <= 0)
            return DCONV_LAUNCH_FAILED;
        const int occ = per_cu > OCC ? OCC : per_cu;
        if (cus * occ >= (1 << 24)) return DCONV_LAUNCH_FAILED;
        seen = key | ((uint32_t)occ << 24) | (uint32_t)(cus * occ);
        cached.store(seen, std::memory_order_relaxed);
    }
    const int chip = (int)((uint32_t)seen & 0xFFFFFFu);
    const int cus = chip / (int)(((uint32_t)seen >> 24) & 0xFFu);

    // Whole tiles when they spread evenly enough, otherwise cut inside tiles.
    int G, split;
    if (sched.mode == 1) split = 0;
    else if (sched.mode == 2) split = 1;
    else {
        // ... when a last round would leave much of the chip idle and a tile is long enough
        // (about 60 us with the workgroups of a CU sharing its matrix cores) for the saving to
        // outweigh the cost of meeting in the workspace; or, with shorter tiles in two rounds
        // or more, when the time the last round leaves the chip idle (its empty part times a
        // tile's time) exceeds that cost (some 12 us).  64 images of 14 x 14 with 512 channels
        // and 512 1x1 filters: 784 tiles of 41 us on 768 slots, 96 us whole, 74 us shared.
        const int64_t rounds = (tiles + chip - 1) / chip;
        const double tile_us = (double)nch * Gm::S * (MW * NW) * 64.0 * OCC / 2400.0;
        const double idle_us = ((double)rounds - (double)tiles / (double)chip) * tile_us;
        const bool long_tiles = tile_us >= 60.0 && (double)tiles < 0.93 * (double)(rounds * chip);
        const bool idle_round = rounds >= 2 && tile_us >= 20.0 && idle_us >= 12.0;
        split = (nch >= 2 && tiles < 8LL * chip && (long_tiles || idle_round)) ? 1 : 0;
    }
    int64_t U = split ? tiles * nch : tiles;
    G = sched.force_G > 0 ? sched.force_G : chip;
    if (G > U) G = (int)U;
    // Fewer tiles than CUs (small batches of deep layers): how many workgroups share the tiles
    // is a trade.  The workgroup that completes a shared tile adds all its parts by itself, one
    // part after the other (`part_us` each, a round trip to the memory side per block), while the
    // matrix-core work per workgroup falls with their number only up to one per CU: beyond, the
    // workgroups of a CU share its matrix cores and gain what latency hiding gives (`eff`).
    // time(G) = units per workgroup x time per unit x workgroups per CU / eff + parts x part_us,
    // fitted to sweeps over the parts per tile on sixteen layers (1 to 16 images of 7 x 7 to
    // 96 x 96, 128 to 2048 channels, 1x1 to 7x7: within 10 % rms).  One image of 20 x 20 with
    // 384 channels and 384 filters of 7x7: 134 -> 82 us; 4 of 17 x 14, 512 channels, 448 1x1
    // filters: 33 -> 18 us.
    if (sched.mode == 0 && sched.force_G <= 0 && nch >= 2 && 4 * tiles < 3LL * cus) {
        constexpr bool kBig = MW * NW >= 4;
        const double eff[4] = {1.0, kBig ? 0.70 : 0.60, kBig ? 0.70 : 0.75, 0.80};
        const double part_us = kBig ? 1.4 : 0.8;
        const double unit_us = (double)Gm::S * (MW * NW) * 64.0 / 2400.0;
        auto per_cu = [&](int64_t g) { return (int)std::min<int64_t>((g + cus - 1) / cus, 3); };
        const int o_whole = per_cu(tiles);
        const double whole = (double)nch * unit_us * o_whole / eff[o_whole];   // one round of tiles
        double best = 1e30;
        int64_t best_g = 0;
        auto consider = [&](int64_t g) {
            g = std::min<int64_t>(std::min<int64_t>(g, chip), tiles * nch);
            if (g <= tiles) return;
            const int o = per_cu(g);
            const double t = (double)(tiles * nch) / (double)g * unit_us * o / eff[o] +
                             part_us * ((double)g / (double)tiles + 1.0);
            if (t < best) { best = t; best_g = g; }
        };
        for (int parts = 2; parts <= 32; ++parts) consider(parts * tiles);
        for (int k = 1; k <= 6; ++k) consider((int64_t)k * cus / 2);
        // (shared only for a tenth or more: the model knows nothing of the cost of a workgroup's
        // passing from one tile to the next; and only for three microseconds or more: with a
        // few short chunks per tile the launch, the first loads and the write-back are most of
        // the kernel's time and sharing adds to them -- kernel times from replayed graphs,
        // 4 x 128 x 56 x 56 with 64 1x1 filters: 20.7 us shared, 13.2 us whole; where the model
        // promises 4.5 us or more, sharing is 25-85 % faster)
        if (best < 0.9 * whole && whole - best >= 3.0) { split = 1; U = tiles * nch; G = (int)best_g; }
        else { split = 0; U = tiles; G = (int)tiles; }
    }

    GenWorkspace ws{nullptr, nullptr};
    if (split && sched.static_ws) {
        const int rc = gen_static_workspace(st, (size_t)G * 2 * MT * NT, (size_t)G, &ws);
        if (rc != DCONV_OK) return rc;
    } else if (split) {
        ws = gen_workspace(st, (size_t)G * 2 * MT * NT, (size_t)G);
        if (!ws.part || !ws.cnt) return DCONV_LAUNCH_FAILED;
    }
    GenParams p{in, filt, out, ws.part, ws.cnt, s.N, s.C, s.H, s.W, s.K, s.Ho, s.Wo,
                pl.bw, pl.nstrips, pl.LS, pl.RS, pl.pt_full, KB, nch, (int)tiles, G, split, aligned, (int)pad_words,
                make_fastdiv(pl.pt_full * KB), make_fastdiv(KB), make_fastdiv(pl.bw),
                make_fastdiv(s.Wo - (pl.nstrips - 1) * pl.bw), make_fastdiv(s.Ho), make_fastdiv(s.Ho + RG - 1),
                make_fastdiv(nch), s.Ho + RG - 1};
    begin_launch();
    hipLaunchKernelGGL(kern, dim3((unsigned)G), dim3(kThreads), (size_t)lds_bytes, st, p);
    return launch_status();
}

// Implemented once per filter side, each in its own translation unit.
template <int F>
int gen_launch_for_F(const float* in, const float* filt, float* out, const Shape& s, hipStream_t st,
                     int tile_cfg, const GenSched& sched, bool dry);

}  // namespace dconv
