// General-case direct convolution for 16-bit inputs (fp16 / bf16) with fp32 accumulation,
// gfx950: the paper's closing remark (Sec. 6) that its model -- match the width of what a
// thread reads from on-chip memory to the width of a bank -- carries over to short data types,
// worked out for CDNA4.
//
// LDS banks are 4 bytes wide, so a lane that read one 2-byte pixel per access would use half
// of every bank cycle and the matrix cores want whole runs of the reduction index per lane
// anyway: v_mfma_f32_32x32x16_{f16,bf16} takes EIGHT consecutive reduction indices per lane
// (16 bytes) for each operand.  The unit that is packed is the CHANNEL run: with channels
// innermost in memory (in[N][H][W][C], filt[K][F][F][C]) the sixteen channels of one pixel are
// 32 contiguous bytes in HBM and in LDS, a lane reads its eight with one 16-byte LDS access at
// any tap offset, and one matrix-core step consumes one tap of sixteen channels.  The rest is
// Algorithm 2 as in the fp32 kernel: (filter block) x (pixel block) tiles, channel chunks
// staged in LDS with the next chunk prefetched into registers during the arithmetic (the
// paper's double buffering, Sec. 4.3), the image block kept as it lies in memory and read at
// shifted addresses.  No transposition is needed on the way into LDS: both blocks are copied
// in 16-byte pieces, pixel after pixel and tap after tap.  What bounds the kernel on chip is
// what the paper names for its general case (Sec. 4.3): the bandwidth of the on-chip memory,
// 16 bytes per lane, operand and matrix-core instruction.
//
//  * tile: 64 filters x 256 output pixels, four waves side by side, each 64 filters x 64
//    pixels = 2 x 2 matrix-core blocks (or 128 x 512 with eight waves of 2 x 4 blocks, see
//    HalfTile); pixels are numbered along (n, y, x) of a column strip as in the fp32 kernel,
//    so narrow maps lose no lanes;
//  * chunk: sixteen channels x RG filter rows; one step per tap (i, j) of the group; the image
//    block of a chunk holds only the input rows its row group touches;
//  * loads go through range-checked buffer descriptors (zero beyond the extent: filters beyond
//    K, rows beyond the batch), so no lane tests anything.
//
// The channel count must be a multiple of sixteen and both inputs 16-byte aligned; other
// shapes run on a plain one-thread-per-output kernel.
//
// The same kernel serves 8-bit integers (v_mfma_i32_32x32x32_i8: sixteen bytes per lane are
// sixteen channels, a pixel's 32-byte run is 32 channels, sums are exact in int32): only the
// element size, the channels per chunk and the matrix-core instruction differ.
#pragma once
#include <algorithm>
#include "common.h"
#include "general_kernel.h"
#include "../../include/dconv.h"

namespace dconv {

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef __bf16 v8b __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// element types of the short-data-type kernels (the values of DCONV_DTYPE_*)
enum : int { kF16 = 0, kBF16 = 1, kI8 = 2 };
constexpr int elem_bytes(int dt) { return dt == kI8 ? 1 : 2; }

// D(32x32) += A(32 x 16 bytes' worth) * B(the same x 32): 16-bit in with fp32 accumulation, or
// 8-bit integers with int32 accumulation (the accumulator registers then hold integers; they
// are only ever moved, never added to outside the matrix cores).  Lane l holds the sixteen
// bytes of reduction indices of half l / 32 of row (A) / column (B) l % 32; D is laid out as
// for mfma_32x32x2.
template <int DT>
__device__ __forceinline__ v16f mfma_16B(v4f a, v4f b, v16f acc) {
    if (DT == kI8)
        return __builtin_bit_cast(v16f, __builtin_amdgcn_mfma_i32_32x32x32_i8(
            __builtin_bit_cast(v4i, a), __builtin_bit_cast(v4i, b), __builtin_bit_cast(v16i, acc), 0, 0, 0));
    if (DT == kBF16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8b, a),
                                                       __builtin_bit_cast(v8b, b), acc, 0, 0, 0);
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, a),
                                                  __builtin_bit_cast(v8h, b), acc, 0, 0, 0);
}

struct HalfParams {
    const char* in;      // [N][H][W][C], 2-byte or 1-byte elements
    const char* filt;    // [K][F][F][C]
    float* out;          // [N][K][Ho][Wo], fp32 (int32 bit patterns for 8-bit inputs)
    int N, C, H, W, K, Ho, Wo;
    int bw;              // width of a column strip of the output (the last strip may be narrower)
    int nstrips;
    int LS;              // pixels per row of the image block: bw + F - 1
    int RS;              // rows of the image block
    int pt_full;         // pixel tiles in a full-width strip
    int KB;              // filter tiles
    int tiles;           // ((nstrips - 1) * pt_full + pt_last) * KB
    int per_xcd;         // tiles per XCD (grid = 8 * per_xcd)
    int Hc;              // image-block rows set aside per image: Ho + RG - 1
    // Layout of the inputs in bytes.  Channels last ([N][H][W][C], [K][F][F][C]): pixels and taps
    // are a whole channel run apart, channel groups 32 bytes.  Channel-blocked
    // ([N][C/cb][H][W][cb], [K][C/cb][F][F][cb] with cb = 32 bytes' worth of channels): pixels
    // and taps are 32 bytes apart, channel groups a whole plane / filter-group.
    int ps, gs;          // image: pixel stride, channel-group stride
    int ts, fgs;         // filters: tap stride, channel-group stride
    FastDiv d_strip;     // by pt_full * KB
    FastDiv d_kb;        // by KB
    FastDiv d_wsf;       // by bw
    FastDiv d_wsl;       // by the width of the last strip
    FastDiv d_ho;        // by Ho
    FastDiv d_hc;        // by Hc
    FastDiv d_ls;        // by LS
};

constexpr int kHalfChunkBytes = 32;            // bytes of a pixel's channel run per chunk: one step
// Filter rows per chunk: 7 to 12 matrix-core steps per chunk where the filter allows it (a step
// is one tap of a 32-byte channel run); the filter block of a chunk is 2 KiB per step and 64 filters.
constexpr int half_row_group(int F) { return F <= 3 ? F : F <= 6 ? 2 : 1; }

// Tile shapes: WM x WN waves per workgroup, each with MW x NW matrix-core blocks; NII: 16-byte
// image pieces a thread stages per chunk, at most.
//   small: 64 filters x 256 pixels, four waves side by side with 2 x 2 blocks each
//   large: 128 filters x 512 pixels, 2 x 4 waves with 2 x 4 blocks each: a quarter fewer LDS
//          operand reads per matrix-core instruction (six per eight instead of four per four),
//          half the staging per instruction, chunks twice as long; 512 threads, one workgroup
//          per CU
template <int MW_, int NW_, int WM_, int WN_, int NII_>
struct HalfTile {
    static constexpr int MW = MW_, NW = NW_, WM = WM_, WN = WN_, NII = NII_;
    static constexpr int THREADS = kWave * WM * WN;
    static constexpr int MT = 32 * MW * WM, NT = 32 * NW * WN;
};
//   mid:   128 filters x 384 pixels, 2 x 4 waves with 2 x 3 blocks each: the large tile with a
//          quarter fewer pixels, for shapes whose large tiles would leave a third of the CUs
//          without one (five operand reads per six instructions)
using HalfTileSmall = HalfTile<2, 2, 1, 4, 6>;
using HalfTileLarge = HalfTile<2, 4, 2, 4, 4>;
using HalfTileMid = HalfTile<2, 3, 2, 4, 4>;

// RG: filter rows per chunk (the last group of a filter may be shorter).
// DIRECT: how a chunk travels from HBM to LDS.
//   true:  16-byte buffer loads with the LDS bit set: lane l of a wave writes piece l of the 64
//          consecutive LDS pieces the instruction is given, whatever HBM offset the lane asks
//          for (out-of-range lanes write zeros).  A staged chunk never sits in registers, the
//          requests are spread over the steps of the previous chunk and have all of it to
//          arrive.  Consecutive lanes must then bring consecutive pieces of an LDS plane, i.e.
//          the same 16-byte half of consecutive pixels (or filters): in HBM that is 16 bytes out
//          of every pixel's run.
//   false: through registers (requested when the previous chunk begins, written to LDS during
//          the second half of its steps).  Lanes 2q and 2q+1 bring the two halves of pixel q,
//          32 contiguous bytes in HBM: half as many memory lines per load instruction, which
//          is what bounds the staging of the small tile when a pixel's channel run is long
//          (channels-last layout; measured: 25-35 % faster there than DIRECT).
template <int F, int RG, int DT, class TL, bool DIRECT>
__global__ void __launch_bounds__(TL::THREADS, 2)
general_half_kernel(HalfParams p)
{
    constexpr int THREADS = TL::THREADS;
    constexpr int CK = kHalfChunkBytes / elem_bytes(DT);    // channels per chunk
    constexpr int NG = (F + RG - 1) / RG, RGL = F - (NG - 1) * RG;
    constexpr int S = RG * F, SL = RGL * F;             // steps of a chunk / of a last-group chunk
    constexpr int MW = TL::MW, NW = TL::NW, WN = TL::WN, MT = TL::MT, NT = TL::NT;
    constexpr int FPIECES = S * MT * 2;                 // 16-byte pieces of the filter block
    constexpr int NFI = (FPIECES + THREADS - 1) / THREADS;
    constexpr int NII = TL::NII;
    constexpr int FB = FPIECES * 4;                     // words of the filter block
    constexpr uint32_t kNowhere = 0xC0000000u;          // beyond every extent (at most 2^31)
    constexpr int kRsrcFlags = 0x00020000;

    extern __shared__ __attribute__((aligned(16))) float lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, l32 = lane & 31;
    const int wm = wave / WN, wn = wave % WN;

    // each XCD (workgroups go to the eight of them round-robin) gets a contiguous run of tiles
    const int tile = (int)(blockIdx.x % 8) * p.per_xcd + (int)(blockIdx.x / 8);
    if (tile >= p.tiles) return;                        // uniform: before any barrier

    const int LS = p.LS;
    // In LDS the two 16-byte halves of a 32-byte channel run lie in two planes, so that the 32
    // lanes of a half-wave (all of one half: that is the matrix-core operand layout) read 512
    // contiguous bytes instead of every other 16-byte piece, which would use half the banks:
    // image block [half][row][col] x 16 B, filter block [tap][half][filter] x 16 B.
    const int img_plane = p.RS * LS;                    // pieces per plane of the image block
    const int img_pieces = 2 * img_plane;
    // words per LDS slot: filter block, image block (DIRECT: rounded up to whole waves of pieces)
    const int SLOT = FB + 4 * (DIRECT ? (img_pieces + 63) & ~63 : img_pieces);
    const int64_t plane = (int64_t)p.Ho * p.Wo;
    const int CB = p.C * elem_bytes(DT);                // bytes per pixel (all channels)

    // ---- where the tile lies -------------------------------------------------------------------
    const int per_strip = p.pt_full * p.KB;
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
    const int Ql = fdiv(min(p0 + NT, total_p) - 1, d_ws);
    const int nl = fdiv(Ql, p.d_ho);
    // block row (n - n_first) * Hc + (y - y_first) + i holds input row y + (group's first filter
    // row) + i of image n; the group's shift goes into the chunk's buffer base
    const int nslots = (nl - n_first) * p.Hc + (Ql - nl * p.Ho) - y_first + RG;
    const int k0 = kb * MT;

    // ---- staging: thread tid brings pieces tid + it * THREADS of each block; their byte offsets
    // in HBM are the same for every chunk.  Piece e is (half, pixel) = (e / img_plane,
    // e % img_plane) of the image block and (tap, half, filter) in that order of the filter block
    // when DIRECT -- the order of the pieces in LDS -- and (pixel e / 2, half e % 2), (tap,
    // filter, half) otherwise -- their order in HBM.
    uint32_t ig[NII];        // from in[n_first][0][0][0] (+ chunk shift), or kNowhere
#pragma unroll
    for (int it = 0; it < NII; ++it) {
        const int e = tid + it * THREADS;
        uint32_t g = kNowhere;
        if (e < img_pieces) {
            const int half = DIRECT ? (e >= img_plane ? 1 : 0) : (e & 1);
            const int pix = DIRECT ? e - half * img_plane : e >> 1;
            const int row = fdiv(pix, p.d_ls), col = pix - row * LS;
            const int dn = fdiv(y_first + row, p.d_hc);
            const int yy = y_first + row - dn * p.Hc;
            if (row < nslots && n_first + dn < p.N && x0 + col < p.W)
                g = (uint32_t)(dn * (p.H * p.W * CB) + (yy * p.W + x0 + col) * p.ps + half * 16);
        }
        ig[it] = g;
    }
    static_assert(THREADS % (2 * MT) == 0, "a thread's filter pieces differ by whole taps");
    uint32_t wg[NFI];        // from filt[k0][group's first row][0][0] (+ channel shift)
#pragma unroll
    for (int it = 0; it < NFI; ++it) {
        const int e = tid + it * THREADS;
        const int t = e / (2 * MT);
        const int half = DIRECT ? (e / MT) & 1 : e & 1, k = DIRECT ? e % MT : (e >> 1) % MT;
        // (filters beyond K lie beyond the end of the bank: the range check returns zero)
        wg[it] = e < FPIECES ? (uint32_t)(k * (F * F) * CB + t * p.ts + half * 16) : kNowhere;
    }
    const int64_t in_bytes = (int64_t)p.N * p.H * p.W * CB;
    const int64_t filt_bytes = (int64_t)p.K * (F * F) * CB;
    const int64_t ifirst = (int64_t)n_first * p.H * p.W * CB;
    const int64_t wfirst = (int64_t)k0 * (F * F) * CB;
    const int nch = p.C / CK * NG;

    __amdgpu_buffer_rsrc_t irs, wrs;                    // descriptors of the chunk being fetched
    auto set_chunk = [&](int chunk) __attribute__((always_inline)) {
        const int cidx = chunk / NG, g = chunk - cidx * NG;
        const int64_t ioff = ifirst + (int64_t)g * RG * p.W * p.ps + (int64_t)cidx * p.gs;
        irs = __builtin_amdgcn_make_buffer_rsrc(
            (void*)(p.in + ioff), 0, (int)min(in_bytes - ioff, (int64_t)0x7FFFFFFF), kRsrcFlags);
        const int64_t woff = wfirst + (int64_t)g * (RG * F) * p.ts + (int64_t)cidx * p.fgs;
        wrs = __builtin_amdgcn_make_buffer_rsrc(
            (void*)(p.filt + woff), 0, (int)min(filt_bytes - woff, (int64_t)0x7FFFFFFF), kRsrcFlags);
    };
    // staging item k < NII is an image piece, item NII + q a filter piece
    constexpr int NI = NII + NFI;

    // DIRECT.  A wave skips the items that lie wholly beyond a block (uniform); the last wave of
    // the image block may write zeros into the padding behind it.  Inside a chunk item k is
    // requested at step k * kSpread / NI.  The large tile spreads its requests over all the steps
    // every chunk has, so that a workgroup's requests do not reach the memory pipeline in one
    // burst (10 % on large layers); the small tile, whose steps are half as long and whose two
    // workgroups per CU already interleave, does better with them in the first steps (measured).
    typedef __attribute__((address_space(3))) void* lds_ptr;
    const int wave_piece = wave * kWave;                // first piece of this wave within an item
    // (The offset argument is cast to the builtin's own type, int: given an unsigned value the
    // host pass of hipcc 7.2 leaves the kernel's launch stub out of the object without a
    // diagnostic, and the library then fails to load.)
    auto fetch_item = [&](int k, float* slot) __attribute__((always_inline)) {
        if (k < NII) {
            if (k * THREADS + wave_piece < img_pieces)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    irs, (lds_ptr)(slot + FB + 4 * (k * THREADS + wave_piece)), 16, (int)ig[k], 0, 0, 0);
        } else {
            const int q = k - NII;
            if (q * THREADS + wave_piece < FPIECES)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    wrs, (lds_ptr)(slot + 4 * (q * THREADS + wave_piece)), 16, (int)wg[q], 0, 0, 0);
        }
    };
    constexpr int kSteps0 = SL < S ? SL : S;
    constexpr int kSpread = THREADS == 512 ? kSteps0 : (kSteps0 > 8 ? kSteps0 - 7 : 1);

    // not DIRECT.  All loads of a chunk are issued when the previous chunk begins; item k goes to
    // LDS at step kFirstCommit + k / kPerStep of it, so that the LDS writes issue between
    // matrix-core instructions.  Pieces beyond the blocks go to sixteen spare bytes behind the
    // slots.
    v4f ireg[DIRECT ? 1 : NII], wreg[DIRECT ? 1 : NFI];
    const int trash = 2 * SLOT;
    const int ipos = (tid & 1) * img_plane + (tid >> 1);                       // + it * THREADS / 2
    const int wpos = (tid / (2 * MT)) * (2 * MT) + (tid & 1) * MT + (tid >> 1) % MT;   // + it * THREADS
    auto load_regs = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < NII; ++it)
            ireg[DIRECT ? 0 : it] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(irs, ig[it], 0, 0));
#pragma unroll
        for (int it = 0; it < NFI; ++it)
            wreg[DIRECT ? 0 : it] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(wrs, wg[it], 0, 0));
    };
    auto commit_item = [&](int k, float* slot) __attribute__((always_inline)) {
        if (k < NII) {
            const int e = tid + k * THREADS;
            *reinterpret_cast<v4f*>(e < img_pieces ? slot + FB + 4 * (ipos + k * (THREADS / 2)) : lds + trash) =
                ireg[DIRECT ? 0 : k];
        } else {
            const int e = tid + (k - NII) * THREADS;
            *reinterpret_cast<v4f*>(e < FPIECES ? slot + 4 * (wpos + (k - NII) * THREADS) : lds + trash) =
                wreg[DIRECT ? 0 : k - NII];
        }
    };
    constexpr int kFirstCommit = S / 2;
    constexpr int kPerStep = (NI + (S - kFirstCommit) - 1) / (S - kFirstCommit);

    // ---- the compute side ------------------------------------------------------------------------
    int base[NW];            // LDS word (within a slot) of the lane's 16 bytes of its pixel at tap (0, 0)
    uint32_t oofs[NW];       // byte offset of out[n][k0 + 32*wm*MW + 4*h][y][x] from out[n_first][k0][0][0]
    bool valid[NW];
    const int kleft = p.K - k0 - 32 * wm * MW - 4 * h;
    float* obase_t = p.out + ((int64_t)n_first * p.K + k0) * plane;
    {
        // one image of the output, in words; where a tile cannot reach a second image (the host
        // checks what lanes add to the tile's base) the product may not fit and meets a zero
        const uint32_t kplane = (uint32_t)p.K * (uint32_t)plane;
#pragma unroll
        for (int nt = 0; nt < NW; ++nt) {
            const int pp = p0 + (wn * NW + nt) * 32 + l32;
            valid[nt] = pp < total_p;
            const int pc = valid[nt] ? pp : total_p - 1;
            const int Q = fdiv(pc, d_ws), xl = pc - Q * ws;
            const int n = fdiv(Q, p.d_ho), y = Q - n * p.Ho;
            base[nt] = FB + (h * (p.RS * LS) + ((n - n_first) * p.Hc + y - y_first) * LS + xl) * 4;
            oofs[nt] = ((uint32_t)(n - n_first) * kplane +
                        (uint32_t)((32 * wm * MW + 4 * h) * (int)plane + y * p.Wo + x0 + xl)) * 4u;
        }
    }
    int wb[MW];
#pragma unroll
    for (int mt = 0; mt < MW; ++mt) wb[mt] = (h * MT + (wm * MW + mt) * 32 + l32) * 4;
    auto load_ops = [&](int s, const float* slot, v4f (&a)[MW], v4f (&b)[NW]) __attribute__((always_inline)) {
        const int i = s / F, j = s % F;
#pragma unroll
        for (int nt = 0; nt < NW; ++nt)
            b[nt] = *reinterpret_cast<const v4f*>(slot + base[nt] + (i * LS + j) * 4);
#pragma unroll
        for (int mt = 0; mt < MW; ++mt)
            a[mt] = *reinterpret_cast<const v4f*>(slot + wb[mt] + s * (MT * 8));
    };

    v16f acc[MW][NW];
#pragma unroll
    for (int mt = 0; mt < MW; ++mt)
#pragma unroll
        for (int nt = 0; nt < NW; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0.f;

    // ---- chunks: compute chunk u from one slot while chunk u+1 travels to the other ------------
    set_chunk(0);
    if constexpr (DIRECT) {
#pragma unroll
        for (int k = 0; k < NI; ++k) fetch_item(k, lds);
        __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0): this wave's pieces are in LDS
    } else {
        load_regs();
#pragma unroll
        for (int k = 0; k < NI; ++k) commit_item(k, lds);
    }
    __syncthreads();
    for (int u = 0; u < nch; ++u) {
        const float* cur = lds + (u & 1) * SLOT;
        // the other slot was last read during chunk u-1, which every wave left before the barrier
        // that ended it
        float* nxt = lds + ((u + 1) & 1) * SLOT;
        const bool more = u + 1 < nch;
        if (more) {
            set_chunk(u + 1);
            if constexpr (!DIRECT) load_regs();
        }
        const bool shortg = SL != S && (u % NG) == NG - 1;     // a last row group: fewer steps
        v4f a0[MW], b0[NW], a1[MW], b1[NW];
        load_ops(0, cur, a0, b0);
#pragma unroll
        for (int s = 0; s < S; ++s) {
            if (s >= SL && shortg) continue;                   // uniform; compiled away when SL == S
            v4f (&a)[MW] = (s & 1) ? a1 : a0;
            v4f (&b)[NW] = (s & 1) ? b1 : b0;
            const bool last_step = s == S - 1 || (s == SL - 1 && shortg);
            if (!last_step) load_ops(s + 1, cur, (s & 1) ? a0 : a1, (s & 1) ? b0 : b1);
            if (more) {
                if constexpr (DIRECT) {
#pragma unroll
                    for (int k = 0; k < NI; ++k)
                        if (k * kSpread / NI == s) fetch_item(k, nxt);
                } else if (s >= kFirstCommit) {
#pragma unroll
                    for (int q = 0; q < kPerStep; ++q)
                        if ((s - kFirstCommit) * kPerStep + q < NI) commit_item((s - kFirstCommit) * kPerStep + q, nxt);
                }
            }
#pragma unroll
            for (int mt = 0; mt < MW; ++mt)
#pragma unroll
                for (int nt = 0; nt < NW; ++nt)
                    acc[mt][nt] = mfma_16B<DT>(a[mt], b[nt], acc[mt][nt]);
        }
        if constexpr (DIRECT) {
            __builtin_amdgcn_s_waitcnt(0x0F70);  // this wave's pieces of chunk u+1 have landed
        } else if (shortg && more) {             // the items of the steps that were left out
#pragma unroll
            for (int k = 0; k < NI; ++k)
                if (kFirstCommit + k / kPerStep >= SL) commit_item(k, nxt);
        }
        __syncthreads();
    }

    // ---- write back: 32 lanes hold 32 consecutive pixels of one output map ---------------------
#pragma unroll
    for (int mt = 0; mt < MW; ++mt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int kk = mt * 32 + mfma_row(r, 0);
            char* ob = (char*)(obase_t + kk * plane);
#pragma unroll
            for (int nt = 0; nt < NW; ++nt)
                if (valid[nt] && kk < kleft)
                    *reinterpret_cast<float*>(ob + oofs[nt]) = acc[mt][nt][r];
        }
    }
}

// One thread per output element, any shape and alignment.
template <int DT>
__global__ void __launch_bounds__(kThreads)
simple_half_kernel(const void* in_, const void* filt_, float* out,
                   int N, int C, int H, int W, int K, int F, int Ho, int Wo, int blocked)
{
    // element index of channel c of pixel / tap `pos` (a flat [N][H][W] or [K][F][F] position
    // within image or filter `outer`, `inner` positions each)
    constexpr int cb = kHalfChunkBytes / elem_bytes(DT);
    auto at = [&](int64_t outer, int64_t inner_count, int64_t pos, int c) -> int64_t {
        if (!blocked) return (outer * inner_count + pos) * C + c;
        return ((outer * (C / cb) + c / cb) * inner_count + pos) * cb + c % cb;
    };
    const int64_t total = (int64_t)N * K * Ho * Wo;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x; o < total; o += stride) {
        const int x = (int)(o % Wo), y = (int)((o / Wo) % Ho);
        const int k = (int)((o / ((int64_t)Wo * Ho)) % K), n = (int)(o / ((int64_t)Wo * Ho * K));
        if (DT == kI8) {
            const signed char* in = (const signed char*)in_;
            const signed char* filt = (const signed char*)filt_;
            int acc = 0;
            for (int i = 0; i < F; ++i)
                for (int j = 0; j < F; ++j)
                    for (int c = 0; c < C; ++c)
                        acc += (int)in[at(n, (int64_t)H * W, (int64_t)(y + i) * W + x + j, c)] *
                               (int)filt[at(k, F * F, i * F + j, c)];
            out[o] = __builtin_bit_cast(float, acc);
            continue;
        }
        const unsigned short* in = (const unsigned short*)in_;
        const unsigned short* filt = (const unsigned short*)filt_;
        auto cvt = [](unsigned short v) {
            if (DT == kBF16) return __builtin_bit_cast(float, (uint32_t)v << 16);
            return (float)__builtin_bit_cast(_Float16, v);
        };
        // sums in three levels (runs of 64 channels, taps, the whole), so that the rounding
        // error grows with the longest level and not with C * F * F
        float acc = 0.f;
        for (int i = 0; i < F; ++i)
            for (int j = 0; j < F; ++j) {
                float tap = 0.f;
                for (int c0 = 0; c0 < C; c0 += 64) {
                    float run = 0.f;
                    const int c1 = c0 + 64 < C ? c0 + 64 : C;
                    for (int c = c0; c < c1; ++c)
                        run = __builtin_fmaf(cvt(in[at(n, (int64_t)H * W, (int64_t)(y + i) * W + x + j, c)]),
                                             cvt(filt[at(k, F * F, i * F + j, c)]), run);
                    tap += run;
                }
                acc += tap;
            }
        out[o] = acc;
    }
}

// ---- host side -----------------------------------------------------------------------------------

struct HalfPlan {
    int bw, nstrips, LS, RS, pt_full, pt_last;
    bool ok;
};

// The widest column strips (at most 128 columns) whose image block a workgroup of `threads`
// threads can stage with `nii` pieces per thread, for tiles of NT pixels.
inline HalfPlan make_half_plan(const Shape& s, int rg, int NT, int nii, int threads)
{
    HalfPlan pl{};
    for (int nstrips = (s.Wo + 127) / 128; nstrips <= s.Wo; ++nstrips) {
        pl.bw = (s.Wo + nstrips - 1) / nstrips;
        pl.nstrips = (s.Wo + pl.bw - 1) / pl.bw;
        pl.LS = pl.bw + s.F - 1;
        const int wmin = s.Wo - (pl.nstrips - 1) * pl.bw;
        const int64_t all_rows = (int64_t)s.N * s.Ho;
        const int rows = (int)std::min<int64_t>((NT - 2) / wmin + 2, all_rows);
        const int cross = std::min(rows >= 2 ? (rows - 2) / s.Ho + 1 : 0, s.N - 1);
        pl.RS = rows + (rg - 1) * (cross + 1);
        pl.pt_full = (int)(((int64_t)s.N * s.Ho * pl.bw + NT - 1) / NT);
        pl.pt_last = (int)(((int64_t)s.N * s.Ho * wmin + NT - 1) / NT);
        if (2LL * pl.RS * pl.LS <= (int64_t)nii * threads) { pl.ok = true; return pl; }
    }
    pl.ok = false;
    return pl;
}

template <int F, int RG, int DT, class TL, bool DIRECT>
int half_try_launch(const void* in, const void* filt, float* out, const Shape& s, hipStream_t st, bool dry,
                    bool blocked)
{
    constexpr int MT = TL::MT, NT = TL::NT, S = RG * F;
    constexpr int EB = elem_bytes(DT);
    if (s.C % (kHalfChunkBytes / EB) != 0) return DCONV_UNSUPPORTED;
    const HalfPlan pl = make_half_plan(s, RG, NT, TL::NII, TL::THREADS);
    if (!pl.ok) return DCONV_UNSUPPORTED;
    // two slots (filter block, image block), as the kernel lays them out
    const int64_t img_pieces = 2LL * pl.RS * pl.LS;
    const int64_t slot_words = (int64_t)S * MT * 8 + 4 * (DIRECT ? (img_pieces + 63) & ~63LL : img_pieces);
    const int64_t lds_bytes = 4 * (2 * slot_words + (DIRECT ? 0 : 4));
    if (lds_bytes > kGenLdsLimit) return DCONV_UNSUPPORTED;
    const int KB = (s.K + MT - 1) / MT;
    const int64_t tiles = ((int64_t)(pl.nstrips - 1) * pl.pt_full + pl.pt_last) * KB;
    if (tiles > 2000000000LL || (int64_t)s.N * s.Ho * s.Wo > 2147483647LL) return DCONV_UNSUPPORTED;
    // lanes address HBM with 32-bit byte offsets from per-tile bases: what a tile can reach from
    // its first image, its first filter and its first output map must lie within 2 GiB
    {
        const int wmin = s.Wo - (pl.nstrips - 1) * pl.bw;
        const int64_t span = std::min<int64_t>(NT / ((int64_t)s.Ho * wmin) + 2, s.N);   // images a tile reaches
        const int64_t plane = (int64_t)s.Ho * s.Wo;
        const int64_t lim = 1LL << 31;
        // (the filter a store belongs to is in its uniform base; a lane adds the image, its wave's
        // first filter, four filters for the upper half-wave, and the pixel)
        if (span * s.H * s.W * s.C * EB >= lim ||
            ((span - 1) * s.K * plane + (32 * (TL::WM - 1) * TL::MW + 6) * plane) * 4 >= lim ||
            (int64_t)(MT + 1) * F * F * s.C * EB >= lim)
            return DCONV_UNSUPPORTED;
    }
    if (dry) return DCONV_OK;
    if ((((uintptr_t)in) & 15) != 0 || (((uintptr_t)filt) & 15) != 0) return DCONV_UNSUPPORTED;

    auto kern = general_half_kernel<F, RG, DT, TL, DIRECT>;
    static std::atomic<uint64_t> lds_limit_raised{0};
    if (!raise_lds_limit((const void*)kern, kGenLdsLimit, lds_limit_raised)) return DCONV_LAUNCH_FAILED;
    const int per_xcd = (int)((tiles + 7) / 8);
    HalfParams p{(const char*)in, (const char*)filt, out, s.N, s.C, s.H, s.W, s.K, s.Ho, s.Wo,
                 pl.bw, pl.nstrips, pl.LS, pl.RS, pl.pt_full, KB, (int)tiles, per_xcd, s.Ho + RG - 1,
                 blocked ? kHalfChunkBytes : s.C * EB, blocked ? s.H * s.W * kHalfChunkBytes : kHalfChunkBytes,
                 blocked ? kHalfChunkBytes : s.C * EB, blocked ? F * F * kHalfChunkBytes : kHalfChunkBytes,
                 make_fastdiv(pl.pt_full * KB), make_fastdiv(KB), make_fastdiv(pl.bw),
                 make_fastdiv(s.Wo - (pl.nstrips - 1) * pl.bw), make_fastdiv(s.Ho),
                 make_fastdiv(s.Ho + RG - 1), make_fastdiv(pl.LS)};
    begin_launch();
    hipLaunchKernelGGL(kern, dim3((unsigned)(per_xcd * 8)), dim3(TL::THREADS), (size_t)lds_bytes, st, p);
    return launch_status();
}

// Tile configurations of the short-data-type kernel (DCONV_VARIANT_TILED_CFG0 + i forces one):
// 0: small tile, 1: large tile, both staged through registers; 2: small tile, 3: large tile,
// 4: mid tile, all three staged directly into LDS.
constexpr int kHalfConfigs = 5;

// Implemented once per filter side, each in its own translation unit.
template <int F>
int half_launch_for_F(const void* in, const void* filt, float* out, const Shape& s, hipStream_t st,
                      int dtype, int config, bool blocked, bool dry);

}  // namespace dconv
