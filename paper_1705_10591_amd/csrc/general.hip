// General-case direct convolution (paper Sec. 4, Algorithm 2) for gfx950.
//
// What is kept from the paper's scheme: a workgroup owns a block of filters
// times a block of output pixels over ALL channels; channels are consumed in
// chunks of CSH; each chunk's image block (with its halo) goes to LDS
// untransposed and the matching filter block goes to LDS transposed, with a
// padded row stride, so that both are read conflict-free; the next chunk is
// prefetched from HBM into registers while the current one is consumed, and
// committed to LDS between two barriers; the image block is read at shifted
// addresses for the F*F taps instead of being unrolled in memory, so every
// input pixel is fetched from HBM once per tile and reused F*F*K times on chip.
//
// What differs (CDNA4 instead of Kepler): the multiply-accumulate runs on the
// matrix cores.  One v_mfma_f32_32x32x2_f32 forms a 32-filter x 32-pixel
// block of partial sums for two reduction indices at once; it is the only
// route to the chip's fp32 peak, and it makes the per-lane register tile of
// the paper (F_T x W_T) a per-wave tile of MW x NW such blocks.  The two
// reduction indices of one instruction are two consecutive entries of the
// flattened (channel, filter row, filter column) list of the chunk, so the
// image operand of lane l is the LDS word of pixel (l % 32) at the tap chosen
// by (l / 32).  Output pixels are numbered along (image, row, column) of a
// column strip, so a 32-pixel block may wrap over rows and images and no
// lanes are wasted on narrow maps (Wo = 26, 54).
#include "common.h"
#include "../../include/dconv.h"

namespace dconv {

struct GenParams {
    const float* in;
    const float* filt;
    float* out;
    int N, C, H, W, K, Ho, Wo;
    int bw;          // width of a column strip of the output (last strip may be narrower)
    int tiles_max;   // pixel tiles per strip (upper bound; surplus workgroups exit)
    int LS;          // LDS row stride of the image block: bw + F - 1
    int RS;          // LDS row slots per channel
    int vec4;        // filter rows can be fetched 16 B at a time
};

// Reduction index t of a chunk <-> (channel in chunk, filter row, filter column).
template <int F> __device__ __forceinline__ constexpr int tap_c(int t) { return t / (F * F); }
template <int F> __device__ __forceinline__ constexpr int tap_i(int t) { return (t % (F * F)) / F; }
template <int F> __device__ __forceinline__ constexpr int tap_j(int t) { return t % F; }

template <int F, int CSH, int MW, int NW, int WM, int WN, int IMAX>
__global__ void __launch_bounds__(kThreads, 2)
general_tiled_kernel(GenParams p)
{
    static_assert(WM * WN * kWave == kThreads, "four waves per workgroup");
    constexpr int MT = 32 * MW * WM;          // filters per workgroup
    constexpr int NT = 32 * NW * WN;          // output pixels per workgroup
    constexpr int FF = F * F;
    constexpr int T = CSH * FF;               // reduction indices per chunk
    constexpr int TP = T + (T & 1);           // padded to a whole number of pairs
    constexpr int S = TP / 2;                 // matrix-core steps per chunk
    constexpr int LDK = MT + 1;               // odd row stride: transposing writes hit 32 banks

    extern __shared__ float lds[];
    float* shFlt = lds;                       // [TP][LDK]   filter block, reduction-major
    float* shImg = lds + TP * LDK;            // [CSH][RS][LS] image block, then one zero word

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: lets wave-level math run on the scalar unit
    const int h = lane >> 5, l32 = lane & 31;
    const int wm = wave / WN, wn = wave % WN;

    const int strip = blockIdx.x / p.tiles_max;
    const int tile = blockIdx.x - strip * p.tiles_max;
    const int x0 = strip * p.bw;
    const int ws = min(p.bw, p.Wo - x0);               // this strip's width
    const int total_p = p.N * p.Ho * ws;               // pixels of the strip
    const int p0 = tile * NT;
    if (p0 >= total_p) return;                          // uniform: before any barrier
    const int k0 = blockIdx.y * MT;

    const int LS = p.LS, PL = p.RS * p.LS;
    // first input row (numbered n*H + y over the batch) the tile touches
    const int Q0 = p0 / ws;
    const int G0 = (Q0 / p.Ho) * p.H + (Q0 % p.Ho);
    const int plast = min(p0 + NT, total_p) - 1;
    const int Ql = plast / ws;
    const int nslots = (Ql / p.Ho) * p.H + (Ql % p.Ho) - G0 + F;

    // ---- per-lane pixel bookkeeping -------------------------------------------------
    int base[NW];            // LDS word of tap (0,0,0) of the lane's pixel
    bool valid[NW];
    int64_t obase[NW];       // out index of (n, k=0, y, x)
#pragma unroll
    for (int nt = 0; nt < NW; ++nt) {
        const int pp = p0 + (wn * NW + nt) * 32 + l32;
        valid[nt] = pp < total_p;
        const int pc = valid[nt] ? pp : total_p - 1;
        const int Q = pc / ws, xl = pc - Q * ws;
        const int n = Q / p.Ho, y = Q - n * p.Ho;
        base[nt] = (n * p.H + y - G0) * LS + xl;
        obase[nt] = ((int64_t)n * p.K * p.Ho + y) * p.Wo + x0 + xl;
    }
    // Offsets of the second tap of a pair relative to the first, by kind of pair.
    const int dX = h;                                         // next column, same row
    const int dY = h * (LS - (F - 1));                        // first column of the next row
    const int dZ = h * (PL - (F - 1) * LS - (F - 1));         // first tap of the next channel
    const int zero_word = CSH * PL;
    const int wbase = h * LDK + wm * (MW * 32) + l32;

    // ---- staging tables: which HBM word each thread brings in per chunk --------------
    int ig[IMAX];            // image: offset from in + c0*H*W, -1 = store zero, -2 = nothing
    const int img_words = CSH * PL;
#pragma unroll
    for (int it = 0; it < IMAX; ++it) {
        const int e = tid + it * kThreads;
        int g = -2;
        if (e < img_words) {
            const int cc = e / PL, rem = e - cc * PL;
            const int slot = rem / LS, col = rem - slot * LS;
            const int G = G0 + slot;
            const int n = G / p.H, yy = G - n * p.H;
            const bool ok = slot < nslots && G < p.N * p.H && x0 + col < p.W;
            g = ok ? ((n * p.C + cc) * p.H + yy) * p.W + x0 + col : -1;
        }
        ig[it] = g;
    }
    const int HW = p.H * p.W;
    const int CFF = p.C * FF;

    // Filter block: TPF threads share one filter; each brings in a contiguous run of EPT of
    // its T reduction indices per chunk (16 B at a time when the layout allows) and scatters
    // it down a column of the transposed LDS block.  All per-element offsets are immediates.
    constexpr int TPF = kThreads / MT;
    constexpr int EPT = (T + TPF - 1) / TPF;
    const int wkl = tid / TPF, we0 = (tid % TPF) * EPT;
    const bool wk_ok = k0 + wkl < p.K;
    const float* wsrc = p.filt + (int64_t)(wk_ok ? k0 + wkl : 0) * CFF + we0;
    float* wdst = shFlt + we0 * LDK + wkl;

    float ireg[IMAX], wreg[EPT];
    auto fetch = [&](int c0) {
        const float* ip = p.in + (int64_t)c0 * HW;
#pragma unroll
        for (int it = 0; it < IMAX; ++it)
            ireg[it] = ig[it] >= 0 ? ip[ig[it]] : 0.f;
        const float* fp = wsrc + (int64_t)c0 * FF;
        if (EPT % 4 == 0 && p.vec4) {
#pragma unroll
            for (int it = 0; it < EPT / 4; ++it) {
                const v4f v = (wk_ok && we0 + 4 * it < T) ? *reinterpret_cast<const v4f*>(fp + 4 * it)
                                                          : (v4f){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int u = 0; u < 4; ++u) wreg[4 * it + u] = v[u];
            }
        } else {
#pragma unroll
            for (int it = 0; it < EPT; ++it)
                wreg[it] = (wk_ok && we0 + it < T) ? fp[it] : 0.f;
        }
    };
    auto commit = [&]() {
#pragma unroll
        for (int it = 0; it < IMAX; ++it)
            if (ig[it] != -2) shImg[tid + it * kThreads] = ireg[it];
#pragma unroll
        for (int it = 0; it < EPT; ++it)
            if (we0 + it < T) wdst[it * LDK] = wreg[it];
    };

    if (tid == 0) shImg[zero_word] = 0.f;
    if (TP != T) {                        // the padding reduction index carries zero weights
        for (int k = tid; k < MT; k += kThreads) shFlt[T * LDK + k] = 0.f;
    }

    v16f acc[MW][NW];
#pragma unroll
    for (int mt = 0; mt < MW; ++mt)
#pragma unroll
        for (int nt = 0; nt < NW; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0.f;

    fetch(0);
    commit();
    __syncthreads();

    for (int c0 = 0; c0 < p.C; c0 += CSH) {
        const bool more = c0 + CSH < p.C;
#if DCONV_GEN_EXP != 1 && DCONV_GEN_EXP != 2
        if (more) fetch(c0 + CSH);
#endif
        // keep the tap addresses from being expanded into one register each outside the loop
#pragma unroll
        for (int nt = 0; nt < NW; ++nt) asm volatile("" : "+v"(base[nt]));

        // Operands of step s+1 are requested from LDS before the matrix-core instructions
        // of step s are issued, so a wave never waits for LDS with the matrix pipe idle.
        auto load_ops = [&](int s, float (&a)[MW], float (&b)[NW]) {
            const int t0 = 2 * s, t1 = 2 * s + 1;
            const int c = tap_c<F>(t0), i = tap_i<F>(t0), j = tap_j<F>(t0);
            const int rowoff = c * PL + i * LS;
#pragma unroll
            for (int nt = 0; nt < NW; ++nt) {
                int addr;
                if (t1 >= T)                                              // pad: second tap reads 0
                    addr = h ? zero_word : base[nt] + rowoff + j;
                else if (tap_c<F>(t1) != c) addr = base[nt] + dZ + rowoff + j;
                else if (tap_i<F>(t1) != i) addr = base[nt] + dY + rowoff + j;
                else                        addr = base[nt] + dX + rowoff + j;
                b[nt] = shImg[addr];
            }
#pragma unroll
            for (int mt = 0; mt < MW; ++mt)
                a[mt] = shFlt[wbase + t0 * LDK + mt * 32];
        };
        float a0[MW], b0[NW], a1[MW], b1[NW];
        load_ops(0, a0, b0);
#pragma unroll
        for (int s = 0; s < S; ++s) {
            float (&a)[MW] = (s & 1) ? a1 : a0;
            float (&b)[NW] = (s & 1) ? b1 : b0;
            if (s + 1 < S) load_ops(s + 1, (s & 1) ? a0 : a1, (s & 1) ? b0 : b1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mt = 0; mt < MW; ++mt)
#pragma unroll
                for (int nt = 0; nt < NW; ++nt)
                    acc[mt][nt] = mfma_32x32x2(a[mt], b[nt], acc[mt][nt]);
            __builtin_amdgcn_sched_barrier(0);
        }

#if DCONV_GEN_EXP != 1 && DCONV_GEN_EXP != 2
        __syncthreads();
        if (more) commit();
        __syncthreads();
#endif
    }

    // ---- write back: 32 lanes hold 32 consecutive pixels of one output map -----------
    const int64_t plane = (int64_t)p.Ho * p.Wo;
#pragma unroll
    for (int mt = 0; mt < MW; ++mt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int k = k0 + (wm * MW + mt) * 32 + mfma_row(r, h);
#pragma unroll
            for (int nt = 0; nt < NW; ++nt)
#if DCONV_GEN_EXP == 2 || DCONV_GEN_EXP == 3
                if (valid[nt] && k < p.K && acc[mt][nt][r] == 1234567.f) p.out[obase[nt] + k * plane] = acc[mt][nt][r];
#else
                if (valid[nt] && k < p.K) p.out[obase[nt] + k * plane] = acc[mt][nt][r];
#endif
        }
    }
}

// ---- host side --------------------------------------------------------------------------

namespace {

constexpr int kLdsLimit = 160 * 1024;
constexpr int kStripMax = 128;      // widest column strip of the output map

struct Plan {
    int bw, nstrips, tiles_max, LS, RS;
};

Plan make_plan(const Shape& s, int NT)
{
    Plan pl;
    pl.nstrips = (s.Wo + kStripMax - 1) / kStripMax;
    pl.bw = (s.Wo + pl.nstrips - 1) / pl.nstrips;
    pl.nstrips = (s.Wo + pl.bw - 1) / pl.bw;
    pl.LS = pl.bw + s.F - 1;
    // A run of NT consecutive strip pixels touches at most this many output rows, taken
    // over every strip width from the narrowest (the last strip) to bw ...
    const int wmin = s.Wo - (pl.nstrips - 1) * pl.bw;
    const int rows = NT >= 2 ? (NT - 2) / wmin + 2 : 1;
    // ... and crosses at most this many image boundaries, each adding F-1 input rows.
    const int cross = rows >= 2 ? (rows - 2) / s.Ho + 1 : 0;
    pl.RS = rows + (s.F - 1) * (cross + 1);
    const int64_t strip_pixels = (int64_t)s.N * s.Ho * pl.bw;
    pl.tiles_max = (int)((strip_pixels + NT - 1) / NT);
    return pl;
}

template <int F, int CSH, int MW, int NW, int WM, int WN, int IMAX>
int try_launch(const float* in, const float* filt, float* out, const Shape& s, hipStream_t st,
               bool dry)
{
    constexpr int MT = 32 * MW * WM, NT = 32 * NW * WN;
    constexpr int T = CSH * F * F, TP = T + (T & 1), LDK = MT + 1;
    if (s.C % CSH != 0) return DCONV_UNSUPPORTED;
    const Plan pl = make_plan(s, NT);
    const int64_t img_words = (int64_t)CSH * pl.RS * pl.LS;
    if (img_words > (int64_t)IMAX * kThreads) return DCONV_UNSUPPORTED;
    const int64_t lds_bytes = 4 * ((int64_t)TP * LDK + img_words + 1);
    if (lds_bytes > kLdsLimit) return DCONV_UNSUPPORTED;
    const int64_t gx = (int64_t)pl.tiles_max * pl.nstrips;
    const int gy = (s.K + MT - 1) / MT;
    if (gx > 2147483647LL || gy > 65535) return DCONV_UNSUPPORTED;
    if (dry) return DCONV_OK;

    auto kern = general_tiled_kernel<F, CSH, MW, NW, WM, WN, IMAX>;
    static bool attr_set = false;     // benign race: the call is idempotent
    if (lds_bytes > 64 * 1024 && !attr_set) {
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                kLdsLimit) != hipSuccess)
            return DCONV_LAUNCH_FAILED;
        attr_set = true;
    }
    const int vec4 = ((int64_t)s.C * F * F) % 4 == 0 && (CSH * F * F) % 4 == 0 &&
                     ((uintptr_t)filt & 15) == 0;
    GenParams p{in, filt, out, s.N, s.C, s.H, s.W, s.K, s.Ho, s.Wo,
                pl.bw, pl.tiles_max, pl.LS, pl.RS, vec4};
    hipLaunchKernelGGL(kern, dim3((unsigned)gx, (unsigned)gy), dim3(kThreads),
                       (size_t)lds_bytes, st, p);
    return hipGetLastError() == hipSuccess ? DCONV_OK : DCONV_LAUNCH_FAILED;
}

// Largest chunk of channels (of those compiled) that divides C.
template <int F>
int launch_for_F(const float* in, const float* filt, float* out, const Shape& s, hipStream_t st,
                 bool dry)
{
    const bool wideK = s.K > 64;
    int rc = DCONV_UNSUPPORTED;
    if constexpr (F <= 3) {
        if (s.C % 8 == 0) {
            rc = wideK ? try_launch<F, 8, 2, 2, 2, 2, 16>(in, filt, out, s, st, dry)
                       : try_launch<F, 8, 1, 2, 2, 2, 16>(in, filt, out, s, st, dry);
            if (rc != DCONV_UNSUPPORTED) return rc;
        }
    }
    if constexpr (F <= 5) {
        if (s.C % 2 == 0) {
            rc = wideK ? try_launch<F, 2, 2, 2, 2, 2, 16>(in, filt, out, s, st, dry)
                       : try_launch<F, 2, 1, 2, 2, 2, 16>(in, filt, out, s, st, dry);
            if (rc != DCONV_UNSUPPORTED) return rc;
        }
    }
    rc = wideK ? try_launch<F, 1, 2, 2, 2, 2, 16>(in, filt, out, s, st, dry)
               : try_launch<F, 1, 1, 2, 2, 2, 16>(in, filt, out, s, st, dry);
    return rc;
}

int launch_any(const float* in, const float* filt, float* out, const Shape& s, hipStream_t st,
               bool dry)
{
    if ((int64_t)s.N * s.Ho * s.Wo > 2147483647LL) return DCONV_UNSUPPORTED;
    switch (s.F) {
    case 1: return launch_for_F<1>(in, filt, out, s, st, dry);
    case 2: return launch_for_F<2>(in, filt, out, s, st, dry);
    case 3: return launch_for_F<3>(in, filt, out, s, st, dry);
    case 4: return launch_for_F<4>(in, filt, out, s, st, dry);
    case 5: return launch_for_F<5>(in, filt, out, s, st, dry);
    case 6: return launch_for_F<6>(in, filt, out, s, st, dry);
    case 7: return launch_for_F<7>(in, filt, out, s, st, dry);
    case 8: return launch_for_F<8>(in, filt, out, s, st, dry);
    case 9: return launch_for_F<9>(in, filt, out, s, st, dry);
    case 10: return launch_for_F<10>(in, filt, out, s, st, dry);
    case 11: return launch_for_F<11>(in, filt, out, s, st, dry);
    default: return DCONV_UNSUPPORTED;
    }
}

}  // namespace

bool general_tiled_supports(const Shape& s)
{
    return launch_any(nullptr, nullptr, nullptr, s, nullptr, true) == DCONV_OK;
}

int general_tile_configs() { return 1; }

int launch_general_tiled(const float* in, const float* filt, float* out, const Shape& s,
                         hipStream_t st, int cfg)
{
    if (cfg > 0) return DCONV_UNSUPPORTED;
    return launch_any(in, filt, out, s, st, false);
}

}  // namespace dconv
