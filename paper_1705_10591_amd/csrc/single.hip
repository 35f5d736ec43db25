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
#include "common.h"
#include "../../include/dconv.h"

namespace dconv {

struct SingleParams {
    const float* img;
    const float* filt;
    float* out;
    int H, W, K, Ho, Wo;
    int tiles_x, tiles_y;
    int fbw;         // 32-filter blocks handled by one workgroup: 1, 2 or 4
};

// TW: tile width in pixels (multiple of 128), TR: tile rows, PAD: extra words per LDS row.
template <int F, int TW, int TR, int PAD>
__global__ void __launch_bounds__(kThreads)
single_tiled_kernel(SingleParams p)
{
    constexpr int FF = F * F;
    constexpr int TP = FF + (FF & 1);
    constexpr int S = TP / 2;                   // matrix-core steps per 32x32 block
    constexpr int LS = TW + F - 1 + PAD;        // LDS row stride
    constexpr int ROWS = TR + F - 1;            // staged image rows; one more row of zeros follows
    constexpr int NB = 4;                       // 32-pixel blocks per wave pass: 128 pixels
    constexpr int CHUNKS = TW / (32 * NB);

    __shared__ float sh[(ROWS + 1) * LS];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, l32 = lane & 31;

    const int tx = blockIdx.x % p.tiles_x;
    const int ty = blockIdx.x / p.tiles_x;
    const int x0 = tx * TW, y0 = ty * TR;
    const int fb = blockIdx.y * p.fbw + wave % p.fbw;     // this wave's 32-filter block
    const int sub = wave / p.fbw, nsub = 4 / p.fbw;       // its share of the tile rows

    // ---- stage the tile (zeros outside the image), coalesced along rows --------------
    const int cols = min(TW + F - 1, p.W - x0);
    for (int r = 0; r < ROWS; ++r) {
        const int gy = y0 + r;
        const float* src = p.img + (int64_t)gy * p.W + x0;
        for (int c = tid; c < LS; c += kThreads)
            sh[r * LS + c] = (gy < p.H && c < cols) ? src[c] : 0.f;
    }
    for (int c = tid; c < LS; c += kThreads) sh[ROWS * LS + c] = 0.f;

    // ---- this wave's filter operands: a[s] = filt[k][tap 2s + h], zero beyond K / F*F --
    float a[S];
    {
        const int k = fb * 32 + l32;
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const int t = 2 * s + h;
            a[s] = (k < p.K && t < FF) ? p.filt[(int64_t)k * FF + t] : 0.f;
        }
    }
    __syncthreads();

    const int64_t plane = (int64_t)p.Ho * p.Wo;
    const int rows_here = min(TR, p.Ho - y0);
    const int dY = h * (LS - (F - 1));          // second tap of a pair sits on the next row

    for (int r = sub; r < rows_here; r += nsub) {
#pragma unroll 1
        for (int ch = 0; ch < CHUNKS; ++ch) {
            const int xc = ch * (32 * NB);                 // first column of this pass, in tile
            if (x0 + xc >= p.Wo) break;
            const int base = r * LS + xc + l32;
            v16f acc[NB];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int q = 0; q < 16; ++q) acc[nb][q] = 0.f;

#pragma unroll
            for (int s = 0; s < S; ++s) {
                const int t0 = 2 * s, t1 = 2 * s + 1;
                const int i = t0 / F, j = t0 % F;
                float b[NB];
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    int addr;
                    if (t1 >= FF)            // pad tap: the zero row (any column of it)
                        addr = h ? (ROWS * LS + l32) : base + i * LS + j + nb * 32;
                    else if (t1 / F != i) addr = base + dY + i * LS + j + nb * 32;
                    else                  addr = base + h + i * LS + j + nb * 32;
                    b[nb] = sh[addr];
                }
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) acc[nb] = mfma_32x32x2(a[s], b[nb], acc[nb]);
            }

            // 32 lanes write 32 consecutive pixels of one output plane
            const int y = y0 + r;
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int k = fb * 32 + mfma_row(q, h);
                float* dst = p.out + k * plane + (int64_t)y * p.Wo + x0 + xc + l32;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const int x = x0 + xc + nb * 32 + l32;
                    if (k < p.K && x < p.Wo) __builtin_nontemporal_store(acc[nb][q], dst + nb * 32);
                }
            }
        }
    }
}

namespace {

template <int F, int TW, int TR, int PAD>
int launch_cfg(const float* img, const float* filt, float* out, const Shape& s, hipStream_t st)
{
    SingleParams p;
    p.img = img; p.filt = filt; p.out = out;
    p.H = s.H; p.W = s.W; p.K = s.K; p.Ho = s.Ho; p.Wo = s.Wo;
    p.tiles_x = (s.Wo + TW - 1) / TW;
    p.tiles_y = (s.Ho + TR - 1) / TR;
    const int fblocks = (s.K + 31) / 32;
    p.fbw = fblocks >= 4 ? 4 : fblocks >= 2 ? 2 : 1;
    const int64_t gx = (int64_t)p.tiles_x * p.tiles_y;
    const int gy = (fblocks + p.fbw - 1) / p.fbw;
    if (gx > 2147483647LL || gy > 65535) return DCONV_UNSUPPORTED;
    hipLaunchKernelGGL((single_tiled_kernel<F, TW, TR, PAD>), dim3((unsigned)gx, (unsigned)gy),
                       dim3(kThreads), 0, st, p);
    return hipGetLastError() == hipSuccess ? DCONV_OK : DCONV_LAUNCH_FAILED;
}

template <int F>
int launch_F(const float* img, const float* filt, float* out, const Shape& s, hipStream_t st)
{
    return launch_cfg<F, 256, 16, 0>(img, filt, out, s, st);
}

}  // namespace

bool single_tiled_supports(const Shape& s)
{
    return s.N == 1 && s.C == 1 && s.F >= 1 && s.F <= 11;
}

int launch_single_tiled(const float* img, const float* filt, float* out, const Shape& s,
                        hipStream_t st)
{
    switch (s.F) {
    case 1: return launch_F<1>(img, filt, out, s, st);
    case 2: return launch_F<2>(img, filt, out, s, st);
    case 3: return launch_F<3>(img, filt, out, s, st);
    case 4: return launch_F<4>(img, filt, out, s, st);
    case 5: return launch_F<5>(img, filt, out, s, st);
    case 6: return launch_F<6>(img, filt, out, s, st);
    case 7: return launch_F<7>(img, filt, out, s, st);
    case 8: return launch_F<8>(img, filt, out, s, st);
    case 9: return launch_F<9>(img, filt, out, s, st);
    case 10: return launch_F<10>(img, filt, out, s, st);
    case 11: return launch_F<11>(img, filt, out, s, st);
    default: return DCONV_UNSUPPORTED;
    }
}

}  // namespace dconv
