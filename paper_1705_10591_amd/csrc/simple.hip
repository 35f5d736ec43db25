// One-thread-per-output direct convolution: the shape-agnostic variant.
//
// Every output element is the triple sum of the paper's Fig. 3a taken by a
// single lane with fp32 fused multiply-adds, level by level (see the kernel).  No tiling and no on-chip
// staging: it exists so that every valid shape has a kernel (filter sides the
// tiled kernels are not compiled for, index ranges beyond their 32-bit
// offsets), not for speed.
#include "common.h"
#include "../../include/dconv.h"

namespace dconv {

__global__ void __launch_bounds__(kThreads)
simple_kernel(const float* __restrict__ in, const float* __restrict__ filt,
              float* __restrict__ out, Shape s)
{
    const int64_t plane = (int64_t)s.Ho * s.Wo;
    const int64_t per_image = plane * s.K;
    const int64_t total = per_image * s.N;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; o < total; o += stride) {
        const int x = (int)(o % s.Wo);
        const int y = (int)((o / s.Wo) % s.Ho);
        const int k = (int)((o / plane) % s.K);
        const int64_t n = o / per_image;
        const float* ip = in + (n * s.C * s.H + y) * s.W + x;
        const float* fp = filt + (int64_t)k * s.C * s.F * s.F;
        // sums in three levels (a filter row, a channel, runs of 16 channels), so that the
        // rounding error grows with the longest level and not with C * F * F
        float acc = 0.f, run = 0.f;
        for (int c = 0; c < s.C; ++c) {
            float chan = 0.f;
            for (int i = 0; i < s.F; ++i) {
                float row = 0.f;
                for (int j = 0; j < s.F; ++j)
                    row = __builtin_fmaf(ip[(int64_t)i * s.W + j], fp[i * s.F + j], row);
                chan += row;
            }
            run += chan;
            if ((c & 15) == 15) { acc += run; run = 0.f; }
            ip += (int64_t)s.H * s.W;
            fp += s.F * s.F;
        }
        acc += run;
        out[o] = acc;
    }
}

int launch_simple(const float* in, const float* filt, float* out, const Shape& s, hipStream_t st)
{
    const int64_t total = (int64_t)s.N * s.K * s.Ho * s.Wo;
    int64_t blocks = (total + kThreads - 1) / kThreads;
    if (blocks > 256 * 64) blocks = 256 * 64;     // grid-stride beyond that
    begin_launch();
    hipLaunchKernelGGL(simple_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, st,
                       in, filt, out, s);
    return launch_status();
}

}  // namespace dconv
