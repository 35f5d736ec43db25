// Shared declarations of the dconv HIP sources (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>
#include "../../include/dconv.h"

namespace dconv {

constexpr int kWave = 64;            // CDNA wavefront width
constexpr int kThreads = 256;        // four waves per workgroup: one per SIMD of a CU

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

// D(32x32) += A(32x2) * B(2x32) on the matrix cores, fp32 in, fp32 accumulate.
// Operand layout for lane l of the wave:
//   a  = A[l % 32][l / 32]          (row of D, reduction index l / 32)
//   b  = B[l / 32][l % 32]          (reduction index l / 32, column of D)
//   acc[r] = D[8 * (r / 4) + 4 * (l / 32) + r % 4][l % 32]
__device__ __forceinline__ v16f mfma_32x32x2(float a, float b, v16f acc) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
}

// Row of D held in accumulator register r by a lane of half h = lane / 32.
__device__ __forceinline__ constexpr int mfma_row(int r, int h) {
    return 8 * (r / 4) + 4 * h + (r % 4);
}

// Status of one kernel launch.  hipGetLastError() also hands back (and clears) an error that
// earlier, unrelated work left behind on this thread: begin_launch() drops such an error before
// the launch, launch_status() reads what the launch itself left.
inline void begin_launch() { (void)hipGetLastError(); }
inline int launch_status() { return hipGetLastError() == hipSuccess ? DCONV_OK : DCONV_LAUNCH_FAILED; }

// Kernels that use more dynamic LDS than the default limit have it raised once per device (the
// attribute belongs to the kernel on the current device): `done` holds one bit per device, one
// word per kernel.  A race between threads only repeats the call.
inline bool raise_lds_limit(const void* kernel, int bytes, std::atomic<uint64_t>& done)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    const uint64_t bit = 1ull << (dev & 63);
    if (dev < 64 && (done.load(std::memory_order_acquire) & bit)) return true;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess)
        return false;
    if (dev < 64) done.fetch_or(bit, std::memory_order_release);
    return true;
}

// Shape of one problem, general layout (the single-channel case has N = C = 1).
struct Shape {
    int N, C, H, W, K, F, Ho, Wo;
};

// Host-side launchers, one per translation unit.  Each returns a dconv_status.
int launch_simple(const float* in, const float* filt, float* out, const Shape& s, hipStream_t st);
// cfg selects one of the compiled tile configurations; cfg < 0 lets the shape decide.
int launch_single_tiled(const float* img, const float* filt, float* out, const Shape& s,
                        hipStream_t st, int cfg);
// static_ws: tiles shared between workgroups meet in the library's static device array instead of
// an allocated workspace (dconv_general_noalloc)
int launch_general_tiled(const float* in, const float* filt, float* out, const Shape& s,
                         hipStream_t st, int cfg, bool static_ws);
int single_tile_configs();
int general_tile_configs();
// what the dispatchers pick by shape: the special case's tile configuration, the general case's
// tile shape (pure host arithmetic)
int single_auto_config(const Shape& s);
int general_auto_shape(const Shape& s);
int launch_single_few(const float* img, const float* filt, float* out, const Shape& s, hipStream_t st);
// the general case with up to eight filters on the vector ALU (general_fewfilters.hip)
int launch_general_few(const float* in, const float* filt, float* out, const Shape& s, hipStream_t st);
bool general_few_supports(const Shape& s);
bool general_few_preferred(const Shape& s);
bool single_few_supports(const Shape& s);      // the few-filters kernel can run the shape
bool single_few_preferred(const Shape& s);     // ... and is the better choice for it
bool single_blocks16_preferred(const Shape& s);   // up to 16 filters: matrix-core blocks of 16 filters are the better choice
bool single_tiled_supports(const Shape& s);
int single_split_filters(const Shape& s);      // filters of the first of two launches of the special-case kernel, 0 for one launch
bool single_general_preferred(const Shape& s); // one image of one channel: the general-case kernel is the better choice
bool single_batch_preferred(const Shape& s);   // dconv_general with up to four channels: the special-case kernel is the better choice
bool general_tiled_supports(const Shape& s);
void release_general_workspaces();
// Short data types (dtype: DCONV_DTYPE_*, layout: DCONV_LAYOUT_*); variant: AUTO, SIMPLE, TILED
// or TILED_CFG0 + i.  `out` receives fp32 values, or int32 bit patterns for 8-bit integer inputs.
int launch_general_half(const void* in, const void* filt, float* out, const Shape& s, hipStream_t st,
                        int dtype, int layout, int variant);

}  // namespace dconv
