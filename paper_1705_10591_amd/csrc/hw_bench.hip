// Microbenchmarks of the hardware rates that shaped the kernels (standalone program, no part of
// libdconv.so):
//   1. HBM: fill, read and copy rates, and the rate of the single-channel kernel's store pattern
//      -- 128-byte runs, 32 consecutive pixels of one output map -- when the rows of a map are a
//      whole number of 128-byte lines long (runs cover lines exactly) and when they are not (most
//      runs straddle two lines, each written in two pieces);
//   2. the fp32 matrix-core loop of the general kernel (two operand pairs from LDS per four
//      v_mfma_f32_32x32x2_f32) bare and with 8, 16, 32 integer vector-ALU instructions added per
//      four matrix-core instructions: what an ordinary vector instruction costs the matrix cores.
//
//   3. the bf16 matrix-core loop (v_mfma_f32_32x32x16_bf16) with operands in registers and fed
//      from LDS, 16 bytes per lane and operand: what the chip sustains of its 16-bit peak.
//   4. fp32 matrix-core waves and store waves on the same SIMD: the two do not overlap -- the
//      stores advance only in the gaps the matrix-core instruction stream leaves -- while a
//      wave's own stores between its own matrix-core instructions do.
//
// `hw_bench --quick` runs only the rates that bench.py quotes as measured achievable peaks
// beside the published ones: fill, read, and the bare fp32 and bf16 matrix-core loops.
#include <hip/hip_runtime.h>
#include <string>
#include <cstdio>
#include <cstring>

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

#define CHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
    fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 1; } } while (0)

// ---- 1. HBM ---------------------------------------------------------------------------------------

__global__ void fill16(v4f* o, size_t n) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) o[i] = (v4f){1, 2, 3, 4};
}
__global__ void read16(const v4f* a, float* o, size_t n) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    float s = 0.f;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) { v4f v = a[i]; s += v[0] + v[3]; }
    if (s == 123.456f) o[0] = s;          // never true for the zeros read: keeps the loads alive
}
__global__ void copy16(const v4f* a, v4f* o, size_t n) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) o[i] = a[i];
}
// 32 maps of `rows` x `w` floats.  A wave takes a 128-pixel segment of one row and writes it to
// all 32 maps: the lanes of half h write 32 consecutive pixels (128 bytes) of map 2 q + h.
template <bool NT>
__global__ void store_runs(float* o, int w, int rows) {
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, lane = threadIdx.x & 63;
    const int h = lane >> 5, l = lane & 31;
    const int segs = (w + 127) / 128, total = rows * segs, nwaves = (gridDim.x * blockDim.x) >> 6;
    for (int it = wave; it < total; it += nwaves) {
        const int r = it / segs, s = it % segs;
        for (int q = 0; q < 16; ++q) {
            float* row = o + ((size_t)(2 * q + h) * rows + r) * w;
            for (int nb = 0; nb < 4; ++nb) {
                const int x = s * 128 + nb * 32 + l;
                if (x < w) {
                    if (NT) __builtin_nontemporal_store(1.f, row + x);
                    else row[x] = 1.f;
                }
            }
        }
    }
}

// ---- 2. matrix cores next to vector-ALU work ----------------------------------------------------

// What the LDS operands of the matrix-core loops hold.  0: a ramp (neighbouring words differ in
// a few low bits), 1: zeros, 2: pseudo-random bits in sign and mantissa, exponents of about one
// (as fp32 words; as pairs of bf16 values in the 16-bit loop).  The instruction stream is the
// same for all three; how fast it runs is not (section 5).
__device__ __forceinline__ float operand_word(int i, int fill, bool halves) {
    if (fill == 0) return i * 0.001f;
    if (fill == 1) return 0.f;
    unsigned x = (unsigned)i * 2654435761u;
    x ^= x >> 15; x *= 2246822519u; x ^= x >> 13;
    if (halves) {
        const unsigned lo = 0x3F80u | (x & 0x807Fu), hi = 0x3F80u | ((x >> 16) & 0x807Fu);
        return __uint_as_float((hi << 16) | lo);
    }
    return __uint_as_float(0x3F800000u | (x & 0x807FFFFFu));
}

// NV integer vector instructions per four matrix-core instructions; 36 steps between barriers.
template <int NV>
__global__ void __launch_bounds__(256, 2) mfma_loop(float* o, int trips, int fill) {
    __shared__ float sh[12288];
    for (int i = threadIdx.x; i < 12288; i += 256) sh[i] = operand_word(i, fill, false);
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int busy[8];
    for (int i = 0; i < 8; ++i) busy[i] = threadIdx.x + i;
    v16f acc[4];
    for (int n = 0; n < 4; ++n) for (int i = 0; i < 16; ++i) acc[n][i] = 0.f;
    const int ba = (lane >> 5) * 129 + (wave & 1) * 64 + (lane & 31);         // weights: 73 rows of 129 words
    const int bb = 9288 + (lane & 31) + (lane >> 5) + (wave >> 1) * 64;       // pixels: rows of 28 words
    for (int t = 0; t < trips; ++t) {
        float a0 = sh[ba], a1 = sh[ba + 32], b0 = sh[bb], b1 = sh[bb + 32];
#pragma unroll
        for (int s = 0; s < 36; ++s) {
            float na0 = 0.f, na1 = 0.f, nb0 = 0.f, nb1 = 0.f;
            if (s + 1 < 36) {         // operands of the next step, requested before this step's arithmetic
                na0 = sh[ba + (2 * s + 2) * 129];
                na1 = sh[ba + (2 * s + 2) * 129 + 32];
                nb0 = sh[bb + ((s + 1) % 9) * 28 + ((s + 1) / 9) * 280];
                nb1 = sh[bb + 32 + ((s + 1) % 9) * 28 + ((s + 1) / 9) * 280];
            }
#pragma unroll
            for (int v = 0; v < NV; ++v) busy[v & 7] = busy[v & 7] * 3 + lane + s;
            __builtin_amdgcn_sched_barrier(0);
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[1], 0, 0, 0);
            acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[2], 0, 0, 0);
            acc[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[3], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            a0 = na0; a1 = na1; b0 = nb0; b1 = nb1;
        }
        __syncthreads();
    }
    float r = 0.f;
    for (int i = 0; i < 8; ++i) r += (float)busy[i];
    for (int n = 0; n < 4; ++n) for (int i = 0; i < 16; ++i) r += acc[n][i];
    o[blockIdx.x * 256 + threadIdx.x] = r;
}

// ---- 3. the 16-bit matrix-core loop ----------------------------------------------------------------

typedef __bf16 v8b __attribute__((ext_vector_type(8)));
// 2 x 2 blocks of v_mfma_f32_32x32x16_bf16 per wave; FEED: operands re-read from LDS every step
// (16 bytes per lane and operand, the next step's requested before this step's arithmetic) or
// kept in registers.  36 steps between barriers.
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
template <bool I8>
__device__ __forceinline__ v16f mfma_short(v4f a, v4f b, v16f c) {
    if (I8) return __builtin_bit_cast(v16f, __builtin_amdgcn_mfma_i32_32x32x32_i8(
        __builtin_bit_cast(v4i, a), __builtin_bit_cast(v4i, b), __builtin_bit_cast(v16i, c), 0, 0, 0));
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8b, a), __builtin_bit_cast(v8b, b), c, 0, 0, 0);
}
template <bool FEED, bool I8 = false>
__global__ void __launch_bounds__(256, 2) mfma16_loop(float* o, int trips, int fill) {
    __shared__ __attribute__((aligned(16))) float sh[12288];
    for (int i = threadIdx.x; i < 12288; i += 256) sh[i] = operand_word(i, fill, !I8);
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    v16f acc[4];
    for (int n = 0; n < 4; ++n) for (int i = 0; i < 16; ++i) acc[n][i] = 0.f;
    const v4f* q = reinterpret_cast<const v4f*>(sh) + lane + (wave & 1) * 64;   // 16-byte pieces
    for (int t = 0; t < trips; ++t) {
        v4f a0 = q[0], a1 = q[128], b0 = q[256], b1 = q[384];
#pragma unroll
        for (int s = 0; s < 36; ++s) {
            v4f na0 = a0, na1 = a1, nb0 = b0, nb1 = b1;
            if (FEED && s + 1 < 36) {
                na0 = q[((s + 1) % 4) * 512];
                na1 = q[((s + 1) % 4) * 512 + 128];
                nb0 = q[((s + 1) % 4) * 512 + 256];
                nb1 = q[((s + 1) % 4) * 512 + 384];
            }
            __builtin_amdgcn_sched_barrier(0);
            acc[0] = mfma_short<I8>(a0, b0, acc[0]);
            acc[1] = mfma_short<I8>(a0, b1, acc[1]);
            acc[2] = mfma_short<I8>(a1, b0, acc[2]);
            acc[3] = mfma_short<I8>(a1, b1, acc[3]);
            __builtin_amdgcn_sched_barrier(0);
            a0 = na0; a1 = na1; b0 = nb0; b1 = nb1;
        }
        __syncthreads();
    }
    float r = 0.f;
    for (int n = 0; n < 4; ++n) for (int i = 0; i < 16; ++i) r += acc[n][i];
    o[blockIdx.x * 256 + threadIdx.x] = r;
}

// ---- 4. matrix cores and a store stream on the same SIMD ------------------------------------------

// Eight waves per workgroup, one workgroup per CU: waves 0-3 (one per SIMD) issue fp32
// matrix-core instructions back to back, four independent chains, with GAP idle slots of 16
// clocks after every four; waves 4-7 (the second wave of each SIMD) store `n4` 16-byte pieces
// from a uniform base with a constant lane offset, so that a store costs no vector-ALU
// instruction.  mode: 1 = only the matrix-core waves work, 2 = only the store waves, 3 = both.
template <int GAP>
__global__ void __launch_bounds__(512, 1) mfma_and_stores(float* o, v4f* big, size_t n4, int iters, int mode) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (wave < 4) {
        if (!(mode & 1)) return;
        float a = lane * 0.1f, b = 1.5f;
        v16f acc[4];
        for (int n = 0; n < 4; ++n) for (int i = 0; i < 16; ++i) acc[n][i] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int q = 0; q < GAP; ++q) asm volatile("s_nop 15");
#pragma unroll
            for (int n = 0; n < 4; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[n], 0, 0, 0);
        }
        float r = 0.f;
        for (int n = 0; n < 4; ++n) for (int i = 0; i < 16; ++i) r += acc[n][i];
        o[blockIdx.x * 256 + threadIdx.x] = r;
    } else {
        if (!(mode & 2)) return;
        const int uw = __builtin_amdgcn_readfirstlane(wave);
        const size_t stp = (size_t)gridDim.x * 4 * 64;
        const v4f v = {1, 2, 3, 4};
        for (size_t i = ((size_t)blockIdx.x * 4 + (uw - 4)) * 64; i + 64 <= n4; i += stp) big[i + lane] = v;
    }
}

// The same two streams in ONE wave per SIMD: after every four matrix-core instructions the wave
// issues SPM of its stores.  mode as above.
template <int SPM>
__global__ void __launch_bounds__(256, 1) mfma_own_stores(float* o, v4f* big, size_t n4, int iters, int mode) {
    const int lane = threadIdx.x & 63;
    const int uw = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    float a = lane * 0.1f, b = 1.5f;
    v16f acc[4];
    for (int n = 0; n < 4; ++n) for (int i = 0; i < 16; ++i) acc[n][i] = 0.f;
    const size_t stp = (size_t)gridDim.x * 4 * 64;
    size_t i = ((size_t)blockIdx.x * 4 + uw) * 64;
    const v4f v = {1, 2, 3, 4};
    for (int it = 0; it < iters; ++it) {
        if (mode & 1) {
#pragma unroll
            for (int n = 0; n < 4; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[n], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (mode & 2) {
#pragma unroll
            for (int q = 0; q < SPM; ++q) {
                if (i + 64 <= n4) big[i + lane] = v;
                i += stp;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    float r = 0.f;
    for (int n = 0; n < 4; ++n) for (int q = 0; q < 16; ++q) r += acc[n][q];
    o[blockIdx.x * 256 + threadIdx.x] = r;
}

template <class L>
int time_ms(L launch, int reps, float* ms) {
    hipEvent_t a, b;
    CHECK(hipEventCreate(&a));
    CHECK(hipEventCreate(&b));
    launch();
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(a));
    for (int i = 0; i < reps; ++i) launch();
    CHECK(hipEventRecord(b));
    CHECK(hipEventSynchronize(b));
    CHECK(hipEventElapsedTime(ms, a, b));
    *ms /= reps;
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int main(int argc, char** argv) {
    const bool quick = argc > 1 && strcmp(argv[1], "--quick") == 0;
    int cus = 0;
    CHECK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, 0));
    const size_t bytes = (size_t)4 << 30, n16 = bytes / 16;
    float *a = nullptr, *b = nullptr;
    CHECK(hipMalloc(&a, bytes));
    CHECK(hipMalloc(&b, bytes));
    CHECK(hipMemset(a, 0, bytes));
    float ms = 0.f;
    printf("# HBM, 4 GiB buffers, %d CUs\n", cus);
    if (time_ms([&] { hipLaunchKernelGGL(fill16, dim3(8192), dim3(256), 0, 0, (v4f*)b, n16); }, 20, &ms)) return 1;
    printf("fill, 16 B per lane:                        %7.3f ms  %6.0f GB/s\n", ms, bytes / ms / 1e6);
    if (time_ms([&] { hipLaunchKernelGGL(read16, dim3(8192), dim3(256), 0, 0, (const v4f*)a, b, n16); }, 20, &ms)) return 1;
    printf("read, 16 B per lane:                        %7.3f ms  %6.0f GB/s\n", ms, bytes / ms / 1e6);
    if (!quick) {
    if (time_ms([&] { hipLaunchKernelGGL(copy16, dim3(8192), dim3(256), 0, 0, (const v4f*)a, (v4f*)b, n16); }, 5, &ms)) return 1;
    printf("copy, 16 B per lane (read + written):       %7.3f ms  %6.0f GB/s\n", ms, 2.0 * bytes / ms / 1e6);
    }
    for (int w : {4096, 4092}) {
        if (quick) break;
        const int rows = w == 4096 ? 8176 : 8184;           // 32 maps just under 4 GiB
        const size_t total = (size_t)32 * rows * w * 4;
        if (total > bytes) return 1;
        if (time_ms([&] { hipLaunchKernelGGL(store_runs<false>, dim3(8192), dim3(256), 0, 0, b, w, rows); }, 3, &ms)) return 1;
        printf("128 B runs, rows of %d floats:              %7.3f ms  %6.0f GB/s\n", w, ms, total / ms / 1e6);
        if (time_ms([&] { hipLaunchKernelGGL(store_runs<true>, dim3(8192), dim3(256), 0, 0, b, w, rows); }, 3, &ms)) return 1;
        printf("128 B runs, rows of %d floats, nontemporal: %7.3f ms  %6.0f GB/s\n", w, ms, total / ms / 1e6);
    }
    printf("# fp32 matrix-core loop fed from LDS, 2 workgroups of 4 waves per CU, 36 steps per barrier\n");
    const int blocks = 2 * cus, trips = 2000;
    const double flop = (double)blocks * 4 * trips * 36 * 4 * 4096.0;
    if (time_ms([&] { hipLaunchKernelGGL(mfma_loop<0>, dim3(blocks), dim3(256), 0, 0, b, trips, 0); }, 2, &ms)) return 1;
    printf("no other vector instructions:               %7.3f ms  %6.1f TFLOP/s\n", ms, flop / ms / 1e9);
    if (!quick) {
    if (time_ms([&] { hipLaunchKernelGGL(mfma_loop<8>, dim3(blocks), dim3(256), 0, 0, b, trips, 0); }, 2, &ms)) return 1;
    printf("+ 8 integer VALU per 4 MFMA:                %7.3f ms  %6.1f TFLOP/s\n", ms, flop / ms / 1e9);
    if (time_ms([&] { hipLaunchKernelGGL(mfma_loop<16>, dim3(blocks), dim3(256), 0, 0, b, trips, 0); }, 2, &ms)) return 1;
    printf("+ 16 integer VALU per 4 MFMA:               %7.3f ms  %6.1f TFLOP/s\n", ms, flop / ms / 1e9);
    if (time_ms([&] { hipLaunchKernelGGL(mfma_loop<32>, dim3(blocks), dim3(256), 0, 0, b, trips, 0); }, 2, &ms)) return 1;
    printf("+ 32 integer VALU per 4 MFMA:               %7.3f ms  %6.1f TFLOP/s\n", ms, flop / ms / 1e9);
    }
    {
        printf("# bf16 matrix-core loop (v_mfma_f32_32x32x16_bf16), 2 workgroups of 4 waves per CU, 2 x 2 blocks per wave\n");
        const int trips16 = 4000;
        const double flop16 = (double)blocks * 4 * trips16 * 36 * 4 * 32768.0;
        if (time_ms([&] { hipLaunchKernelGGL(mfma16_loop<false>, dim3(blocks), dim3(256), 0, 0, b, trips16, 0); }, 2, &ms)) return 1;
        printf("bf16, operands in registers:                %7.3f ms  %6.1f TFLOP/s\n", ms, flop16 / ms / 1e9);
        if (time_ms([&] { hipLaunchKernelGGL(mfma16_loop<true>, dim3(blocks), dim3(256), 0, 0, b, trips16, 0); }, 2, &ms)) return 1;
        printf("bf16, operands from LDS every step:         %7.3f ms  %6.1f TFLOP/s\n", ms, flop16 / ms / 1e9);
        // (the 8-bit instruction does twice the operations per instruction)
        if (time_ms([&] { hipLaunchKernelGGL((mfma16_loop<true, true>), dim3(blocks), dim3(256), 0, 0, b, trips16, 0); }, 2, &ms)) return 1;
        printf("int8, operands from LDS every step:         %7.3f ms  %6.1f TOP/s\n", ms, 2.0 * flop16 / ms / 1e9);
    }
    if (quick) {
        CHECK(hipFree(a));
        CHECK(hipFree(b));
        return 0;
    }
    printf("# fp32 matrix-core waves and store waves sharing every SIMD (one of each), 4 GiB stored, 12000 matrix-core instructions per wave\n");
    {
        const int iters = 3000;
        for (int gap = 0; gap < 3; ++gap) {
            float t[3];
            for (int mode = 1; mode <= 3; ++mode) {
                auto go = [&] {
                    if (gap == 0) hipLaunchKernelGGL(mfma_and_stores<0>, dim3(cus), dim3(512), 0, 0, a, (v4f*)b, n16, iters, mode);
                    else if (gap == 1) hipLaunchKernelGGL(mfma_and_stores<2>, dim3(cus), dim3(512), 0, 0, a, (v4f*)b, n16, iters, mode);
                    else hipLaunchKernelGGL(mfma_and_stores<8>, dim3(cus), dim3(512), 0, 0, a, (v4f*)b, n16, iters, mode);
                };
                if (time_ms(go, 3, &t[mode - 1])) return 1;
            }
            printf("%3d idle clocks per 4 MFMA: matrix cores alone %6.3f ms, stores alone %6.3f ms, together %6.3f ms\n",
                   gap == 0 ? 0 : gap == 1 ? 32 : 128, t[0], t[1], t[2]);
        }
    }
    printf("# the same in ONE wave per SIMD: its own stores between its matrix-core instructions, 4 GiB stored\n");
    {
        float t[3];
        for (int mode = 1; mode <= 3; ++mode)
            if (time_ms([&] { hipLaunchKernelGGL(mfma_own_stores<1>, dim3(cus), dim3(256), 0, 0, a, (v4f*)b, n16, 4096, mode); }, 3, &t[mode - 1])) return 1;
        printf("1 store per 4 MFMA:  matrix cores alone %6.3f ms, stores alone %6.3f ms, interleaved %6.3f ms\n", t[0], t[1], t[2]);
        for (int mode = 1; mode <= 3; ++mode)
            if (time_ms([&] { hipLaunchKernelGGL(mfma_own_stores<2>, dim3(cus), dim3(256), 0, 0, a, (v4f*)b, n16, 2048, mode); }, 3, &t[mode - 1])) return 1;
        printf("2 stores per 4 MFMA: matrix cores alone %6.3f ms, stores alone %6.3f ms, interleaved %6.3f ms\n", t[0], t[1], t[2]);
    }
    {
        // 5. the same matrix-core loops on other operand VALUES: the chip's clock is managed by
        // power, and what a multiplier array draws depends on the bits it is fed.  Ten launches
        // each (some 150 ms), so that the clock has settled.
        printf("# the matrix-core loops of sections 2 and 3 by what their operands hold (same instructions; 10 launches each)\n");
        const int trips16 = 4000;
        const double flop16 = (double)blocks * 4 * trips16 * 36 * 4 * 32768.0;
        const char* names[3] = {"a ramp", "zeros", "random bits"};
        for (int fill = 1; fill <= 2; ++fill) {
            if (time_ms([&] { hipLaunchKernelGGL(mfma_loop<0>, dim3(blocks), dim3(256), 0, 0, b, trips, fill); }, 10, &ms)) return 1;
            printf("fp32 loop, operands %-12s           %7.3f ms  %6.1f TFLOP/s\n", (std::string(names[fill]) + ":").c_str(), ms, flop / ms / 1e9);
        }
        for (int fill = 1; fill <= 2; ++fill) {
            if (time_ms([&] { hipLaunchKernelGGL(mfma16_loop<true>, dim3(blocks), dim3(256), 0, 0, b, trips16, fill); }, 10, &ms)) return 1;
            printf("bf16 loop, operands %-12s           %7.3f ms  %6.1f TFLOP/s\n", (std::string(names[fill]) + ":").c_str(), ms, flop16 / ms / 1e9);
        }
    }
    CHECK(hipFree(a));
    CHECK(hipFree(b));
    return 0;
}
