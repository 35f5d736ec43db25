// The paper's bank-width experiment (Sec. 2-3: a thread should read units as wide as a bank of
// the on-chip memory, or bandwidth is lost), repeated on the LDS of a CDNA4 compute unit: how
// many bytes per clock and CU do stride-1 reads (and writes) of 2, 4, 8 and 16 bytes per lane
// reach?  LDS banks are 4 bytes wide, so the 2-byte case is the paper's "unmatched" one.
//
// Standalone program (no part of libdconv.so): four waves per workgroup, two workgroups per CU,
// sixteen accesses per loop trip, each through its own address register.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));

constexpr int kWords = 16384;         // 64 KiB of LDS per workgroup: 16 KiB per wave
constexpr int kUnroll = 16;
#define LDS_PTR(T) __attribute__((address_space(3))) T*

// BYTES per lane and access; WRITE: stores instead of loads.  Lane l of wave w touches
// bytes [l * BYTES, (l + 1) * BYTES) of its wave's 16 KiB region, plus u * 64 * BYTES for the
// u-th access of a trip.
template <int BYTES, bool WRITE>
__global__ void __launch_bounds__(256) lds_width_kernel(float* sink, int trips)
{
    __shared__ __attribute__((aligned(16))) float sh[kWords];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < kWords; i += 256) sh[i] = (float)i;
    __syncthreads();
    constexpr int kStep = 64 * BYTES;                 // bytes one access of a wave covers
    // every access of a trip goes through an address register of its own that the compiler
    // cannot relate to the others, so that it does not pair accesses into two-address
    // instructions (ds_read2 / ds_write2)
    LDS_PTR(char) addr[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        addr[u] = (LDS_PTR(char))(sh + wave * 4096) + lane * BYTES + u * kStep;
        asm volatile("" : "+v"(addr[u]));
    }
    float acc = 0.f;
    const float val = (float)lane;
    for (int t = 0; t < trips; ++t) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            LDS_PTR(char) p = addr[u];
            if (WRITE) {
                if (BYTES == 2) *(LDS_PTR(unsigned short))p = (unsigned short)lane;
                if (BYTES == 4) *(LDS_PTR(float))p = val;
                if (BYTES == 8) *(LDS_PTR(v2f))p = (v2f){val, val};
                if (BYTES == 16) *(LDS_PTR(v4f))p = (v4f){val, val, val, val};
            } else {
                if (BYTES == 2) acc += (float)*(LDS_PTR(unsigned short))p;
                if (BYTES == 4) acc += *(LDS_PTR(float))p;
                if (BYTES == 8) { v2f v = *(LDS_PTR(v2f))p; acc += v[0] + v[1]; }
                if (BYTES == 16) { v4f v = *(LDS_PTR(v4f))p; acc += v[0] + v[3]; }
            }
        }
        // (the compiler may not carry loaded values or pending stores over to the next trip)
        asm volatile("" ::: "memory");
    }
    sink[blockIdx.x * 256 + threadIdx.x] = acc + sh[threadIdx.x];
}

#define CHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
    fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 1; } } while (0)

template <int BYTES, bool WRITE>
int run(float* sink, int blocks, int trips, int cus, double ghz)
{
    hipEvent_t a, b;
    CHECK(hipEventCreate(&a));
    CHECK(hipEventCreate(&b));
    hipLaunchKernelGGL((lds_width_kernel<BYTES, WRITE>), dim3(blocks), dim3(256), 0, 0, sink, trips);
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(a));
    for (int r = 0; r < 3; ++r)
        hipLaunchKernelGGL((lds_width_kernel<BYTES, WRITE>), dim3(blocks), dim3(256), 0, 0, sink, trips);
    CHECK(hipEventRecord(b));
    CHECK(hipEventSynchronize(b));
    float ms = 0.f;
    CHECK(hipEventElapsedTime(&ms, a, b));
    ms /= 3.f;
    const double bytes = (double)blocks * 256 * trips * kUnroll * BYTES;
    printf("%-5s %2d B per lane: %8.3f ms  %6.1f B/clk/CU\n", WRITE ? "write" : "read", BYTES, ms,
           bytes / (ms * 1e-3) / cus / (ghz * 1e9));
    return 0;
}

int main(int argc, char** argv)
{
    const double ghz = argc > 1 ? atof(argv[1]) : 2.4;      // clock the rates are quoted at
    int cus = 0;
    CHECK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, 0));
    const int blocks = 2 * cus, trips = 2000;
    float* sink = nullptr;
    CHECK(hipMalloc(&sink, (size_t)blocks * 256 * sizeof(float)));
    printf("# LDS stride-1 access rates, %d CUs, %d workgroups of 256 threads, quoted at %.2f GHz\n", cus, blocks, ghz);
    if (run<2, false>(sink, blocks, trips, cus, ghz) || run<4, false>(sink, blocks, trips, cus, ghz) ||
        run<8, false>(sink, blocks, trips, cus, ghz) || run<16, false>(sink, blocks, trips, cus, ghz) ||
        run<2, true>(sink, blocks, trips, cus, ghz) || run<4, true>(sink, blocks, trips, cus, ghz) ||
        run<8, true>(sink, blocks, trips, cus, ghz) || run<16, true>(sink, blocks, trips, cus, ghz))
        return 1;
    CHECK(hipFree(sink));
    return 0;
}
