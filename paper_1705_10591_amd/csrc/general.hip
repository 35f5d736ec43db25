// General-case direct convolution: dispatch over filter side, tile shape and schedule, and
// the workspace that shared tiles are summed through.  The kernel is in general_kernel.h.
#include <map>
#include <mutex>
#include <utility>
#include <vector>
#include "general_kernel.h"

namespace dconv {

// ---- workspace ---------------------------------------------------------------------------------
// One per (device, stream): launches on one stream run in order and may share it; launches on
// different streams may overlap and must not.  It holds the partial sums of tiles shared by
// several workgroups and one arrival counter per workgroup.  The counters are zero between
// launches: the workgroup that completes a tile resets its counter.
//
// A block, once handed out, keeps its address until release_general_workspaces(): kernel
// arguments hold it by value, so a HIP graph captured on the stream refers to it for as long as
// the graph lives.  The first request on a (device, stream) therefore allocates what the
// largest launch on that device can need (a launch has at most OCC workgroups per CU, each with
// two partial tiles), and later requests find it large enough.  Should a request ever exceed it
// (a forced grid), a larger block is allocated beside the old one, which is kept until release.
namespace {

// floats of partial sums and counters per CU that cover every compiled tile shape:
// 64 x 256 tiles at two workgroups per CU (2 * 2 * 16384), 64 x 128 or 32 x 256 at three
constexpr size_t kPartFloatsPerCu = 2 * 2 * 64 * 256;
constexpr size_t kCountersPerCu = 4;

struct WsEntry {
    float* part = nullptr;
    size_t part_floats = 0;
    int* cnt = nullptr;
    size_t ncnt = 0;
    std::vector<void*> retired;      // outgrown blocks: freed only by release_general_workspaces()
};
std::mutex g_ws_mutex;
std::map<std::pair<int, hipStream_t>, WsEntry> g_ws;

}  // namespace

GenWorkspace gen_workspace(hipStream_t st, size_t part_floats, size_t ncnt)
{
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return {nullptr, nullptr};
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    WsEntry& e = g_ws[{dev, st}];
    if (e.part_floats >= part_floats && e.ncnt >= ncnt) return {e.part, e.cnt};
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return {nullptr, nullptr};
    if (e.part_floats < part_floats) {
        const size_t want = std::max(part_floats, kPartFloatsPerCu * (size_t)cus);
        float* fresh = nullptr;
        if (hipMalloc((void**)&fresh, want * sizeof(float)) != hipSuccess) {
            (void)hipGetLastError();
            return {nullptr, nullptr};
        }
        if (e.part) e.retired.push_back(e.part);
        e.part = fresh;
        e.part_floats = want;
    }
    if (e.ncnt < ncnt) {
        const size_t want = std::max(ncnt, kCountersPerCu * (size_t)cus);
        int* fresh = nullptr;
        // (the one place where a call may not be captured into a graph: first use on a stream)
        if (hipMalloc((void**)&fresh, want * sizeof(int)) != hipSuccess ||
            hipMemsetAsync(fresh, 0, want * sizeof(int), st) != hipSuccess) {
            if (fresh) (void)hipFree(fresh);
            (void)hipGetLastError();
            return {nullptr, nullptr};
        }
        if (e.cnt) e.retired.push_back(e.cnt);
        e.cnt = fresh;
        e.ncnt = want;
    }
    return {e.part, e.cnt};
}

void release_general_workspaces()
{
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    for (auto& kv : g_ws) {
        if (kv.second.part) (void)hipFree(kv.second.part);
        if (kv.second.cnt) (void)hipFree(kv.second.cnt);
        for (void* q : kv.second.retired) (void)hipFree(q);
    }
    g_ws.clear();
}

// ---- the static scratch array of dconv_general_noalloc --------------------------------------------
// The same two things as the workspace above -- arrival counters, then partial sums -- in device
// memory that comes with the library's code object: every GPU the library runs on holds its own
// copy of the array, at its own address, from the moment the code object is loaded there until
// the process ends.  In host code the array's name only stands for the symbol; its address on
// the current device is looked up once per device and that pointer is what kernels are given.
// All calls on a device share the array (one call at a time, see dconv.h) and it keeps what the
// last call left: the counters a launch uses are cleared on its stream before it, by a kernel,
// so that the call can be captured into a graph.
namespace {

constexpr size_t kScratchCounters = 4096;               // ints: 16 KiB, then the partial sums
constexpr size_t kScratchPartFloats = (size_t)16 << 20; // 64 MiB: 512 workgroups x 2 x (64 x 256)
constexpr size_t kScratchBytes = 4 * (kScratchCounters + kScratchPartFloats);
constexpr int kMaxDevices = 64;

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices] = {};         // device address of `scratch`, per device

__global__ void clear_counters_kernel(int* cnt, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) cnt[i] = 0;
}

}  // namespace

int gen_static_workspace(hipStream_t st, size_t part_floats, size_t ncnt, GenWorkspace* ws)
{
    if (part_floats > kScratchPartFloats || ncnt > kScratchCounters) return DCONV_SCRATCH_EXCEEDED;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DCONV_LAUNCH_FAILED;
    unsigned char* base;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            void* q = nullptr;
            if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || !q) {
                (void)hipGetLastError();
                return DCONV_LAUNCH_FAILED;
            }
            g_scratch_ptr[dev] = (unsigned char*)q;
        }
        base = g_scratch_ptr[dev];
    }
    ws->cnt = (int*)base;
    ws->part = (float*)(base + 4 * kScratchCounters);
    begin_launch();
    hipLaunchKernelGGL(clear_counters_kernel, dim3((unsigned)((ncnt + kThreads - 1) / kThreads)),
                       dim3(kThreads), 0, st, ws->cnt, (int)ncnt);
    return launch_status();
}

// ---- dispatch ----------------------------------------------------------------------------------

namespace {

// Tile configurations offered through the ABI: tile shape x schedule.
//   shape    0: 64 filters x 128 pixels, 1: 64 x 256, 2: 32 x 256
//   schedule 0: by shape, 1: whole tiles only, 2: tiles cut over channels wherever the even
//            split of the work falls, 3: the same on a grid of 7 workgroups (so that small
//            test shapes exercise every way a tile can be shared)
//   write-back: configurations 0 to 11 store straight from the accumulators, 12 to 23 are the
//            same twelve with tiles written back in whole 128-byte lines through LDS (the
//            reorganisation through on-chip memory that the paper leaves open, Sec. 4.2).
//            Measured against each other (paper_1705_10591_amd.tune writeback): the second is
//            never faster, so no shape gets it by itself.  Outputs that fit the 256 MB
//            memory-side cache do not care about line alignment at all; larger ones of narrow
//            maps break even at best, because every accumulator then passes the register file's
//            ports three times (to LDS, back, to memory) instead of once, and those ports are
//            what stores compete for with the matrix cores; wide maps lose up to 40 %, because
//            column strips cut every row into segments whose ends are partial lines anyway.
constexpr int kShapes = 3, kSchedules = 4, kWriteBacks = 2;

int launch_any(const float* in, const float* filt, float* out, const Shape& s, hipStream_t st,
               int tile_cfg, const GenSched& sched, bool dry)
{
    switch (s.F) {
    case 1: return gen_launch_for_F<1>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 2: return gen_launch_for_F<2>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 3: return gen_launch_for_F<3>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 4: return gen_launch_for_F<4>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 5: return gen_launch_for_F<5>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 6: return gen_launch_for_F<6>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 7: return gen_launch_for_F<7>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 8: return gen_launch_for_F<8>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 9: return gen_launch_for_F<9>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 10: return gen_launch_for_F<10>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 11: return gen_launch_for_F<11>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 12: return gen_launch_for_F<12>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 13: return gen_launch_for_F<13>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 14: return gen_launch_for_F<14>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 15: return gen_launch_for_F<15>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 16: return gen_launch_for_F<16>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 17: return gen_launch_for_F<17>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 18: return gen_launch_for_F<18>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 19: return gen_launch_for_F<19>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 20: return gen_launch_for_F<20>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 21: return gen_launch_for_F<21>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 22: return gen_launch_for_F<22>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 23: return gen_launch_for_F<23>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 24: return gen_launch_for_F<24>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 25: return gen_launch_for_F<25>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 26: return gen_launch_for_F<26>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 27: return gen_launch_for_F<27>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 28: return gen_launch_for_F<28>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 29: return gen_launch_for_F<29>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 30: return gen_launch_for_F<30>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 31: return gen_launch_for_F<31>(in, filt, out, s, st, tile_cfg, sched, dry);
    case 32: return gen_launch_for_F<32>(in, filt, out, s, st, tile_cfg, sched, dry);
    default: return DCONV_UNSUPPORTED;
    }
}

// Tile shape by problem shape, from the tile search (paper_1705_10591_amd.tune) over forty layer
// shapes and from timing the three shapes on 630 layers drawn at random (3 to 512 channels, 16 to
// 512 filters of 1x1 to 7x7, 7 x 7 to 224 x 224 maps, 0.5 to 30 GFLOP); the rule below is within
// 1 % of the fastest shape on their average (4 % before it was refitted on them).
int shape_for(const Shape& s)
{
    const int64_t px = (int64_t)s.N * s.Ho * s.Wo;
    const int64_t wide_tiles = (px + 255) / 256, fblocks = (s.K + 63) / 64;
    const int64_t tiles = wide_tiles * fblocks;           // of the 64 x 256 shape
    const int taps = s.C * s.F * s.F;                      // multiply-adds per output element
    const int64_t chunks = ((int64_t)taps + 35) / 36;
    const bool tiny = (int64_t)s.Ho * s.Wo < 100;
    // Up to 32 filters: the 32 x 256 tile, so that half of every filter block is not padding
    // (1x1 filters on tiny maps, where a 256-pixel tile reaches over several images: 64 x 128).
    // (and 1x1 filters on 64 channels or more in a launch of under a hundred wide tiles: the
    // 64 x 128 tile's three workgroups per CU hide the barrier per chunk, which counts for more
    // than the padded half block -- kernel times from replayed graphs, 8 x 64 x 28 x 28 with 32
    // filters: 11.7 -> 8.8 us)
    if (s.K <= 32) return (s.F == 1 && (tiny || (s.C >= 64 && wide_tiles < 100))) ? 0 : 2;
    // Filter counts whose last block of 64 is at most half full (96, 160, 224, 288): the 32 x 256
    // tile computes 25, 17, 12, 10 % fewer padded filters and is 20, 10, 5, 4 % faster from 3x3
    // on (and for the smaller filters with few channels); on tiny maps only for 96.
    // (with few tiles only where a quarter is saved)
    if (s.K % 64 != 0 && s.K % 64 <= 32 && (s.F >= 3 || taps <= 64)) {
        const int k32 = (s.K + 31) / 32 * 32, k64 = (int)fblocks * 64;
        const bool quarter = k32 * 100 <= k64 * 76;
        if (tiles >= (quarter ? 20 : 100) && (quarter || (!tiny && k32 * 100 <= k64 * 91))) return 2;
    }
    // 1x1 filters: a chunk is sixteen channels, eight matrix-core steps and a barrier, whatever
    // the tile, and the 64 x 128 tile's three workgroups per CU hide that better than the four
    // matrix-core instructions per step of the 64 x 256 tile pay: 10-80 % faster from 128
    // channels on, and from 64 on maps up to 64 wide (14 x 14 .. 224 x 224 maps, 32 to 512
    // channels, 64 to 512 filters); with fewer channels or on wider maps the large tile's
    // fewer, longer output runs win by up to 30 %.
    // (a launch of a few tiles: the 32 x 256 tile, twice the tiles, 10-25 % faster in kernel
    // time on 7 x 7 .. 56 x 56 maps with 16 or 32 channels)
    if (s.F == 1) return (s.C >= 128 || (s.C >= 64 && s.Wo <= 64)) ? 0 : tiles < 64 ? 2 : 1;
    // Tiny maps (under a hundred outputs per image): a 256-pixel tile reaches over several
    // images, each with its halo rows in the image block; the 128-pixel tile is 20-35 % faster
    // (7 x 7 outputs, 64 to 512 channels and filters, hundreds of images).
    if (tiny) return 0;
    // 2x2 filters are like 1x1 ones: eight channels a chunk, and beyond 40 channels the small
    // tile is 13-34 % faster (maps up to 60 wide; a tie on the widest).
    if (s.F == 2 && taps > 160) return 0;
    // Few multiply-adds per output element (up to 160): the stores bound the time and the
    // 64 x 256 tile's longer runs win as soon as there are tiles enough for the CUs.
    const bool few_taps = taps <= 160;
    if (s.K <= 64) {
        // 64 x 256 when the work divides finely enough over the chip with it (many tiles, or so
        // many chunks per tile that sharing tiles is cheap), else 64 x 128, which doubles the
        // number of tiles and fits three workgroups per CU.  (With a few dozen wide tiles only,
        // sharing them leaves the chip unevenly loaded however many chunks they have: 512
        // channels, 64 filters of 5x5, 57 wide tiles: 9 % slower.)
        return (wide_tiles >= 1024 || (wide_tiles >= 200 && wide_tiles * chunks >= 12000) ||
                (few_taps && wide_tiles >= 300)) ? 1 : 0;
    }
    if (few_taps) return tiles >= 150 ? 1 : 0;
    return (tiles >= 400 || (tiles >= 100 && chunks >= 100)) ? 1 : 0;
}

}  // namespace

int general_tile_configs() { return kShapes * kSchedules * kWriteBacks; }

int general_auto_shape(const Shape& s) { return shape_for(s); }

namespace {

bool whole_batch_supported(const Shape& s)
{
    const GenSched sched{0, 0, false, false, 0};
    return launch_any(nullptr, nullptr, nullptr, s, nullptr, shape_for(s), sched, true) == DCONV_OK ||
           launch_any(nullptr, nullptr, nullptr, s, nullptr, 0, sched, true) == DCONV_OK;
}

// A batch whose images are so large that a tile reaching from one image into the next would need
// more than 32 bits of lane offset runs image by image (each launch is long: nothing is lost).
bool per_image_supported(const Shape& s, Shape* one)
{
    *one = s;
    one->N = 1;
    return s.N > 1 && whole_batch_supported(*one);
}

}  // namespace

bool general_tiled_supports(const Shape& s)
{
    Shape one;
    return whole_batch_supported(s) || per_image_supported(s, &one);
}

int launch_general_tiled(const float* in, const float* filt, float* out, const Shape& s,
                         hipStream_t st, int cfg, bool static_ws)
{
    if (cfg >= kShapes * kSchedules * kWriteBacks) return DCONV_UNSUPPORTED;
    Shape one;
    if (!whole_batch_supported(s) && per_image_supported(s, &one)) {
        const int64_t in_image = (int64_t)s.C * s.H * s.W, out_image = (int64_t)s.K * s.Ho * s.Wo;
        for (int n = 0; n < s.N; ++n) {
            const int rc = launch_general_tiled(in + n * in_image, filt, out + n * out_image, one, st, cfg,
                                                static_ws);
            if (rc != DCONV_OK) return rc;
        }
        return DCONV_OK;
    }
    if (cfg < 0) {
        const GenSched sched{0, 0, false, static_ws, 0};
        int rc = launch_any(in, filt, out, s, st, shape_for(s), sched, false);
        if (rc == DCONV_UNSUPPORTED)
            rc = launch_any(in, filt, out, s, st, 0, sched, false);
        return rc;
    }
    const int schedule = cfg / kShapes % kSchedules;
    const int wb = cfg / (kShapes * kSchedules) + 1;
    const GenSched sched{schedule == 3 ? 2 : schedule, schedule == 3 ? 7 : 0, false, static_ws, wb};
    return launch_any(in, filt, out, s, st, cfg % kShapes, sched, false);
}

}  // namespace dconv
