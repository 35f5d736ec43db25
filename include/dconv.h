/*
 * dconv -- direct (no GEMM lowering, no FFT, no Winograd) fp32 2D convolution
 * for AMD MI355X (gfx950), after "Optimizing Memory Efficiency for
 * Convolution Kernels on Kepler GPUs" (Chen, Chen, Chen, Hu, DAC'17).
 *
 * C ABI of libdconv.so.  Letters: batch N, channels C, image H x W, K filters
 * of side F.  (The paper's Fig. 3 caption writes K for the filter side and F
 * for the number of filters; this header uses the letters above throughout.)
 *
 * Common rules for every compute entry point
 *   - Every data pointer is a DEVICE pointer to dense, row-major fp32 in HBM.
 *     The caller owns all buffers; the library neither allocates, frees nor
 *     keeps them.  `out` must not overlap an input.  Base pointers must be
 *     4-byte aligned (anything hipMalloc or a torch tensor returns is).
 *   - Semantics: cross-correlation (no filter flip), stride 1, no padding,
 *     window anchored at the top-left output position:
 *         Ho = H - F + 1,  Wo = W - F + 1
 *         out[n][k][y][x] = sum_c sum_i sum_j in[n][c][y+i][x+j] * filt[k][c][i][j]
 *     Every element of `out` is overwritten (no bias, no scaling, no
 *     accumulation into old contents).  Arithmetic is fp32 multiply-add with
 *     fp32 accumulation; the order of additions is unspecified, so results
 *     agree with an exact sum to within rounding of an fp32 sum of C*F*F
 *     terms, and are bit-exact whenever all partial sums are exactly
 *     representable.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued on it and the call returns without synchronising.
 *     The launch happens on the device that is current in the calling thread;
 *     the buffers must live on that device.
 *   - The return value is a dconv_status; nothing is launched unless
 *     validation passed.  The library never aborts or throws across the ABI.
 *   - Calls are thread-safe: any number of host threads may call any entry
 *     point at once, on the same or on different streams (the only shared
 *     host state, the workspace table of dconv_general, is guarded, and a
 *     workspace block never moves once a call has been given it).
 */
#ifndef DCONV_H
#define DCONV_H

#ifdef __cplusplus
extern "C" {
#endif

typedef enum dconv_status {
    DCONV_OK = 0,
    DCONV_NULL_POINTER = 1,   /* a required pointer argument was NULL            */
    DCONV_BAD_SHAPE = 2,      /* a dimension <= 0, F > H, F > W, or a size that
                                 does not fit the kernels' 32-bit indexing       */
    DCONV_UNSUPPORTED = 3,    /* the requested variant cannot run this shape     */
    DCONV_LAUNCH_FAILED = 4,  /* the HIP runtime reported an error at launch     */
    DCONV_SCRATCH_EXCEEDED = 5/* dconv_general_noalloc only: the launch would need
                                 more scratch memory than the static array holds */
} dconv_status;

/* Kernel variants accepted by the *_v entry points. */
enum {
    DCONV_VARIANT_AUTO = 0,   /* pick by shape (what the plain entry points do)  */
    DCONV_VARIANT_SIMPLE = 1, /* one thread per output element; any shape        */
    DCONV_VARIANT_TILED = 2,  /* LDS-staged, matrix-core tiled kernel, tile
                                 configuration picked by shape                   */
    DCONV_VARIANT_FEW_FILTERS = 3,
                              /* F <= 7: vector-ALU kernels with a sliding
                                 register window and wave-uniform weights.
                                 dconv_single_channel_v: the paper's Algorithm 1
                                 as it stands; what AUTO picks for few filters
                                 (at most 20; how many depends on filter and
                                 image size) where it beats the matrix-core
                                 kernel.  dconv_general_v: the paper's
                                 Algorithm 2 with all filters in a thread's
                                 register tile, K <= 16 only; what AUTO picks for
                                 such layers where its estimated kernel time is
                                 below the matrix-core kernel's, whose 32-filter
                                 block would be mostly padding (few filters, or
                                 up to sixteen on few channels)                  */
    DCONV_VARIANT_SPECIAL_CASE = 4,
                              /* dconv_general with C = 1 (any filter up to
                                 11x11) or C <= 4 (filters up to 5x5) only: the
                                 tiled kernel of the single-channel case, the N
                                 images as further work items and the channels
                                 as further taps; what AUTO picks for large
                                 output volumes of wide images with small filters */
    DCONV_VARIANT_TILED_CFG0 = 0x100,
                              /* DCONV_VARIANT_TILED_CFG0 + i: the tiled kernel
                                 with tile configuration i forced, 0 <= i <
                                 dconv_tile_config_count(); for tests and tuners */
    DCONV_VARIANT_SPECIAL_CASE_CFG0 = 0x200
                              /* + i: DCONV_VARIANT_SPECIAL_CASE with tile
                                 configuration i of the single-channel case,
                                 0 <= i < dconv_tile_config_count(1) (with more
                                 than one channel only 0 and 3 to 6 exist; the
                                 others return DCONV_UNSUPPORTED)                */
};

/*
 * Special case of the paper's Sec. 3 (Algorithm 1): ONE input channel
 * convolved with K filters.
 *   img  [H][W]            device, read
 *   filt [K][F][F]         device, read
 *   out  [K][H-F+1][W-F+1] device, written
 * Errors: NULL img/filt/out -> DCONV_NULL_POINTER; H, W, K, F <= 0, F > H or
 * F > W, or more than 2^31-1 elements in img or in the whole output
 * [K][Ho][Wo] -> DCONV_BAD_SHAPE.
 * Filters up to 11 x 11 run on the kernels of the special case, or, where
 * that is the faster one (narrow or short images, large filters: the choice is
 * made from the shape), on the general-case kernel with one channel; 12 x 12
 * to 32 x 32 always on the latter (it may allocate its workspace, see
 * dconv_release_workspace); larger ones on the one-thread-per-output kernel.
 */
int dconv_single_channel(const float *img, int H, int W,
                         const float *filt, int K, int F,
                         float *out, void *stream);

/*
 * General case of the paper's Sec. 4 (Algorithm 2, Fig. 3a): C channels,
 * K filters, with a batch of N independent images sharing the filters (the
 * batch is this ABI's addition; the paper treats one image).
 *   in   [N][C][H][W]            device, read
 *   filt [K][C][F][F]            device, read
 *   out  [N][K][H-F+1][W-F+1]    device, written
 * Errors as above; additionally N, C <= 0, or more than 2^31-1 elements in
 * `in`, in `filt` or in one image's output [K][Ho][Wo], -> DCONV_BAD_SHAPE.
 * With C = 1 this is the special case of Sec. 3 applied to N images: the
 * automatic choice runs them on the single-channel kernel (all images in one
 * launch) where that is the faster one, and likewise two to four channels
 * with small filters, see DCONV_VARIANT_SPECIAL_CASE.  With up to sixteen
 * filters the automatic choice is the vector-ALU kernel of
 * DCONV_VARIANT_FEW_FILTERS wherever it is the faster one.
 * The tiled kernel is compiled for filters up to 32 x 32; larger ones (and
 * shapes beyond its 32-bit index limits) run on the one-thread-per-output
 * kernel.
 */
int dconv_general(const float *in, int N, int C, int H, int W,
                  const float *filt, int K, int F,
                  float *out, void *stream);

/*
 * The same two operations with the kernel variant chosen by the caller
 * (DCONV_VARIANT_*), for tests and tuning.  A variant that cannot handle the
 * shape returns DCONV_UNSUPPORTED without launching anything;
 * DCONV_VARIANT_SIMPLE accepts every valid shape.
 */
int dconv_single_channel_v(const float *img, int H, int W,
                           const float *filt, int K, int F,
                           float *out, int variant, void *stream);
int dconv_general_v(const float *in, int N, int C, int H, int W,
                    const float *filt, int K, int F,
                    float *out, int variant, void *stream);

/*
 * General case for 16-bit inputs with fp32 accumulation: the paper's closing
 * remark (Sec. 6) that its width-matching model carries over to short data
 * types.  The packed unit is the channel run, so channels are innermost:
 *   in   [N][H][W][C]            device, read, fp16 or bf16 bit patterns
 *   filt [K][F][F][C]            device, read, same type
 *   out  [N][K][H-F+1][W-F+1]    device, written, fp32
 *   out[n][k][y][x] = sum_i sum_j sum_c in[n][y+i][x+j][c] * filt[k][i][j][c]
 * Products of two 16-bit values are exact in fp32; sums are fp32 in
 * unspecified order.  The matrix-core kernel needs C to be a multiple of 16,
 * F <= 32 (and, beyond 27 x 27, an image block small enough for a filter row
 * of a chunk to fit in LDS beside it) and 16-byte aligned inputs; other
 * shapes run on a one-thread-per-output kernel (any valid shape, 2-byte
 * alignment), which is some thousand times slower: pad the channels.
 * Errors as for dconv_general; a base pointer that is not 2-byte aligned ->
 * DCONV_BAD_SHAPE.
 */
enum { DCONV_DTYPE_F16 = 0, DCONV_DTYPE_BF16 = 1, DCONV_DTYPE_I8 = 2 };
int dconv_general_f16(const void *in, int N, int C, int H, int W,
                      const void *filt, int K, int F,
                      float *out, void *stream);
int dconv_general_bf16(const void *in, int N, int C, int H, int W,
                       const void *filt, int K, int F,
                       float *out, void *stream);
/* dtype: DCONV_DTYPE_F16 or _BF16; variant: DCONV_VARIANT_AUTO, _SIMPLE, _TILED, or
 * DCONV_VARIANT_TILED_CFG0 + i to force a tile configuration of the matrix-core
 * kernel, for tests and tuning (0: 64 filters x 256 pixels, 1: 128 x 512, both
 * with chunks staged through registers; 2 and 3: the same tiles staged by loads
 * that write LDS directly; 4: 128 x 384, staged directly). */
int dconv_general_half_v(const void *in, int N, int C, int H, int W,
                         const void *filt, int K, int F,
                         float *out, int dtype, int variant, void *stream);

/*
 * The same with signed 8-bit integer inputs and exact int32 sums:
 *   in   [N][H][W][C] int8, filt [K][F][F][C] int8, out [N][K][Ho][Wo] int32
 * (|sum| <= C*F*F*2^14 must fit int32, which it does for every shape the
 * 2^31-1 element limits admit with C*F*F < 2^17; larger reductions wrap as
 * int32 arithmetic does).  The matrix-core kernel needs C to be a multiple of
 * 32, F <= 32 (as above) and 16-byte aligned inputs; other shapes run on the
 * one-thread-per-output kernel.  variant as for dconv_general_half_v.
 */
int dconv_general_i8(const void *in, int N, int C, int H, int W,
                     const void *filt, int K, int F,
                     int *out, void *stream);
int dconv_general_i8_v(const void *in, int N, int C, int H, int W,
                       const void *filt, int K, int F,
                       int *out, int variant, void *stream);

/*
 * The general case on short data types with every choice explicit: dtype
 * (DCONV_DTYPE_*), layout, variant (as for dconv_general_half_v); `out` is fp32
 * for the 16-bit types and int32 for int8.  Layouts:
 *   DCONV_LAYOUT_CHANNELS_LAST    in [N][H][W][C],        filt [K][F][F][C]
 *   DCONV_LAYOUT_CHANNEL_BLOCKED  in [N][C/cb][H][W][cb], filt [K][C/cb][F][F][cb]
 * with cb = 16 channels for the 16-bit types and 32 for int8 (32 bytes: the
 * unit a matrix-core step consumes per pixel).  In the blocked layout the
 * kernel's staging loads are contiguous along image rows instead of gathering
 * 32 bytes out of every pixel's channel run; C must be a multiple of cb
 * (otherwise DCONV_BAD_SHAPE).  Everything else as for dconv_general_f16.
 */
enum { DCONV_LAYOUT_CHANNELS_LAST = 0, DCONV_LAYOUT_CHANNEL_BLOCKED = 1 };
int dconv_general_lowp(const void *in, int N, int C, int H, int W,
                       const void *filt, int K, int F,
                       void *out, int dtype, int layout, int variant, void *stream);

/*
 * Number of tile configurations compiled into the tiled kernel of the
 * single-channel case (single_channel != 0) or of the general case
 * (single_channel == 0).  The paper picks its tile sizes by exploring the
 * design space per device (Sec. 5, Table 1); this is the hook for doing the
 * same here: time DCONV_VARIANT_TILED_CFG0 + i for every i.  A configuration
 * that cannot hold a given shape returns DCONV_UNSUPPORTED without launching.
 */
int dconv_tile_config_count(int single_channel);

/*
 * What DCONV_VARIANT_AUTO picks for a shape, decided on the host from the shape
 * alone: nothing is launched and no GPU is needed.  For tuners, and for tests
 * that pin the dispatcher's rules (the rules are where the paper's per-device
 * design-space exploration, Sec. 5 and Table 1, ends up in this library).
 *   single_channel != 0: the shape of dconv_single_channel (N and C must be 1);
 *   single_channel == 0: the shape of dconv_general.
 * Returns the tile configuration i (as in DCONV_VARIANT_TILED_CFG0 + i) of that
 * entry point's tiled kernel -- for dconv_general the tile shape only, 0 to 2:
 * how its tiles are shared between workgroups is decided at launch from the
 * device's CU count -- or one of the negative values below.
 */
enum dconv_choice {
    DCONV_CHOICE_FEW_FILTERS = -1,  /* the vector-ALU kernel for few filters of that entry point */
    DCONV_CHOICE_SPECIAL_CASE = -2, /* dconv_general hands the shape to the special-case
                                       kernel (one channel, or a few with small filters)   */
    DCONV_CHOICE_SIMPLE = -3,       /* the one-thread-per-output kernel                    */
    DCONV_CHOICE_INVALID = -4,      /* not a valid shape (the entry point would return
                                       DCONV_BAD_SHAPE)                                    */
    DCONV_CHOICE_GENERAL_CASE = -5  /* one channel on the general-case kernel: filters
                                       beyond the special-case kernel's 11 x 11, and
                                       shapes where it is the faster one (narrow or short
                                       images, large filters)                              */
};
int dconv_tile_choice(int single_channel, int N, int C, int H, int W, int K, int F);

/*
 * HIP graph capture.  Every entry point only enqueues kernels on `stream` (no
 * synchronisation, no host-side reads), so calls can be captured into a graph
 * and replayed.  The one exception is the workspace of dconv_general described
 * below: the first call that needs it on a stream allocates and clears it,
 * which is not allowed while that stream is capturing.  Run the calls once on
 * the stream before capturing on it.
 */

/*
 * dconv_general keeps one device workspace per (device, stream) it has been
 * called on: when the tiles of a shape do not spread evenly over the chip, a
 * tile is summed over channels by several workgroups and their partial sums
 * meet there.  The first call that needs it on a stream allocates, with
 * hipMalloc, what the largest launch on that device can need (256 KiB of
 * partial sums and four counters per compute unit: 64 MiB + 4 KiB on a 256-CU
 * chip) and clears the counters on that stream; no other entry point
 * allocates (dconv_single_channel counts as dconv_general here where it runs
 * on the same kernel, see there), and no call
 * synchronises.  The block keeps its address from then
 * on: later calls on the stream, whatever their shape, use the same block (they
 * run in order, so they share it safely; calls on different streams use
 * different blocks), and a graph captured on the stream stays valid while
 * other calls are made on it.
 * dconv_release_workspace frees all blocks.  The caller must make sure that no
 * dconv_general launch is still running and that every graph that holds
 * captured dconv_general calls has been destroyed (or is never launched
 * again): a replay after the release would write to freed memory.  Always
 * returns DCONV_OK.
 */
int dconv_release_workspace(void);

/*
 * dconv_general_v for callers that cannot allocate device memory: code that is
 * under HIP graph capture from its first call on, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same results (bit for bit:
 * the same kernels in the same launch configuration) and same errors as
 * dconv_general_v, but it never calls hipMalloc, hipFree or any allocating
 * routine: where dconv_general_v would use its workspace, the partial sums and
 * arrival counters of shared tiles go to a static device array that is part of
 * the library's code object -- 64 MiB + 16 KiB on every GPU the library runs on,
 * held until the process ends.  That is room for 512 workgroups with two 64 x 256
 * partial tiles each and 4096 counters, i.e. for every launch configuration on
 * a chip of up to 256 compute units; a launch that would need more returns
 * DCONV_SCRATCH_EXCEEDED and nothing is launched.  Variants that never share
 * tiles (DCONV_VARIANT_SIMPLE, the special-case kernels) do not touch the array.
 * The counters a launch uses are cleared on `stream`, by a kernel, before it.
 * All calls on one GPU share the one array: two dconv_general_noalloc calls
 * that overlap in time on the same GPU (different streams, or different host
 * threads whose launches run concurrently) race on it and give wrong results;
 * the caller must order them.  Calls of the other entry points are unaffected.
 */
int dconv_general_noalloc(const float *in, int N, int C, int H, int W,
                          const float *filt, int K, int F,
                          float *out, int variant, void *stream);

/* Human-readable name of a status code; static storage, never NULL. */
const char *dconv_status_string(int status);

/* ABI version: major * 1000 + minor. */
int dconv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DCONV_H */
