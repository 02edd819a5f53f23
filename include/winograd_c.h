/*
 * C ABI of the MI355X (gfx950) integer complex-Winograd convolution library.
 *
 * The library computes 3x3, stride-1, dilation-1, zero-pad-1 convolution
 * (correlation, no kernel flip) of int8 activations with int8 filters into
 * int32 outputs with the complex Winograd algorithm F(4x4,3x3) over the
 * Gaussian integers of Meng & Brothers, "Efficient Winograd Convolution via
 * Integer Arithmetic" (SysML 2019), Sections 3.3-3.4 and 4.2.
 *
 * Conventions shared by every entry point
 *   - Every *_dev pointer is DEVICE memory owned by the caller; the library
 *     never allocates, frees or keeps it.  Activation, filter and output
 *     pointers must be 4-byte aligned, packed_dev and workspace_dev 256-byte.
 *   - hip_stream is a hipStream_t passed as void* (NULL = the null stream).
 *     All work is enqueued on it; no call synchronises unless it says so.
 *   - Return value: WG_OK, or a negative wg_status; on error nothing has been
 *     enqueued.  Validation happens on the host before the first launch.
 *   - layout WG_NCHW: activations [N][C][H][W], filters [K][C][3][3],
 *     outputs [N][K][H][W].  layout WG_NHWC: activations [N][H][W][C], filters
 *     [K][3][3][C], outputs [N][H][W][K].  All dense, no strides.
 *   - 1 <= C <= WG_MAX_CHANNELS keeps every int32 accumulator exact for any
 *     int8 data (16 * 9 * C * 128 * 128 < 2^31).
 *   - Threads and devices: launches go to the device that is current in the
 *     calling thread.  The first call of a kernel variant raises that kernel's
 *     shared-memory limit, once per process and under a lock, so calls may come
 *     from several threads; a process should drive one device through this
 *     library (the build targets one GPU).  The winograd_debug_* switches are
 *     process-wide: a call in flight on another thread may see either value.
 */
#ifndef WINOGRAD_C_H
#define WINOGRAD_C_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum wg_status {
    WG_OK = 0,
    WG_EINVAL = -1,        /* null pointer, non-positive size, unknown enum, misaligned pointer */
    WG_EUNSUPPORTED = -2,  /* C > WG_MAX_CHANNELS, tensor too large for 32-bit indexing, odd H/W with pooling */
    WG_ESMALLBUF = -3,     /* packed_bytes / workspace_bytes below what the query functions return */
    WG_EBLOB = -4,         /* packed filter blob does not match (K, C, mode) */
    WG_ERUNTIME = -5       /* a HIP launch failed */
};
enum wg_layout { WG_NCHW = 0, WG_NHWC = 1 };
enum wg_mode {
    WG_LOSSLESS = 0, /* exact: equals the direct convolution bit for bit (Section 3.3-3.4) */
    WG_SCALED = 1    /* Winograd-domain filters scaled back into int8 per output channel and
                        location, inverse applied before the output transform (Section 4.2) */
};
#define WG_MAX_CHANNELS 896

/* Human-readable name of a status code; never NULL. */
const char* winograd_status_string(int status);

/* Size in bytes of the packed Winograd-domain filter blob for K filters of C
   channels in the given mode; 0 if the arguments are invalid. */
size_t winograd_packed_filter_bytes(int K, int C, int mode);

/* Size in bytes of the scratch workspace winograd_conv2d_int8 needs for this
   problem (transformed activations and Winograd-domain accumulators); 0 if
   the arguments are invalid. */
size_t winograd_workspace_bytes(int N, int C, int H, int W, int K, int mode);

/*
 * Filter transform W = G' g G'^T with G' = 4G (Section 3.3; the conjugate
 * structure of W is the one printed in Section 3.4), done once per layer and
 * reused by every convolution call (Section 4.3 notes it is off the
 * inference path).  Only the 26 free entries of each 6x6 tile are kept
 * (16 real, 10 complex), already split into the int8 operand planes the
 * contraction consumes.
 *   WG_LOSSLESS: 12-bit entries as exact int8 limbs.
 *   WG_SCALED:   Section 4.2's precision scaling for int8 filters: per output
 *                channel and location, the largest max(|Re|,|Im|) over input
 *                channels; if above 127 every entry there is multiplied by the
 *                largest n/2^p (4-bit n) that brings it back within +-127,
 *                rounding half up; the blob also holds the 8-bit reciprocal
 *                r/2^q applied later.
 * w_dev: int8 filters in `layout`.  packed_dev: blob of at least
 * winograd_packed_filter_bytes(K, C, mode) bytes, fully overwritten.
 */
int winograd_filter_transform(const int8_t* w_dev, int K, int C, int layout, int mode,
                              void* packed_dev, size_t packed_bytes, void* hip_stream);

/*
 * Synchronous check that a blob was produced by winograd_filter_transform
 * for exactly (K, C, mode): copies the blob header to the host (blocks on
 * hip_stream).  WG_OK or WG_EBLOB.  The convolution entry points do not do
 * this themselves because they never synchronise; their kernels re-check the
 * header on the device and leave the output untouched on a mismatch.
 */
int winograd_packed_filter_check(const void* packed_dev, int K, int C, int mode, void* hip_stream);

/*
 * The whole hot path Y = A^T [ sum_c W (.) (B^T d B) ] A (Section 3.4) for
 * every 4x4 output tile: input transform of the overlapping 6x6 tiles,
 * Winograd-domain contraction over input channels on the int8 matrix cores
 * (16 real and 10 complex products per tile and channel pair, three real
 * multiplications per complex one, partial products kept separate until the
 * channel sum is complete), the inverse filter scaling in WG_SCALED mode, and
 * the output transform followed by the rescale by 2^-4 (G' = 4G twice).
 * WG_LOSSLESS results equal direct_conv2d_int8's bit for bit.  WG_SCALED
 * rounds half up at the inverse scaling and at the final shift.
 * x_dev: int8 activations; packed_dev: blob from winograd_filter_transform
 * with the same (K, C, mode); y_dev: int32 output, every element written.
 * workspace_dev: at least winograd_workspace_bytes(...) bytes; contents are
 * scratch and calls sharing a workspace must not overlap in time.
 */
int winograd_conv2d_int8(const int8_t* x_dev, const void* packed_dev, int32_t* y_dev,
                         int N, int C, int H, int W, int K, int layout, int mode,
                         void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/*
 * The same path on the quantised tensors of Section 4.1: unsigned int8 bytes
 * with a zero point (0..255) that is subtracted from every byte, i.e. integers
 * in [-255, 255] (int9): y = sum (x - zero_x) (w - zero_w) in int32, with padding
 * pixels contributing nothing (they read as the zero point).  G' g G'^T then
 * reaches 16 * 255 = 4080 (13 bits, the 4 extra bits of Section 3.4 on top of
 * int9) and B^T d B likewise; WG_SCALED brings the 13-bit filters into +-127
 * (factors down to 15/2^9) and keeps the activations as two int8 limbs.
 * winograd_filter_transform_u8: w_dev uint8 in `layout`; same blob size, alignment
 * and error codes as winograd_filter_transform.  winograd_conv2d_u8: x_dev uint8,
 * y_dev int32, every element written; needs no workspace.  The two go together:
 * winograd_conv2d_u8 accepts only blobs from winograd_filter_transform_u8 and
 * winograd_conv2d_int8 only blobs from winograd_filter_transform (a mismatch
 * leaves y untouched; winograd_packed_filter_check accepts both kinds).  Signed
 * int8 filters w enter as the bytes w + 128 with zero point 128.
 * Channels: the path forms 16 y in int32 and |y| can reach 9 C 255^2, so
 * C <= 229 (16 * 9 * 229 * 255^2 < 2^31); more return WG_EUNSUPPORTED.  Up to
 * there WG_LOSSLESS equals the int9 direct convolution bit for bit (sums inside
 * the path may wrap modulo 2^32; the result does not).  WG_SCALED results
 * approximate it and are exact functions of the inputs as in winograd_conv2d_int8;
 * data that drive 16 |y| to within about 1 % of 2^31 can wrap there.
 */
int winograd_filter_transform_u8(const uint8_t* w_dev, int zero_point, int K, int C, int layout, int mode,
                                 void* packed_dev, size_t packed_bytes, void* hip_stream);
int winograd_conv2d_u8(const uint8_t* x_dev, int zero_point, const void* packed_dev, int32_t* y_dev,
                       int N, int C, int H, int W, int K, int layout, int mode, void* hip_stream);

/*
 * The path with the activations scaled as well.  Section 4.1 ends with the
 * remark that the analysis of Section 4.2 carries over to the activation
 * transform B^T d B (12 bits here for int8 data) and leaves it out because it
 * cannot be prepared offline; here it runs inside the convolution kernel.  The
 * rule is that section's with a tile in the place of an output feature map: for
 * each tile and each of its 26 free entries the largest max(|Re|, |Im|) over the
 * input channels decides n/2^p (4-bit n; nothing if the maximum is within
 * +-127), Re and Im of every channel's value there are multiplied by it,
 * rounding half up, and a channel sum is multiplied back first by the filter's
 * reciprocal r/2^q, then by the tile's (each step rounds half up).  Both
 * operands of the Winograd-domain products are then single int8 values: half
 * the matrix-core work of WG_SCALED, at the price of a second pass over the
 * input transform.
 * packed_dev: a WG_SCALED blob of winograd_filter_transform (signed int8
 * filters; a mismatch leaves y untouched).  x_dev, y_dev, layout, limits and
 * error codes as for winograd_conv2d_int8; no workspace.  act_table_dev: NULL,
 * or int32 [T][26][4] = (n, p, r, q) per tile t = (n*ceil(H/4) + ty)*ceil(W/4)
 * + tx and free entry in the library's order (the 16 real entries (r, c), r, c
 * in {0,1,2,5}, row-major; then (r,3) for r in {0,1,2,5}; (3,c) for c in
 * {0,1,2,5}; (3,3); (3,4)), (0,0,1,0) where nothing was scaled, which the kernel
 * fills for tests (DEVICE memory, 16-byte aligned).
 */
int winograd_conv2d_int8_act_scaled(const int8_t* x_dev, const void* packed_dev, int32_t* y_dev,
                                    int N, int C, int H, int W, int K, int layout,
                                    int32_t* act_table_dev, void* hip_stream);

/*
 * For callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid it): winograd_conv2d_int8's staged
 * pipeline (input transform, contraction, output transform) with its workspace
 * in a buffer of winograd_static_workspace_limit() bytes (64 MiB) that is part
 * of the library's device image, one per GPU, held until the process ends.  The
 * call allocates nothing; its first use on a device asks the runtime for the
 * buffer's address there.  Same arguments, results and error codes as
 * winograd_conv2d_int8 without the workspace pair; WG_ESMALLBUF if
 * winograd_workspace_bytes(N, C, H, W, K, mode) exceeds the limit, nothing
 * enqueued.  Every call on a GPU uses that GPU's one buffer, whatever the
 * stream: calls that overlap in time on one GPU race.  The buffer keeps the
 * last call's contents; no call depends on them.
 */
size_t winograd_static_workspace_limit(void);
int winograd_conv2d_int8_static_workspace(const int8_t* x_dev, const void* packed_dev, int32_t* y_dev,
                                          int N, int C, int H, int W, int K, int layout, int mode,
                                          void* hip_stream);

/*
 * The same convolution with the requantisation that follows each quantised
 * convolution in a network (Section 4.4) applied before the store, so a layer
 * stack passes int8 from layer to layer and the int32 outputs never reach
 * memory.  The result equals winograd_conv2d_int8 followed by
 * requant_relu_pool_int8 with the same (shift, relu, pool) bit for bit:
 *   v = (y + 2^(shift-1)) >> shift (shift = 0: v = y), clamped to [0,127] if
 *   relu else [-128,127], then an optional 2x2 stride-2 maximum (H and W must
 *   then be even, else WG_EUNSUPPORTED).
 * out_dev: int8 in `layout`, [N][K][H][W] or [N][H][W][K], with H/2 and W/2
 * when pool != 0; every element written.  0 <= shift <= 31.  Always runs the
 * single-kernel path and needs no workspace.
 */
int winograd_conv2d_int8_requant(const int8_t* x_dev, const void* packed_dev, int8_t* out_dev,
                                 int N, int C, int H, int W, int K, int layout, int mode,
                                 int shift, int relu, int pool, void* hip_stream);

/*
 * The same convolution with the rational Winograd algorithm F(2x2,3x3) in
 * integer arithmetic: the running example of Sections 4.1-4.2 and the variant
 * the evaluation of Section 4.4 used.  G' = 2G is the filter transform matrix
 * printed in Section 4.1; all 16 Winograd-domain entries are real.
 *   WG_LOSSLESS: 12-bit transformed filters and 11-bit transformed activations
 *                as exact int8 limbs; the result equals direct_conv2d_int8's bit
 *                for bit.
 *   WG_SCALED:   Section 4.2 with 16 factors per filter (one per X-Y location,
 *                from the largest magnitude over the input channels): filters
 *                scaled into +-127 by n/2^p with a 4-bit n, rounding half up;
 *                the channel sums multiplied back by the 8-bit reciprocal r/2^q
 *                before the output transform; the final division by 4 (G' = 2G
 *                on both sides) rounds half up.
 * winograd_f2x2_filter_transform fills a blob of at least
 * winograd_f2x2_packed_filter_bytes(K, C, mode) bytes (256-byte aligned; 0 from
 * the size query means invalid arguments); winograd_f2x2_conv2d_int8 consumes it
 * (WG_EBLOB-style mismatches leave y untouched) and needs no workspace.  Layouts,
 * limits and error codes are those of the F(4x4,3x3) entry points.
 * winograd_f2x2_debug_filter_operands exports what the blob holds:
 * planes_dev int8 [planes][K][C] (lossless: 32 planes, entry e = 4 row + column
 * as high limb 2e and low limb 2e+1; scaled: 16 planes) and table_dev int32
 * [K][16][4] = (n, p, r, q).
 */
size_t winograd_f2x2_packed_filter_bytes(int K, int C, int mode);
/*
 * The *_u8 variants take the quantised tensors of Section 4.1: unsigned int8
 * bytes with a zero point (0..255), i.e. the integers byte - zero_point in
 * [-255, 255] (int9).  y = sum (x - zx) (w - zw) in int32, exact in
 * WG_LOSSLESS mode (G' g G'^T then reaches the 1020/1530/2295 of the
 * section's table and travels as two int8 limbs); WG_SCALED brings the
 * 13-bit Winograd-domain filters into +-127, the operand range of the
 * matrix cores.  Blobs are interchangeable: either convolution entry point
 * accepts a blob made by either filter transform.
 */
int winograd_f2x2_filter_transform(const int8_t* w_dev, int K, int C, int layout, int mode,
                                   void* packed_dev, size_t packed_bytes, void* hip_stream);
int winograd_f2x2_conv2d_int8(const int8_t* x_dev, const void* packed_dev, int32_t* y_dev,
                              int N, int C, int H, int W, int K, int layout, int mode,
                              void* hip_stream);
int winograd_f2x2_filter_transform_u8(const uint8_t* w_dev, int zero_point, int K, int C, int layout,
                                      int mode, void* packed_dev, size_t packed_bytes, void* hip_stream);
int winograd_f2x2_conv2d_u8(const uint8_t* x_dev, int zero_point, const void* packed_dev, int32_t* y_dev,
                            int N, int C, int H, int W, int K, int layout, int mode, void* hip_stream);
int winograd_f2x2_debug_filter_operands(const void* packed_dev, int K, int C, int mode,
                                        int8_t* planes_dev, int32_t* table_dev, void* hip_stream);
/*
 * winograd_f2x2_conv2d_int8 with the requantisation that follows a quantised
 * convolution in a network (Section 4.4) applied before the store, as in
 * winograd_conv2d_int8_requant: out = clamp((y + 2^(shift-1)) >> shift, lo, 127)
 * with lo = 0 if relu else -128, then an optional 2x2 stride-2 maximum (pool != 0:
 * H and W even; a 2x2 output tile is exactly one pooling window).  out_dev: int8
 * in `layout` with K channels, [N][K][H/2][W/2] or [N][H/2][W/2][K] when pooling,
 * every element written, 4-byte aligned.  0 <= shift <= 31.  Signed int8 inputs.
 */
int winograd_f2x2_conv2d_int8_requant(const int8_t* x_dev, const void* packed_dev, int8_t* out_dev,
                                      int N, int C, int H, int W, int K, int layout, int mode,
                                      int shift, int relu, int pool, void* hip_stream);

/*
 * F(2x2,3x3) with the activations scaled as well.  Section 4.1 ends with the
 * remark that the analysis of Section 4.2 carries over to the activation
 * transform B^T d B (11 bits for int8 data) and leaves it out because it cannot
 * be prepared offline; here it runs inside the convolution kernel.  The rule is
 * that section's with a tile in the place of an output feature map: for each
 * tile and each of its 16 X-Y locations the largest magnitude over the input
 * channels decides n/2^p (4-bit n; nothing if the maximum is within +-127),
 * every channel's value there is multiplied by it, rounding half up, and a
 * channel sum is multiplied back first by the filter's reciprocal r/2^q, then
 * by the tile's (each step rounds half up).  Both operands of the
 * Winograd-domain products are then single int8 values.
 * packed_dev: a WG_SCALED blob of winograd_f2x2_filter_transform (signed int8
 * filters; WG_EBLOB-style mismatches leave y untouched).  x_dev, y_dev, layout,
 * limits and error codes as for winograd_f2x2_conv2d_int8.  act_table_dev: NULL,
 * or int32 [T][16][4] = (n, p, r, q) per tile t = (n*ceil(H/2) + ty)*ceil(W/2)
 * + tx and location 4 row + column ((0,0,1,0) where nothing was scaled), which
 * the kernel fills for tests (DEVICE memory, 16-byte aligned).
 */
int winograd_f2x2_conv2d_int8_act_scaled(const int8_t* x_dev, const void* packed_dev, int32_t* y_dev,
                                         int N, int C, int H, int W, int K, int layout,
                                         int32_t* act_table_dev, void* hip_stream);

/*
 * Direct evaluation of the same convolution (the 144-multiplication method
 * that Section 3.4 compares against):
 *   y[n,k,h,w] = sum_{c,a,b} x[n,c,h+a-1,w+b-1] * g[k,c,a,b],  x = 0 outside.
 * w_dev: the untransformed int8 filters in `layout`.
 */
int direct_conv2d_int8(const int8_t* x_dev, const int8_t* w_dev, int32_t* y_dev,
                       int N, int C, int H, int W, int K, int layout, void* hip_stream);

/*
 * Glue for stacking layers (a requantisation follows each quantised
 * convolution, Section 4.4): v = (y + 2^(shift-1)) >> shift (shift = 0: v = y),
 * clamped to [0,127] if relu else [-128,127], then an optional 2x2 stride-2
 * max-pool (H and W must then be even).  y_dev int32 and out_dev int8 use
 * `layout` with K channels; out is [N][K][H/2][W/2] (or NHWC) when pool != 0.
 * 0 <= shift <= 31.
 */
int requant_relu_pool_int8(const int32_t* y_dev, int8_t* out_dev, int N, int K, int H, int W,
                           int layout, int shift, int relu, int pool, void* hip_stream);

/*
 * Which implementation winograd_conv2d_int8 runs for this problem: 1 = staged
 * (input transform, contraction, output transform through the workspace),
 * 2 = fused single kernel; negative status on invalid arguments.
 */
int winograd_conv2d_path(int N, int C, int H, int W, int K, int mode);

/*
 * Measurement aid for benchmarks: enqueues ONE kernel of winograd_conv2d_int8 (same arguments and
 * launch configuration as in that call) `iters` times back to back on hip_stream and returns; the
 * caller brackets the call with its own events on that stream.  stage 0: the staged pipeline's input
 * transform (Section 3.4's B^T d B), 1: its contraction, 2: its output transform, 3: the single
 * fused kernel.  Stages 1 and 2 consume what the stage before them left in the workspace, so run
 * the stages in order once before timing them.  Never synchronises, creates nothing.  iters >= 1.
 */
int winograd_conv2d_int8_enqueue_stage(const int8_t* x_dev, const void* packed_dev, int32_t* y_dev,
                                       int N, int C, int H, int W, int K, int layout, int mode,
                                       void* workspace_dev, size_t workspace_bytes, void* hip_stream,
                                       int stage, int iters);

/* ---- stage exports used by the stage-level parity tests ------------------
 * Operand-plane numbering.  The 26 free entries of a transformed tile are
 * ordered: real entries (r,c), r,c in {0,1,2,5}, row-major (index 4*ri+ci),
 * then the complex ones (0,3) (1,3) (2,3) (5,3) (3,0) (3,1) (3,2) (3,5) (3,3)
 * (3,4).  "Values": one per real entry (0..15), three per complex entry j
 * (16+3j: Re, +1: Im, +2: Re+Im, the extra operand of the three-multiplication
 * complex product of Section 3.1).
 *   WG_LOSSLESS operand planes, both sides: 3*value + {0: high limb v>>6,
 *     1: low limb v&63, 2: high+low}, 138 planes.
 *   WG_SCALED activation planes: real entry p: 2p + {0: high, 1: low};
 *     complex entry j: 32 + 4j + {Re high, Re low, Im high, Im low}; 72 planes.
 *   WG_SCALED filter planes: real entry p: p; complex entry j: 16 + 3j +
 *     {Re, Im, -Im}; 46 planes.
 * Accumulator planes (36): real entry p: p; complex entry j: 16 + 2j + {Re, Im}.
 */
int winograd_num_activation_planes(int mode);

/* winograd_conv2d_int8 has two implementations of the same arithmetic: a fused
   single kernel, which the library runs by default, and a staged pipeline
   (input transform, contraction, output transform as three kernels through
   the workspace) whose intermediate arrays the stage exports below expose.
   path 0 = library's choice (default), 1 = always staged, 2 = always fused.
   Process-wide (an atomic flag); for tests and benchmarks.  Returns WG_EINVAL
   for any other value. */
int winograd_debug_force_path(int path);
/* Test hook for the single-kernel path's streaming variant (one workgroup walks over many tile
   blocks of a 32-filter block; the library picks it by itself only for large layers): n > 0
   makes every call whose layout allows it (channels-last, C % 4 = 0, K % 4 = 0) use it with n
   workgroups per filter block; 0 restores the library's own choice.  Process-wide, like
   winograd_debug_force_path. */
int winograd_debug_stream_workgroups(int n);
/* Test hook for the single-kernel path in WG_LOSSLESS mode, which has two forms of the product phase: one whose
   matrix-core filter operand carries both int8 limbs of eight filters (a wave owns complete outputs; channels-last
   inputs with C % 4 = 0), and one with 16 filters per operand and the rows of the Winograd-domain tile split over two
   waves (any layout).  0: the library's choice, 1: the first form wherever the layout allows, 2: never the first
   form.  Process-wide, like winograd_debug_force_path. */
int winograd_debug_lossless_variant(int variant);
/* A switch of the same kind for the role-specialised single-kernel form (transform and products on separate waves), which
   exists with four product waves and 32 filters per workgroup and with eight product waves and 64 filters (channels-last
   inputs with C % 4 = 0 and K % 4 = 0; both modes, whatever the name says).  0: the library's choice, 1: the second form
   wherever the layout allows, 2: never the second form. */
int winograd_debug_scaled_variant(int variant);
/* The same switch for the streaming form of that kernel (a workgroup walks over many tile blocks; chosen for large
   layers), which also exists with 64 filters per workgroup (each product wave owns every entry of 16 filters; lossless
   mode, or one channel block).  0: the library's choice, 1: the 64-filter form wherever a layer streams and the form
   applies, 2: never. */
int winograd_debug_stream_variant(int variant);
int winograd_num_filter_planes(int mode);

/* Host-only: the (n, ty, tx) the kernels derive from tile index t = (n*TH + ty)*TW + tx for
   this problem (they divide by multiply-and-shift with constants prepared on the host; this
   lets a CPU test compare that arithmetic against plain division).  out3_host: 3 ints. */
int winograd_debug_tile_decode(int N, int C, int H, int W, int K, int t, int* out3_host);

/* Runs only the input transform D = B^T d B (Section 3.4) and writes its int8
   operand planes as a dense [planes][T][C] array, T = N*ceil(H/4)*ceil(W/4),
   tile index (n*TH + ty)*TW + tx. */
int winograd_debug_input_operands(const int8_t* x_dev, int8_t* planes_dev, int N, int C, int H,
                                  int W, int layout, int mode, void* workspace_dev,
                                  size_t workspace_bytes, void* hip_stream);

/* Unpacks a filter blob into dense int8 [planes][K][C] and the scaling table
   int32 [K][26][4] = (n, p, r, q) per output channel and free entry
   (all zero-scaling entries (0,0,1,0); WG_LOSSLESS fills the table the same way). */
int winograd_debug_filter_operands(const void* packed_dev, int K, int C, int mode,
                                   int8_t* planes_dev, int32_t* table_dev, void* hip_stream);

/* Runs input transform and contraction (and the inverse scaling in WG_SCALED)
   and writes the 36 accumulator planes as dense int32 [36][T][K]. */
int winograd_debug_contraction(const int8_t* x_dev, const void* packed_dev, int32_t* m_dev,
                               int N, int C, int H, int W, int K, int layout, int mode,
                               void* workspace_dev, size_t workspace_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* WINOGRAD_C_H */
