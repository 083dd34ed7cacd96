/*
 * hb -- five image-processing stages recast as dense products with fixed
 * Toeplitz / strided-Toeplitz / phase / triangular coefficient matrices and run
 * on the MI355X (gfx950) matrix units, after "Pushing Tensor Accelerators
 * beyond MatMul in a User-Schedulable Language" (Sec. V-A, V-B).
 *
 * C ABI.  Plain pointers and sizes only.
 *
 * Common conventions
 * ------------------
 *  - hb_half is an IEEE binary16 bit pattern.
 *  - Every `in`, `out`, `residual`, `down`, `w`, `workspace` pointer is a DEVICE
 *    pointer owned by the caller.  `taps*_host` pointers are HOST pointers; they
 *    are read during the call and travel to the GPU inside the kernel arguments,
 *    so the caller may free or change them as soon as the call returns.
 *  - Single-channel images are row-major; pitches are in ELEMENTS (not bytes) and
 *    must be >= the width (at most 2^26; hb_fir1d and hb_sepblur also want
 *    H * in_pitch < 2^31 and H * out_pitch < 2^30, HB_ERR_UNSUPPORTED beyond).
 *    Any H, W >= 1 is computed correctly.
 *    Base pointers need the alignment of their element type only (2 bytes for fp16,
 *    4 for fp32); the kernels run fastest when fp16 base pointers and pitches are
 *    multiples of 4 bytes and fp32 ones multiples of 16 bytes (torch allocations
 *    and even pitches are).  Images narrower than one window of the matrix
 *    formulation (32 to 96 pixels, depending on the taps) run the vector-ALU kernel.
 *  - Orientation is correlation, as the paper prints it: O(x) = sum_r I(x + r) K(r).
 *    `anchor` shifts the window, tap r reads x + r - anchor; anchor = 0 is the
 *    paper's formula verbatim.  Output has the size of the input; out-of-range
 *    reads clamp the INPUT index to the edge (zero padding for hb_conv3x3).
 *  - Arithmetic: fp16 operands, fp32 accumulation on the matrix units.
 *  - `stream` is a hipStream_t (passed as void* so that this header needs no HIP
 *    include).  All work is enqueued on it; no call synchronises, allocates, frees
 *    or keeps a pointer.  Input and output buffers must not overlap.
 *  - Errors: the return code only.  Arguments are validated before any HIP call
 *    (HB_ERR_INVALID_ARG / HB_ERR_UNSUPPORTED / HB_ERR_WORKSPACE); a launch failure
 *    reported by the runtime gives HB_ERR_HIP.  Faults inside a kernel surface at
 *    the caller's next synchronisation, as for any asynchronous launch.
 *  - Thread safety: calls from several host threads and on different streams may run
 *    concurrently provided their buffers and workspaces are distinct.  The state the
 *    library keeps is small and guarded by locks or atomics: per device, the
 *    number of compute units, the LDS limit already granted to each kernel, how many
 *    workgroups of the one-launch summed-area kernel are resident at once, and the
 *    address of hb_sat2d_noalloc's array (each looked up at the first call that needs
 *    it on that device); process-wide, the wait limit of hb_sat2d_set_wait_limit.
 *    None of it depends on the data of a call.
 *  - Every stage has a `_valu` twin with the same signature and results that uses
 *    only vector-ALU FMAs (no MFMA): the ablation that shows what the matrix units
 *    buy.
 */
#ifndef HB_H
#define HB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HB_OK = 0,
    HB_ERR_INVALID_ARG = 1,   /* null pointer, non-positive size, pitch < width, bad taps/anchor ... */
    HB_ERR_UNSUPPORTED = 2,   /* valid request outside what the kernels implement */
    HB_ERR_WORKSPACE = 3,     /* workspace missing, misaligned or too small */
    HB_ERR_HIP = 4            /* the HIP runtime rejected a launch */
} hb_status;

typedef uint16_t hb_half;
typedef void *hb_stream;      /* hipStream_t */

#define HB_MAX_TAPS 64          /* per axis, hb_sepblur */
#define HB_MAX_TAPS_FIR1D 256   /* hb_fir1d: the large-tap regime of Sec. V-A */
#define HB_MAX_TAPS_CONV2D 32   /* per axis, hb_conv2d, hb_down2, hb_up2 */
#define HB_RESIZE_MAX_SPAN 512   /* hb_resize: largest band; input samples of a group handled per round */

/* Human-readable name of a status code (static storage). */
const char *hb_status_string(hb_status s);

/*
 * Row-wise 1-D FIR (Sec. V-A, 1-D convolution as a product with the Toeplitz
 * matrix A_K(x, y) = K(y - x)):
 *     out[y][x] = sum_{r < ntaps} taps[r] * in[y][clampW(x + r - anchor)]
 * in: H x W fp16, out: H x W fp32.  1 <= ntaps <= HB_MAX_TAPS_FIR1D, 0 <= anchor < ntaps.
 */
hb_status hb_fir1d(const hb_half *in, float *out, int H, int W,
                   int64_t in_pitch, int64_t out_pitch,
                   const hb_half *taps_host, int ntaps, int anchor, hb_stream stream);
hb_status hb_fir1d_valu(const hb_half *in, float *out, int H, int W,
                        int64_t in_pitch, int64_t out_pitch,
                        const hb_half *taps_host, int ntaps, int anchor, hb_stream stream);

/*
 * Single-channel 2-D convolution with an arbitrary, non-separable kernel (Sec. V-A,
 * the 2-D form; on the matrix units it runs as the serial loop over the kernel
 * rows r_y, one Toeplitz product per kernel row into the same accumulator):
 *     out[y][x] = sum_{ry < kh} sum_{rx < kw} taps[ry * kw + rx]
 *                 * in[clampH(y + ry - anchor_y)][clampW(x + rx - anchor_x)]
 * in: H x W fp16, out: H x W fp32.  taps_host: kh x kw fp16 bit patterns, row-major,
 * HOST memory, read before the call returns.  1 <= kh, kw <= HB_MAX_TAPS_CONV2D,
 * 0 <= anchor_y < kh, 0 <= anchor_x < kw; otherwise HB_ERR_INVALID_ARG.  Size
 * limits as for hb_fir1d (HB_ERR_UNSUPPORTED beyond them).  One launch: strips whose
 * windows reach over the left or right image border load their pixels with clamped
 * column indices inside the same kernel.
 */
hb_status hb_conv2d(const hb_half *in, float *out, int H, int W,
                    int64_t in_pitch, int64_t out_pitch,
                    const hb_half *taps_host, int kh, int kw, int anchor_y, int anchor_x,
                    hb_stream stream);
hb_status hb_conv2d_valu(const hb_half *in, float *out, int H, int W,
                         int64_t in_pitch, int64_t out_pitch,
                         const hb_half *taps_host, int kh, int kw, int anchor_y, int anchor_x,
                         hb_stream stream);

/*
 * Resampling by a factor of two with an arbitrary 2-D kernel (Sec. V-B).
 *
 * hb_down2, the strided convolution (per kernel row a product with the
 * Toeplitz-like matrix A^down_K(x, y) = K(y - 2x)):
 *     out[y][x] = sum_{ry < kh} sum_{rx < kw} taps[ry * kw + rx]
 *                 * in[clampH(2y + ry - anchor_y)][clampW(2x + rx - anchor_x)]
 * in: H x W fp16, out: ceil(H/2) x ceil(W/2) fp32; 0 <= anchor_y < kh, 0 <= anchor_x < kw.
 *
 * hb_up2, the multiphase filter K^phase(x, y, dx, dy) = K(2x + dx, 2y + dy):
 *     out[y][x] = sum_{ry < kh/2} sum_{rx < kw/2} taps[(2 ry + y%2) * kw + 2 rx + x%2]
 *                 * in[clampH(y/2 + ry - anchor_y)][clampW(x/2 + rx - anchor_x)]
 * in: H x W fp16, out: 2H x 2W fp32; kh and kw even; anchors count input pixels:
 * 0 <= anchor_y < kh/2, 0 <= anchor_x < kw/2.
 *
 * Both: taps_host is kh x kw fp16 bit patterns, row-major, HOST memory, read
 * before the call returns; 1 <= kh, kw <= HB_MAX_TAPS_CONV2D; pitches in elements
 * of the respective image; HB_ERR_INVALID_ARG for bad shapes, taps or anchors,
 * HB_ERR_UNSUPPORTED beyond the size limits of hb_fir1d (applied to the input and
 * to the output image).
 */
hb_status hb_down2(const hb_half *in, float *out, int H, int W,
                   int64_t in_pitch, int64_t out_pitch,
                   const hb_half *taps_host, int kh, int kw, int anchor_y, int anchor_x,
                   hb_stream stream);
hb_status hb_down2_valu(const hb_half *in, float *out, int H, int W,
                        int64_t in_pitch, int64_t out_pitch,
                        const hb_half *taps_host, int kh, int kw, int anchor_y, int anchor_x,
                        hb_stream stream);
hb_status hb_up2(const hb_half *in, float *out, int H, int W,
                 int64_t in_pitch, int64_t out_pitch,
                 const hb_half *taps_host, int kh, int kw, int anchor_y, int anchor_x,
                 hb_stream stream);
hb_status hb_up2_valu(const hb_half *in, float *out, int H, int W,
                      int64_t in_pitch, int64_t out_pitch,
                      const hb_half *taps_host, int kh, int kw, int anchor_y, int anchor_x,
                      hb_stream stream);

/*
 * Separable 2-D blur (Sec. V-A, the 2-D form with K(rx, ry) = kx[rx] ky[ry]; the
 * second axis is a second Toeplitz product with the coefficient matrix on the
 * left):
 *     tmp[y][x] = sum_r taps_x[r] * in[y][clampW(x + r - anchor_x)]    (rounded to fp16)
 *     out[y][x] = sum_r taps_y[r] * tmp[clampH(y + r - anchor_y)][x]
 * in: H x W fp16, out: H x W fp32; tmp never leaves the chip.
 */
hb_status hb_sepblur(const hb_half *in, float *out, int H, int W,
                     int64_t in_pitch, int64_t out_pitch,
                     const hb_half *taps_x_host, int ntaps_x, int anchor_x,
                     const hb_half *taps_y_host, int ntaps_y, int anchor_y, hb_stream stream);
hb_status hb_sepblur_valu(const hb_half *in, float *out, int H, int W,
                          int64_t in_pitch, int64_t out_pitch,
                          const hb_half *taps_x_host, int ntaps_x, int anchor_x,
                          const hb_half *taps_y_host, int ntaps_y, int anchor_y, hb_stream stream);

/*
 * Resampling by a non-integer factor with precomputed banded matrices (Sec. V-C:
 * vertical and horizontal resizing are separate sparse matrices with a band of
 * known width; groups of 16 rows are treated as one dense block):
 *     out[c][yo][xo] = sum_{i < band_y} sum_{j < band_x} coef_y[yo * band_y + i] * coef_x[xo * band_x + j]
 *                      * in[c][clampH(start_y[yo] + i)][clampW(start_x[xo] + j)]
 * The horizontal pass runs first; its result is rounded to fp16 and kept, transposed,
 * in `workspace`.  in: C planes of H x W fp16 (row pitch in_pitch, plane stride in_plane,
 * in elements); out: C planes of Ho x Wo fp32 (out_pitch, out_plane).
 * start_y / start_x: Ho / Wo int32; coef_y / coef_x: Ho x band_y / Wo x band_x fp16,
 * row-major.  All four are DEVICE pointers, read by the kernels on `stream`.
 * `workspace`: device scratch of at least hb_resize_workspace_size(C, H, Wo) bytes,
 * 256-byte aligned; contents undefined on exit; concurrent calls need their own.
 * 1 <= band <= HB_RESIZE_MAX_SPAN.  Every read is clamped into the image whatever
 * the matrices hold, and any starts are computed correctly: an aligned group of 16
 * outputs whose rows together span more than HB_RESIZE_MAX_SPAN input samples is
 * processed in several rounds of that many samples (slower, same result).
 */
size_t hb_resize_workspace_size(int C, int H, int Wo);
hb_status hb_resize(const hb_half *in, float *out, void *workspace, size_t workspace_bytes,
                    int C, int H, int W, int Ho, int Wo,
                    int64_t in_pitch, int64_t in_plane, int64_t out_pitch, int64_t out_plane,
                    const int32_t *start_y, const hb_half *coef_y, int band_y,
                    const int32_t *start_x, const hb_half *coef_x, int band_x, hb_stream stream);
hb_status hb_resize_valu(const hb_half *in, float *out, void *workspace, size_t workspace_bytes,
                         int C, int H, int W, int Ho, int Wo,
                         int64_t in_pitch, int64_t in_plane, int64_t out_pitch, int64_t out_plane,
                         const int32_t *start_y, const hb_half *coef_y, int band_y,
                         const int32_t *start_x, const hb_half *coef_x, int band_x, hb_stream stream);

/*
 * The banded matrix of a three-lobed Lanczos pre-filter, sinc(x) sinc(x/3) on [-3, 3]
 * (Sec. V-C), that resamples n_in samples to n_out <= n_in: output o sits at input
 * position (o + 1/2) n_in/n_out - 1/2, the window is stretched by n_in/n_out, every
 * row is normalised to sum 1 (in double) and rounded once to fp16.  HOST function and
 * HOST arrays: start_host[n_out], coef_host[n_out * hb_lanczos3_band(n_in, n_out)].
 * hb_lanczos3_band returns the entries per row, floor(6 n_in/n_out) + 1, or 0 for
 * bad sizes; hb_lanczos3_matrix returns HB_ERR_UNSUPPORTED if that exceeds
 * HB_RESIZE_MAX_SPAN.
 */
int hb_lanczos3_band(int n_in, int n_out);
hb_status hb_lanczos3_matrix(int n_in, int n_out, int32_t *start_host, hb_half *coef_host);

/*
 * Second-order recursive filter over C independent channels (Sec. V-D):
 *     out[c][t] = in[c][t] + alpha * out[c][t-1] + beta * out[c][t-2],   out[c][-1] = out[c][-2] = 0
 * computed in tiles with a fix-up from the preceding tiles; inside a tile the
 * recursion over a block of 32 samples is a product with the triangular Toeplitz
 * matrix of the impulse response.  in: C x T fp16, out: C x T fp32 (row pitches in
 * elements, >= T).  |alpha|, |beta| <= 4; filters whose 32-sample impulse response
 * leaves the fp16 range, or whose tile-to-tile state maps overflow, are
 * HB_ERR_UNSUPPORTED (stable filters never are).  All sums are fp32, and a rounding
 * error made at one sample passes through the filter like an input: the absolute
 * error is bounded by about 2^-24 * G * max|out|, G = sum over i < T of |h[i]| (h the
 * impulse response).  The call computes G on the host and returns
 * HB_ERR_UNSUPPORTED when G > 16384 (= 1e-3 * 2^24: beyond it that bound no longer
 * stays within 1e-3 * max|out|); a complex pole pair of radius 0.95 has G of a few
 * hundred, the running sum (alpha = 1, beta = 0) has G = T.  hb_iir2_abs_gain
 * returns the G that the call would check (host only; -1 for arguments outside
 * the ranges above).
 * `workspace`: device scratch of at
 * least hb_iir2_workspace_size(C, T) bytes, 256-byte aligned; contents undefined on
 * exit; concurrent calls need their own.
 */
size_t hb_iir2_workspace_size(int C, int64_t T);
double hb_iir2_abs_gain(float alpha, float beta, int64_t T);
hb_status hb_iir2(const hb_half *in, float *out, int C, int64_t T, int64_t in_pitch, int64_t out_pitch,
                  float alpha, float beta, void *workspace, size_t workspace_bytes, hb_stream stream);
hb_status hb_iir2_valu(const hb_half *in, float *out, int C, int64_t T, int64_t in_pitch, int64_t out_pitch,
                       float alpha, float beta, void *workspace, size_t workspace_bytes, hb_stream stream);

/*
 * DCT-domain denoising by coring (Sec. V-E): 16 x 16 tiles at stride 8; a tile is
 * multiplied by the separable window w(i) = sin(pi (i + 1/2) / 16), transformed by
 * the orthonormal 2-D DCT-II (D T D^T), every bin except DC with magnitude below
 * `threshold` is set to zero, the tile is transformed back (D^T Y D), windowed again,
 * and the overlapping tiles are blended:
 *     out = sum_tiles(w * reconstruction) / sum_tiles(w^2)
 * Tile origins are (8 ty, 8 tx), 0 <= ty < H/8 - 1, 0 <= tx < W/8 - 1.  (The paper
 * fixes the tile size, the four fused products and the separate blend; window,
 * stride and the treatment of DC are this library's choices.)  in: C planes of H x W
 * fp16, out: C planes of H x W fp32 (row pitches and plane strides in elements);
 * H and W multiples of 8 and >= 16; threshold >= 0.  `workspace`: device scratch of
 * at least hb_dct_denoise_workspace_size(C, H, W) bytes, 256-byte aligned; contents
 * undefined on exit; concurrent calls need their own.  (hb_dct_denoise blends inside
 * its one kernel and leaves the workspace untouched; the twin keeps its tiles there.
 * Both check it the same way.)
 */
size_t hb_dct_denoise_workspace_size(int C, int H, int W);
hb_status hb_dct_denoise(const hb_half *in, float *out, int C, int H, int W,
                         int64_t in_pitch, int64_t in_plane, int64_t out_pitch, int64_t out_plane,
                         float threshold, void *workspace, size_t workspace_bytes, hb_stream stream);
hb_status hb_dct_denoise_valu(const hb_half *in, float *out, int C, int H, int W,
                              int64_t in_pitch, int64_t in_plane, int64_t out_pitch, int64_t out_plane,
                              float threshold, void *workspace, size_t workspace_bytes, hb_stream stream);

/*
 * Summed-area table (inclusive prefix sum over rows and columns; a product
 * L * X * U with triangular all-ones matrices per tile plus inter-tile carries --
 * the tile-then-fix-up structure of Sec. V-D applied to a first-order recursion):
 *     out[i][j] = sum_{y <= i} sum_{x <= j} in[y][x]
 * in: H x W fp16, out: H x W fp32.  `workspace` is device scratch of at least
 * hb_sat2d_workspace_size(H, W) bytes, 256-byte aligned; its contents on entry do
 * not matter and are undefined on exit.  Two calls that run concurrently need
 * two workspaces.
 * Images of up to 1024 regions of 256 x 256 pixels whose workgroups are all resident
 * at once (4096 x 4096 is 256 regions) run as ONE kernel that reads the image once:
 * every workgroup forms the local table of its region in registers, publishes the
 * region's row, column and total sums in the workspace, waits until all regions have
 * published, adds the sums of the regions to its left and above, and stores.  The
 * wait is bounded (hb_sat2d_set_wait_limit): a workgroup that reaches the bound marks
 * its region and exits, and the workgroups that got through finish the marked regions
 * from memory, so the kernel ends whatever the scheduling.  A small kernel ahead of it
 * on the same stream clears the wait's counters.  Larger images take three launches
 * (tile sums, scans of the carries, apply) and read the image twice.
 */
size_t hb_sat2d_workspace_size(int H, int W);
hb_status hb_sat2d(const hb_half *in, float *out, int H, int W,
                   int64_t in_pitch, int64_t out_pitch,
                   void *workspace, size_t workspace_bytes, hb_stream stream);
hb_status hb_sat2d_valu(const hb_half *in, float *out, int H, int W,
                        int64_t in_pitch, int64_t out_pitch,
                        void *workspace, size_t workspace_bytes, hb_stream stream);

/*
 * hb_sat2d for callers that cannot allocate device memory or pass a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments (minus the workspace), same kernels and bit-identical results; the carry
 * tables live in a fixed array of HB_SAT2D_NOALLOC_SCRATCH_BYTES inside the library's
 * code object, which every GPU the library runs on holds until the process ends.  The
 * call allocates and frees nothing.  Images whose hb_sat2d_workspace_size(H, W) exceeds
 * HB_SAT2D_NOALLOC_SCRATCH_BYTES (4096 x 4096 needs 4.6 MiB and fits) return
 * HB_ERR_UNSUPPORTED.  All calls on one GPU share
 * that GPU's array: two such calls that overlap in time on one GPU (different streams)
 * race; calls on one stream, or ordered by events, are fine.  The first call on a device
 * looks the array's address up (make it outside a graph capture).
 */
#define HB_SAT2D_NOALLOC_SCRATCH_BYTES (5u << 20)
hb_status hb_sat2d_noalloc(const hb_half *in, float *out, int H, int W,
                           int64_t in_pitch, int64_t out_pitch, hb_stream stream);

/*
 * Tuning and test hook of hb_sat2d's one-launch kernel (see hb_sat2d): how many polls a
 * workgroup spends in the grid-wide wait before it hands its region to a finisher.
 * polls > 0 sets the limit, 0 restores the default (16384), a negative value makes every
 * workgroup that does not find the wait already over stop at once (tests use it to run
 * the finisher path).  Whatever the value, every kernel exits and the result is the same.
 * Process-wide; read when a call is enqueued.  Returns the previous limit.
 */
int hb_sat2d_set_wait_limit(int polls);

/*
 * Multi-channel 3x3 convolution, stride 1, zero padding 1 (Sec. V-A 2-D form summed
 * over input channels; the conv layer of Sec. IV without bias and activation), as an
 * implicit GEMM with M = pixels, N = Cout, K = 9 * Cin:
 *     out[n][y][x][co] = sum_{ky,kx < 3} sum_ci in[n][y+ky-1][x+kx-1][ci] * w[ky][kx][ci][co]
 * in: N x H x W x Cin fp16 (NHWC, dense), w: 3 x 3 x Cin x Cout fp16 (HWIO, dense),
 * out: N x H x W x Cout fp16 (fp32 accumulator rounded to nearest even).
 * Cin and Cout must both be 64 (HB_ERR_UNSUPPORTED otherwise); pointers 16-byte aligned;
 * one image at most 2 GiB (H * W < 2^24 pixels; HB_ERR_UNSUPPORTED beyond).
 */
hb_status hb_conv3x3(const hb_half *in_nhwc, const hb_half *w_hwio, hb_half *out_nhwc,
                     int N, int H, int W, int Cin, int Cout, hb_stream stream);
hb_status hb_conv3x3_valu(const hb_half *in_nhwc, const hb_half *w_hwio, hb_half *out_nhwc,
                          int N, int H, int W, int Cin, int Cout, hb_stream stream);

/*
 * One Laplacian-pyramid level with the fixed kernel w = [1,4,6,4,1]/16 (Sec. V-B:
 * 2x downsample as a product with A_down(x, y) = K(y - 2x), 2x upsample as a
 * two-phase filter K_phase(x, dx) = K(2x + dx) whose phases are interleaved before
 * the store):
 *     D[m][n]  = sum_{i,j=-2..2} w[i] w[j] in[clampH(2m+i)][clampW(2n+j)]      (H/2 x W/2, fp16 on chip)
 *     per axis:  U[2n] = (D[c(n-1)] + 6 D[n] + D[c(n+1)]) / 8,  U[2n+1] = (D[n] + D[c(n+1)]) / 2
 *                (c clamps the D index to its extent), along x then along y
 *     residual = in - U                                                        (H x W, fp32)
 * H and W must be even.  `down_or_null`, when not null, receives D rounded to fp16
 * (H/2 x W/2, pitch down_pitch); pass NULL (and any pitch) to skip it.
 */
hb_status hb_pyr_level(const hb_half *in, float *residual, hb_half *down_or_null,
                       int H, int W, int64_t in_pitch, int64_t res_pitch, int64_t down_pitch,
                       hb_stream stream);
hb_status hb_pyr_level_valu(const hb_half *in, float *residual, hb_half *down_or_null,
                            int H, int W, int64_t in_pitch, int64_t res_pitch, int64_t down_pitch,
                            hb_stream stream);

/*
 * Measurement helper, not a stage: out[i] = (float) in[i] for n elements with 16-byte
 * vector accesses.  It moves the same 2 B in + 4 B out per element as the streaming
 * stages and serves as the achievable-bandwidth reference.  n >= 1; pointers 16-byte
 * aligned.
 */
hb_status hb_copy_f16_f32(const hb_half *in, float *out, int64_t n, hb_stream stream);

/*
 * Self-check helper, not a stage: runs one v_mfma_f32_16x16x32_f16 (which = 0),
 * one v_mfma_f32_16x16x16_f16 (which = 1), one v_mfma_f32_32x32x16_f16 (which = 2) or
 * one v_mfma_f32_16x16x4_f32 (which = 3) on dense row-major operands A (M x K) and
 * B (K x N) gathered through the operand-to-lane maps the kernels assume, and
 * scatters the accumulator to row-major D (M x N, fp32).  A test multiplies random
 * matrices and compares with a host product, which checks those maps.  A and B are
 * fp16 for which 0..2 and fp32 for which 3.  which = 4 chains two products of
 * different shape on one accumulator, back to back (an order the stage kernels never
 * use): D = A1 B1 + A2 B2 with A = A1 (16 x 32) followed by A2 (16 x 16), B = B1
 * (32 x 16) followed by B2 (16 x 16), each part dense row-major fp16, D 16 x 16.
 */
hb_status hb_mfma_probe(int which, const void *A, const void *B, float *D, hb_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* HB_H */
