/*
 * znni.h -- C ABI of the pruned-FFT 3D convolutional layer for AMD MI355X (gfx950).
 *
 * The layer (paper Section IV): a batch of S inputs, each a tuple of f images of n^3 voxels, is turned into
 * S tuples of f' images of n'^3 voxels, n' = n - k + 1, by
 *
 *     O[s][j] = act( bias[j] + sum_{i<f} w[j][i] * I[s][i] )          (* = valid convolution, kernel flipped)
 *
 * computed with the convolution theorem (Section III-A) in three stages, as in the GPU algorithm of
 * Section IV-B-2 (Algorithm 3): forward transforms of the S*f images, a multiply-accumulate over the input
 * images in every frequency bin, inverse transforms of the S*f' accumulated spectra.  Kernel transforms are
 * pruned as in Section III-A (k^2, then k*n~, then n~^2 one-dimensional transforms) and their last stage is
 * evaluated inside the multiply-accumulate kernel, so no full-size kernel spectrum is ever stored.  Along x
 * (the slowest axis, transformed last) the common transform size of images and kernels is the library's choice
 * per layer shape: the full n~ for batches; blocks of eight or no transform at all (the kx-tap sum written out)
 * where a full-length kernel spectrum value would serve one input only.  The valid outputs are the same numbers
 * up to fp32 rounding whichever is taken.  Bias and transfer function are applied where the inverse transform
 * finishes an output image (Section IV-A-3).
 *
 * Limits (every call validates them on the host and returns the status named)
 *   - transform size per axis at most ZNNI_MAX_FFT = 1024, i.e. image edges up to 1024 (ZNNI_ERR_UNSUPPORTED_SIZE);
 *   - S*f and S*f' at most 65535 (launch grid), (f'+15)*(f+3)*kmax^2 and S*max(f,f')*nmax at most 2^30
 *     (32-bit index products inside the kernels) (ZNNI_ERR_SHAPE);
 *   - direct primitive: kernels whose staged image tile fits the 160 KB of LDS, about 6^3 taps and below
 *     (ZNNI_ERR_UNSUPPORTED_SIZE); pooling: window at most 4 and image edge at most 4096 per axis;
 *   - znni_conv3d_fft_static_v: layers whose workspace fits ZNNI_STATIC_SCRATCH_BYTES (ZNNI_ERR_WORKSPACE);
 *   - the workspace size reported by the *_workspace calls includes (f~ + 64) * f'~ zeroed complex elements
 *     (f~ = f rounded up to 4, f'~ = f' to 16) after the stored kernel transforms, which two multiply-accumulate kernels
 *     read (and discard) one iteration past the last frequency bin; nothing is read or written outside the
 *     workspace and the tensors for any shape within these limits.
 *
 * Conventions for every function below
 *   - Returns a znni_status; never throws, aborts or prints.
 *   - Every argument is validated on the host BEFORE the first HIP call, so argument errors are reported the
 *     same way on a machine without a GPU.
 *   - Pointers named in/w/bias/out/workspace are DEVICE pointers owned by the caller.  The library never
 *     allocates, frees or reallocates device memory and keeps no device state between calls.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default stream) and the call
 *     returns without synchronising, except znni_conv3d_fft_profile, which synchronises the stream.
 *   - Results are deterministic: no floating-point atomics, fixed summation order.
 *   - Tensors are dense, row-major, last index fastest; all arithmetic is fp32.
 */
#ifndef ZNNI_H
#define ZNNI_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ZNNI_OK = 0,
    ZNNI_ERR_NULL = -1,             /* a required pointer is NULL                                         */
    ZNNI_ERR_SHAPE = -2,            /* S, f, f' < 1, k < 1 or k > n on an axis, or a count too large for the launch grid */
    ZNNI_ERR_UNSUPPORTED_SIZE = -3, /* no supported transform size n~ >= n                                 */
    ZNNI_ERR_WORKSPACE = -4,        /* workspace smaller than znni_conv3d_fft_workspace reports            */
    ZNNI_ERR_FLAGS = -5,            /* unknown flag bit, or more than one of the ZNNI_MAC_* bits           */
    ZNNI_ERR_HIP = -6,              /* a HIP call or kernel launch failed                                  */
    ZNNI_ERR_ALIGN = -7             /* a device pointer is not 16-byte aligned (workspace: 256-byte)       */
} znni_status;

/* flags */
enum {
    ZNNI_RELU = 1u,                 /* transfer function max(0, .) (Section V); without it: identity       */
    ZNNI_MAC_REFERENCE = 2u,        /* diagnostic: run the multiply-accumulate stage with the plain one-thread- */
                                    /* per-bin kernel instead of the matrix-core kernel (same result up to     */
                                    /* rounding, much slower)                                                   */
    ZNNI_MAC_SINGLE = 4u,           /* force the multiply-accumulate form built for S = 1 (work grows with k*S) */
    ZNNI_MAC_BATCH = 8u,            /* force the form built for batches (kernel spectrum generated once per    */
                                    /* bin, shared by the S inputs; ignored where that form does not exist:    */
                                    /* more than 12 kernel taps, or up to 8 inputs with an odd transform       */
                                    /* length along x)                                                          */
    ZNNI_MAC_XDIRECT = 16u,         /* force the route that does not transform the x axis at all: transforms    */
                                    /* along z and y only, and the kernel's taps along x applied as a short     */
                                    /* valid convolution inside the multiply-accumulate (same contraction       */
                                    /* length as ZNNI_MAC_SINGLE, no x passes; ignored where it does not exist: */
                                    /* more than 9 taps along x, or a y transform length without an in-register */
                                    /* pass kernel)                                                             */
    ZNNI_KEEP_KERNELS = 64u,        /* skip the kernel transform: the workspace still holds the stored kernel   */
                                    /* transforms of an earlier call with the same w, layer shape and           */
                                    /* multiply-accumulate form, and nothing else has written to it since.      */
                                    /* For inference, where one set of kernels meets every patch of a volume    */
                                    /* (Section II), so that the pruned kernel transform of Section III-A is    */
                                    /* paid once per network and not once per patch.  The caller vouches: the   */
                                    /* library cannot tell stale transforms from fresh ones.  w is not read.    */
                                    /* Rejected by znni_conv3d_fft_budget_v (its sub-layers share the space).   */
    ZNNI_PASSES_REFERENCE = 128u,   /* diagnostic: run every transform pass with the generic kernels (lines staged in  */
                                    /* LDS, radix-2/3/4/5/7/8 stages) instead of the in-register ones, which serve all */
                                    /* transform sizes from 8 up: an independent implementation of the same passes,    */
                                    /* about half as fast.  Excludes the routes that do not transform x at full length */
    ZNNI_MAC_XBLOCK = 32u           /* force the route that transforms the x axis in overlapping blocks of      */
                                    /* eight inside the multiply-accumulate (transforms along z and y as for    */
                                    /* ZNNI_MAC_XDIRECT; 8 / (9 - kx) multiply-adds per output instead of kx;   */
                                    /* ignored where it does not exist: other than 4 or 5 taps along x, fewer   */
                                    /* than 16 input images, or no in-register y pass kernel); without any of   */
                                    /* these flags the library picks                                            */
};

/* Stages reported by znni_conv3d_fft_profile, in execution order (Algorithm 3 of Section IV-B-2). */
enum {
    ZNNI_STAGE_KERNEL_PREP = 0,     /* pruned kernel transform, first two axes (Section III-A)             */
    ZNNI_STAGE_FWD_Z = 1,           /* image transform, real-to-complex along z (Section III-C)            */
    ZNNI_STAGE_FWD_Y = 2,
    ZNNI_STAGE_FWD_X = 3,
    ZNNI_STAGE_MAC = 4,             /* last kernel-transform stage + per-bin multiply-accumulate           */
    ZNNI_STAGE_INV_X = 5,           /* inverse transforms, pruned to the valid outputs (Section III-B)     */
    ZNNI_STAGE_INV_Y = 6,
    ZNNI_STAGE_INV_Z = 7,           /* complex-to-real along z + bias + transfer function                  */
    ZNNI_NUM_STAGES = 8
};

/* Library version, major*10000 + minor*100 + patch. */
int znni_version(void);

/* Static string for a status code (never NULL; any integer may be passed, unknown ones give "unknown status"). */
const char* znni_status_string(int st);

/*
 * Transform size n~ used for an image edge n.  Members of the family 2^a 3^b 5^c 7^d that Section III-D names for
 * GPU transforms, up to ZNNI_MAX_FFT.  The valid outputs of a circular convolution of any length n~ >= n never wrap,
 * so the choice is one of speed only: the smallest of the 46 lengths that the in-register pass kernels serve (8, 10,
 * 12, 14, 16, 20, 24, 28, 32, 36, 40, 48, 56, 64, 72, 80, 84, 96, 100, 112, 120, 128, 144, 160, 168, 192, 200, 224,
 * 240, 256, 288, 320, 336, 384, 400, 448, 480, 512, 576, 640, 720, 768, 840, 896, 960, 1024) that is >= n, at most
 * 20 % above n; n itself for n < 7.  Returns 0 if there is no supported size (n < 1 or n > ZNNI_MAX_FFT).  Host only.
 */
#define ZNNI_MAX_FFT 1024
int znni_fft_size(int n);

/*
 * Bytes of device workspace znni_conv3d_fft needs for this layer shape (Table II's GPU-FFT row plays the
 * same role in the paper: spectra of the inputs and outputs plus per-call scratch).  Host only.
 *   S, f, fo (= f'), n, k : layer shape as in Section IV.        bytes : out, host pointer.
 */
znni_status znni_conv3d_fft_workspace(int S, int f, int fo, int n, int k, size_t* bytes);

/*
 * The layer (Section IV equation; Algorithm 3).  Asynchronous on `stream`.
 *   in        [S][f][n][n][n]          device, read-only
 *   w         [fo][f][k][k][k]         device, read-only
 *   bias      [fo] device, read-only, or NULL for zero bias
 *   out       [S][fo][n-k+1]^3         device, written (every element)
 *   flags     bitwise OR of ZNNI_RELU, ZNNI_KEEP_KERNELS, ZNNI_PASSES_REFERENCE and at most one of the ZNNI_MAC_*
 *             flags, or 0
 *   workspace device scratch of at least znni_conv3d_fft_workspace() bytes, 256-byte aligned; contents on
 *             entry are ignored, contents on return are unspecified.  Calls that share a workspace must
 *             not overlap in time.
 */
znni_status znni_conv3d_fft(int S, int f, int fo, int n, int k,
                            const float* in, const float* w, const float* bias, float* out,
                            unsigned flags, void* workspace, size_t workspace_bytes, void* stream);

/*
 * znni_conv3d_fft_v for callers that cannot allocate device memory and have no workspace to pass: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same tensors, flags, result (bit for bit)
 * and status codes as znni_conv3d_fft_v, but the workspace is an array of ZNNI_STATIC_SCRATCH_BYTES bytes that
 * is part of the library's device code: every GPU the library runs on holds one copy from the moment the code is
 * loaded there until the process ends.  The call allocates and frees nothing.
 *   - ZNNI_ERR_WORKSPACE if the layer needs more than ZNNI_STATIC_SCRATCH_BYTES (znni_conv3d_fft_workspace_v
 *     tells what a shape needs; the second benchmark-sized layer, 8 -> 8 images of 64^3 with 5^3 kernels, fits).
 *   - The array belongs to the GPU that is current when the call is made; `stream` must be a stream of that GPU.
 *     Its address is looked up on the first call on each GPU (make that call outside a graph capture).
 *   - All calls on one GPU share the array, which keeps whatever the last call left in it (no call depends on
 *     that): two calls that overlap in time on one GPU, on any streams, race.  Calls on one stream do not overlap.
 */
#define ZNNI_STATIC_SCRATCH_BYTES (64u << 20)
znni_status znni_conv3d_fft_static_v(int S, int f, int fo, const int n[3], const int k[3],
                                     const float* in, const float* w, const float* bias, float* out,
                                     unsigned flags, void* stream);

/*
 * Same computation, with a HIP event recorded on `stream` between stages; synchronises `stream` before
 * returning and writes the elapsed milliseconds of each stage to stage_ms[ZNNI_NUM_STAGES] (HOST pointer).
 * Meant for measurement: creates and destroys its events on every call.  For small images the z and y
 * transforms of each side run as one kernel; its time is then reported under ZNNI_STAGE_FWD_Z (forward) and
 * ZNNI_STAGE_INV_Y (inverse), and ZNNI_STAGE_FWD_Y / ZNNI_STAGE_INV_Z read about zero.
 */
znni_status znni_conv3d_fft_profile(int S, int f, int fo, int n, int k,
                                    const float* in, const float* w, const float* bias, float* out,
                                    unsigned flags, void* workspace, size_t workspace_bytes, void* stream,
                                    float* stage_ms);

/*
 * Measurement aid (host only): the work the method itself has to do in each stage of a layer call with these
 * flags, for the kernels that call would run.  hbm_bytes[s] = bytes stage s must read plus write once (its input
 * and output tensors, unpadded); flops[s] = floating-point operations of the contraction in the
 * multiply-accumulate stage, counting 8 per complex multiply-add: (8 S + 8 (kx - 1)) f f' per bin of the transformed
 * image when the x axis is transformed (the per-bin product of Algorithm 3 plus the kx-term sum that stands in for a
 * stored kernel spectrum), 8 kx S f f' per bin of the image transformed along y and z only when it is not, 64 S f f'
 * per block of 9 - kx outputs where x is transformed in blocks of eight.  Stages a
 * call does not run (the y or z stage where one kernel does both, the x stages where the x axis is not transformed)
 * get 0.  Both arrays have ZNNI_NUM_STAGES elements, indexed like stage_ms above.
 */
znni_status znni_conv3d_fft_stage_work_v(int S, int f, int fo, const int n[3], const int k[3], unsigned flags,
                                         double hbm_bytes[ZNNI_NUM_STAGES], double flops[ZNNI_NUM_STAGES]);

/*
 * General image and kernel sizes (Section IV: an image has size n = <nx,ny,nz>, a kernel k = <kx,ky,kz>, the
 * output n' = n - k + 1 on every axis).  n and k are HOST pointers to three ints in the order x, y, z, where x
 * is the slowest and z the fastest (contiguous) index of the tensors:
 *   in   [S][f][nx][ny][nz]      w   [fo][f][kx][ky][kz]      out  [S][fo][nx-kx+1][ny-ky+1][nz-kz+1]
 * Each axis gets its own transform size znni_fft_size(n[axis]).  Everything else (pointer ownership, flags,
 * workspace, stream, status codes) is as for the cubic calls above, which are these calls with
 * n = <n,n,n>, k = <k,k,k>.  ZNNI_ERR_NULL if n or k is NULL.
 */
znni_status znni_conv3d_fft_workspace_v(int S, int f, int fo, const int n[3], const int k[3], size_t* bytes);

znni_status znni_conv3d_fft_v(int S, int f, int fo, const int n[3], const int k[3],
                              const float* in, const float* w, const float* bias, float* out,
                              unsigned flags, void* workspace, size_t workspace_bytes, void* stream);

znni_status znni_conv3d_fft_profile_v(int S, int f, int fo, const int n[3], const int k[3],
                                      const float* in, const float* w, const float* bias, float* out,
                                      unsigned flags, void* workspace, size_t workspace_bytes, void* stream,
                                      float* stage_ms);

/*
 * The layer under a memory budget (Section VII-A: a layer of shape (S, f, f') computed as sub-layers of shapes
 * (S_i, f_i, f'_i), each small enough for the memory at hand).  The budget is the workspace the caller can
 * spare.  The division follows the preference stated there: the whole layer if it fits; else sub-batches
 * (f_i = f, f'_i = f', the largest S_i that fits), which transform every input and output image once; else
 * S_i = 1 with blocks of f_i input and f'_i output images (f_i from {f, multiples of 4, 2, 1}, f'_i from
 * {f', multiples of 16, 8, 4, 2, 1}), chosen to move the fewest bytes.  In the last case the sub-layers of one block of output images add their
 * products into that block's spectra, which are inverse-transformed once, after the last input block; bias and
 * transfer function are applied there.  The result equals znni_conv3d_fft_v's up to fp32 rounding (the sum over
 * input images is taken in a different order).
 *
 * znni_conv3d_fft_sublayers_v: host only.  Writes the division for `budget_bytes` to sub[3] = {S_i, f_i, f'_i}
 *   and the workspace it needs (<= budget_bytes) to *bytes.  ZNNI_ERR_WORKSPACE if even the smallest division
 *   (S_i = f_i = f'_i = 1) does not fit; *bytes then holds what that division needs.
 * znni_conv3d_fft_budget_v: runs the layer with the division chosen for workspace_bytes.  Arguments, ownership,
 *   alignment and status codes as for znni_conv3d_fft_v; ZNNI_ERR_WORKSPACE if no division fits.
 */
znni_status znni_conv3d_fft_sublayers_v(int S, int f, int fo, const int n[3], const int k[3],
                                        size_t budget_bytes, int sub[3], size_t* bytes);

znni_status znni_conv3d_fft_budget_v(int S, int f, int fo, const int n[3], const int k[3],
                                     const float* in, const float* w, const float* bias, float* out,
                                     unsigned flags, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same layer by direct convolution (Section IV-A-1): no transforms, the sum over input images and kernel taps
 * is evaluated as written, on the matrix cores.  Meant for small kernels and few input images, where it beats the
 * transform route (Section VII: the choice of primitive per layer).  Tensors, flags (ZNNI_RELU only), ownership and
 * status codes as for znni_conv3d_fft_v, except that in, w and out need 4-byte alignment only.  The workspace
 * (znni_conv3d_direct_workspace_v bytes, 256-byte aligned) holds the kernel bank rearranged for the matrix cores.
 * ZNNI_ERR_UNSUPPORTED_SIZE if the kernel is too large for this primitive (about 7^3 and up).
 */
znni_status znni_conv3d_direct_workspace_v(int S, int f, int fo, const int n[3], const int k[3], size_t* bytes);

znni_status znni_conv3d_direct_v(int S, int f, int fo, const int n[3], const int k[3],
                                 const float* in, const float* w, const float* bias, float* out,
                                 unsigned flags, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Choice of primitive per layer (Section VII: each layer is run by whichever primitive is fastest for its shape).
 * znni_conv3d_choose_v (host only) ranks the transform route and the direct route with a cost model whose rates
 * were measured on MI355X and writes the pick to *primitive; est_ms, if not NULL, receives the two estimates in
 * milliseconds (index = primitive; negative = that primitive does not take this shape).
 * znni_conv3d_workspace_v / znni_conv3d_v are the workspace query and the layer call of the picked primitive;
 * arguments as for znni_conv3d_fft_v.  When the direct route is picked, ZNNI_MAC_SINGLE, _BATCH, _XDIRECT and
 * _XBLOCK are accepted (at most one) and ignored: they choose between forms of the transform route only.
 * ZNNI_KEEP_KERNELS is ignored there too (that route keeps nothing a later call could reuse and rearranges the bank
 * on every call), and ZNNI_MAC_REFERENCE is rejected with ZNNI_ERR_FLAGS.
 */
enum { ZNNI_PRIMITIVE_FFT = 0, ZNNI_PRIMITIVE_DIRECT = 1 };

znni_status znni_conv3d_choose_v(int S, int f, int fo, const int n[3], const int k[3], int* primitive,
                                 float est_ms[2]);

znni_status znni_conv3d_workspace_v(int S, int f, int fo, const int n[3], const int k[3], size_t* bytes);

znni_status znni_conv3d_v(int S, int f, int fo, const int n[3], const int k[3],
                          const float* in, const float* w, const float* bias, float* out,
                          unsigned flags, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Max-pooling fragments (Section VI, second paragraph).  For every offset o = (ox,oy,oz), 0 <= o < p, the image
 * is max-pooled with window p = <px,py,pz> starting at o:
 *     F[o][a][b][c] = max over the p-block of I starting at (ox + px a, oy + py b, oz + pz c),   a,b,c < m,
 * where n + 1 must be divisible by p on every axis with p > 1, so that every fragment has size
 * m = floor(n / p) per axis (the case the paper states).  A batch of S tuples of f images becomes a batch of
 * S*px*py*pz tuples (the most significant dimension grows, Section VII-A):
 *     in   [S][f][nx][ny][nz]                       device, read-only, 4-byte aligned
 *     out  [S*px*py*pz][f][mx][my][mz]              device, written (every element);
 *          tuple s*px*py*pz + (ox*py + oy)*pz + oz holds the fragments of offset (ox,oy,oz) of input s
 *   n, p  HOST pointers to three ints (x, y, z; z contiguous); 1 <= p <= 4 and p <= n <= 4096 per axis
 * Needs no workspace; asynchronous on `stream`.  ZNNI_ERR_SHAPE if the divisibility rule fails,
 * ZNNI_ERR_UNSUPPORTED_SIZE for a window above 4.
 */
znni_status znni_mpf(int S, int f, const int n[3], const int p[3], const float* in, float* out, void* stream);

/*
 * Max pooling (Section VI, first paragraph): the image is cut into blocks of size p and each block is replaced by
 * its maximum; n must be divisible by p on every axis.
 *     in [S][f][nx][ny][nz]  ->  out [S][f][nx/px][ny/py][nz/pz]      (device pointers, 4-byte aligned)
 * Needs no workspace; asynchronous on `stream`.
 */
znni_status znni_maxpool(int S, int f, const int n[3], const int p[3], const float* in, float* out, void* stream);

/*
 * Measurement aid: a plain device-to-device copy of `bytes` bytes (a multiple of 16; both pointers 16-byte
 * aligned device pointers) done by one simple kernel on `stream`.  Hardware counters that report HBM traffic are
 * calibrated against this kernel, whose traffic is known exactly: `bytes` read and `bytes` written.
 */
znni_status znni_copy_probe(void* dst, const void* src, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ZNNI_H */
