/*
 * znni_ref.c -- CPU ORACLE for the 3D convolutional layer.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain, obviously-correct definition the GPU library is checked against.
 * It is never linked into, imported by, or called from the product path; it shares no code, header,
 * table or helper with the HIP kernels.  Only tests, the smoke check and the benchmark's cpu_baseline
 * leg may load it.
 *
 * What it computes (paper Section IV, layer equation and tensor shapes):
 *
 *     O[s][j] = sum_{i<f}  w[j][i] * I[s][i]          ("*" = true convolution, kernel flipped)
 *
 * restricted to the positions where the kernel lies entirely inside the image ("valid" convolution,
 * Section II), so an image of size n = <nx,ny,nz> and a kernel of size k = <kx,ky,kz> give an output of
 * size n' = n - k + 1 (Section IV).  Written out per output voxel:
 *
 *     pre[s][j][x][y][z] = bias[j]
 *         + sum_{i<f} sum_{a<kx} sum_{b<ky} sum_{c<kz}
 *               w[j][i][a][b][c] * I[s][i][x + kx-1 - a][y + ky-1 - b][z + kz-1 - c]
 *     O = max(0, pre) when the rectified-linear transfer function is selected, else pre.
 *
 * The bias is one scalar per output image and is added, followed by the transfer function, in the same
 * step that finishes an output image (Section IV-A-3, "output image transform" task); the networks of
 * Section V use the rectified-linear function.
 *
 * Loop structure follows the direct-convolution algorithm of Section IV-A-1 (Algorithm 1): the two outer
 * loops over the batch index s and the output image j run in parallel, the loop over the input image i is
 * serial and accumulates Convolve(I[s][i], w[j][i]) into O[s][j].
 *
 * Arithmetic: inputs are the caller's fp32 arrays promoted to fp64; every product and sum is fp64.
 * No FFT, no BLAS, no blocking, no reordering beyond the loops stated above.
 *
 * All pointers are HOST pointers.  Tensors are dense row-major with the last index fastest:
 *     in  [S][f ][nx][ny][nz]   float
 *     w   [fo][f][kx][ky][kz]   float
 *     bias[fo] float, or NULL meaning zero
 *     out [S][fo][nx-kx+1][ny-ky+1][nz-kz+1]   double
 * Return value: 0 on success, -1 null pointer, -2 bad shape, -5 unknown flag bit.
 */
#include <stddef.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ZNNI_REF_RELU 1u

static int check_args(int S, int f, int fo, int nx, int ny, int nz, int kx, int ky, int kz,
                      const void* in, const void* w, const void* out, unsigned flags)
{
    if (!in || !w || !out) return -1;
    if (S < 1 || f < 1 || fo < 1) return -2;
    if (kx < 1 || ky < 1 || kz < 1) return -2;
    if (kx > nx || ky > ny || kz > nz) return -2;
    if (flags & ~ZNNI_REF_RELU) return -5;
    return 0;
}

/* One "Convolve(I[s][i], w[j][i])" of Algorithm 1, accumulated into the output image o (n' voxels). */
static void convolve_accumulate(const float* img, const float* ker, double* o,
                                int nx, int ny, int nz, int kx, int ky, int kz)
{
    const int ox = nx - kx + 1, oy = ny - ky + 1, oz = nz - kz + 1;
    (void)nx;
    for (int a = 0; a < kx; ++a)
        for (int b = 0; b < ky; ++b)
            for (int c = 0; c < kz; ++c) {
                const double wv = (double)ker[((size_t)a * ky + b) * kz + c];
                for (int x = 0; x < ox; ++x)
                    for (int y = 0; y < oy; ++y) {
                        const float* src = img + ((size_t)(x + kx - 1 - a) * ny + (y + ky - 1 - b)) * nz
                                               + (kz - 1 - c);
                        double* dst = o + ((size_t)x * oy + y) * oz;
                        for (int z = 0; z < oz; ++z) dst[z] += wv * (double)src[z];
                    }
            }
}

/* General (anisotropic) layer: image size <nx,ny,nz>, kernel size <kx,ky,kz>. */
int znni_ref_conv3d_f64_v(int S, int f, int fo, int nx, int ny, int nz, int kx, int ky, int kz,
                          const float* in, const float* w, const float* bias, double* out,
                          unsigned flags, int nthreads)
{
    int rc = check_args(S, f, fo, nx, ny, nz, kx, ky, kz, in, w, out, flags);
    if (rc) return rc;
    const size_t nvox = (size_t)nx * ny * nz;
    const size_t kvox = (size_t)kx * ky * kz;
    const size_t ovox = (size_t)(nx - kx + 1) * (ny - ky + 1) * (nz - kz + 1);
#ifdef _OPENMP
    if (nthreads < 1) nthreads = omp_get_max_threads();
#else
    (void)nthreads;
#endif
    const long jobs = (long)S * fo;
    #pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (long sj = 0; sj < jobs; ++sj) {
        const int s = (int)(sj / fo), j = (int)(sj % fo);
        double* o = out + ((size_t)s * fo + j) * ovox;
        for (size_t v = 0; v < ovox; ++v) o[v] = 0.0;
        for (int i = 0; i < f; ++i)
            convolve_accumulate(in + ((size_t)s * f + i) * nvox, w + ((size_t)j * f + i) * kvox, o,
                                nx, ny, nz, kx, ky, kz);
        const double bj = bias ? (double)bias[j] : 0.0;
        for (size_t v = 0; v < ovox; ++v) {
            double pre = o[v] + bj;
            o[v] = ((flags & ZNNI_REF_RELU) && pre < 0.0) ? 0.0 : pre;
        }
    }
    return 0;
}

/* Cubic layer: image n^3, kernel k^3 (the shape used by Table I and by every workload here). */
int znni_ref_conv3d_f64(int S, int f, int fo, int n, int k,
                        const float* in, const float* w, const float* bias, double* out,
                        unsigned flags, int nthreads)
{
    return znni_ref_conv3d_f64_v(S, f, fo, n, n, n, k, k, k, in, w, bias, out, flags, nthreads);
}

/*
 * The same definition evaluated one output voxel at a time at caller-chosen positions, for layers whose
 * full direct convolution is too slow to run in a test.  pts holds npts records (s, j, x, y, z) of int;
 * out[p] receives O[s][j][x][y][z].  Summation order per voxel: i, a, b, c.
 * Returns -2 if any position lies outside the output tensor.
 */
int znni_ref_conv3d_points_f64(int S, int f, int fo, int nx, int ny, int nz, int kx, int ky, int kz,
                               const float* in, const float* w, const float* bias,
                               const int* pts, long npts, double* out, unsigned flags, int nthreads)
{
    int rc = check_args(S, f, fo, nx, ny, nz, kx, ky, kz, in, w, out, flags);
    if (rc) return rc;
    if (!pts || npts < 0) return -1;
    const int ox = nx - kx + 1, oy = ny - ky + 1, oz = nz - kz + 1;
    const size_t nvox = (size_t)nx * ny * nz;
    const size_t kvox = (size_t)kx * ky * kz;
    for (long p = 0; p < npts; ++p) {
        const int* q = pts + 5 * p;
        if (q[0] < 0 || q[0] >= S || q[1] < 0 || q[1] >= fo || q[2] < 0 || q[2] >= ox ||
            q[3] < 0 || q[3] >= oy || q[4] < 0 || q[4] >= oz)
            return -2;
    }
#ifdef _OPENMP
    if (nthreads < 1) nthreads = omp_get_max_threads();
#else
    (void)nthreads;
#endif
    #pragma omp parallel for schedule(static) num_threads(nthreads)
    for (long p = 0; p < npts; ++p) {
        const int s = pts[5 * p], j = pts[5 * p + 1];
        const int x = pts[5 * p + 2], y = pts[5 * p + 3], z = pts[5 * p + 4];
        double acc = 0.0;
        for (int i = 0; i < f; ++i) {
            const float* img = in + ((size_t)s * f + i) * nvox;
            const float* ker = w + ((size_t)j * f + i) * kvox;
            for (int a = 0; a < kx; ++a)
                for (int b = 0; b < ky; ++b)
                    for (int c = 0; c < kz; ++c)
                        acc += (double)ker[((size_t)a * ky + b) * kz + c] *
                               (double)img[((size_t)(x + kx - 1 - a) * ny + (y + ky - 1 - b)) * nz
                                           + (z + kz - 1 - c)];
        }
        double pre = acc + (bias ? (double)bias[j] : 0.0);
        out[p] = ((flags & ZNNI_REF_RELU) && pre < 0.0) ? 0.0 : pre;
    }
    return 0;
}

/* Number of threads a call with nthreads < 1 would use (reported next to the CPU baseline timing). */
int znni_ref_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
