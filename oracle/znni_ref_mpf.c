/*
 * znni_ref_mpf.c -- CPU ORACLE for max-pooling and max-pooling fragments.  TEST INFRASTRUCTURE ONLY.
 *
 * Slow, plain, obviously-correct definition the GPU library's pooling kernels are checked against.  Never
 * linked into, imported by, or called from the product path; shares no code, header or helper with the HIP
 * kernels.  Only tests, the smoke check and the benchmark's cpu_baseline leg may load it.
 *
 * What it computes (paper Section VI, "Max-pooling and max-pooling fragments"):
 *
 *   Max pooling of an image of size n = <nx,ny,nz> with window p = <px,py,pz> cuts the image into blocks of
 *   size p and takes the maximum of each block; n must be divisible by p; the result has size n / p.
 *
 *   Max-pooling fragmentation performs that max pooling at every offset o = (ox,oy,oz), 0 <= o < p: fragment
 *   o is the max pooling of the image with its first o voxels per axis cut away (and whatever does not fill a
 *   whole block at the far end dropped).  It yields px*py*pz output images per input image.  When n + 1 is
 *   divisible by p on every axis all fragments have the size m = floor(n / p); this is the only case accepted
 *   here (a window of 1 on an axis is always accepted: then m = n on that axis).  Per output voxel:
 *
 *     F[o][a][b][c] = max_{0<=u<px, 0<=v<py, 0<=t<pz}  I[ox + px*a + u][oy + py*b + v][oz + pz*c + t],
 *                     0 <= a < mx, 0 <= b < my, 0 <= c < mz.
 *
 *   The layer turns a batch of S tuples of f images into a batch of S * px*py*pz tuples of f images
 *   (Section VII-A: the most significant dimension grows, each of the S inputs giving px*py*pz fragments):
 *
 *     O[s * (px py pz) + (ox * py + oy) * pz + oz][i] = F[(ox,oy,oz)] of I[s][i]
 *
 *   The order of the fragments inside one input's group (offset z fastest) is a convention of this build.
 *
 * Arithmetic: the maximum of fp32 values is one of them, so the result is exact; no promotion is needed.
 * Comparison uses '>' on floats; the inputs of the tests hold no NaN.
 *
 * All pointers are HOST pointers; tensors dense row-major, last index fastest:
 *     in  [S][f][nx][ny][nz]                                  float
 *     out (fragments) [S*px*py*pz][f][mx][my][mz]             float
 *     out (max pooling) [S][f][nx/px][ny/py][nz/pz]           float
 * Return value: 0 on success, -1 null pointer, -2 bad shape.
 */
#include <stddef.h>

static float window_max(const float* img, int ny, int nz, int x0, int y0, int z0, int px, int py, int pz)
{
    float m = img[((size_t)x0 * ny + y0) * nz + z0];
    for (int u = 0; u < px; ++u)
        for (int v = 0; v < py; ++v)
            for (int t = 0; t < pz; ++t) {
                const float val = img[((size_t)(x0 + u) * ny + (y0 + v)) * nz + (z0 + t)];
                if (val > m) m = val;
            }
    return m;
}

/* Plain max pooling (first paragraph of Section VI): n divisible by p on every axis. */
int znni_ref_maxpool(int S, int f, int nx, int ny, int nz, int px, int py, int pz,
                     const float* in, float* out)
{
    if (!in || !out) return -1;
    if (S < 1 || f < 1 || nx < 1 || ny < 1 || nz < 1 || px < 1 || py < 1 || pz < 1) return -2;
    if (nx % px || ny % py || nz % pz) return -2;
    const int mx = nx / px, my = ny / py, mz = nz / pz;
    for (long img = 0; img < (long)S * f; ++img) {
        const float* I = in + (size_t)img * nx * ny * nz;
        float* O = out + (size_t)img * mx * my * mz;
        for (int a = 0; a < mx; ++a)
            for (int b = 0; b < my; ++b)
                for (int c = 0; c < mz; ++c)
                    O[((size_t)a * my + b) * mz + c] = window_max(I, ny, nz, px * a, py * b, pz * c, px, py, pz);
    }
    return 0;
}

/* Max-pooling fragments (second paragraph of Section VI), batch layout as described above. */
int znni_ref_mpf(int S, int f, int nx, int ny, int nz, int px, int py, int pz,
                 const float* in, float* out)
{
    if (!in || !out) return -1;
    if (S < 1 || f < 1 || nx < 1 || ny < 1 || nz < 1 || px < 1 || py < 1 || pz < 1) return -2;
    if (px > nx || py > ny || pz > nz) return -2;
    if ((px > 1 && (nx + 1) % px) || (py > 1 && (ny + 1) % py) || (pz > 1 && (nz + 1) % pz)) return -2;
    const int mx = nx / px, my = ny / py, mz = nz / pz;
    const int nfrag = px * py * pz;
    const size_t fragvox = (size_t)mx * my * mz;
    for (int s = 0; s < S; ++s)
        for (int i = 0; i < f; ++i) {
            const float* I = in + ((size_t)s * f + i) * nx * ny * nz;
            for (int ox = 0; ox < px; ++ox)
                for (int oy = 0; oy < py; ++oy)
                    for (int oz = 0; oz < pz; ++oz) {
                        const int frag = (ox * py + oy) * pz + oz;
                        float* O = out + (((size_t)s * nfrag + frag) * f + i) * fragvox;
                        for (int a = 0; a < mx; ++a)
                            for (int b = 0; b < my; ++b)
                                for (int c = 0; c < mz; ++c)
                                    O[((size_t)a * my + b) * mz + c] =
                                        window_max(I, ny, nz, ox + px * a, oy + py * b, oz + pz * c, px, py, pz);
                    }
        }
    return 0;
}
