// mac.hip -- pruned kernel transform and the per-bin multiply-accumulate.
//
// Kernel side of the layer (Sections III-A and IV-B-2).  A k^3 kernel zero-padded to N^3 is transformed
// axis by axis, touching only lines that are not all zero: k^2 lines along z, then k*zc lines along y, then
// N*zc lines along x.  With k small each of these one-dimensional transforms of a k-sample line is evaluated
// directly from its k non-zero inputs.  The first two stages are stored (array A, k*N*zc values per kernel
// instead of N*N*zc); the third is evaluated where it is consumed, inside the multiply-accumulate
//
//     Yt[s][j](ox,oy,oz) = sum_i  Wt[j][i](ox,oy,oz) * Xt[s][i](ox,oy,oz),
//     Wt[j][i](ox,oy,oz) = sum_{a<k} A[oz][oy][j][i][a] * exp(-2 pi i a ox / N)
//
// which is the second stage of Algorithm 3 (multiply the f image spectra by the f kernel spectra of output
// image j, accumulate over the f products) without a stored kernel spectrum.  The 1/N^3 of the unnormalised
// transforms is folded into A.
#include "znni_internal.h"

namespace znni {

// A1[oz][row][.] with row = ((j*f+i)*k + a)*k + b :  sum_c w[row][c] exp(-2 pi i oz c / N)
__global__ void k_kprep_z(const float* __restrict__ w, float2* __restrict__ A1, const float2* __restrict__ tw,
                          int N, int nrows, int k)
{
    const int row = blockIdx.x * blockDim.x + threadIdx.x;
    const int oz = blockIdx.y;
    if (row >= nrows) return;
    const float* wr = w + (size_t)row * k;
    float2 acc = make_float2(0.f, 0.f);
    for (int c = 0; c < k; ++c) acc = caxpy(acc, wr[c], tw[(oz * c) % N]);
    A1[(size_t)oz * nrows + row] = acc;
}

// A[oz][oy][jia] = scale * sum_b A1[oz][jia][b] exp(-2 pi i oy b / N),   jia = (j*f+i)*k + a
__global__ void k_kprep_y(const float2* __restrict__ A1, float2* __restrict__ A, const float2* __restrict__ tw,
                          int N, int njia, int k, float scale)
{
    const int jia = blockIdx.x * blockDim.x + threadIdx.x;
    const int oy = blockIdx.y, oz = blockIdx.z;
    if (jia >= njia) return;
    const float2* a1 = A1 + ((size_t)oz * njia + jia) * k;
    float2 acc = make_float2(0.f, 0.f);
    for (int b = 0; b < k; ++b) acc = cadd(acc, cmul(a1[b], tw[(oy * b) % N]));
    A[((size_t)oz * N + oy) * njia + jia] = cscale(acc, scale);
}

// Plain multiply-accumulate, one workgroup per (oz, oy) pencil, one thread per ox.  Slow and simple: it is
// the fallback for shapes the tiled kernel does not take, and the form the tiled kernel is checked against.
__global__ void k_mac_simple(const float2* __restrict__ Xt, const float2* __restrict__ A, float2* __restrict__ Yt,
                             const float2* __restrict__ tw, int N, int S, int f, int fo, int k)
{
    const size_t pencil = (size_t)blockIdx.y * N + blockIdx.x;
    const float2* Xp = Xt + pencil * S * f * N;
    const float2* Ap = A + pencil * fo * f * k;
    float2* Yp = Yt + pencil * S * fo * N;
    for (int ox = threadIdx.x; ox < N; ox += blockDim.x) {
        for (int s = 0; s < S; ++s)
            for (int j = 0; j < fo; ++j) {
                float2 acc = make_float2(0.f, 0.f);
                for (int i = 0; i < f; ++i) {
                    const float2* aji = Ap + (size_t)(j * f + i) * k;
                    float2 W = make_float2(0.f, 0.f);
                    for (int a = 0; a < k; ++a) W = cadd(W, cmul(aji[a], tw[(a * ox) % N]));
                    acc = cadd(acc, cmul(W, Xp[(size_t)(s * f + i) * N + ox]));
                }
                Yp[(size_t)(s * fo + j) * N + ox] = acc;
            }
    }
}

#define ZNNI_LAUNCH_CHECK()                         \
    do {                                            \
        if (hipGetLastError() != hipSuccess) return ZNNI_ERR_HIP; \
    } while (0)

znni_status launch_kernel_prep(const LayerPlan& L, const float* w, hipStream_t st)
{
    const int njia = L.fo * L.f * L.k;
    const int nrows = njia * L.k;
    k_kprep_z<<<dim3((nrows + 255) / 256, L.zc), dim3(256), 0, st>>>(w, L.A1, L.tw, L.N, nrows, L.k);
    ZNNI_LAUNCH_CHECK();
    const float scale = (float)(1.0 / ((double)L.N * L.N * L.N));
    k_kprep_y<<<dim3((njia + 255) / 256, L.N, L.zc), dim3(256), 0, st>>>(L.A1, L.A, L.tw, L.N, njia, L.k, scale);
    ZNNI_LAUNCH_CHECK();
    return ZNNI_OK;
}

znni_status launch_mac(const LayerPlan& L, hipStream_t st)
{
    k_mac_simple<<<dim3(L.N, L.zc), dim3(256), 0, st>>>(L.buf0, L.A, L.buf1, L.tw, L.N, L.S, L.f, L.fo, L.k);
    ZNNI_LAUNCH_CHECK();
    return ZNNI_OK;
}

}  // namespace znni
