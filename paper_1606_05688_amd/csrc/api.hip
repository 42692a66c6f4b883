// api.hip -- the exported C ABI: argument validation, workspace planning, and the stage sequence of the
// GPU algorithm of Section IV-B-2 (Algorithm 3): transform the images, multiply-accumulate per bin with the
// kernel transforms, inverse-transform the output images.  All validation happens before the first HIP call.
#include <stdint.h>

#include "znni_internal.h"

namespace znni {

static bool smooth7(int m)
{
    for (int p : {2, 3, 5, 7})
        while (m % p == 0) m /= p;
    return m == 1;
}

static int fft_size(int n)
{
    if (n < 1) return 0;
    for (int m = n; m <= ZNNI_MAX_FFT; ++m)
        if (smooth7(m)) return m;
    return 0;
}

// Radix schedule: odd primes first, then the power of two as 8s with a 4,4 / 4 / 2 tail.
static void make_fft_plan(int N, FftPlan* P)
{
    P->N = N;
    P->nstages = 0;
    int m = N;
    for (int p : {7, 5, 3})
        while (m % p == 0) { P->radix[P->nstages++] = p; m /= p; }
    int a = 0;
    while (m > 1) { m >>= 1; ++a; }
    if (a == 1) { P->radix[P->nstages++] = 2; a = 0; }
    if (a % 3 == 1) { P->radix[P->nstages++] = 4; P->radix[P->nstages++] = 4; a -= 4; }
    if (a % 3 == 2) { P->radix[P->nstages++] = 4; a -= 2; }
    while (a > 0) { P->radix[P->nstages++] = 8; a -= 3; }
}

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

znni_status make_plan(int S, int f, int fo, const int n[3], const int k[3], void* base, LayerPlan* L)
{
    if (!n || !k) return ZNNI_ERR_NULL;
    if (S < 1 || f < 1 || fo < 1) return ZNNI_ERR_SHAPE;
    for (int a = 0; a < 3; ++a)
        if (n[a] < 1 || k[a] < 1 || k[a] > n[a]) return ZNNI_ERR_SHAPE;
    Dims& d = L->d;
    d.nx = n[0]; d.ny = n[1]; d.nz = n[2];
    d.kx = k[0]; d.ky = k[1]; d.kz = k[2];
    d.Nx = fft_size(d.nx); d.Ny = fft_size(d.ny); d.Nz = fft_size(d.nz);
    if (d.Nx == 0 || d.Ny == 0 || d.Nz == 0) return ZNNI_ERR_UNSUPPORTED_SIZE;
    // launch-grid limits (grid y/z <= 65535) and 32-bit index products used inside the kernels
    if ((long long)S * f > 65535 || (long long)S * fo > 65535) return ZNNI_ERR_SHAPE;
    const int kmax = d.kx > d.ky ? (d.kx > d.kz ? d.kx : d.kz) : (d.ky > d.kz ? d.ky : d.kz);
    const int nmax = d.nx > d.ny ? (d.nx > d.nz ? d.nx : d.nz) : (d.ny > d.nz ? d.ny : d.nz);
    if (((long long)fo + 15) * (f + 3) * kmax * kmax > (1ll << 30)) return ZNNI_ERR_SHAPE;
    if ((long long)S * (f > fo ? f : fo) * nmax > (1ll << 30)) return ZNNI_ERR_SHAPE;
    L->S = S; L->f = f; L->fo = fo;
    d.zc = d.Nz / 2 + 1;
    d.nox = d.nx - d.kx + 1; d.noy = d.ny - d.ky + 1; d.noz = d.nz - d.kz + 1;
    d.ldz = (d.zc + 15) & ~15;       // Y1 rows start on 128-byte boundaries
    L->nimg = S * f;
    L->nimgo = S * fo;
    L->fp = (f + 3) & ~3;
    plan_mac(L);        // also sets Mp
    make_fft_plan(d.Nx, &L->fftx);
    make_fft_plan(d.Ny, &L->ffty);
    make_fft_plan(d.Nz, &L->fftz);

    const size_t c = sizeof(float2);
    const size_t zc = d.zc, nimg = L->nimg, nimgo = L->nimgo;
    const size_t sz_A1 = zc * d.ky * d.kx * L->fp * L->Mp * c;
    // + room for the operand requests the multiply-accumulate issues one group of steps past the end
    const size_t sz_A = zc * d.Ny * d.kx * L->fp * L->Mp * c + (size_t)(L->fp + 64) * L->Mp * c;
    size_t b0 = nimg * d.nx * zc * d.ny;                             // X1
    size_t t = zc * d.Ny * nimg * d.Nx; if (t > b0) b0 = t;          // Xt
    t = nimgo * zc * d.nox * d.Ny; if (t > b0) b0 = t;               // Y2
    size_t b1 = nimg * zc * d.Ny * d.nx;                             // X2
    t = zc * d.Ny * nimgo * d.Nx; if (t > b1) b1 = t;                // Yt
    t = nimgo * d.nox * d.noy * d.ldz; if (t > b1) b1 = t;           // Y1
    size_t off = 0;
    char* p = (char*)base;
    L->twx = (float2*)(p + off); off += align_up((size_t)d.Nx * c, 256);
    L->twy = (float2*)(p + off); off += align_up((size_t)d.Ny * c, 256);
    L->twz = (float2*)(p + off); off += align_up((size_t)d.Nz * c, 256);
    L->A1 = (float2*)(p + off); off += align_up(sz_A1, 256);
    L->A = (float2*)(p + off); off += align_up(sz_A, 256);
    L->buf0 = (float2*)(p + off); off += align_up(b0 * c, 256);
    L->buf1 = (float2*)(p + off); off += align_up(b1 * c, 256);
    L->bytes = off;
    return ZNNI_OK;
}

static znni_status validate(int S, int f, int fo, const int n[3], const int k[3], const float* in,
                            const float* w, float* out, unsigned flags, void* workspace,
                            size_t workspace_bytes, LayerPlan* L)
{
    if (!in || !w || !out || !workspace) return ZNNI_ERR_NULL;
    if (flags & ~(unsigned)(ZNNI_RELU | ZNNI_MAC_REFERENCE)) return ZNNI_ERR_FLAGS;
    znni_status rc = make_plan(S, f, fo, n, k, workspace, L);
    if (rc) return rc;
    if (((uintptr_t)in | (uintptr_t)w | (uintptr_t)out) & 15u) return ZNNI_ERR_ALIGN;
    if ((uintptr_t)workspace & 255u) return ZNNI_ERR_ALIGN;
    if (workspace_bytes < L->bytes) return ZNNI_ERR_WORKSPACE;
    return ZNNI_OK;
}

// Runs the stages in order; if ev != NULL records ev[s] before stage s and ev[ZNNI_NUM_STAGES] at the end.
static znni_status run(const LayerPlan& L, const float* in, const float* w, const float* bias, float* out,
                       unsigned flags, hipStream_t st, hipEvent_t* ev)
{
    znni_status rc;
#define ZNNI_MARK(s)                                                          \
    do {                                                                      \
        if (ev && hipEventRecord(ev[s], st) != hipSuccess) return ZNNI_ERR_HIP; \
    } while (0)
#define ZNNI_DO(call)          \
    do {                       \
        rc = (call);           \
        if (rc) return rc;     \
    } while (0)
    ZNNI_DO(launch_twiddles(L, st));
    ZNNI_MARK(ZNNI_STAGE_KERNEL_PREP);
    ZNNI_DO(launch_kernel_prep(L, w, st));
    ZNNI_MARK(ZNNI_STAGE_FWD_Z);
    ZNNI_DO(launch_fwd_z(L, in, st));
    ZNNI_MARK(ZNNI_STAGE_FWD_Y);
    ZNNI_DO(launch_fwd_y(L, st));
    ZNNI_MARK(ZNNI_STAGE_FWD_X);
    ZNNI_DO(launch_fwd_x(L, st));
    ZNNI_MARK(ZNNI_STAGE_MAC);
    ZNNI_DO(launch_mac(L, flags, st));
    ZNNI_MARK(ZNNI_STAGE_INV_X);
    ZNNI_DO(launch_inv_x(L, st));
    ZNNI_MARK(ZNNI_STAGE_INV_Y);
    ZNNI_DO(launch_inv_y(L, st));
    ZNNI_MARK(ZNNI_STAGE_INV_Z);
    ZNNI_DO(launch_inv_z(L, bias, out, flags, st));
    ZNNI_MARK(ZNNI_NUM_STAGES);
#undef ZNNI_MARK
#undef ZNNI_DO
    return ZNNI_OK;
}

__global__ void k_copy_probe(float4* __restrict__ dst, const float4* __restrict__ src, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace znni

using namespace znni;

extern "C" {

int znni_version(void) { return 200; }

const char* znni_status_string(znni_status st)
{
    switch (st) {
        case ZNNI_OK: return "ok";
        case ZNNI_ERR_NULL: return "a required pointer is NULL";
        case ZNNI_ERR_SHAPE: return "bad layer shape (need S,f,f' >= 1 and 1 <= k <= n on every axis, counts within launch limits)";
        case ZNNI_ERR_UNSUPPORTED_SIZE: return "no supported transform size for this image edge";
        case ZNNI_ERR_WORKSPACE: return "workspace too small";
        case ZNNI_ERR_FLAGS: return "unknown flag bit";
        case ZNNI_ERR_HIP: return "HIP call or kernel launch failed";
        case ZNNI_ERR_ALIGN: return "device pointer not sufficiently aligned";
    }
    return "unknown status";
}

int znni_fft_size(int n) { return fft_size(n); }

znni_status znni_conv3d_fft_workspace_v(int S, int f, int fo, const int n[3], const int k[3], size_t* bytes)
{
    if (!bytes) return ZNNI_ERR_NULL;
    LayerPlan L;
    znni_status rc = make_plan(S, f, fo, n, k, nullptr, &L);
    if (rc) return rc;
    *bytes = L.bytes;
    return ZNNI_OK;
}

znni_status znni_conv3d_fft_v(int S, int f, int fo, const int n[3], const int k[3], const float* in,
                              const float* w, const float* bias, float* out, unsigned flags, void* workspace,
                              size_t workspace_bytes, void* stream)
{
    LayerPlan L;
    znni_status rc = validate(S, f, fo, n, k, in, w, out, flags, workspace, workspace_bytes, &L);
    if (rc) return rc;
    return run(L, in, w, bias, out, flags, (hipStream_t)stream, nullptr);
}

znni_status znni_conv3d_fft_profile_v(int S, int f, int fo, const int n[3], const int k[3], const float* in,
                                      const float* w, const float* bias, float* out, unsigned flags,
                                      void* workspace, size_t workspace_bytes, void* stream, float* stage_ms)
{
    if (!stage_ms) return ZNNI_ERR_NULL;
    LayerPlan L;
    znni_status rc = validate(S, f, fo, n, k, in, w, out, flags, workspace, workspace_bytes, &L);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    hipEvent_t ev[ZNNI_NUM_STAGES + 1];
    int made = 0;
    for (; made <= ZNNI_NUM_STAGES; ++made)
        if (hipEventCreate(&ev[made]) != hipSuccess) break;
    if (made <= ZNNI_NUM_STAGES) rc = ZNNI_ERR_HIP;
    if (!rc) rc = run(L, in, w, bias, out, flags, st, ev);
    if (!rc && hipStreamSynchronize(st) != hipSuccess) rc = ZNNI_ERR_HIP;
    if (!rc)
        for (int s = 0; s < ZNNI_NUM_STAGES; ++s)
            if (hipEventElapsedTime(&stage_ms[s], ev[s], ev[s + 1]) != hipSuccess) rc = ZNNI_ERR_HIP;
    for (int e = 0; e < made; ++e) (void)hipEventDestroy(ev[e]);
    return rc;
}

znni_status znni_conv3d_fft_workspace(int S, int f, int fo, int n, int k, size_t* bytes)
{
    const int nn[3] = {n, n, n}, kk[3] = {k, k, k};
    return znni_conv3d_fft_workspace_v(S, f, fo, nn, kk, bytes);
}

znni_status znni_conv3d_fft(int S, int f, int fo, int n, int k, const float* in, const float* w,
                            const float* bias, float* out, unsigned flags, void* workspace,
                            size_t workspace_bytes, void* stream)
{
    const int nn[3] = {n, n, n}, kk[3] = {k, k, k};
    return znni_conv3d_fft_v(S, f, fo, nn, kk, in, w, bias, out, flags, workspace, workspace_bytes, stream);
}

znni_status znni_conv3d_fft_profile(int S, int f, int fo, int n, int k, const float* in, const float* w,
                                    const float* bias, float* out, unsigned flags, void* workspace,
                                    size_t workspace_bytes, void* stream, float* stage_ms)
{
    const int nn[3] = {n, n, n}, kk[3] = {k, k, k};
    return znni_conv3d_fft_profile_v(S, f, fo, nn, kk, in, w, bias, out, flags, workspace, workspace_bytes,
                                     stream, stage_ms);
}

znni_status znni_copy_probe(void* dst, const void* src, size_t bytes, void* stream)
{
    if (!dst || !src) return ZNNI_ERR_NULL;
    if (bytes == 0 || (bytes & 15u)) return ZNNI_ERR_SHAPE;
    if (((uintptr_t)dst | (uintptr_t)src) & 15u) return ZNNI_ERR_ALIGN;
    const size_t n16 = bytes / 16;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;
    k_copy_probe<<<dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream>>>((float4*)dst, (const float4*)src, n16);
    if (hipGetLastError() != hipSuccess) return ZNNI_ERR_HIP;
    return ZNNI_OK;
}

}  // extern "C"
