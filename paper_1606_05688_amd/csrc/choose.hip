// choose.hip -- which primitive to run a convolutional layer with (host only), and the call that does so.
//
// Section VII: every layer can be computed by several primitives and the fastest one is picked per layer; the
// paper measures each candidate (Table IV lists the winners) and prunes the search with a kernel-size rule.
// Here the pick comes from a two-term cost model per primitive, with rates measured on one MI355X:
//
//   transform route:  bytes moved by the six transform passes and the kernel preparation over the HBM rate those
//                     kernels reach (lower for transform lengths served by the generic pass kernel), plus the
//                     multiply-accumulate's matrix-core work, plus a fixed cost for its dozen launches;
//   direct route:     its matrix-core work over the rate the kernel reaches (lower for windows of fewer than 27
//                     taps, where staging the image tiles weighs more per product) plus the output write, plus
//                     two launches.
//
// The model only has to rank the two; it is not used for anything else.
#include "znni_internal.h"

namespace znni {

// measured rates (MI355X)
constexpr double kPassBytesPerSecFast = 5.3e12;     // in-register pass kernels
constexpr double kPassBytesPerSecGeneric = 2.0e12;  // generic LDS pass kernels
constexpr double kPrepBytesPerSec = 4.5e12;         // kernel preparation (write-bound)
constexpr double kMacFlopsPerSec = 110e12;          // issued matrix-core flops of the multiply-accumulate (S = 1 form)
constexpr double kMacBatchSecPerValue = 2.1e-12;    // batch form: per kernel-spectrum value and 16 inputs
constexpr double kDirectFlopsPerSec = 80e12;        // direct convolution, windows of 27 taps and more
constexpr double kDirectFlopsPerSecSmall = 60e12;   // ... of fewer taps
constexpr double kDirectWriteBytesPerSec = 3.6e12;  // direct convolution, output write
constexpr double kLaunchSec = 3.5e-6;

static double fft_seconds(int S, int f, int fo, const int n[3], const int k[3])
{
    const double Nx = znni_fft_size(n[0]), Ny = znni_fft_size(n[1]), Nz = znni_fft_size(n[2]);
    const double zc = (int)Nz / 2 + 1;
    const double nox = n[0] - k[0] + 1, noy = n[1] - k[1] + 1, noz = n[2] - k[2] + 1;
    const double c = 8.0;
    struct { double bytes; int N; } pass[6] = {
        {(double)S * f * (4.0 * n[0] * n[1] * n[2] + c * n[0] * n[1] * zc), (int)Nz},
        {(double)S * f * (c * n[0] * n[1] * zc + c * n[0] * Ny * zc), (int)Ny},
        {(double)S * f * (c * n[0] * Ny * zc + c * Nx * Ny * zc), (int)Nx},
        {(double)S * fo * (c * Nx * Ny * zc + c * nox * Ny * zc), (int)Nx},
        {(double)S * fo * (c * nox * Ny * zc + c * nox * noy * zc), (int)Ny},
        {(double)S * fo * (c * nox * noy * zc + 4.0 * nox * noy * noz), (int)Nz},
    };
    double t = 12 * kLaunchSec;
    for (auto& p : pass) t += p.bytes / (fast_pass_available(p.N) ? kPassBytesPerSecFast : kPassBytesPerSecGeneric);
    const double fp = (f + 3) / 4 * 4, Mp = (fo + 15) / 16 * 16;
    t += c * zc * Ny * k[0] * fp * Mp / kPrepBytesPerSec;
    // S = 1 form: three real matrix products per complex one, contraction over (input image, x tap), every
    // column; batch form (taken from k*S = 32 on): cost per kernel-spectrum value, once per 16 inputs
    if (k[0] * S >= 32 && k[0] <= 12)
        t += kMacBatchSecPerValue * fp * Mp * Nx * Ny * zc * ((S + 15) / 16);
    else
        t += 6.0 * k[0] * fp * Mp * (double)S * Nx * Ny * zc / kMacFlopsPerSec;
    return t;
}

static double direct_seconds(int S, int f, int fo, const int n[3], const int k[3])
{
    const double ovox = (double)(n[0] - k[0] + 1) * (n[1] - k[1] + 1) * (n[2] - k[2] + 1);
    const double taps4 = (k[0] * k[1] * k[2] + 3) / 4 * 4, Mp = (fo + 15) / 16 * 16;
    const double flops = 2.0 * S * f * taps4 * Mp * ovox;
    const double wr = 4.0 * S * fo * ovox;
    const double rate = k[0] * k[1] * k[2] >= 27 ? kDirectFlopsPerSec : kDirectFlopsPerSecSmall;
    return flops / rate + wr / kDirectWriteBytesPerSec + 2 * kLaunchSec;
}

}  // namespace znni

using namespace znni;

extern "C" {

znni_status znni_conv3d_choose_v(int S, int f, int fo, const int n[3], const int k[3], int* primitive,
                                 float est_ms[2])
{
    if (!primitive) return ZNNI_ERR_NULL;
    size_t bf = 0, bd = 0;
    const znni_status rf = znni_conv3d_fft_workspace_v(S, f, fo, n, k, &bf);
    const znni_status rd = znni_conv3d_direct_workspace_v(S, f, fo, n, k, &bd);
    if (rf != ZNNI_OK && rd != ZNNI_OK) return rf;          // bad shape, or neither primitive takes it
    const double tf = rf == ZNNI_OK ? fft_seconds(S, f, fo, n, k) : -1.0;
    const double td = rd == ZNNI_OK ? direct_seconds(S, f, fo, n, k) : -1.0;
    if (est_ms) { est_ms[ZNNI_PRIMITIVE_FFT] = (float)(tf * 1e3); est_ms[ZNNI_PRIMITIVE_DIRECT] = (float)(td * 1e3); }
    if (tf < 0) *primitive = ZNNI_PRIMITIVE_DIRECT;
    else if (td < 0) *primitive = ZNNI_PRIMITIVE_FFT;
    else *primitive = td < tf ? ZNNI_PRIMITIVE_DIRECT : ZNNI_PRIMITIVE_FFT;
    return ZNNI_OK;
}

znni_status znni_conv3d_workspace_v(int S, int f, int fo, const int n[3], const int k[3], size_t* bytes)
{
    if (!bytes) return ZNNI_ERR_NULL;
    int prim = 0;
    znni_status rc = znni_conv3d_choose_v(S, f, fo, n, k, &prim, nullptr);
    if (rc) return rc;
    return prim == ZNNI_PRIMITIVE_DIRECT ? znni_conv3d_direct_workspace_v(S, f, fo, n, k, bytes)
                                         : znni_conv3d_fft_workspace_v(S, f, fo, n, k, bytes);
}

znni_status znni_conv3d_v(int S, int f, int fo, const int n[3], const int k[3], const float* in, const float* w,
                          const float* bias, float* out, unsigned flags, void* workspace, size_t workspace_bytes,
                          void* stream)
{
    int prim = 0;
    znni_status rc = znni_conv3d_choose_v(S, f, fo, n, k, &prim, nullptr);
    if (rc) return rc;
    if (prim == ZNNI_PRIMITIVE_DIRECT) {
        if (flags & ZNNI_MAC_REFERENCE) return ZNNI_ERR_FLAGS;
        // the transform route's stricter alignment is asked of both, so a call does not depend on the pick
        if (in && w && out && (((uintptr_t)in | (uintptr_t)w | (uintptr_t)out) & 15u)) return ZNNI_ERR_ALIGN;
        // the hints that pick a multiply-accumulate form mean nothing to the direct route: validated, then dropped
        // (at most one, as on the transform route); the direct route stores no kernel transforms a later call
        // could reuse, so ZNNI_KEEP_KERNELS is dropped as well: the bank is rearranged again, which is always right; it
        // has no transform passes either
        const unsigned forms = flags & (unsigned)(ZNNI_MAC_SINGLE | ZNNI_MAC_BATCH | ZNNI_MAC_XDIRECT | ZNNI_MAC_XBLOCK);
        if (forms & (forms - 1)) return ZNNI_ERR_FLAGS;
        return znni_conv3d_direct_v(S, f, fo, n, k, in, w, bias, out,
                                    flags & ~(forms | (unsigned)(ZNNI_KEEP_KERNELS | ZNNI_PASSES_REFERENCE)), workspace,
                                    workspace_bytes, stream);
    }
    return znni_conv3d_fft_v(S, f, fo, n, k, in, w, bias, out, flags, workspace, workspace_bytes, stream);
}

}  // extern "C"
