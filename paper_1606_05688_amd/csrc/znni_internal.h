// znni_internal.h -- host-side plan of one layer call and the launchers of its stages (library-internal).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

#include "../../include/znni.h"
#include "fft_core.h"

namespace znni {

// Sizes of one layer, per axis (Section IV: image size <nx,ny,nz>, kernel size <kx,ky,kz>, output size
// n' = n - k + 1 per axis).  x is the slowest axis of the tensors, z the contiguous one.  Passed to kernels by value.
struct Dims {
    int nx, ny, nz;       // image
    int kx, ky, kz;       // kernel
    int Nx, Ny, Nz;       // transform sizes n~ >= n
    int zc;               // Nz/2 + 1 bins along the halved axis
    int nox, noy, noz;    // output n - k + 1
    int ldy, ldx, ldo;    // row strides of X1, X2 and Y1: ny, nx and noy rounded up to a multiple of 16 complex
    int ldn;              // row stride of Y2: Ny, rounded up likewise where Ny is not a multiple of 8
                          // (128 bytes)
    int ldxo;             // row stride of Yd (layers whose x axis is not transformed): nox rounded up likewise
    int x2i, x2o;         // row (img, oz, oy) of X2 is row number img*x2i + oz*x2o + oy
    int ydi, ydo;         // row (imgo, oz, oy) of Yd is row number imgo*ydi + oz*ydo + oy
};

// Everything one call needs: sizes, the radix schedules, and where each buffer lives in the workspace.
// Buffers buf0/buf1 are reused in turn by the stages (X1 -> X2 -> Xt, then Yt -> Y2 -> Y1), the way the
// paper reuses its transform scratch (Section III-D, last paragraphs).
struct LayerPlan {
    int S, f, fo;
    Dims d;
    // The x axis is not transformed (mac_xd.hip): in -> X1 -> X2, multiply-accumulate with the kx taps as shifted
    // reads of X2 -> Yd[imgo][oz][oy][xo] (in Yt), inverse y pass reading Yd transposed -> Y1 -> out.
    bool xdirect;
    // ... and the kx taps are applied through length-8 transforms of overlapping blocks of X2 rows (mac_xb.hip)
    // instead of shifted reads; A then holds the length-8 transforms of the taps.  Implies xdirect.
    bool xblock;
    // Diagnostic (ZNNI_PASSES_REFERENCE): every transform pass by the generic kernels of passes.hip, no fused z+y
    // kernels, x axis transformed at full length.
    bool generic_passes;
    int nimg;     // S * f
    int nimgo;    // S * fo
    int fp;       // f rounded up to a multiple of 4   (matrix-core k-step)
    int Mp;       // fo rounded up to whole row blocks of the matrix-core kernel (a multiple of 16)
    // tiling of the matrix-core multiply-accumulate (see mac.hip): the S*Nx columns of a pencil are cut into
    // mac_n2 blocks of 128 columns followed by mac_n1 blocks of 64
    int mac_RTW, mac_FC, mac_nmblk, mac_n2, mac_n1;
    FftPlan fftx, ffty, fftz;
    // workspace carving (device pointers)
    float2* twx;  // [Nx] exp(-2 pi i q / Nx)
    float2* twy;  // [Ny]
    float2* twz;  // [Nz]
    float2* A1;   // [zc][ky(b)][kx(a)][fp][Mp]      kernel transform after the z stage
    float2* A;    // [zc][Ny][fp/4][kx][4][Mp]       after the z and y stages, scaled by 1/(Nx Ny Nz)
    float2* buf0;
    float2* buf1;
    float2* Yt;   // accumulated output spectra: buf1 itself for a whole-layer call (buf0 where the x axis is not
                  // transformed: the multiply-accumulate then reads X2 from buf1); a buffer of its own when the
                  // layer runs as sub-layers, because it must then survive the forward passes of later input chunks
    size_t sz[5]; // bytes of A1, A, buf0, buf1 and of a separate Yt
    size_t bytes; // total workspace bytes
};

// Host-only: validate the shape and fill every field; pointers are offsets from `base` (may be NULL when
// only the size is wanted).
// flags: the call's flags (only the bits that pick a multiply-accumulate form matter: they decide `xdirect`).
znni_status make_plan(int S, int f, int fo, const int n[3], const int k[3], unsigned flags, void* base,
                      LayerPlan* out);

int lines_per_tile(int N);

znni_status launch_twiddles(const LayerPlan& L, hipStream_t st);
// w points at kernel (j0, i0) of the bank; wj_stride = floats between the kernels of consecutive output images
// (f_total * kx*ky*kz), so a sub-bank of a larger bank can be transformed in place.
znni_status launch_kernel_prep(const LayerPlan& L, const float* w, size_t wj_stride, hipStream_t st);
znni_status launch_fwd_z(const LayerPlan& L, const float* in, hipStream_t st);
znni_status launch_fwd_y(const LayerPlan& L, hipStream_t st);
znni_status launch_fwd_x(const LayerPlan& L, hipStream_t st);
void plan_mac(LayerPlan* L);
// accumulate != 0: add to the spectra already in L.Yt instead of overwriting them (later chunks of input images).
znni_status launch_mac(const LayerPlan& L, unsigned flags, int accumulate, hipStream_t st);
znni_status launch_inv_x(const LayerPlan& L, hipStream_t st);
znni_status launch_inv_y(const LayerPlan& L, hipStream_t st);
// Inverse y pass for layers whose x axis is not transformed: reads Yd[imgo][oz][oy][xo] from L.Yt with a
// transposing load, writes Y1 to buf1.  Exists for the in-register transform lengths only.
znni_status launch_fast_inv_yt(const LayerPlan& L, hipStream_t st);
znni_status launch_inv_z(const LayerPlan& L, const float* bias, float* out, unsigned flags, hipStream_t st);

// Forward z and y transforms in one kernel when a (oz, oy) plane fits LDS (passes_fused.hip): in -> X2' in buf1,
// laid out [img][x][oz][oy]; launch_fast_fwd_xt is the x pass that reads it (buf1 -> Xt in buf0).
bool fused_fwd_zy_available(const LayerPlan& L);
znni_status launch_fwd_zy(const LayerPlan& L, const float* in, hipStream_t st);
znni_status launch_fast_fwd_xt(const LayerPlan& L, hipStream_t st);

// Inverse y and z transforms in one kernel when a (oz, oy) plane fits LDS (passes_fused.hip); reads Y2 from buf0.
bool fused_inv_yz_available(const LayerPlan& L);
znni_status launch_inv_yz(const LayerPlan& L, const float* bias, float* out, unsigned flags, hipStream_t st);

// Two-step in-register passes for selected transform lengths (passes_fast.hip).
bool fast_pass_available(int N);
znni_status launch_fast_fwd_z(const LayerPlan& L, const float* in, hipStream_t st);
znni_status launch_fast_fwd_y(const LayerPlan& L, hipStream_t st);
znni_status launch_fast_fwd_x(const LayerPlan& L, hipStream_t st);
znni_status launch_fast_inv_x(const LayerPlan& L, hipStream_t st);
znni_status launch_fast_inv_y(const LayerPlan& L, hipStream_t st);
znni_status launch_fast_inv_z(const LayerPlan& L, const float* bias, float* out, unsigned flags, hipStream_t st);

}  // namespace znni
