// api.hip -- the exported C ABI: argument validation, workspace planning, and the stage sequence of the
// GPU algorithm of Section IV-B-2 (Algorithm 3): transform the images, multiply-accumulate per bin with the
// kernel transforms, inverse-transform the output images.  All validation happens before the first HIP call.
#include <stdint.h>

#include <mutex>

#include "mac_common.h"
#include "znni_internal.h"

// Scratch memory of znni_conv3d_fft_static_v, the entry point for callers that cannot allocate: one array per GPU,
// placed by the loader when the library's code is loaded on that GPU and held until the process ends.  In host
// code this name is only a handle for hipGetSymbolAddress; kernels are given the address that call returns.
static __device__ __align__(256) unsigned char scratch[ZNNI_STATIC_SCRATCH_BYTES];

namespace znni {

// Transform size for an image edge n: the smallest length >= n that the in-register pass kernels serve (46
// members of the 2^a 3^b 5^c 7^d family from 8 to 1024, never more than 20 % above n); below 7 the edge itself (all
// of 1..6 are members), transformed by the generic pass kernels.  A layer's cost grows in proportion to the length,
// and the generic kernels run at well under half the speed per element, so a nearer generic length never pays.
static int fft_size(int n)
{
    if (n < 1) return 0;
    if (n < 7) return n;
    for (int m = n; m <= ZNNI_MAX_FFT; ++m)
        if (fast_pass_available(m)) return m;
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

// Whether a layer runs without transforming its x axis (mac_xd.hip).  A flag that names a multiply-accumulate form
// decides; otherwise that route is taken where each kernel-spectrum value would serve too few inputs to be worth
// generating (the same rule that picks between the two forms of the fully transformed route), provided the y
// transform has an in-register kernel (only those read the transposed layout).  Measured on 48 -> 48 images of
// 320^3 with 5^3 kernels: 20.9 ms against 25.0 ms; 40 -> 40 images of 128^3, 3^3 kernels: 0.98 against 1.10 ms.
static bool pick_untransformed_x(const LayerPlan& L, unsigned flags)
{
    if (flags & (ZNNI_MAC_REFERENCE | ZNNI_MAC_SINGLE | ZNNI_MAC_BATCH)) return false;
    // small images, where one kernel per side does the z and y transforms: the two routes were measured within
    // a few per cent of each other (lengths 64 and 100), the fully transformed one ahead
    if (fused_fwd_zy_available(L) && fused_inv_yz_available(L)) return false;
    return !mac_batch_preferred(L);
}

// ... and whether it applies the kernel's taps along x through length-8 transforms of overlapping blocks
// (mac_xb.hip) rather than as shifted reads: wherever that form exists (4 or 5 taps).  Measured, whole layer:
// 48 -> 48 images of 320^3, 5^3 kernels 18.6 against 20.9 ms; 48 -> 48 of 240^3, 4^3: 7.8 against 8.2 ms;
// 2 x 32 -> 32 of 128^3, 5^3: 1.49 against 1.55 ms; 80 -> 80 of 200^3, 5^3 (row blocks of three and two tiles):
// 12.0 against 14.4 ms, with 4^3 kernels 11.2 against 12.4 ms.
static bool pick_xblock(const LayerPlan& L, unsigned flags)
{
    if (L.generic_passes || !mac_xb_available(L) || !fast_pass_available(L.d.Ny)) return false;
    if (flags & ZNNI_MAC_XBLOCK) return true;
    if (flags & ZNNI_MAC_XDIRECT) return false;
    if (pick_untransformed_x(L, flags)) return true;
    // small images (one kernel per side for the z and y transforms of the fully transformed route): ahead only with
    // five taps and at least 24 blocks along x.  Measured, blocks against full length: 80 -> 80 images of 100^3, 5^3
    // kernels 1.81 against 2.08 ms; 4 x 48 -> 48 of 100^3 2.57 against 2.91; 48 -> 48 of 120^3 1.31 against 1.39;
    // but 80 -> 80 of 120^3 with 4^3 kernels 2.75 against 2.69, 80 -> 80 of 60^3 with 5^3 0.67 against 0.52.
    if (flags & (ZNNI_MAC_REFERENCE | ZNNI_MAC_SINGLE | ZNNI_MAC_BATCH)) return false;
    return L.d.kx == 5 && L.d.nox >= 96 && !mac_batch_preferred(L);
}

static bool pick_xdirect(const LayerPlan& L, unsigned flags)
{
    if (L.xblock) return true;
    if (L.generic_passes || !mac_xd_available(L) || !fast_pass_available(L.d.Ny)) return false;
    if (flags & ZNNI_MAC_XDIRECT) return true;
    if (flags & ZNNI_MAC_XBLOCK) return false;
    return pick_untransformed_x(L, flags);
}

// Shape part of a plan: validates, fills every size and the array sizes sz[]; assigns no pointers.
static znni_status shape_plan(int S, int f, int fo, const int n[3], const int k[3], unsigned flags, LayerPlan* L)
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
    d.ldy = (d.ny + 15) & ~15;       // X1, X2 and Y1 rows start on 128-byte boundaries
    d.ldx = (d.nx + 15) & ~15;
    d.ldo = (d.noy + 15) & ~15;
    // Y2 rows: padded to 128-byte boundaries only where they would not even start on 64-byte ones (lengths
    // like 100: the inverse x pass, which stores 128-byte runs into them, is then 20 % faster); where rows are
    // 64-byte aligned anyway the extra bytes cost more than the alignment gains (measured at 40 and 72)
    d.ldn = (d.Ny % 8 == 0) ? d.Ny : ((d.Ny + 15) & ~15);
    d.ldxo = (d.nox + 15) & ~15;
    L->nimg = S * f;
    L->nimgo = S * fo;
    L->fp = (f + 3) & ~3;
    plan_mac(L);        // also sets Mp
    L->generic_passes = (flags & ZNNI_PASSES_REFERENCE) != 0;
    L->xblock = pick_xblock(*L, flags);
    L->xdirect = pick_xdirect(*L, flags);
    // X2 and Yd are ordered [image][oz][oy]; the order [oz][image][oy] was measured too: 2 % faster for the
    // multiply-accumulate that reads X2 and writes Yd, 6 % slower for the y passes on the other side of them
    d.x2i = d.zc * d.Ny; d.x2o = d.Ny;
    d.ydi = d.zc * d.Ny; d.ydo = d.Ny;
    make_fft_plan(d.Nx, &L->fftx);
    make_fft_plan(d.Ny, &L->ffty);
    make_fft_plan(d.Nz, &L->fftz);

    const size_t c = sizeof(float2);
    const size_t zc = d.zc, nimg = L->nimg, nimgo = L->nimgo;
    L->sz[0] = zc * d.ky * d.kx * L->fp * L->Mp * c;                                    // A1
    // A + room for the operand requests the multiply-accumulate issues one group of steps past the end
    L->sz[1] = zc * d.Ny * d.kx * L->fp * L->Mp * c + (size_t)(L->fp + 64) * L->Mp * c;
    if (mac_xb_available(*L) && mac_xb_kernel_bytes(*L) > L->sz[1]) L->sz[1] = mac_xb_kernel_bytes(*L);
    // Sized for either route (x axis transformed or not), so that the workspace a shape needs does not depend on
    // the flags of the call.
    size_t b0 = nimg * d.nx * zc * d.ldy;                            // X1
    size_t t = zc * d.Ny * nimg * d.Nx; if (t > b0) b0 = t;          // Xt
    t = nimgo * zc * d.nox * d.ldn; if (t > b0) b0 = t;              // Y2
    const size_t yd = nimgo * zc * d.Ny * d.ldxo;                    // Yd
    if (yd > b0) b0 = yd;
    size_t b1 = nimg * zc * d.Ny * d.ldx;                            // X2
    t = nimgo * d.nox * zc * d.ldo; if (t > b1) b1 = t;              // Y1
    L->sz[2] = b0 * c;
    L->sz[3] = b1 * c;
    t = zc * d.Ny * nimgo * d.Nx;                                    // Yt
    L->sz[4] = (t > yd ? t : yd) * c;
    return ZNNI_OK;
}

// Pointer part: carve the workspace at `base` into arrays of the given byte sizes.  own_yt = false: the output
// spectra share buf1 (a whole-layer call never needs X2 or Y1 while Yt is alive), or buf0 where the x axis is not
// transformed (X1 is dead by then and X2, in buf1, is being read).
static void place_plan(LayerPlan* L, void* base, const size_t sz[5], bool own_yt)
{
    const Dims& d = L->d;
    const size_t c = sizeof(float2);
    size_t off = 0;
    // addresses as integers: a size query carves from a null base
    const uintptr_t p = (uintptr_t)base;
    L->twx = (float2*)(p + off); off += align_up((size_t)d.Nx * c, 256);
    L->twy = (float2*)(p + off); off += align_up((size_t)d.Ny * c, 256);
    L->twz = (float2*)(p + off); off += align_up((size_t)d.Nz * c, 256);
    L->A1 = (float2*)(p + off); off += align_up(sz[0], 256);
    L->A = (float2*)(p + off); off += align_up(sz[1], 256);
    L->buf0 = (float2*)(p + off); off += align_up(sz[2], 256);
    // (sz[2] already covers Yd, so nothing is added for the layers whose x axis is not transformed)
    const size_t b1 = own_yt ? sz[3] : (sz[3] > sz[4] ? sz[3] : sz[4]);
    L->buf1 = (float2*)(p + off); off += align_up(b1, 256);
    if (own_yt) { L->Yt = (float2*)(p + off); off += align_up(sz[4], 256); }
    else L->Yt = L->xdirect ? L->buf0 : L->buf1;
    L->bytes = off;
}

znni_status make_plan(int S, int f, int fo, const int n[3], const int k[3], unsigned flags, void* base,
                      LayerPlan* L)
{
    znni_status rc = shape_plan(S, f, fo, n, k, flags, L);
    if (rc) return rc;
    place_plan(L, base, L->sz, false);
    return ZNNI_OK;
}

// ------------------------------------------------------------------------------------------- sub-layers
// Section VII-A: a layer of shape (S, f, f') can be computed as sub-layers of shapes (S_i, f_i, f'_i), each small
// enough for the memory at hand.  Here the memory at hand is the caller's workspace.  The division follows the
// paper's preference: whole-layer if it fits; else sub-batches (f_i = f, f'_i = f', S_i < S), which transform
// every input and output once; else S_i = 1 with blocks of f_a input and f'_a output images.  In the last case
// the sub-layers of one output block accumulate their products in the output spectra (kept in a buffer of their
// own), so each output block is inverse-transformed once, and the input transforms are repeated once per output
// block.
struct Division {
    int Si, fi, foi;
    bool own_yt;
    size_t sz[5];
    size_t bytes;
};

// Workspace of a division: arrays sized for its largest sub-layer (the ragged last chunks are smaller).
static znni_status division_bytes(int S, int f, int fo, const int n[3], const int k[3], Division* D)
{
    D->own_yt = D->fi < f;
    for (int q = 0; q < 5; ++q) D->sz[q] = 0;
    // distinct sub-layer shapes: full or ragged in each of S, f, f'
    const int Ss[2] = {D->Si, S % D->Si}, fs[2] = {D->fi, f % D->fi}, fos[2] = {D->foi, fo % D->foi};
    LayerPlan L;
    for (int a = 0; a < 2; ++a)
        for (int b = 0; b < 2; ++b)
            for (int c = 0; c < 2; ++c) {
                if (Ss[a] == 0 || fs[b] == 0 || fos[c] == 0) continue;
                znni_status rc = shape_plan(Ss[a], fs[b], fos[c], n, k, 0, &L);
                if (rc) return rc;
                for (int q = 0; q < 5; ++q)
                    if (L.sz[q] > D->sz[q]) D->sz[q] = L.sz[q];
            }
    place_plan(&L, nullptr, D->sz, D->own_yt);
    D->bytes = L.bytes;
    return ZNNI_OK;
}

// Rough HBM traffic of a division in units of one transformed image (what the choice between blockings is
// based on): three forward passes per input image and output block, one read-modify-write of the output spectra
// per input block, three inverse passes per output image.
static double division_cost(int f, int fo, int fi, int foi)
{
    const double nfo = (fo + foi - 1) / foi, nfi = (f + fi - 1) / fi;
    return 5.0 * f * nfo + 2.0 * fo * (nfi - 1) + 5.0 * fo;
}

static znni_status choose_division(int S, int f, int fo, const int n[3], const int k[3], size_t budget,
                                   Division* D)
{
    if (!n || !k) return ZNNI_ERR_NULL;
    if (S < 1 || f < 1 || fo < 1) return ZNNI_ERR_SHAPE;
    D->Si = S; D->fi = f; D->foi = fo;
    znni_status rc = division_bytes(S, f, fo, n, k, D);
    if (rc) return rc;
    if (D->bytes <= budget) return ZNNI_OK;
    // sub-batches: the largest S_i that fits
    if (S > 1) {
        int lo = 0, hi = S;             // lo fits (0 = none), hi does not
        while (hi - lo > 1) {
            const int mid = (lo + hi) / 2;
            D->Si = mid;
            rc = division_bytes(S, f, fo, n, k, D);
            if (rc) return rc;
            if (D->bytes <= budget) lo = mid; else hi = mid;
        }
        if (lo >= 1) {
            D->Si = lo;
            return division_bytes(S, f, fo, n, k, D);
        }
    }
    // blocks of input and output images, one input at a time: input blocks of f, then multiples of 4 (the
    // matrix-core contraction step), then 2 and 1; output blocks of f', then multiples of 16 (the matrix-core
    // tile), then 8, 4, 2, 1
    D->Si = 1;
    Division best;
    double best_cost = -1.0;
    auto next = [](int cur, int full, int step) {
        if (cur > step) return cur == full && full % step ? full / step * step : cur - step;
        return cur / 2;                 // step, step/2, ..., 1, 0
    };
    for (int foi = fo; foi >= 1; foi = next(foi, fo, 16)) {
        // the largest input block that fits with this output block
        int fit = 0;
        for (int fi = f; fi >= 1; fi = next(fi, f, 4)) {
            D->fi = fi; D->foi = foi;
            rc = division_bytes(S, f, fo, n, k, D);
            if (rc) return rc;
            if (D->bytes <= budget) { fit = fi; break; }
        }
        if (fit) {
            const double cost = division_cost(f, fo, fit, foi);
            if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = *D; }
        }
    }
    if (best_cost < 0) return ZNNI_ERR_WORKSPACE;
    *D = best;
    return ZNNI_OK;
}

// Known bits only, and at most one of the three bits that pick a multiply-accumulate form.
static bool flags_ok(unsigned flags)
{
    const unsigned all_forms = ZNNI_MAC_REFERENCE | ZNNI_MAC_SINGLE | ZNNI_MAC_BATCH | ZNNI_MAC_XDIRECT | ZNNI_MAC_XBLOCK;
    if (flags & ~(unsigned)(ZNNI_RELU | ZNNI_KEEP_KERNELS | ZNNI_PASSES_REFERENCE | all_forms)) return false;
    const unsigned forms = flags & all_forms;
    return (forms & (forms - 1)) == 0;
}

static znni_status validate(int S, int f, int fo, const int n[3], const int k[3], const float* in,
                            const float* w, float* out, unsigned flags, void* workspace,
                            size_t workspace_bytes, LayerPlan* L)
{
    if (!in || !w || !out || !workspace) return ZNNI_ERR_NULL;
    if (!flags_ok(flags)) return ZNNI_ERR_FLAGS;
    znni_status rc = make_plan(S, f, fo, n, k, flags, workspace, L);
    if (rc) return rc;
    if (((uintptr_t)in | (uintptr_t)w | (uintptr_t)out) & 15u) return ZNNI_ERR_ALIGN;
    if ((uintptr_t)workspace & 255u) return ZNNI_ERR_ALIGN;
    if (workspace_bytes < L->bytes) return ZNNI_ERR_WORKSPACE;
    return ZNNI_OK;
}

#define ZNNI_DO(call)          \
    do {                       \
        rc = (call);           \
        if (rc) return rc;     \
    } while (0)

// Runs the stages in order; if ev != NULL records ev[s] before stage s and ev[ZNNI_NUM_STAGES] at the end.
static znni_status run(const LayerPlan& L, const float* in, const float* w, const float* bias, float* out,
                       unsigned flags, hipStream_t st, hipEvent_t* ev)
{
    znni_status rc;
#define ZNNI_MARK(s)                                                          \
    do {                                                                      \
        if (ev && hipEventRecord(ev[s], st) != hipSuccess) return ZNNI_ERR_HIP; \
    } while (0)
    ZNNI_DO(launch_twiddles(L, st));
    ZNNI_MARK(ZNNI_STAGE_KERNEL_PREP);
    // the stored kernel transforms of an earlier call on this workspace may be kept (same w, shape and form)
    if (!(flags & ZNNI_KEEP_KERNELS)) ZNNI_DO(launch_kernel_prep(L, w, (size_t)L.f * L.d.kx * L.d.ky * L.d.kz, st));
    if (L.xdirect) {
        // x axis not transformed: the x stages do nothing and read about zero
        ZNNI_MARK(ZNNI_STAGE_FWD_Z);
        ZNNI_DO(launch_fwd_z(L, in, st));
        ZNNI_MARK(ZNNI_STAGE_FWD_Y);
        ZNNI_DO(launch_fwd_y(L, st));
        ZNNI_MARK(ZNNI_STAGE_FWD_X);
        ZNNI_MARK(ZNNI_STAGE_MAC);
        ZNNI_DO(L.xblock ? launch_mac_xb(L, 0, st) : launch_mac_xd(L, 0, st));
        ZNNI_MARK(ZNNI_STAGE_INV_X);
        ZNNI_MARK(ZNNI_STAGE_INV_Y);
        ZNNI_DO(launch_fast_inv_yt(L, st));
        ZNNI_MARK(ZNNI_STAGE_INV_Z);
        ZNNI_DO(launch_inv_z(L, bias, out, flags, st));
        ZNNI_MARK(ZNNI_NUM_STAGES);
        return ZNNI_OK;
    }
    const bool fused_zy = fused_fwd_zy_available(L);       // then the z stage's time covers z and y
    ZNNI_MARK(ZNNI_STAGE_FWD_Z);
    if (fused_zy) ZNNI_DO(launch_fwd_zy(L, in, st));
    else ZNNI_DO(launch_fwd_z(L, in, st));
    ZNNI_MARK(ZNNI_STAGE_FWD_Y);
    if (!fused_zy) ZNNI_DO(launch_fwd_y(L, st));
    ZNNI_MARK(ZNNI_STAGE_FWD_X);
    if (fused_zy) ZNNI_DO(launch_fast_fwd_xt(L, st));
    else ZNNI_DO(launch_fwd_x(L, st));
    ZNNI_MARK(ZNNI_STAGE_MAC);
    ZNNI_DO(launch_mac(L, flags, 0, st));
    ZNNI_MARK(ZNNI_STAGE_INV_X);
    ZNNI_DO(launch_inv_x(L, st));
    const bool fused_yz = fused_inv_yz_available(L);       // then the y stage's time covers both
    ZNNI_MARK(ZNNI_STAGE_INV_Y);
    if (fused_yz) ZNNI_DO(launch_inv_yz(L, bias, out, flags, st));
    else ZNNI_DO(launch_inv_y(L, st));
    ZNNI_MARK(ZNNI_STAGE_INV_Z);
    if (!fused_yz) ZNNI_DO(launch_inv_z(L, bias, out, flags, st));
    ZNNI_MARK(ZNNI_NUM_STAGES);
#undef ZNNI_MARK
    return ZNNI_OK;
}

// The layer as the sub-layers of division D, all on one workspace.
static znni_status run_divided(const Division& D, int S, int f, int fo, const int n[3], const int k[3],
                               const float* in, const float* w, const float* bias, float* out, unsigned flags,
                               void* workspace, hipStream_t st)
{
    znni_status rc;
    const size_t nvox = (size_t)n[0] * n[1] * n[2], kvol = (size_t)k[0] * k[1] * k[2];
    const size_t ovox = (size_t)(n[0] - k[0] + 1) * (n[1] - k[1] + 1) * (n[2] - k[2] + 1);
    for (int s0 = 0; s0 < S; s0 += D.Si) {
        const int Sc = S - s0 < D.Si ? S - s0 : D.Si;
        for (int j0 = 0; j0 < fo; j0 += D.foi) {
            const int foc = fo - j0 < D.foi ? fo - j0 : D.foi;
            LayerPlan L;
            for (int i0 = 0; i0 < f; i0 += D.fi) {
                const int fc = f - i0 < D.fi ? f - i0 : D.fi;
                // a block of images is one contiguous tensor only if it spans all images of a tuple or one tuple
                if (Sc > 1 && (fc != f || foc != fo)) return ZNNI_ERR_SHAPE;
                ZNNI_DO(shape_plan(Sc, fc, foc, n, k, flags, &L));
                for (int q = 0; q < 5; ++q)
                    if (L.sz[q] > D.sz[q]) return ZNNI_ERR_WORKSPACE;
                place_plan(&L, workspace, D.sz, D.own_yt);
                ZNNI_DO(launch_twiddles(L, st));      // also zeroes the padding behind this chunk's A
                ZNNI_DO(launch_kernel_prep(L, w + ((size_t)j0 * f + i0) * kvol, (size_t)f * kvol, st));
                const float* isub = in + ((size_t)s0 * f + i0) * nvox;
                if (L.xdirect) {
                    ZNNI_DO(launch_fwd_z(L, isub, st));
                    ZNNI_DO(launch_fwd_y(L, st));
                    ZNNI_DO(L.xblock ? launch_mac_xb(L, i0 > 0, st) : launch_mac_xd(L, i0 > 0, st));
                    continue;
                }
                if (fused_fwd_zy_available(L)) {
                    ZNNI_DO(launch_fwd_zy(L, isub, st));
                    ZNNI_DO(launch_fast_fwd_xt(L, st));
                } else {
                    ZNNI_DO(launch_fwd_z(L, isub, st));
                    ZNNI_DO(launch_fwd_y(L, st));
                    ZNNI_DO(launch_fwd_x(L, st));
                }
                ZNNI_DO(launch_mac(L, flags, i0 > 0, st));
            }
            const float* bsub = bias ? bias + j0 : nullptr;
            float* osub = out + ((size_t)s0 * fo + j0) * ovox;
            if (L.xdirect) {
                ZNNI_DO(launch_fast_inv_yt(L, st));
                ZNNI_DO(launch_inv_z(L, bsub, osub, flags, st));
                continue;
            }
            ZNNI_DO(launch_inv_x(L, st));
            if (fused_inv_yz_available(L)) {
                ZNNI_DO(launch_inv_yz(L, bsub, osub, flags, st));
            } else {
                ZNNI_DO(launch_inv_y(L, st));
                ZNNI_DO(launch_inv_z(L, bsub, osub, flags, st));
            }
        }
    }
    return ZNNI_OK;
}
#undef ZNNI_DO

// Device address of `scratch` on the current GPU, looked up once per GPU (each GPU holds its own copy of the
// array at its own address).
static znni_status static_scratch(void** out)
{
    constexpr int kMaxDevices = 64;
    static void* ptr[kMaxDevices];          // zero-initialised
    static std::mutex mu;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ZNNI_ERR_HIP;
    std::lock_guard<std::mutex> guard(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return ZNNI_ERR_HIP;
        if ((uintptr_t)p & 255u) return ZNNI_ERR_ALIGN;
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return ZNNI_OK;
}

// One 16-byte element per thread and as many workgroups as that takes: the launch shape that moved the most bytes
// per second of those tried (6.2 TB/s on 6 GiB; 8 elements per thread 5.3, grid-stride loops of 1024 to 4096
// workgroups 4.8 to 5.1, hipMemcpyAsync 4.5).
__global__ __launch_bounds__(256) void k_copy_probe(float4* __restrict__ dst, const float4* __restrict__ src, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace znni

using namespace znni;

extern "C" {

int znni_version(void) { return 200; }

const char* znni_status_string(int st)
{
    switch (st) {
        case ZNNI_OK: return "ok";
        case ZNNI_ERR_NULL: return "a required pointer is NULL";
        case ZNNI_ERR_SHAPE: return "bad layer shape (need S,f,f' >= 1 and 1 <= k <= n on every axis, counts within launch limits)";
        case ZNNI_ERR_UNSUPPORTED_SIZE: return "no supported transform size for this image edge";
        case ZNNI_ERR_WORKSPACE: return "workspace too small";
        case ZNNI_ERR_FLAGS: return "unknown flag bit, or more than one multiply-accumulate form requested";
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
    znni_status rc = make_plan(S, f, fo, n, k, 0, nullptr, &L);
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

znni_status znni_conv3d_fft_stage_work_v(int S, int f, int fo, const int n[3], const int k[3], unsigned flags,
                                         double hbm_bytes[ZNNI_NUM_STAGES], double flops[ZNNI_NUM_STAGES])
{
    if (!hbm_bytes || !flops) return ZNNI_ERR_NULL;
    if (!flags_ok(flags)) return ZNNI_ERR_FLAGS;
    LayerPlan L;
    znni_status rc = make_plan(S, f, fo, n, k, flags, nullptr, &L);
    if (rc) return rc;
    const Dims& d = L.d;
    const double c = sizeof(float2), ni = L.nimg, no = L.nimgo, zc = d.zc;
    const double vox = (double)d.nx * d.ny * d.nz, ovox = (double)d.nox * d.noy * d.noz;
    const double x1 = c * d.nx * d.ny * zc, x2 = c * d.nx * d.Ny * zc, xt = c * (double)d.Nx * d.Ny * zc;
    const double y2 = c * zc * d.nox * d.Ny, y1 = c * (double)d.nox * d.noy * zc;
    // stored kernel transforms, unpadded: kx values per kernel column along x, or 8 where x goes in blocks of eight
    const double a = c * zc * d.Ny * (double)f * fo * (L.xblock ? 8 : d.kx);
    for (int q = 0; q < ZNNI_NUM_STAGES; ++q) hbm_bytes[q] = flops[q] = 0.0;
    if (!(flags & ZNNI_KEEP_KERNELS)) hbm_bytes[ZNNI_STAGE_KERNEL_PREP] = 4.0 * f * fo * d.kx * d.ky * d.kz + a;
    const bool fused_zy = !L.xdirect && fused_fwd_zy_available(L), fused_yz = !L.xdirect && fused_inv_yz_available(L);
    if (fused_zy) hbm_bytes[ZNNI_STAGE_FWD_Z] = ni * (4.0 * vox + x2);
    else {
        hbm_bytes[ZNNI_STAGE_FWD_Z] = ni * (4.0 * vox + x1);
        hbm_bytes[ZNNI_STAGE_FWD_Y] = ni * (x1 + x2);
    }
    if (fused_yz) hbm_bytes[ZNNI_STAGE_INV_Y] = no * (y2 + 4.0 * ovox);
    else {
        hbm_bytes[ZNNI_STAGE_INV_Y] = no * (y2 + y1);
        hbm_bytes[ZNNI_STAGE_INV_Z] = no * (y1 + 4.0 * ovox);
    }
    if (L.xdirect) {
        // the spectra between the y passes and the multiply-accumulate keep the x axis as it is
        const double bins = zc * d.Ny * d.nox;
        hbm_bytes[ZNNI_STAGE_MAC] = ni * x2 + a + no * y2;
        flops[ZNNI_STAGE_MAC] = 8.0 * d.kx * S * (double)f * fo * bins;
        if (L.xblock) {
            // one length-8 product per block of V = 9 - kx outputs
            const int V = 9 - d.kx;
            flops[ZNNI_STAGE_MAC] = 8.0 * 8 * S * (double)f * fo * zc * d.Ny * ((d.nox + V - 1) / V);
        }
    } else {
        const double bins = zc * d.Ny * d.Nx;
        hbm_bytes[ZNNI_STAGE_FWD_X] = ni * (x2 + xt);
        hbm_bytes[ZNNI_STAGE_INV_X] = no * (xt + y2);
        hbm_bytes[ZNNI_STAGE_MAC] = ni * xt + a + no * xt;
        flops[ZNNI_STAGE_MAC] = (8.0 * S + 8.0 * (d.kx - 1)) * (double)f * fo * bins;
    }
    return ZNNI_OK;
}

znni_status znni_conv3d_fft_static_v(int S, int f, int fo, const int n[3], const int k[3], const float* in,
                                     const float* w, const float* bias, float* out, unsigned flags, void* stream)
{
    // host-only checks first, against a stand-in workspace address (only its alignment matters to them)
    LayerPlan L;
    znni_status rc = validate(S, f, fo, n, k, in, w, out, flags, (void*)(uintptr_t)256, ZNNI_STATIC_SCRATCH_BYTES, &L);
    if (rc) return rc;                       // ZNNI_ERR_WORKSPACE: the layer needs more than the array holds
    void* base = nullptr;
    rc = static_scratch(&base);
    if (rc) return rc;
    rc = make_plan(S, f, fo, n, k, flags, base, &L);
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

znni_status znni_conv3d_fft_sublayers_v(int S, int f, int fo, const int n[3], const int k[3],
                                        size_t budget_bytes, int sub[3], size_t* bytes)
{
    if (!sub || !bytes) return ZNNI_ERR_NULL;
    Division D;
    znni_status rc = choose_division(S, f, fo, n, k, budget_bytes, &D);
    if (rc == ZNNI_ERR_WORKSPACE) {
        // report what the smallest division would need
        D.Si = 1; D.fi = 1; D.foi = 1;
        if (division_bytes(S, f, fo, n, k, &D) == ZNNI_OK) *bytes = D.bytes;
        return rc;
    }
    if (rc) return rc;
    sub[0] = D.Si; sub[1] = D.fi; sub[2] = D.foi;
    *bytes = D.bytes;
    return ZNNI_OK;
}

znni_status znni_conv3d_fft_budget_v(int S, int f, int fo, const int n[3], const int k[3], const float* in,
                                     const float* w, const float* bias, float* out, unsigned flags,
                                     void* workspace, size_t workspace_bytes, void* stream)
{
    if (!in || !w || !out || !workspace) return ZNNI_ERR_NULL;
    // sub-layers take turns in the workspace, so there are no stored kernel transforms to keep between calls
    if (!flags_ok(flags) || (flags & ZNNI_KEEP_KERNELS)) return ZNNI_ERR_FLAGS;
    Division D;
    znni_status rc = choose_division(S, f, fo, n, k, workspace_bytes, &D);
    if (rc) return rc;
    if (((uintptr_t)in | (uintptr_t)w | (uintptr_t)out) & 15u) return ZNNI_ERR_ALIGN;
    if ((uintptr_t)workspace & 255u) return ZNNI_ERR_ALIGN;
    return run_divided(D, S, f, fo, n, k, in, w, bias, out, flags, workspace, (hipStream_t)stream);
}

znni_status znni_copy_probe(void* dst, const void* src, size_t bytes, void* stream)
{
    if (!dst || !src) return ZNNI_ERR_NULL;
    if (bytes == 0 || (bytes & 15u)) return ZNNI_ERR_SHAPE;
    if (((uintptr_t)dst | (uintptr_t)src) & 15u) return ZNNI_ERR_ALIGN;
    const size_t n16 = bytes / 16;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 0x7fffffffull) blocks = 0x7fffffffull;     // beyond 8 TiB the kernel's loop takes over
    k_copy_probe<<<dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream>>>((float4*)dst, (const float4*)src, n16);
    if (hipGetLastError() != hipSuccess) return ZNNI_ERR_HIP;
    return ZNNI_OK;
}

}  // extern "C"
