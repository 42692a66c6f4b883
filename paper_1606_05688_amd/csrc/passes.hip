// passes.hip -- the six transform passes of the layer, for any supported transform length.
//
// Forward (Section III-C order: the contiguous axis z first, real-to-complex, then y, then x) and inverse
// (the same steps in reverse, Section III-B/C).  Where the paper permutes the 4-D tensor between
// library calls, each pass here reads TL whole lines that are contiguous along the axis being transformed,
// transforms them in LDS, and writes them back with the NEXT axis contiguous, so every pass both reads and
// writes HBM in contiguous runs and the tensor is touched exactly once per pass.  Like the paper's GPU
// transform, the result is left in permuted order because only bin-wise work follows.
//
// Pruning (Section III-A): lines that are zero padding are never read or transformed (they only exist when
// n~ > n); on the inverse side only the n' = n-k+1 valid outputs of a line are stored, so the later passes
// run nox/Nx (y) and nox*noy/(Nx*Ny) (z) of the lines.
//
// Layouts (image <nx,ny,nz>, transform sizes <Nx,Ny,Nz>, zc = Nz/2+1, valid outputs <nox,noy,noz>,
// img = s*f + i, imgo = s*f' + j; all complex interleaved fp32):
//   in  [img][x<nx][y<ny][z<nz]             real
//   X1  [img][x<nx][oz<zc][y<ny (ldy)]      after z     (ldy, ldx, ldo: row pitches rounded up to 16 elements,
//   X2  [img][oz][oy<Ny][x<nx (ldx)]        after y      so that every row starts on a 128-byte boundary)
//   Xt  [oz][oy][img][ox<Nx]                after x   ("pencil" order: one (oz,oy) pair holds all images)
//   Yt  [oz][oy][imgo][ox<Nx]               accumulated output spectra
//   Y2  [imgo][oz][xo<nox][oy<Ny]           after inverse x, cropped to valid x (row pitch ldn)
//   Y1  [imgo][xo][oz<zc][yo<noy (ldo)]     after inverse y, cropped to valid y
//   out [imgo][xo][yo][zo<noz]              real, after inverse z + bias + transfer function
#include "znni_internal.h"

namespace znni {

// The three twiddle tables exp(-2 pi i q / N) of a layer (x, y, z axis) in one launch; blockIdx.y picks the axis.
// A's zeroed padding behind the last pencil (pad elements at `padp`) is written by the same launch.
__global__ void k_twiddles(float2* twx, int Nx, float2* twy, int Ny, float2* twz, int Nz, float2* padp, size_t pad)
{
    const size_t q = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (blockIdx.y == 3) {
        if (q < pad) padp[q] = make_float2(0.f, 0.f);
        return;
    }
    float2* tw = blockIdx.y == 0 ? twx : (blockIdx.y == 1 ? twy : twz);
    const int N = blockIdx.y == 0 ? Nx : (blockIdx.y == 1 ? Ny : Nz);
    if (q < (size_t)N) {
        double s, c;
        sincospi(2.0 * (double)q / (double)N, &s, &c);
        tw[q] = make_float2((float)c, (float)(-s));
    }
}

struct Lds {
    float2* tw;
    float2* a;
    float2* b;
    int ld;
};

__device__ __forceinline__ Lds carve(float2* base, int N, int nlines, const float2* __restrict__ twg)
{
    Lds L;
    L.ld = N | 1;
    L.tw = base;
    L.a = base + N;
    L.b = L.a + nlines * L.ld;
    for (int q = threadIdx.x; q < N; q += blockDim.x) L.tw[q] = twg[q];
    return L;
}

// ---- forward, axis z: real -> complex.  Two real lines ride through one complex transform.
__global__ void k_fwd_z(const float* __restrict__ in, float2* __restrict__ X1, const float2* __restrict__ twg,
                        FftPlan P, Dims d, int TL)
{
    extern __shared__ float2 lds[];
    const int N = P.N, nl = TL >> 1;
    Lds L = carve(lds, N, nl, twg);
    const int y0 = blockIdx.x * TL, x = blockIdx.y, img = blockIdx.z;
    const int ny = d.ny, nz = d.nz, zc = d.zc;
    const int nvalid = min(TL, ny - y0);
    const float* src = in + (((size_t)img * d.nx + x) * ny + y0) * nz;
    for (int e = threadIdx.x; e < nl * N; e += blockDim.x) {
        const int p = e / N, z = e - p * N;
        float re = 0.f, im = 0.f;
        if (z < nz) {
            if (2 * p < nvalid) re = src[(size_t)(2 * p) * nz + z];
            if (2 * p + 1 < nvalid) im = src[(size_t)(2 * p + 1) * nz + z];
        }
        L.a[p * L.ld + z] = make_float2(re, im);
    }
    __syncthreads();
    const float2* r = fft_lines(L.a, L.b, L.tw, nl, L.ld, P);
    float2* dst = X1 + ((size_t)img * d.nx + x) * zc * d.ldy + y0;
    for (int e = threadIdx.x; e < zc * TL; e += blockDim.x) {
        const int l = e & (TL - 1), oz = e / TL;
        if (l >= nvalid) continue;
        const float2* row = r + (l >> 1) * L.ld;
        const float2 z1 = row[oz], z2 = cconj(row[oz ? N - oz : 0]);
        const float2 v = (l & 1) ? cscale(mul_mi(csub(z1, z2)), 0.5f) : cscale(cadd(z1, z2), 0.5f);
        dst[(size_t)oz * d.ldy + l] = v;
    }
}

// ---- forward, axis y
__global__ void k_fwd_y(const float2* __restrict__ X1, float2* __restrict__ X2, const float2* __restrict__ twg,
                        FftPlan P, Dims d, int TL)
{
    extern __shared__ float2 lds[];
    const int N = P.N;
    Lds L = carve(lds, N, TL, twg);
    const int x0 = blockIdx.x * TL, oz = blockIdx.y, img = blockIdx.z;
    const int nx = d.nx, ny = d.ny, zc = d.zc;
    const int nvalid = min(TL, nx - x0);
    for (int e = threadIdx.x; e < TL * N; e += blockDim.x) {
        const int l = e / N, y = e - l * N;
        float2 v = make_float2(0.f, 0.f);
        if (l < nvalid && y < ny) v = X1[(((size_t)img * nx + x0 + l) * zc + oz) * d.ldy + y];
        L.a[l * L.ld + y] = v;
    }
    __syncthreads();
    const float2* r = fft_lines(L.a, L.b, L.tw, TL, L.ld, P);
    float2* dst = X2 + ((size_t)img * d.x2i + (size_t)oz * d.x2o) * d.ldx + x0;
    for (int e = threadIdx.x; e < N * TL; e += blockDim.x) {
        const int l = e & (TL - 1), oy = e / TL;
        if (l < nvalid) dst[(size_t)oy * d.ldx + l] = r[l * L.ld + oy];
    }
}

// ---- forward, axis x; writes pencil order
__global__ void k_fwd_x(const float2* __restrict__ X2, float2* __restrict__ Xt, const float2* __restrict__ twg,
                        FftPlan P, Dims d, int nimg, int TL)
{
    extern __shared__ float2 lds[];
    const int N = P.N;
    Lds L = carve(lds, N, TL, twg);
    const int oy0 = blockIdx.x * TL, oz = blockIdx.y, img = blockIdx.z;
    const int nx = d.nx, Ny = d.Ny;
    const int nvalid = min(TL, Ny - oy0);
    const float2* src = X2 + ((size_t)img * d.x2i + (size_t)oz * d.x2o + oy0) * d.ldx;
    for (int e = threadIdx.x; e < TL * N; e += blockDim.x) {
        const int l = e / N, x = e - l * N;
        float2 v = make_float2(0.f, 0.f);
        if (l < nvalid && x < nx) v = src[(size_t)l * d.ldx + x];
        L.a[l * L.ld + x] = v;
    }
    __syncthreads();
    const float2* r = fft_lines(L.a, L.b, L.tw, TL, L.ld, P);
    for (int e = threadIdx.x; e < TL * N; e += blockDim.x) {
        const int l = e / N, ox = e - l * N;
        if (l < nvalid) Xt[(((size_t)oz * Ny + oy0 + l) * nimg + img) * N + ox] = r[l * L.ld + ox];
    }
}

// The inverse transform of a line is conj(forward(conj(line))); the 1/(Nx Ny Nz) factor is folded into the
// kernel spectra.

// ---- inverse, axis x; keeps x in [kx-1, nx-1]
__global__ void k_inv_x(const float2* __restrict__ Yt, float2* __restrict__ Y2, const float2* __restrict__ twg,
                        FftPlan P, Dims d, int nimgo, int TL)
{
    extern __shared__ float2 lds[];
    const int N = P.N;
    Lds L = carve(lds, N, TL, twg);
    const int oy0 = blockIdx.x * TL, oz = blockIdx.y, img = blockIdx.z;
    const int Ny = d.Ny, zc = d.zc, nox = d.nox;
    const int nvalid = min(TL, Ny - oy0);
    for (int e = threadIdx.x; e < TL * N; e += blockDim.x) {
        const int l = e / N, ox = e - l * N;
        float2 v = make_float2(0.f, 0.f);
        if (l < nvalid) v = cconj(Yt[(((size_t)oz * Ny + oy0 + l) * nimgo + img) * N + ox]);
        L.a[l * L.ld + ox] = v;
    }
    __syncthreads();
    const float2* r = fft_lines(L.a, L.b, L.tw, TL, L.ld, P);
    float2* dst = Y2 + ((size_t)img * zc + oz) * nox * d.ldn + oy0;
    for (int e = threadIdx.x; e < nox * TL; e += blockDim.x) {
        const int l = e & (TL - 1), xo = e / TL;
        if (l < nvalid) dst[(size_t)xo * d.ldn + l] = cconj(r[l * L.ld + xo + d.kx - 1]);
    }
}

// ---- inverse, axis y; keeps y in [ky-1, ny-1]; only lines with valid x exist.  Tile: TL consecutive xo of one
// (imgo, oz), which lie next to each other in Y2; each transformed line is written as it is (yo contiguous).
__global__ void k_inv_y(const float2* __restrict__ Y2, float2* __restrict__ Y1, const float2* __restrict__ twg,
                        FftPlan P, Dims d, int TL)
{
    extern __shared__ float2 lds[];
    const int N = P.N;
    Lds L = carve(lds, N, TL, twg);
    const int xo0 = blockIdx.x * TL, oz = blockIdx.y, img = blockIdx.z;
    const int zc = d.zc, nox = d.nox, noy = d.noy;
    const int nvalid = min(TL, nox - xo0);
    const float2* src = Y2 + (((size_t)img * zc + oz) * nox + xo0) * d.ldn;
    for (int e = threadIdx.x; e < TL * N; e += blockDim.x) {
        const int l = e / N, oy = e - l * N;
        float2 v = make_float2(0.f, 0.f);
        if (l < nvalid) v = cconj(src[(size_t)l * d.ldn + oy]);
        L.a[l * L.ld + oy] = v;
    }
    __syncthreads();
    const float2* r = fft_lines(L.a, L.b, L.tw, TL, L.ld, P);
    for (int e = threadIdx.x; e < TL * noy; e += blockDim.x) {
        const int l = e / noy, yo = e - l * noy;
        if (l < nvalid)
            Y1[(((size_t)img * nox + xo0 + l) * zc + oz) * d.ldo + yo] = cconj(r[l * L.ld + yo + d.ky - 1]);
    }
}

// ---- inverse, axis z: complex -> real for two lines at once; keeps z in [kz-1, nz-1]; bias + transfer.
// Tile: TL consecutive yo of one (imgo, xo); in Y1 they are adjacent elements of every oz row.
__global__ void k_inv_z(const float2* __restrict__ Y1, float* __restrict__ out, const float* __restrict__ bias,
                        const float2* __restrict__ twg, FftPlan P, Dims d, int fo, int relu, int TL)
{
    extern __shared__ float2 lds[];
    const int N = P.N, nl = TL >> 1;
    Lds L = carve(lds, N, nl, twg);
    const int yo0 = blockIdx.x * TL, xo = blockIdx.y, img = blockIdx.z;
    const int zc = d.zc, nox = d.nox, noy = d.noy, noz = d.noz;
    const int nvalid = min(TL, noy - yo0);
    const float2* src = Y1 + (((size_t)img * nox + xo) * zc) * d.ldo + yo0;
    for (int e = threadIdx.x; e < nl * N; e += blockDim.x) {
        const int p = e % nl, o = e / nl;          // the line pair fastest: neighbouring lanes read neighbouring yo
        const bool direct = o < zc;
        const int oo = direct ? o : N - o;
        // rows are 128-byte aligned and yo0 + 2p is even: the pair (A, B) is one aligned 16-byte load; the pitch
        // covers the element behind an odd last line
        const float4 ab = *reinterpret_cast<const float4*>(src + (size_t)oo * d.ldo + 2 * p);
        float2 A = make_float2(0.f, 0.f), B = A;
        if (2 * p < nvalid) A = make_float2(ab.x, ab.y);
        if (2 * p + 1 < nvalid) B = make_float2(ab.z, ab.w);
        if (!direct) { A = cconj(A); B = cconj(B); }
        // Z = A + iB carries line 2p in its real part and line 2p+1 in its imaginary part after the
        // inverse transform; stored conjugated for the forward-transform route.
        L.a[p * L.ld + o] = cconj(cadd(A, mul_pi(B)));
    }
    __syncthreads();
    const float2* r = fft_lines(L.a, L.b, L.tw, nl, L.ld, P);
    const float bj = bias ? bias[img % fo] : 0.f;
    float* dst = out + (((size_t)img * nox + xo) * noy + yo0) * noz;
    for (int e = threadIdx.x; e < TL * noz; e += blockDim.x) {
        const int l = e / noz, zo = e - l * noz;
        if (l >= nvalid) continue;
        const float2 t = r[(l >> 1) * L.ld + zo + d.kz - 1];
        float v = ((l & 1) ? -t.y : t.x) + bj;
        if (relu) v = fmaxf(v, 0.f);
        dst[(size_t)l * noz + zo] = v;
    }
}

// ------------------------------------------------------------------------------------------- host side
static size_t pass_lds_bytes(int N, int nlines) { return sizeof(float2) * ((size_t)N + 2 * (size_t)nlines * (N | 1)); }

int lines_per_tile(int N)
{
    // largest power of two <= 16 whose two LDS buffers stay within ~72 KB, so several tiles share a CU
    int TL = 16;
    while (TL > 2 && pass_lds_bytes(N, TL) > 72 * 1024) TL >>= 1;
    return TL;
}

#define ZNNI_LAUNCH_CHECK()                         \
    do {                                            \
        if (hipGetLastError() != hipSuccess) return ZNNI_ERR_HIP; \
    } while (0)

static znni_status allow_lds(const void* fn, size_t bytes)
{
    if (bytes > 48 * 1024) {
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess)
            return ZNNI_ERR_HIP;
    }
    return ZNNI_OK;
}

znni_status launch_twiddles(const LayerPlan& L, hipStream_t st)
{
    const Dims& d = L.d;
    // the multiply-accumulate reads a little past A's last pencil (values multiplied by zero at most): that
    // padding is zeroed here
    // (the block-transform route keeps another array in A and reads nothing behind it)
    const size_t pad = L.xblock ? 0 : (size_t)(L.fp + 64) * L.Mp;
    const size_t per = (size_t)d.kx * L.fp * L.Mp;
    size_t most = pad > 0 ? pad : 1;
    for (int N : {d.Nx, d.Ny, d.Nz})
        if ((size_t)N > most) most = N;
    k_twiddles<<<dim3((unsigned)((most + 255) / 256), 4), dim3(256), 0, st>>>(
        L.twx, d.Nx, L.twy, d.Ny, L.twz, d.Nz, L.A + (size_t)d.zc * d.Ny * per, pad);
    ZNNI_LAUNCH_CHECK();
    return ZNNI_OK;
}

znni_status launch_fwd_z(const LayerPlan& L, const float* in, hipStream_t st)
{
    const Dims& d = L.d;
    if (!L.generic_passes && fast_pass_available(d.Nz)) return launch_fast_fwd_z(L, in, st);
    const int TL = lines_per_tile(d.Nz);
    const size_t lds = pass_lds_bytes(d.Nz, TL / 2);
    znni_status rc = allow_lds((const void*)k_fwd_z, lds);
    if (rc) return rc;
    dim3 grid((d.ny + TL - 1) / TL, d.nx, L.nimg);
    k_fwd_z<<<grid, dim3(256), lds, st>>>(in, L.buf0, L.twz, L.fftz, d, TL);
    ZNNI_LAUNCH_CHECK();
    return ZNNI_OK;
}

znni_status launch_fwd_y(const LayerPlan& L, hipStream_t st)
{
    const Dims& d = L.d;
    if (!L.generic_passes && fast_pass_available(d.Ny)) return launch_fast_fwd_y(L, st);
    const int TL = lines_per_tile(d.Ny);
    const size_t lds = pass_lds_bytes(d.Ny, TL);
    znni_status rc = allow_lds((const void*)k_fwd_y, lds);
    if (rc) return rc;
    dim3 grid((d.nx + TL - 1) / TL, d.zc, L.nimg);
    k_fwd_y<<<grid, dim3(256), lds, st>>>(L.buf0, L.buf1, L.twy, L.ffty, d, TL);
    ZNNI_LAUNCH_CHECK();
    return ZNNI_OK;
}

znni_status launch_fwd_x(const LayerPlan& L, hipStream_t st)
{
    const Dims& d = L.d;
    if (!L.generic_passes && fast_pass_available(d.Nx)) return launch_fast_fwd_x(L, st);
    const int TL = lines_per_tile(d.Nx);
    const size_t lds = pass_lds_bytes(d.Nx, TL);
    znni_status rc = allow_lds((const void*)k_fwd_x, lds);
    if (rc) return rc;
    dim3 grid((d.Ny + TL - 1) / TL, d.zc, L.nimg);
    k_fwd_x<<<grid, dim3(256), lds, st>>>(L.buf1, L.buf0, L.twx, L.fftx, d, L.nimg, TL);
    ZNNI_LAUNCH_CHECK();
    return ZNNI_OK;
}

znni_status launch_inv_x(const LayerPlan& L, hipStream_t st)
{
    const Dims& d = L.d;
    if (!L.generic_passes && fast_pass_available(d.Nx)) return launch_fast_inv_x(L, st);
    const int TL = lines_per_tile(d.Nx);
    const size_t lds = pass_lds_bytes(d.Nx, TL);
    znni_status rc = allow_lds((const void*)k_inv_x, lds);
    if (rc) return rc;
    dim3 grid((d.Ny + TL - 1) / TL, d.zc, L.nimgo);
    k_inv_x<<<grid, dim3(256), lds, st>>>(L.Yt, L.buf0, L.twx, L.fftx, d, L.nimgo, TL);
    ZNNI_LAUNCH_CHECK();
    return ZNNI_OK;
}

znni_status launch_inv_y(const LayerPlan& L, hipStream_t st)
{
    const Dims& d = L.d;
    if (!L.generic_passes && fast_pass_available(d.Ny)) return launch_fast_inv_y(L, st);
    const int TL = lines_per_tile(d.Ny);
    const size_t lds = pass_lds_bytes(d.Ny, TL);
    znni_status rc = allow_lds((const void*)k_inv_y, lds);
    if (rc) return rc;
    dim3 grid((d.nox + TL - 1) / TL, d.zc, L.nimgo);
    k_inv_y<<<grid, dim3(256), lds, st>>>(L.buf0, L.buf1, L.twy, L.ffty, d, TL);
    ZNNI_LAUNCH_CHECK();
    return ZNNI_OK;
}

znni_status launch_inv_z(const LayerPlan& L, const float* bias, float* out, unsigned flags, hipStream_t st)
{
    const Dims& d = L.d;
    if (!L.generic_passes && fast_pass_available(d.Nz)) return launch_fast_inv_z(L, bias, out, flags, st);
    const int TL = lines_per_tile(d.Nz);
    const size_t lds = pass_lds_bytes(d.Nz, TL / 2);
    znni_status rc = allow_lds((const void*)k_inv_z, lds);
    if (rc) return rc;
    dim3 grid((d.noy + TL - 1) / TL, d.nox, L.nimgo);
    k_inv_z<<<grid, dim3(256), lds, st>>>(L.buf1, out, bias, L.twz, L.fftz, d, L.fo, (flags & ZNNI_RELU) ? 1 : 0,
                                          TL);
    ZNNI_LAUNCH_CHECK();
    return ZNNI_OK;
}

}  // namespace znni
