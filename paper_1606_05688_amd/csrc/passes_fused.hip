// passes_fused.hip -- the transforms along y and z in one kernel, for images whose (oz, oy) plane fits LDS.
//
// Inverse side:
// When the transform lengths along y and z are equal and at most about 120, the plane Y2[imgo][.][xo][.] of one
// (output image, xo) -- zc rows of N complex values, 58 KB at N = 120 -- fits the 160 KB of LDS of a CU more than
// once.  One workgroup
// then does what the separate inverse y and inverse z passes do (Section III-B/C, the last two steps of the
// inverse transform, pruned to the valid outputs, with bias and transfer function, Section IV-A-3) without the
// intermediate tensor Y1 going to HBM and back: it reads the plane's rows as they lie, inverse-transforms them
// along y keeping the valid yo in LDS, then takes pairs of yo columns through the complex-to-real inverse along z
// and writes the (yo, zo) plane of the output image, which is contiguous.  Per output image that moves
// 8 N zc nox + 4 nox noy noz bytes instead of that plus 16 zc nox noy.
//
// Forward side, the mirror image: one workgroup reads the (y, z) plane of one (input image, x) -- contiguous in
// the input tensor --, transforms pairs of rows real-to-complex along z into LDS, then every oz column along y, and
// writes X2'[img][x][oz][oy] as whole rows; the intermediate tensor X1 never exists.  The forward x pass that
// follows reads X2' with a transposing load (P_FWD_XT in passes_fast.hip).
//
// Every line is transformed by the same two in-register steps as in passes_fast.hip (two_step.h).
#include "two_step.h"
#include <algorithm>
#include "znni_internal.h"

namespace znni {

struct FusedArgs {
    const float2* src;     // Y2[imgo][oz][xo][oy]
    float* out;
    const float2* tw;      // [N]
    const float* bias;
    Dims d;
    int fo, relu;
    int LG;                // lines (rows, then yo pairs) per round
    int QP;                // pitch of the plane kept in LDS (noy + 1 or + 2, even)
};

template <int R1, int R2>
__global__ __launch_bounds__(1024) void k_inv_yz(FusedArgs a)
{
    using TS = TwoStep<R1, R2>;
    constexpr int N = TS::N, P = TS::P, ZC = N / 2 + 1;
    extern __shared__ float2 lds[];
    const int LG = a.LG, QP = a.QP;
    float2* tws = lds;                 // [N]
    float2* buf = lds + N;             // [LG][P]
    float2* Q = buf + LG * P;          // [ZC][QP]: the plane after the inverse along y, valid yo only
    const int t = threadIdx.x, NTH = blockDim.x;
    const int xo = blockIdx.x, img = blockIdx.y;
    const Dims& d = a.d;
    const int nox = d.nox, noy = d.noy, noz = d.noz;

    for (int q = t; q < N; q += NTH) tws[q] = a.tw[q];
    for (int e = t; e < ZC * (QP - noy); e += NTH) {         // the spare columns read by the last yo pair
        const int row = e / (QP - noy), c = e - row * (QP - noy);
        Q[row * QP + noy + c] = make_float2(0.f, 0.f);
    }

    const int ja = t % R2, la = t / R2;       // step A: (line la, sample offset ja)
    const bool in_a = la < LG;
    const int lb = t % LG, q = t / LG;        // step B: (line lb, output offset q); work only for q < R1
    float2 v[R1];

    // ---- inverse along y: rows oz of the plane, conj . forward . conj
    for (int l0 = 0; l0 < ZC; l0 += LG) {
        const int nl = min(LG, ZC - l0);
        if (in_a) {
            const float ml = la < nl ? 1.f : 0.f;
            const float2* row = a.src + (((size_t)img * ZC + l0 + min(la, nl - 1)) * nox + xo) * N;
#pragma unroll
            for (int m = 0; m < R1; ++m) {
                const float2 x = row[ja + R2 * m];
                v[m] = make_float2(x.x * ml, -(x.y * ml));
            }
        }
        __syncthreads();                      // twiddles are in LDS; the previous round has left buf
        if (in_a) TS::step_a(v, la, ja, tws, buf);
        __syncthreads();
        if (q < R1 && lb < nl) {
            float2 u[R2];
            TS::step_b(u, lb, q, buf);
#pragma unroll
            for (int r = 0; r < R2; ++r) {
                const int yo = q + R1 * r - (d.ky - 1);
                if (yo >= 0 && yo < noy) Q[(l0 + lb) * QP + yo] = cconj(u[r]);
            }
        }
    }
    __syncthreads();

    // ---- inverse along z, complex to real: yo columns 2p and 2p+1 ride as real and imaginary part of one line
    const int npairs = (noy + 1) >> 1;
    const float bj = a.bias ? a.bias[img % a.fo] : 0.f;
    for (int p0 = 0; p0 < npairs; p0 += LG) {
        const int np = min(LG, npairs - p0);
        if (in_a) {
            const float mp = la < np ? 1.f : 0.f;
            const float2* col = Q + 2 * (p0 + min(la, np - 1));
#pragma unroll
            for (int m = 0; m < R1; ++m) {
                const int e = ja + R2 * m;
                const bool direct = e < ZC;
                const int ee = direct ? e : N - e;
                const float4 ab = *reinterpret_cast<const float4*>(col + ee * QP);
                float2 A = make_float2(ab.x * mp, ab.y * mp), B = make_float2(ab.z * mp, ab.w * mp);
                if (!direct) { A = cconj(A); B = cconj(B); }
                v[m] = cconj(cadd(A, mul_pi(B)));
            }
        }
        __syncthreads();                      // the previous round's rows have been stored from buf
        if (in_a) TS::step_a(v, la, ja, tws, buf);
        __syncthreads();
        float2 u[R2];
        if (q < R1) TS::step_b(u, lb, q, buf);
        __syncthreads();
        if (q < R1) {
#pragma unroll
            for (int r = 0; r < R2; ++r) buf[lb * P + q + R1 * r] = u[r];     // natural order per line
        }
        __syncthreads();
        // rows yo = 2*p0 .. of out[imgo][xo]: real part -> row 2l, minus imaginary part -> row 2l+1
        const int rows = min(2 * np, noy - 2 * p0);
        float* dst = a.out + (((size_t)img * nox + xo) * noy + 2 * p0) * noz;
        for (int ll = t / 64; ll < rows; ll += NTH / 64) {
            const float2* row = buf + (ll >> 1) * P + (d.kz - 1);
            for (int zo = t % 64; zo < noz; zo += 64) {
                const float2 c = row[zo];
                float val = ((ll & 1) ? -c.y : c.x) + bj;
                if (a.relu) val = fmaxf(val, 0.f);
                dst[(size_t)ll * noz + zo] = val;
            }
        }
    }
}

struct FusedFwdArgs {
    const float* in;       // [img][x][y][z]
    float2* dst;           // X2'[img][x][oz][oy]
    const float2* tw;      // [N]
    Dims d;
    int LG;                // lines per round; at least (ny + 1) / 2, so that the z transforms take one round
    int PP;                // pitch of the plane kept in LDS (ny + 1 or + 2, even)
    int RP;                // pitch, in floats, of the raw input plane in LDS
};

template <int R1, int R2>
__global__ __launch_bounds__(1024) void k_fwd_zy(FusedFwdArgs a)
{
    using TS = TwoStep<R1, R2>;
    constexpr int N = TS::N, P = TS::P, ZC = N / 2 + 1;
    extern __shared__ float2 lds[];
    const int LG = a.LG, PP = a.PP;
    float2* tws = lds;                 // [N]
    float2* buf = lds + N;             // [LG][P]
    float2* Pl = buf + LG * P;         // [ZC][PP]: the plane after the transform along z, Pl[oz][y]
    const int t = threadIdx.x, NTH = blockDim.x;
    const int x = blockIdx.x, img = blockIdx.y;
    const Dims& d = a.d;
    const int ny = d.ny, nz = d.nz;
    const float* plane = a.in + (((size_t)img * d.nx + x) * ny) * nz;

    for (int q = t; q < N; q += NTH) tws[q] = a.tw[q];

    const int ja = t % R2, la = t / R2;
    const bool in_a = la < LG;
    const int lb = t % LG, q = t / LG;
    float2 v[R1];

    // ---- the (y, z) plane, contiguous in the input tensor, into LDS with fully coalesced loads.  (Reading each
    // line's samples straight into the registers of the first step, as the separate z pass does, touches every
    // cache line from four instructions and, for row lengths near a multiple of 256 bytes, from rows that
    // all fall into the same few sets of the vector cache: measured up to 2.8x slower.)
    float* raw = reinterpret_cast<float*>(Pl);     // [ny][RP]; overlaid on the plane it turns into
    {
        const int tot = ny * nz, RP = a.RP;
        const float inv_nz = 1.f / (float)nz;
        for (int i0 = 0; i0 < tot; i0 += 8 * NTH) {
            float r[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) r[k] = plane[min(i0 + k * NTH + t, tot - 1)];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int i = i0 + k * NTH + t;
                int row = (int)((float)i * inv_nz);
                row -= row * nz > i ? 1 : 0;
                row += (row + 1) * nz <= i ? 1 : 0;
                if (i < tot) raw[row * RP + (i - row * nz)] = r[k];
            }
        }
    }
    __syncthreads();

    // ---- along z, real to complex: rows 2p and 2p+1 ride as real and imaginary part of one line; all
    // (ny + 1) / 2 <= LG lines in one round
    {
        const int np = (ny + 1) >> 1;
        if (in_a) {
            const int ya = 2 * min(la, np - 1);
            const float ma = la < np ? 1.f : 0.f, mb = (la < np && ya + 1 < ny) ? 1.f : 0.f;
            const float* ra = raw + ya * a.RP;
            const float* rb = raw + min(ya + 1, ny - 1) * a.RP;
#pragma unroll
            for (int m = 0; m < R1; ++m) {
                const int e = ja + R2 * m, ec = min(e, nz - 1);
                const float me = e < nz ? 1.f : 0.f;
                v[m] = make_float2(ra[ec] * (me * ma), rb[ec] * (me * mb));
            }
        }
        __syncthreads();                      // raw has been consumed (it is overwritten by the untangling below)
        if (in_a) TS::step_a(v, la, ja, tws, buf);
        __syncthreads();
        float2 u[R2];
        if (q < R1) TS::step_b(u, lb, q, buf);
        __syncthreads();
        if (q < R1) {
#pragma unroll
            for (int r = 0; r < R2; ++r) buf[lb * P + q + R1 * r] = u[r];     // natural order per line
        }
        __syncthreads();
        // untangle the two rows of every line and park them as two neighbouring y of each oz row
        for (int e = t; e < np * ZC; e += NTH) {          // lines fastest: neighbouring lanes write neighbours
            const int oz = e / np, l = e - oz * np;
            const float2* row = buf + l * P;
            const float2 z1 = row[oz], z2 = cconj(row[oz ? N - oz : 0]);
            const float2 ev = cscale(cadd(z1, z2), 0.5f), od = cscale(mul_mi(csub(z1, z2)), 0.5f);
            *reinterpret_cast<float4*>(Pl + oz * PP + 2 * l) = make_float4(ev.x, ev.y, od.x, od.y);
        }
    }
    __syncthreads();

    // ---- along y: one line per oz
    for (int l0 = 0; l0 < ZC; l0 += LG) {
        const int nl = min(LG, ZC - l0);
        if (in_a) {
            const float ml = la < nl ? 1.f : 0.f;
            const float2* line = Pl + (l0 + min(la, nl - 1)) * PP;
#pragma unroll
            for (int m = 0; m < R1; ++m) {
                const int y = ja + R2 * m;
                const float mk = y < ny ? ml : 0.f;
                const float2 c = line[min(y, ny - 1)];
                v[m] = make_float2(c.x * mk, c.y * mk);
            }
        }
        __syncthreads();                      // the previous round's rows have been stored from buf
        if (in_a) TS::step_a(v, la, ja, tws, buf);
        __syncthreads();
        float2 u[R2];
        if (q < R1) TS::step_b(u, lb, q, buf);
        __syncthreads();
        if (q < R1) {
#pragma unroll
            for (int r = 0; r < R2; ++r) buf[lb * P + q + R1 * r] = u[r];
        }
        __syncthreads();
        float2* dst = a.dst + (((size_t)img * d.nx + x) * ZC + l0) * N;
        for (int l = t / 64; l < nl; l += NTH / 64)
            for (int e = t % 64; e < N; e += 64) dst[(size_t)l * N + e] = buf[l * P + e];
    }
}

// ------------------------------------------------------------------------------------------- host side
struct FusedShape { int LG, QP, nth; size_t lds; };

// forward = true: the plane holds ny columns instead of noy, and the x pass after it must be an in-register one
static bool fused_shape(const LayerPlan& L, FusedShape* F, bool forward = false)
{
    const Dims& d = L.d;
    if (forward && (!fast_pass_available(d.Nx) || d.nx > 65535 || L.nimg > 65535)) return false;
    // Measured on MI355X against the two separate passes (32 output images per input, batches filling 2 GB):
    // 1.3x to 2.1x faster up to N = 64, 1.25x at 80, 1.1x at 96, 1.2x at 100 and 120, even at 112, 10 % slower at
    // 128, where the plane leaves room for only one workgroup per CU.
    if (d.Ny != d.Nz || !fast_pass_available(d.Ny)) return false;
    if (d.Ny > 100 && d.Ny != 120) return false;
    if (d.nox > 65535 * 1 || L.nimgo > 65535) return false;
    const int N = d.Ny, zc = d.zc;
    int T = 0;
    switch (N) {      // threads per line = the larger factor of the in-register split (passes_fast.hip)
        case 8: T = 4; break;    case 10: T = 5; break;   case 12: T = 4; break;   case 14: T = 7; break;
        case 16: T = 4; break;   case 20: T = 5; break;   case 24: T = 6; break;   case 28: T = 7; break;
        case 32: T = 8; break;   case 36: T = 9; break;   case 40: T = 8; break;   case 48: T = 8; break;
        case 56: T = 8; break;   case 64: T = 8; break;   case 72: T = 9; break;   case 80: T = 10; break;
        case 96: T = 12; break;  case 100: T = 10; break; case 112: T = 14; break; case 120: T = 15; break;
        case 128: T = 16; break;
        default: return false;
    }
    int LG = 1024 / T;
    if (LG > zc) LG = zc;
    const int rounds = (zc + LG - 1) / LG;
    LG = (zc + rounds - 1) / rounds;
    F->LG = LG;
    const int cols = forward ? d.ny : d.noy;
    F->QP = cols + 2 - (cols & 1);
    F->nth = (LG * T + 63) / 64 * 64;
    size_t plane = sizeof(float2) * (size_t)zc * F->QP;
    if (forward) {
        if (LG < zc) return false;                         // all row pairs of the plane in one round
        plane = std::max(plane, sizeof(float) * (size_t)d.ny * (d.nz + 8));     // the raw plane, any pitch
    }
    F->lds = sizeof(float2) * ((size_t)N + (size_t)LG * (N + 2)) + plane;
    return F->nth <= 1024 && F->lds <= 150 * 1024;
}

bool fused_inv_yz_available(const LayerPlan& L)
{
    FusedShape F;
    return fused_shape(L, &F);
}

template <int R1, int R2>
static znni_status launch_yz(const FusedArgs& a, const FusedShape& F, dim3 grid, hipStream_t st)
{
    const void* fn = (const void*)k_inv_yz<R1, R2>;
    if (F.lds > 48 * 1024 &&
        hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)F.lds) != hipSuccess)
        return ZNNI_ERR_HIP;
    k_inv_yz<R1, R2><<<grid, dim3(F.nth), F.lds, st>>>(a);
    if (hipGetLastError() != hipSuccess) return ZNNI_ERR_HIP;
    return ZNNI_OK;
}

bool fused_fwd_zy_available(const LayerPlan& L)
{
    FusedShape F;
    return fused_shape(L, &F, true);
}

template <int R1, int R2>
static znni_status launch_zy(const FusedFwdArgs& a0, const FusedShape& F, dim3 grid, hipStream_t st)
{
    // rows of the raw plane 2*RP floats apart must spread the R2 neighbouring samples of the lines that a
    // wave reads together over all LDS banks: RP = 2 mod 4 for R2 = 4, 4 mod 8 otherwise
    FusedFwdArgs a = a0;
    const int mod = R2 == 4 ? 4 : 8;
    a.RP = a.d.nz + ((mod / 2 - a.d.nz) % mod + mod) % mod;
    const void* fn = (const void*)k_fwd_zy<R1, R2>;
    if (F.lds > 48 * 1024 &&
        hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)F.lds) != hipSuccess)
        return ZNNI_ERR_HIP;
    k_fwd_zy<R1, R2><<<grid, dim3(F.nth), F.lds, st>>>(a);
    if (hipGetLastError() != hipSuccess) return ZNNI_ERR_HIP;
    return ZNNI_OK;
}

// in -> X2' (buf1); to be followed by launch_fast_fwd_xt
znni_status launch_fwd_zy(const LayerPlan& L, const float* in, hipStream_t st)
{
    FusedShape F;
    if (!fused_shape(L, &F, true)) return ZNNI_ERR_UNSUPPORTED_SIZE;
    const Dims& d = L.d;
    FusedFwdArgs a;
    a.in = in; a.dst = L.buf1; a.tw = L.twy; a.d = d; a.LG = F.LG; a.PP = F.QP; a.RP = 0;
    const dim3 grid(d.nx, L.nimg);
    switch (d.Ny) {
        case 8: return launch_zy<2, 4>(a, F, grid, st);
        case 10: return launch_zy<5, 2>(a, F, grid, st);
        case 12: return launch_zy<3, 4>(a, F, grid, st);
        case 14: return launch_zy<7, 2>(a, F, grid, st);
        case 16: return launch_zy<4, 4>(a, F, grid, st);
        case 20: return launch_zy<5, 4>(a, F, grid, st);
        case 24: return launch_zy<6, 4>(a, F, grid, st);
        case 28: return launch_zy<7, 4>(a, F, grid, st);
        case 32: return launch_zy<4, 8>(a, F, grid, st);
        case 36: return launch_zy<9, 4>(a, F, grid, st);
        case 40: return launch_zy<5, 8>(a, F, grid, st);
        case 48: return launch_zy<6, 8>(a, F, grid, st);
        case 56: return launch_zy<7, 8>(a, F, grid, st);
        case 64: return launch_zy<8, 8>(a, F, grid, st);
        case 72: return launch_zy<9, 8>(a, F, grid, st);
        case 80: return launch_zy<10, 8>(a, F, grid, st);
        case 96: return launch_zy<12, 8>(a, F, grid, st);
        case 100: return launch_zy<10, 10>(a, F, grid, st);
        case 120: return launch_zy<15, 8>(a, F, grid, st);
    }
    return ZNNI_ERR_UNSUPPORTED_SIZE;
}

znni_status launch_inv_yz(const LayerPlan& L, const float* bias, float* out, unsigned flags, hipStream_t st)
{
    FusedShape F;
    if (!fused_shape(L, &F)) return ZNNI_ERR_UNSUPPORTED_SIZE;
    const Dims& d = L.d;
    FusedArgs a;
    a.src = L.buf0; a.out = out; a.tw = L.twy; a.bias = bias;
    a.d = d; a.fo = L.fo; a.relu = (flags & ZNNI_RELU) ? 1 : 0;
    a.LG = F.LG; a.QP = F.QP;
    const dim3 grid(d.nox, L.nimgo);
    switch (d.Ny) {       // the splits of the separate passes, except that R2 stays at 8 for the long lengths
        case 8: return launch_yz<2, 4>(a, F, grid, st);
        case 10: return launch_yz<5, 2>(a, F, grid, st);
        case 12: return launch_yz<3, 4>(a, F, grid, st);
        case 14: return launch_yz<7, 2>(a, F, grid, st);
        case 16: return launch_yz<4, 4>(a, F, grid, st);
        case 20: return launch_yz<5, 4>(a, F, grid, st);
        case 24: return launch_yz<6, 4>(a, F, grid, st);
        case 28: return launch_yz<7, 4>(a, F, grid, st);
        case 32: return launch_yz<4, 8>(a, F, grid, st);
        case 36: return launch_yz<9, 4>(a, F, grid, st);
        case 40: return launch_yz<5, 8>(a, F, grid, st);
        case 48: return launch_yz<6, 8>(a, F, grid, st);
        case 56: return launch_yz<7, 8>(a, F, grid, st);
        case 64: return launch_yz<8, 8>(a, F, grid, st);
        case 72: return launch_yz<9, 8>(a, F, grid, st);
        case 80: return launch_yz<10, 8>(a, F, grid, st);
        case 96: return launch_yz<12, 8>(a, F, grid, st);
        case 100: return launch_yz<10, 10>(a, F, grid, st);
        case 112: return launch_yz<14, 8>(a, F, grid, st);
        case 120: return launch_yz<15, 8>(a, F, grid, st);
        case 128: return launch_yz<16, 8>(a, F, grid, st);
    }
    return ZNNI_ERR_UNSUPPORTED_SIZE;
}

}  // namespace znni
