// passes_fused.hip -- the transforms along y and z in one kernel, for images whose (oz, oy) plane fits LDS.
//
// Inverse side:
// When the transform lengths along y and z are equal and at most about 120, the plane Y2[imgo][.][xo][.] of one
// (output image, xo) -- zc rows of N complex values, 58 KB at N = 120 -- fits the 160 KB of LDS of a CU more than
// once.  One workgroup then does what the separate inverse y and inverse z passes do (Section III-B/C, the last
// two steps of the inverse transform, pruned to the valid outputs, with bias and transfer function,
// Section IV-A-3) without the intermediate tensor Y1 going to HBM and back: it reads the plane's rows as they
// lie, inverse-transforms them along y keeping the valid yo in LDS, then takes pairs of yo columns through the
// complex-to-real inverse along z and writes the (yo, zo) plane of the output image, which is contiguous.  Per
// output image that moves 8 N zc nox + 4 nox noy noz bytes instead of that plus 16 zc nox noy.
//
// Forward side, the mirror image: one workgroup reads the (y, z) plane of one (input image, x) -- contiguous in
// the input tensor --, transforms pairs of rows real-to-complex along z into LDS, then every oz column along y, and
// writes X2'[img][x][oz][oy] as whole rows; the intermediate tensor X1 never exists.  The forward x pass that
// follows reads X2' with a transposing load (P_FWD_XT in passes_fast.hip).
//
// Every line is transformed by the same two in-register steps as in passes_fast.hip (two_step.h), all lines of the
// plane in one round (one thread per (line, sample offset); zc lines, or N / 2 where the two real ones ride as one,
// see the kernels).  The exchange buffer of the two steps, the plane between the two transforms (inverse) and the
// raw input plane (forward) take turns in ONE region of zc x (N + 2) complex values: whatever is read next sits in
// registers across the barrier that hands the region over.  That is 42 KB at N = 100 -- three workgroups per CU,
// where separate regions (83 KB) left room for one, and a workgroup's life is a chain of memory round trips and
// barriers that only other workgroups can fill.  The forward kernel exists up to length 128, the inverse up to 120.
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
    int QP;                // pitch of the plane kept in LDS (noy + 1 or + 2, even)
};

// Threads of a workgroup, and the number of waves per SIMD the register allocation is held to.  By default four
// (128 registers); the listed kernels sit a few registers above the step that lets one more workgroup share the
// CU and are held below it.
template <int R1, int R2>
constexpr int fused_nth() { return ((R1 * R2 / 2 + 1) * (R1 > R2 ? R1 : R2) + 63) / 64 * 64; }
// The forward kernel can do with N / 2 lines per direction instead of N / 2 + 1 (see there).  It does where that
// saves a wave per workgroup and was measured faster (7 to 21 % at 32, 48, 64; 2 % at 96) and at 128, which then fits
// one round of 1024 threads; where no wave is saved the special cases cost up to 10 % (24), and at 112 it was 5 %
// slower in spite of the wave saved.
constexpr bool fused_fwd_packs(int N) { return N == 32 || N == 48 || N == 64 || N == 96 || N == 128; }
template <int R1, int R2>
constexpr int fused_nth_fwd()
{
    return ((R1 * R2 / 2 + (fused_fwd_packs(R1 * R2) ? 0 : 1)) * (R1 > R2 ? R1 : R2) + 63) / 64 * 64;
}
template <int R1, int R2, bool FWD>
constexpr int fused_waves()
{
    constexpr int N = R1 * R2;
    // measured (32 -> 32 images, batches of 1.5 GB): inverse at 96 held to 64 registers (two over; three workgroups
    // per CU instead of two) 14 % faster, inverse at 112 3-4 %; where the step is further away the spills cost 5 to
    // 25 %.  (The forward kernels need no budget: since they untangle on the way into the y transform they use 38
    // to 68 registers.)
    if (!FWD && (N == 96 || N == 112)) return 8;
    // forward at 128: 1024 threads; at 76 registers one workgroup has a CU to itself, held to 64 (16 bytes of
    // scratch) two share it: 0.24 -> 0.19 ms for 40 images of 128^3
    if (FWD && N == 128) return 8;
    return 4;
}

// The inverse kernel can pack the same two lines: rows oz = 0 and N / 2 of the plane are spectra of real sequences,
// so c = row 0 + i row N/2 comes back from the inverse y transform as (row 0's values, row N/2's values).  Measured:
// 11-12 % faster at 32 and 64 (a wave less per workgroup), a tie at 48, 3 % slower at 96; at 128 the kernel it makes
// possible (1024 threads, held to 64 registers with 36 bytes of scratch) is 13 % slower than the two separate
// passes on 40 images of 128^3 and 16-19 % faster on 32 or 8 images: not used there.
constexpr bool fused_inv_packs(int N) { return N == 32 || N == 64; }
template <int R1, int R2>
constexpr int fused_nth_inv()
{
    return ((R1 * R2 / 2 + (fused_inv_packs(R1 * R2) ? 0 : 1)) * (R1 > R2 ? R1 : R2) + 63) / 64 * 64;
}

template <int R1, int R2>
__global__ __launch_bounds__((fused_nth_inv<R1, R2>())) __attribute__((amdgpu_waves_per_eu((fused_waves<R1, R2, false>()))))
void k_inv_yz(FusedArgs a)
{
    using TS = TwoStep<R1, R2>;
    constexpr int N = TS::N, P = TS::P, ZC = N / 2 + 1;
    constexpr bool PACK = fused_inv_packs(N);
    constexpr int NL = PACK ? N / 2 : ZC;     // lines per transform
    extern __shared__ float2 lds[];
    const int QP = a.QP;
    float2* tws = lds;                 // [N]
    float2* R = lds + N;               // [ZC][P] exchange buffer; between the transforms the plane Q[ZC][QP]
    const int t = threadIdx.x, NTH = blockDim.x;
    const int xo = blockIdx.x, img = blockIdx.y;
    const Dims& d = a.d;
    const int nox = d.nox, noy = d.noy, noz = d.noz;

    for (int q = t; q < N; q += NTH) tws[q] = a.tw[q];

    const int ja = t % R2, la = t / R2;       // step A: (line la, sample offset ja)
    const bool in_a = la < NL;
    const int lb = t % NL, q = t / NL;        // step B: (line lb, output offset q); work only for q < R1
    float2 v[R1];
    float2 u[R2];

    // ---- inverse along y: the rows oz of the plane, conj . forward . conj
    if (in_a) {
        const float2* row = a.src + (((size_t)img * ZC + la) * nox + xo) * d.ldn;
        if (!PACK || la) {
#pragma unroll
            for (int m = 0; m < R1; ++m) {
                const float2 x = row[ja + R2 * m];
                v[m] = make_float2(x.x, -x.y);
            }
        } else {                              // line 0 = row 0 + i row N/2, conjugated
            const float2* rown = row + (size_t)(N / 2) * nox * d.ldn;
#pragma unroll
            for (int m = 0; m < R1; ++m) {
                const float2 x = row[ja + R2 * m], y = rown[ja + R2 * m];
                v[m] = make_float2(x.x - y.y, -(x.y + y.x));
            }
        }
    }
    __syncthreads();                          // twiddles are in LDS
    if (in_a) TS::step_a(v, la, ja, tws, R);
    __syncthreads();
    if (q < R1) TS::step_b(u, lb, q, R);
    __syncthreads();                          // the exchange buffer has been read: the region becomes Q
    if (q < R1) {
#pragma unroll
        for (int r = 0; r < R2; ++r) {
            const int yo = q + R1 * r - (d.ky - 1);
            if (yo >= 0 && yo < noy) {
                if (!PACK || lb) {
                    R[lb * QP + yo] = cconj(u[r]);
                } else {                      // real part: row 0, imaginary part of the conjugate: row N/2
                    R[yo] = make_float2(u[r].x, 0.f);
                    R[(N / 2) * QP + yo] = make_float2(-u[r].y, 0.f);
                }
            }
        }
    }
    {
        const int sh = QP - noy - 1;                         // one or two spare columns, read by the last yo pair
        for (int e = t; e < (ZC << sh); e += NTH) R[(e >> sh) * QP + noy + (e & sh)] = make_float2(0.f, 0.f);
    }
    __syncthreads();

    // ---- inverse along z, complex to real: yo columns 2p and 2p+1 ride as real and imaginary part of one line
    const int np = (noy + 1) >> 1;            // <= N / 2 < ZC lines
    if (in_a) {
        const float mp = la < np ? 1.f : 0.f;
        const float2* col = R + 2 * min(la, np - 1);
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
    __syncthreads();                          // Q has been read: the region is the exchange buffer again
    if (in_a) TS::step_a(v, la, ja, tws, R);
    __syncthreads();
    if (q < R1) TS::step_b(u, lb, q, R);
    __syncthreads();
    if (q < R1) {
#pragma unroll
        for (int r = 0; r < R2; ++r) R[lb * P + q + R1 * r] = u[r];           // natural order per line
    }
    __syncthreads();
    // rows yo of out[imgo][xo]: real part of line l -> row 2l, minus imaginary part -> row 2l+1
    const float bj = a.bias ? a.bias[img % a.fo] : 0.f;
    float* dst = a.out + (((size_t)img * nox + xo) * noy) * noz;
    // a wave per line = pair of rows (one LDS read serves both), or per two or four lines where rows are at most 32
    // or 16 long
    constexpr int LW = N <= 16 ? 16 : N <= 32 ? 32 : 64, RPI = 64 / LW;
    for (int l = (t / 64) * RPI + (t % 64) / LW; l < np; l += (NTH / 64) * RPI) {
        const float2* row = R + l * P + (d.kz - 1);
        float* d0 = dst + (size_t)(2 * l) * noz;
        const bool two = 2 * l + 1 < noy;
        for (int zo = t % LW; zo < noz; zo += LW) {
            const float2 c = row[zo];
            float v0 = c.x + bj, v1 = bj - c.y;
            if (a.relu) { v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); }
            d0[zo] = v0;
            if (two) d0[noz + zo] = v1;
        }
    }
}

struct FusedFwdArgs {
    const float* in;       // [img][x][y][z]
    float2* dst;           // X2'[img][x][oz][oy]
    const float2* tw;      // [N]
    Dims d;
};

// Lines per transform: along z two real rows ride in one complex line, N / 2 lines at most.  Along y the plane has
// N / 2 + 1 lines (oz = 0 ... N / 2), but the first and the last are real sequences (sums and alternating sums of
// real rows): with PACK they ride together as real and imaginary part of line 0 and are separated, by the same
// symmetry, when the rows are stored -- N / 2 lines in both directions.
template <int R1, int R2>
__global__ __launch_bounds__((fused_nth_fwd<R1, R2>())) __attribute__((amdgpu_waves_per_eu((fused_waves<R1, R2, true>()))))
void k_fwd_zy(FusedFwdArgs a)
{
    using TS = TwoStep<R1, R2>;
    constexpr int N = TS::N, P = TS::P, ZC = N / 2 + 1;
    constexpr bool PACK = fused_fwd_packs(N);
    constexpr int NL = PACK ? N / 2 : ZC;
    extern __shared__ float2 lds[];
    const int RP = a.d.nz;             // the raw plane keeps its pitch
    float2* tws = lds;                 // [N]
    float2* R = lds + N;               // in turn: raw plane [ny][RP] floats, exchange buffer and lines [NL][P]
    const int t = threadIdx.x, NTH = blockDim.x;
    const int x = blockIdx.x, img = blockIdx.y;
    const Dims& d = a.d;
    const int ny = d.ny, nz = d.nz;
    const float* plane = a.in + (((size_t)img * d.nx + x) * ny) * nz;

    for (int q = t; q < N; q += NTH) tws[q] = a.tw[q];

    const int ja = t % R2, la = t / R2;
    const bool in_a = la < NL;
    const int lb = t % NL, q = t / NL;
    float2 v[R1];
    float2 u[R2];

    // ---- the (y, z) plane, contiguous in the input tensor, into LDS with fully coalesced loads.  (Reading each
    // line's samples straight into the registers of the first step, as the separate z pass does, touches every
    // cache line from four instructions and, for some row lengths, evicts it in between: measured up to 2.8x
    // slower with a whole plane per workgroup.)
    float* raw = reinterpret_cast<float*>(R);
    {
        // a flat copy, rows at their pitch in memory.  (Padding the rows in LDS so that the lines a wave reads
        // together spread over all banks costs index arithmetic per element -- these kernels are bound by issuing
        // instructions, not by LDS -- and was measured 3-8 % slower at almost every length.)
        const int tot = ny * nz;
        for (int i0 = 0; i0 < tot; i0 += 8 * NTH) {
            float r[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) r[k] = plane[min(i0 + k * NTH + t, tot - 1)];
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (i0 + k * NTH + t < tot) raw[i0 + k * NTH + t] = r[k];
        }
    }
    __syncthreads();

    // ---- along z, real to complex: rows 2p and 2p+1 ride as real and imaginary part of line p
    const int np = (ny + 1) >> 1;             // <= N / 2 < ZC lines
    if (in_a) {
        const int ya = 2 * min(la, np - 1);
        const float ma = la < np ? 1.f : 0.f, mb = (la < np && ya + 1 < ny) ? 1.f : 0.f;
        const float* ra = raw + ya * RP;
        const float* rb = raw + min(ya + 1, ny - 1) * RP;
        // rows that fill the transform length: constant offsets, no padding in z
        if (nz == N) {
#pragma unroll
            for (int m = 0; m < R1; ++m) v[m] = make_float2(ra[ja + R2 * m] * ma, rb[ja + R2 * m] * mb);
        } else {
#pragma unroll
            for (int m = 0; m < R1; ++m) {
                const int e = ja + R2 * m, ec = min(e, nz - 1);
                const float me = e < nz ? 1.f : 0.f;
                v[m] = make_float2(ra[ec] * (me * ma), rb[ec] * (me * mb));
            }
        }
    }
    __syncthreads();                          // the raw plane has been read: the region becomes the exchange buffer
    if (in_a) TS::step_a(v, la, ja, tws, R);
    __syncthreads();
    if (q < R1) TS::step_b(u, lb, q, R);
    __syncthreads();
    if (q < R1) {
#pragma unroll
        for (int r = 0; r < R2; ++r) R[lb * P + q + R1 * r] = u[r];           // natural order per line
    }
    __syncthreads();
    // ---- along y: one line per oz.  Its sample y = 2l + h is row h of line l above, untangled on the way in:
    // with Z = line l and W = conj(Z[N - oz]), row 0 is (Z[oz] + W) / 2 and row 1 is -i (Z[oz] - W) / 2.  R2 is even,
    // so a thread sees rows of one parity only, and its lines l advance by R2 / 2 per sample: two addresses, then
    // constant offsets.  (Untangling into a plane of its own first cost a pass through LDS each way, a barrier and
    // index arithmetic per element.)
    static_assert(R2 % 2 == 0, "a thread's samples must have one parity");
    if (in_a) {
        const int oz = la;
        const bool odd = ja & 1;
        if (!PACK || oz) {
            const float sg = odd ? -1.f : 1.f;
            const float2* pz = R + (ja >> 1) * P + oz;
            const float2* pw = R + (ja >> 1) * P + (oz ? N - oz : 0);
#pragma unroll
            for (int m = 0; m < R1; ++m) {
                const float mk = ja + R2 * m < ny ? 0.5f : 0.f;
                const float2 z = pz[(R2 / 2) * P * m], w = pw[(R2 / 2) * P * m];
                const float pr = fmaf(sg, w.x, z.x) * mk, qi = fmaf(-sg, w.y, z.y) * mk;
                v[m] = odd ? make_float2(qi, -pr) : make_float2(pr, qi);
            }
        } else {
            // line 0 carries oz = 0 (real part) and oz = N / 2 (imaginary part): at these two bins the rows of a
            // line are simply the real and the imaginary part of the line's value
            const float2* pz = R + (ja >> 1) * P;
#pragma unroll
            for (int m = 0; m < R1; ++m) {
                const float mk = ja + R2 * m < ny ? 1.f : 0.f;
                const float2 z = pz[(R2 / 2) * P * m], w = pz[(R2 / 2) * P * m + N / 2];
                v[m] = odd ? make_float2(z.y * mk, w.y * mk) : make_float2(z.x * mk, w.x * mk);
            }
        }
    }
    __syncthreads();                          // the lines have been read: the region is the exchange buffer again
    if (in_a) TS::step_a(v, la, ja, tws, R);
    __syncthreads();
    if (q < R1) TS::step_b(u, lb, q, R);
    __syncthreads();
    if (q < R1) {
#pragma unroll
        for (int r = 0; r < R2; ++r) R[lb * P + q + R1 * r] = u[r];
    }
    __syncthreads();
    float2* dst = a.dst + (((size_t)img * d.nx + x) * ZC) * N;
    // a wave per row, or per two or four rows where rows are at most 32 or 16 long; rows 0 and N / 2 come out of
    // line 0 = C: (C[oy] + conj(C[N - oy])) / 2 and -i (C[oy] - conj(C[N - oy])) / 2
    constexpr int LW = N <= 16 ? 16 : N <= 32 ? 32 : 64, RPI = 64 / LW;
    for (int l = (t / 64) * RPI + (t % 64) / LW; l < ZC; l += (NTH / 64) * RPI) {
        if (!PACK || (l != 0 && l != N / 2)) {
            for (int e = t % LW; e < N; e += LW) dst[(size_t)l * N + e] = R[l * P + e];
        } else {
            for (int e = t % LW; e < N; e += LW) {
                const float2 c = R[e], m = cconj(R[e ? N - e : 0]);
                dst[(size_t)l * N + e] = l ? cscale(mul_mi(csub(c, m)), 0.5f) : cscale(cadd(c, m), 0.5f);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------- host side
struct FusedShape { int R1, R2, QP, RP, nth; size_t lds; };

// The in-register split of each supported length, measured best per length (32 -> 32 images, batches of 1.5 GB):
// mostly R1 x 8 -- fewer, fatter threads than the separate passes use would not cover a plane's lines in one
// round --, with the squarer splits 6 x 6, 8 x 10 and 8 x 12 10 to 15 % ahead at 36, 80 and 96.  At 120 both
// kernels take 10 x 12 (12 threads per line instead of 15): the inverse kernel then runs two workgroups per CU instead
// of one and is 40 % faster, the forward kernel is 10 % faster with it than with 15 x 8.
static bool fused_split(int N, bool forward, int* R1, int* R2)
{
    static const int tab[][3] = {{8, 2, 4},    {10, 5, 2},  {12, 3, 4},  {14, 7, 2},  {16, 4, 4},  {20, 5, 4},
                                 {24, 6, 4},   {28, 7, 4},  {32, 4, 8},  {36, 6, 6},  {40, 5, 8},  {48, 6, 8},
                                 {56, 7, 8},   {64, 8, 8},  {72, 9, 8},  {80, 8, 10}, {96, 8, 12}, {100, 10, 10},
                                 {112, 7, 16}, {120, 15, 8}};
    if (N == 120) { *R1 = 10; *R2 = 12; return true; }
    if (N == 128 && forward) { *R1 = 8; *R2 = 16; return true; }    // one round of 1024 threads: 64 lines x 16
    for (const auto& e : tab)
        if (e[0] == N) { *R1 = e[1]; *R2 = e[2]; return true; }
    return false;
}

// forward = true: the plane holds ny columns instead of noy, and the x pass after it must be an in-register one
static bool fused_shape(const LayerPlan& L, FusedShape* F, bool forward = false)
{
    const Dims& d = L.d;
    if (L.generic_passes || d.Ny != d.Nz) return false;
    int R1, R2;
    if (!fused_split(d.Ny, forward, &R1, &R2)) return false;
    F->R1 = R1; F->R2 = R2;
    if (forward) {
        if (!fast_pass_available(d.Nx) || d.nx > 65535 || L.nimg > 65535) return false;
    } else {
        if (d.nox > 65535 || L.nimgo > 65535) return false;
    }
    const int N = d.Ny, zc = d.zc;
    const int cols = forward ? d.ny : d.noy;
    F->QP = cols + 2 - (cols & 1);
    F->RP = d.nz;
    const int lines = (forward ? fused_fwd_packs(N) : fused_inv_packs(N)) ? N / 2 : zc;   // two lines may ride as one
    F->nth = (lines * std::max(R1, R2) + 63) / 64 * 64;
    size_t region = sizeof(float2) * (size_t)(forward ? lines : zc) * (N + 2);      // the inverse plane Q has zc rows
    if (forward) region = std::max(region, sizeof(float) * (size_t)d.ny * F->RP);
    F->lds = sizeof(float2) * (size_t)N + region;
    return F->nth <= 1024 && F->lds <= 80 * 1024;             // two workgroups per CU at least
}

bool fused_inv_yz_available(const LayerPlan& L)
{
    FusedShape F;
    return fused_shape(L, &F);
}

bool fused_fwd_zy_available(const LayerPlan& L)
{
    FusedShape F;
    return fused_shape(L, &F, true);
}

template <typename Args>
static znni_status launch_fused(void (*kernel)(Args), const Args& a, const FusedShape& F, dim3 grid, hipStream_t st)
{
    if (F.lds > 48 * 1024 &&
        hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)F.lds) != hipSuccess)
        return ZNNI_ERR_HIP;
    kernel<<<grid, dim3(F.nth), F.lds, st>>>(a);
    if (hipGetLastError() != hipSuccess) return ZNNI_ERR_HIP;
    return ZNNI_OK;
}

// dispatch on the split that fused_split chose (R1 * 100 + R2)
#define ZNNI_FUSED_CASES(KERNEL)                                                                   \
    switch (F.R1 * 100 + F.R2) {                                                                   \
        case 204: return launch_fused(KERNEL<2, 4>, a, F, grid, st);                               \
        case 502: return launch_fused(KERNEL<5, 2>, a, F, grid, st);                               \
        case 304: return launch_fused(KERNEL<3, 4>, a, F, grid, st);                               \
        case 702: return launch_fused(KERNEL<7, 2>, a, F, grid, st);                               \
        case 404: return launch_fused(KERNEL<4, 4>, a, F, grid, st);                               \
        case 504: return launch_fused(KERNEL<5, 4>, a, F, grid, st);                               \
        case 604: return launch_fused(KERNEL<6, 4>, a, F, grid, st);                               \
        case 704: return launch_fused(KERNEL<7, 4>, a, F, grid, st);                               \
        case 408: return launch_fused(KERNEL<4, 8>, a, F, grid, st);                               \
        case 606: return launch_fused(KERNEL<6, 6>, a, F, grid, st);                               \
        case 508: return launch_fused(KERNEL<5, 8>, a, F, grid, st);                               \
        case 608: return launch_fused(KERNEL<6, 8>, a, F, grid, st);                               \
        case 708: return launch_fused(KERNEL<7, 8>, a, F, grid, st);                               \
        case 808: return launch_fused(KERNEL<8, 8>, a, F, grid, st);                               \
        case 908: return launch_fused(KERNEL<9, 8>, a, F, grid, st);                               \
        case 810: return launch_fused(KERNEL<8, 10>, a, F, grid, st);                              \
        case 812: return launch_fused(KERNEL<8, 12>, a, F, grid, st);                              \
        case 1010: return launch_fused(KERNEL<10, 10>, a, F, grid, st);                            \
        case 716: return launch_fused(KERNEL<7, 16>, a, F, grid, st);                              \
        case 1508: return launch_fused(KERNEL<15, 8>, a, F, grid, st);                             \
        case 1012: return launch_fused(KERNEL<10, 12>, a, F, grid, st);                            \
        case 816: return launch_fused(KERNEL<8, 16>, a, F, grid, st);                              \
    }                                                                                              \
    return ZNNI_ERR_UNSUPPORTED_SIZE;

// in -> X2' (buf1); to be followed by launch_fast_fwd_xt
znni_status launch_fwd_zy(const LayerPlan& L, const float* in, hipStream_t st)
{
    FusedShape F;
    if (!fused_shape(L, &F, true)) return ZNNI_ERR_UNSUPPORTED_SIZE;
    const Dims& d = L.d;
    FusedFwdArgs a;
    a.in = in; a.dst = L.buf1; a.tw = L.twy; a.d = d;
    const dim3 grid(d.nx, L.nimg);
    ZNNI_FUSED_CASES(k_fwd_zy)
}

znni_status launch_inv_yz(const LayerPlan& L, const float* bias, float* out, unsigned flags, hipStream_t st)
{
    FusedShape F;
    if (!fused_shape(L, &F)) return ZNNI_ERR_UNSUPPORTED_SIZE;
    const Dims& d = L.d;
    FusedArgs a;
    a.src = L.buf0; a.out = out; a.tw = L.twy; a.bias = bias;
    a.d = d; a.fo = L.fo; a.relu = (flags & ZNNI_RELU) ? 1 : 0;
    a.QP = F.QP;
    const dim3 grid(d.nox, L.nimgo);
    ZNNI_FUSED_CASES(k_inv_yz)
}

}  // namespace znni
