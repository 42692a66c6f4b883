// mac.hip -- pruned kernel transform and the per-bin multiply-accumulate.
//
// Kernel side of the layer (Sections III-A and IV-B-2).  A kx*ky*kz kernel zero-padded to Nx*Ny*Nz is
// transformed axis by axis, touching only lines that are not all zero: kx*ky lines along z, then kx*zc lines
// along y, then Ny*zc lines along x (for a cubic layer: k^2, k*zc, N*zc).  With k small each of these
// one-dimensional transforms of a k-sample line is evaluated directly from its k non-zero inputs.  The first
// two stages are stored (array A, kx*Ny*zc values per kernel instead of Nx*Ny*zc); the third is evaluated
// where it is consumed, inside the multiply-accumulate
//
//     Yt[s][j](ox,oy,oz) = sum_i  Wt[j][i](ox,oy,oz) * Xt[s][i](ox,oy,oz),
//     Wt[j][i](ox,oy,oz) = sum_{a<kx} A[oz][oy](a,i,j) * exp(-2 pi i a ox / Nx)
//
// which is the second stage of Algorithm 3 (multiply the f image spectra by the f kernel spectra of output
// image j, accumulate over the f products) without a stored kernel spectrum.  The 1/(Nx Ny Nz) of the
// unnormalised transforms is folded into A.  Below, N stands for Nx and k for kx.
//
// For one (oz,oy) pencil this is one dense complex matrix product
//
//     Yt[j][col] = sum_{(i,a)} A(a,i,j) * ( T[a*ox(col)] * X[i][col] ),     T[q] = exp(-2 pi i q / N),
//
// with col = s*N + ox running over all images of the batch and the contraction index running over the f*k
// (input image, tap) pairs: the left operand does not depend on the column, the right operand is the image
// spectrum times a twiddle that depends on the tap and the column only.  That is a contraction, so it runs on
// the matrix cores (v_mfma_f32_16x16x4_f32), each complex product done as three real ones:
//     P1 = Ar Br, P2 = Ai Bi, P3 = (Ar+Ai)(Br+Bi);  Re = P1 - P2, Im = P3 - P1 - P2.
// A is stored in the order the contraction walks it: [oz][oy][i/4][a][i%4][j<Mp].
#include <algorithm>
#include "mac_common.h"

namespace znni {

// Both stages below need few twiddles per workgroup -- exp(-2 pi i o c / N) for the workgroup's KPREP_OZ (KPREP_OY)
// consecutive outputs o and the taps c -- and every thread needs the same one at the same time.  They are gathered
// once into LDS as tw2[c][o], KPREP_TAPS taps at a time, and the inner loops read them at constant offsets: no
// index arithmetic per product (it was half of the vector instructions of kernels that are bound by issuing them).
constexpr int KPREP_TAPS = 64;
template <int NO>
__device__ __forceinline__ void kprep_gather(float2* tw2, const float2* __restrict__ tw, int N, int o0, int c0, int nc)
{
    for (int e = threadIdx.x; e < nc * NO; e += 256) {
        const int c = e / NO, o = e - c * NO;
        tw2[e] = tw[(unsigned)((o0 + o) * (c0 + c)) % (unsigned)N];      // both factors below 1024
    }
}

// A1[oz][b<ky][a<kx][i<fp][j<Mp] = sum_{c<kz} w[j][i][a][b][c] exp(-2 pi i oz c / Nz); zero where i >= f or
// j >= fo.  (j fastest, so the y stage below reads and writes contiguous runs.)
// One thread produces KPREP_OZ consecutive oz for one (b,a,i,j): its kz kernel values -- a short run of w, far
// from the runs of the neighbouring lanes -- are read once per KPREP_OZ outputs.  (One thread per output re-read w
// for every oz: 3.2 ms for 80 x 80 kernels of 9^3 at length 100.)
constexpr int KPREP_OZ = 16;
__global__ __launch_bounds__(256) void k_kprep_z(const float* __restrict__ w, float2* __restrict__ A1,
                                                 const float2* __restrict__ twz, Dims d, int f, int fo, int fp,
                                                 int Mp, size_t wj_stride)
{
    extern __shared__ float2 tw2[];                            // [taps of the chunk][KPREP_OZ]
    const int N = d.Nz;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    const int oz0 = blockIdx.y * KPREP_OZ;
    const int per = d.ky * d.kx * fp * Mp;
    const int j = idx % Mp;
    const int i = (idx / Mp) % fp;
    const int ba = idx / (Mp * fp);
    const int a = ba % d.kx, b = ba / d.kx;
    const bool live = idx < per && i < f && j < fo;
    float2 acc[KPREP_OZ];
#pragma unroll
    for (int o = 0; o < KPREP_OZ; ++o) acc[o] = make_float2(0.f, 0.f);
    const float* wr = w + (live ? (size_t)j * wj_stride + ((((size_t)i) * d.kx + a) * d.ky + b) * d.kz : 0);
    for (int c0 = 0; c0 < d.kz; c0 += KPREP_TAPS) {
        const int nc = min(KPREP_TAPS, d.kz - c0);
        if (c0) __syncthreads();                               // the previous chunk's twiddles have been used
        kprep_gather<KPREP_OZ>(tw2, twz, N, oz0, c0, nc);
        __syncthreads();
        if (live) {
            for (int c = 0; c < nc; ++c) {
                const float v = wr[c0 + c];
                const float2* tc = tw2 + c * KPREP_OZ;
#pragma unroll
                for (int o = 0; o < KPREP_OZ; ++o) acc[o] = caxpy(acc[o], v, tc[o]);
            }
        }
    }
    if (idx >= per) return;
#pragma unroll
    for (int o = 0; o < KPREP_OZ; ++o)
        if (oz0 + o < d.zc) A1[(size_t)(oz0 + o) * per + idx] = acc[o];
}

// A[oz][oy<Ny][i/4][a<kx][i%4][j<Mp] = scale * sum_{b<ky} A1[oz][b][a][i][j] exp(-2 pi i oy b / Ny)
// (i < fp, j < Mp: f and fo rounded up to the matrix-core tiles; the padding holds zeros).
// One thread produces KPREP_OY consecutive oy for one (a,i,j): each A1 value is loaded once, and per product the
// thread issues the four multiply-adds and nothing else.
constexpr int KPREP_OY = 32;
__global__ __launch_bounds__(256) void k_kprep_y(const float2* __restrict__ A1, float2* __restrict__ A,
                                                 const float2* __restrict__ tw, int N, int k, int ky, int fp, int Mp,
                                                 int per, float scale)
{
    // N = Ny, k = kx (taps left for the multiply-accumulate), ky = taps summed here, per = kx*fp*Mp
    extern __shared__ float2 tw2[];                            // [taps of the chunk][KPREP_OY]
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;     // (a, i, j) as laid out in A1
    const int oy0 = blockIdx.y * KPREP_OY, oz = blockIdx.z;
    const bool live = idx < per;
    const float2* a1 = A1 + (size_t)oz * ky * per + (live ? idx : 0);
    float2 acc[KPREP_OY];
#pragma unroll
    for (int o = 0; o < KPREP_OY; ++o) acc[o] = make_float2(0.f, 0.f);
    for (int b0 = 0; b0 < ky; b0 += KPREP_TAPS) {
        const int nb = min(KPREP_TAPS, ky - b0);
        if (b0) __syncthreads();                               // the previous chunk's twiddles have been used
        kprep_gather<KPREP_OY>(tw2, tw, N, oy0, b0, nb);
        __syncthreads();
        if (live) {
            for (int b = 0; b < nb; ++b) {
                const float2 v = a1[(size_t)(b0 + b) * per];
                const float2* tb = tw2 + b * KPREP_OY;
#pragma unroll
                for (int o = 0; o < KPREP_OY; ++o) acc[o] = cfma(acc[o], v, tb[o]);
            }
        }
    }
    if (!live) return;
    const int j = idx % Mp, i = (idx / Mp) % fp, a = idx / (Mp * fp);
    float2* d = A + ((size_t)oz * N + oy0) * per + (size_t)(((i >> 2) * k + a) * 4 + (i & 3)) * Mp + j;
#pragma unroll
    for (int o = 0; o < KPREP_OY; ++o)
        if (oy0 + o < N) st_stream(d + (size_t)o * per, cscale(acc[o], scale));
}

// Plain multiply-accumulate, one workgroup per (oz, oy) pencil, one thread per ox.  Slow and simple; kept as
// a diagnostic path (flag ZNNI_MAC_REFERENCE) the matrix-core kernel can be compared with.
__global__ void k_mac_simple(const float2* __restrict__ Xt, const float2* __restrict__ A, float2* __restrict__ Yt,
                             const float2* __restrict__ tw, int N, int S, int f, int fo, int k, int fp, int Mp,
                             int accumulate)
{
    // N = Nx, k = kx; grid = (Ny, zc)
    const size_t pencil = (size_t)blockIdx.y * gridDim.x + blockIdx.x;
    const float2* Xp = Xt + pencil * S * f * N;
    const float2* Ap = A + pencil * k * fp * Mp;
    float2* Yp = Yt + pencil * S * fo * N;
    for (int ox = threadIdx.x; ox < N; ox += blockDim.x) {
        for (int s = 0; s < S; ++s)
            for (int j = 0; j < fo; ++j) {
                float2 acc = make_float2(0.f, 0.f);
                for (int i = 0; i < f; ++i) {
                    float2 W = make_float2(0.f, 0.f);
                    for (int a = 0; a < k; ++a)
                        W = cadd(W, cmul(Ap[(size_t)(((i >> 2) * k + a) * 4 + (i & 3)) * Mp + j], tw[(a * ox) % N]));
                    acc = cadd(acc, cmul(W, Xp[(size_t)(s * f + i) * N + ox]));
                }
                float2* dst = Yp + (size_t)(s * fo + j) * N + ox;
                *dst = accumulate ? cadd(*dst, acc) : acc;
            }
    }
}

// Matrix-core multiply-accumulate for any number of taps k (work split: see mac_common.h).
//
// The fp x NW block of image spectra stays in LDS for the whole call (in chunks of FC input images if it does
// not fit); A is streamed from global memory straight into the matrix-core operand layout (lane l supplies
// A[row l%16][k-index l/16]); the four waves of a workgroup read the same A values, which the vector L1 serves.
//
// The contraction is a flat sequence of steps s = (i/4)*k + a, four contraction indices (input images) per
// step.  On this hardware every instruction a wave issues costs matrix-core time (vector and matrix
// instructions do not overlap), so the loop is built to need few of them: A addresses advance by a constant,
// A registers are reloaded in two alternating sets of four steps (no copies), the right operand of step s+1
// (image fragment times twiddle, and their sum for the three-product scheme) is prepared during step s, and
// the three partial products are combined once, after the last step.
template <int RTW, int CTW>
__device__ __forceinline__ void mac_body(float2* lds, const float2* __restrict__ Xt, const float2* __restrict__ A,
                                         float2* __restrict__ Yt, const float2* __restrict__ twg, int N, int S,
                                         int f, int fo, int k, int fp, int Mp, int FC, int col0, int ncolblk,
                                         int pencil, int sub, int accumulate)
{
    constexpr int NW = 64 * CTW;
    float2* tws = lds;              // [N]
    float2* Xs = lds + N;           // [FC][NW]

    MacWork w;
    mac_decode<RTW, CTW>(w, Xt, A, Yt, N, S, f, fo, k, fp, Mp, col0, ncolblk, pencil, sub);
    const int l16 = w.l16, kk = w.kk, m0 = w.m0, cw0 = w.cw0, colbase = w.colbase;
    const float2* Ap = w.Ap;

    for (int q = threadIdx.x; q < N; q += 256) tws[q] = twg[q];

    int oxs[CTW];
#pragma unroll
    for (int c = 0; c < CTW; ++c) oxs[c] = (colbase + cw0 + c * 16 + l16) % N;

    floatx4 p1[RTW][CTW], p2[RTW][CTW], p3[RTW][CTW];
#pragma unroll
    for (int r = 0; r < RTW; ++r)
#pragma unroll
        for (int c = 0; c < CTW; ++c) {
            p1[r][c] = floatx4{0.f, 0.f, 0.f, 0.f}; p2[r][c] = p1[r][c]; p3[r][c] = p1[r][c];
        }

    for (int ic0 = 0; ic0 < fp; ic0 += FC) {
        const int fc = min(FC, fp - ic0);           // multiple of 4
        __syncthreads();
        mac_stage_x<NW>(Xs, w, ic0, fc, f, N);
        __syncthreads();

        // ---- ST = (fc/4)*k steps.  Step s uses A[ic0/4*k + s][kk][m0 + 16r + l16], rows 4*(s/k)..+3 of the
        // staged block and the twiddle of tap a = s % k.
        const int ST = (fc >> 2) * k;
        const size_t jstride = (size_t)4 * Mp;
        const float2* Ab = Ap + ((size_t)(ic0 >> 2) * k * 4 + kk) * Mp + m0 + l16;
        const float2* Xw = Xs + kk * NW + cw0 + l16;

        // right-operand pipeline state: (i4n, an) = block row and tap of the step being prepared
        int i4n = 0, an = 0;
        int tix[CTW];
        float2 bn[CTW];             // prepared right operand
        float bsn[CTW];             // its real + imaginary part
#pragma unroll
        for (int c = 0; c < CTW; ++c) tix[c] = 0;

        // prepare the operand of the step (i4n, an) into bn/bsn, then advance the state by one step
#define ZNNI_MAC_PREP()                                                                                   \
    {                                                                                                     \
        const float2* xr_ = Xw + i4n * 4 * NW;                                                            \
        _Pragma("unroll") for (int c = 0; c < CTW; ++c) {                                                 \
            const float2 x_ = xr_[c * 16];                                                                \
            const float2 t_ = tws[tix[c]];                                                                \
            bn[c] = make_float2(x_.x * t_.x - x_.y * t_.y, x_.x * t_.y + x_.y * t_.x);                    \
            bsn[c] = bn[c].x + bn[c].y;                                                                   \
        }                                                                                                 \
        const bool wrap_ = (an + 1 == k);                                                                 \
        an = wrap_ ? 0 : an + 1;                                                                          \
        i4n = wrap_ ? min(i4n + 1, (fc >> 2) - 1) : i4n;                                                  \
        _Pragma("unroll") for (int c = 0; c < CTW; ++c) {                                                 \
            int t_ = tix[c] + oxs[c];                                                                     \
            t_ = t_ >= N ? t_ - N : t_;                                                                   \
            tix[c] = wrap_ ? 0 : t_;                                                                      \
        }                                                                                                 \
    }
        // one step: consume AR (A operand registers of this step) and the prepared right operand, prepare the
        // next right operand.  MK: 1 for real steps, 0 for the surplus steps of a masked group.
#define ZNNI_MAC_STEP(AR, MASKED, MK)                                                                     \
    {                                                                                                     \
        float2 b_[CTW]; float bs_[CTW];                                                                   \
        _Pragma("unroll") for (int c = 0; c < CTW; ++c) { b_[c] = bn[c]; bs_[c] = bsn[c]; }               \
        float ax_[RTW], ay_[RTW], as_[RTW];                                                               \
        _Pragma("unroll") for (int r = 0; r < RTW; ++r) {                                                 \
            ax_[r] = MASKED ? AR[r].x * (MK) : AR[r].x;                                                   \
            ay_[r] = MASKED ? AR[r].y * (MK) : AR[r].y;                                                   \
            as_[r] = ax_[r] + ay_[r];                                                                     \
        }                                                                                                 \
        ZNNI_MAC_PREP()                                                                                   \
        _Pragma("unroll") for (int c = 0; c < CTW; ++c) {                                                 \
            _Pragma("unroll") for (int r = 0; r < RTW; ++r) {                                             \
                p1[r][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(ax_[r], b_[c].x, p1[r][c], 0, 0, 0);      \
                p2[r][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(ay_[r], b_[c].y, p2[r][c], 0, 0, 0);      \
                p3[r][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(as_[r], bs_[c], p3[r][c], 0, 0, 0);       \
            }                                                                                             \
        }                                                                                                 \
        __builtin_amdgcn_sched_barrier(0);                                                                \
    }
        // a group of four steps starting at step S0: request the A operands of the following group into NXT
        // (they get four steps to arrive), then run the four steps on CUR
#define ZNNI_MAC_GROUP(CUR, NXT, S0, MASKED)                                                              \
    {                                                                                                     \
        const float2* an_ = Ab + (size_t)((S0) + 4) * jstride;                                            \
        _Pragma("unroll") for (int q = 0; q < 4; ++q)                                                     \
            _Pragma("unroll") for (int r = 0; r < RTW; ++r) NXT[q][r] = an_[(size_t)q * jstride + r * 16];\
        __builtin_amdgcn_sched_barrier(0);                                                                \
        ZNNI_MAC_STEP(CUR[0], MASKED, 1.f)                                                                \
        ZNNI_MAC_STEP(CUR[1], MASKED, ((S0) + 1 < ST ? 1.f : 0.f))                                        \
        ZNNI_MAC_STEP(CUR[2], MASKED, ((S0) + 2 < ST ? 1.f : 0.f))                                        \
        ZNNI_MAC_STEP(CUR[3], MASKED, ((S0) + 3 < ST ? 1.f : 0.f))                                        \
    }
        float2 ga[4][RTW], gb[4][RTW];
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int r = 0; r < RTW; ++r) ga[q][r] = Ab[(size_t)q * jstride + r * 16];
        ZNNI_MAC_PREP()                             // operand of step 0
        int s = 0;
        for (; s + 8 <= ST; s += 8) {
            ZNNI_MAC_GROUP(ga, gb, s, false)
            ZNNI_MAC_GROUP(gb, ga, s + 4, false)
        }
        // 0..7 steps left.  Requests past the last step read the following pencil or the zeroed padding
        // behind A; surplus steps of a masked group multiply such values by zero.
        if (ST - s >= 4) {
            ZNNI_MAC_GROUP(ga, gb, s, false)
            s += 4;
            if (s < ST) ZNNI_MAC_GROUP(gb, ga, s, true)
        } else if (s < ST) {
            ZNNI_MAC_GROUP(ga, gb, s, true)
        }
#undef ZNNI_MAC_GROUP
#undef ZNNI_MAC_STEP
#undef ZNNI_MAC_PREP
    }
    mac_store<RTW, CTW>(w, p1, p2, p3, N, fo, accumulate);
}

// One launch for all column blocks of all pencils: pieces [0, n2*nmblk) of a pencil are 128-wide blocks, the rest
// 64-wide blocks behind them.  WIDE = false leaves the 128-wide path out (row blocks too tall for it).
template <int RTW, bool WIDE>
__global__ __launch_bounds__(256, RTW * (WIDE ? 2 : 1) <= 3 ? 3 : 2)
void k_mac_mfma(const float2* __restrict__ Xt, const float2* __restrict__ A, float2* __restrict__ Yt,
                const float2* __restrict__ twg, int N, int S, int f, int fo, int k, int fp, int Mp, int FC, int n2,
                int n1, int nmblk, int npencils, int accumulate)
{
    extern __shared__ float2 lds[];
    int pencil, sub;
    if (!mac_block((n2 + n1) * nmblk, npencils, pencil, sub)) return;
    if constexpr (WIDE) {
        if (sub < n2 * nmblk) {
            mac_body<RTW, 2>(lds, Xt, A, Yt, twg, N, S, f, fo, k, fp, Mp, FC, 0, n2, pencil, sub, accumulate);
            return;
        }
    }
    mac_body<RTW, 1>(lds, Xt, A, Yt, twg, N, S, f, fo, k, fp, Mp, FC, n2 * 128, n1, pencil, sub - n2 * nmblk,
                     accumulate);
}

#define ZNNI_LAUNCH_CHECK()                         \
    do {                                            \
        if (hipGetLastError() != hipSuccess) return ZNNI_ERR_HIP; \
    } while (0)

znni_status launch_kernel_prep(const LayerPlan& L, const float* w, size_t wj_stride, hipStream_t st)
{
    const Dims& d = L.d;
    const int per = d.kx * L.fp * L.Mp;
    const int per1 = per * d.ky;
    k_kprep_z<<<dim3((per1 + 255) / 256, (d.zc + KPREP_OZ - 1) / KPREP_OZ), dim3(256),
                sizeof(float2) * KPREP_OZ * (size_t)std::min(d.kz, KPREP_TAPS), st>>>(
        w, L.A1, L.twz, d, L.f, L.fo, L.fp, L.Mp, wj_stride);
    ZNNI_LAUNCH_CHECK();
    if (L.xblock) return launch_kprep_yb(L, st);
    // the unnormalised transforms' factor: one per transformed axis
    const float scale = (float)(1.0 / ((L.xdirect ? 1.0 : (double)d.Nx) * d.Ny * d.Nz));
    k_kprep_y<<<dim3((per + 255) / 256, (d.Ny + KPREP_OY - 1) / KPREP_OY, d.zc), dim3(256),
                sizeof(float2) * KPREP_OY * (size_t)std::min(d.ky, KPREP_TAPS), st>>>(
        L.A1, L.A, L.twy, d.Ny, d.kx, d.ky, L.fp, L.Mp, per, scale);
    ZNNI_LAUNCH_CHECK();
    return ZNNI_OK;
}

// Tiling of the matrix-core kernel for a layer shape (host only): rows per wave RTW, row padding Mp, and the
// columns cut into blocks of 128 (two column tiles per wave) with a 64-wide remainder where that wastes less.
void plan_mac(LayerPlan* L)
{
    const int rt = (L->fo + 15) / 16;                   // 16-row tiles needed
    const int nmblk = (rt + 4) / 5;                     // at most 5 row tiles per wave
    const int RTW = (rt + nmblk - 1) / nmblk;
    L->mac_RTW = RTW;
    L->mac_nmblk = nmblk;
    L->Mp = nmblk * RTW * 16;
    const int Ct = L->S * L->d.Nx;
    // 128-wide column blocks where there is room for 2 x RTW accumulator tiles per wave; a remainder of more than 64
    // columns goes to one more of them, ragged, rather than to two 64-wide blocks
    L->mac_n2 = (RTW <= 3 && Ct > 64) ? (Ct + 63) / 128 : 0;
    L->mac_n1 = Ct > L->mac_n2 * 128 ? (Ct - L->mac_n2 * 128 + 63) / 64 : 0;
    // image-spectrum block kept in LDS: about 48 KB at most, so that three workgroups share a CU
    const int nwmax = L->mac_n2 ? 128 : 64;
    int FC = (48 * 1024) / (nwmax * (int)sizeof(float2));
    FC &= ~3;
    if (FC < 4) FC = 4;
    if (FC > L->fp) FC = L->fp;
    L->mac_FC = FC;
}

template <int RTW, bool WIDE>
static znni_status launch_mac_t(const LayerPlan& L, int accumulate, hipStream_t st)
{
    const void* fn = (const void*)k_mac_mfma<RTW, WIDE>;
    const size_t lds = sizeof(float2) * ((size_t)L.d.Nx + (size_t)L.mac_FC * (WIDE ? 128 : 64));
    if (lds > 48 * 1024 &&
        hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return ZNNI_ERR_HIP;
    const int npencils = L.d.zc * L.d.Ny;
    const int per_pencil = (L.mac_n2 + L.mac_n1) * L.mac_nmblk;
    const long long blocks = (long long)((npencils + 7) / 8) * per_pencil * 8;
    k_mac_mfma<RTW, WIDE><<<dim3((unsigned)blocks), dim3(256), lds, st>>>(
        L.buf0, L.A, L.Yt, L.twx, L.d.Nx, L.S, L.f, L.fo, L.d.kx, L.fp, L.Mp, L.mac_FC, L.mac_n2, L.mac_n1,
        L.mac_nmblk, npencils, accumulate);
    ZNNI_LAUNCH_CHECK();
    return ZNNI_OK;
}

znni_status launch_mac(const LayerPlan& L, unsigned flags, int accumulate, hipStream_t st)
{
    if (flags & ZNNI_MAC_REFERENCE) {
        k_mac_simple<<<dim3(L.d.Ny, L.d.zc), dim3(256), 0, st>>>(L.buf0, L.A, L.Yt, L.twx, L.d.Nx, L.S, L.f,
                                                                 L.fo, L.d.kx, L.fp, L.Mp, accumulate);
        ZNNI_LAUNCH_CHECK();
        return ZNNI_OK;
    }
    if (((flags & ZNNI_MAC_BATCH) && mac_batch_available(L)) ||
        (!(flags & ZNNI_MAC_SINGLE) && mac_batch_preferred(L)))
        return launch_mac_batch(L, accumulate, st);
    if (mac_k_available(L)) return launch_mac_k(L, accumulate, st);
    if (L.mac_n2 > 0) {
        switch (L.mac_RTW) {
            case 1: return launch_mac_t<1, true>(L, accumulate, st);
            case 2: return launch_mac_t<2, true>(L, accumulate, st);
            case 3: return launch_mac_t<3, true>(L, accumulate, st);
        }
        return ZNNI_ERR_SHAPE;
    }
    switch (L.mac_RTW) {
        case 1: return launch_mac_t<1, false>(L, accumulate, st);
        case 2: return launch_mac_t<2, false>(L, accumulate, st);
        case 3: return launch_mac_t<3, false>(L, accumulate, st);
        case 4: return launch_mac_t<4, false>(L, accumulate, st);
        case 5: return launch_mac_t<5, false>(L, accumulate, st);
    }
    return ZNNI_ERR_SHAPE;
}

}  // namespace znni
