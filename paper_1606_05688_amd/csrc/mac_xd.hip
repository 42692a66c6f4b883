// mac_xd.hip -- multiply-accumulate for layers whose x axis is never transformed.
//
// For one input of the batch the work of the last kernel-transform stage plus the per-bin multiply-accumulate
// (Algorithm 3, second stage; kernel transform pruned as in Section III-A) is, per (oz, oy) pencil,
//
//     Yt[j][ox] = sum_{(i,a)} A(a,i,j) * exp(-2 pi i a ox / Nx) * Xt[i][ox],
//
// a contraction of length f*kx per bin.  The inverse x transform of that product, kept on the valid outputs
// xo = 0 .. nx-kx (Section III-B), is exactly the kx-tap valid convolution along x
//
//     Yd[j][xo] = sum_{(i,a)} A(a,i,j) * X2[i][xo + kx-1 - a],
//
// where X2 is the image transformed along z and y only: the same contraction length per output, with no x
// transform on either side and no twiddle products.  So when every kernel-spectrum value would be used once
// (few inputs per batch) the x axis is never transformed: the forward x pass, the inverse x pass and the tensors
// between them disappear, and the right operand of the matrix product is the image row itself, read at kx
// shifted offsets.  (With many inputs per batch a kernel-spectrum value generated once per bin serves them all,
// and the fully transformed route of mac_batch.hip does less work.)
//
// Layouts: X2[img][oz][oy][x < ldx] as the forward y pass leaves it, A[oz][oy][i/4][a][i%4][j<Mp] scaled by
// 1/(Ny Nz), Yd[imgo][oz][oy][xo < ldxo], which the inverse y pass reads with a transposing load.
//
// Work split, operand layout and the three-real-products scheme are those of the kernels in mac_k.hip; the
// number of taps is a compile-time constant (1 to 9).
#include "mac_common.h"

namespace znni {

struct XdArgs {
    const float2* X2;
    const float2* A;
    float2* Yd;
    size_t ximg, yimg;          // elements between the rows of consecutive images in X2 / Yd
    size_t xpen, ypen;          // elements between the rows of pencils (oz, oy) and (oz + 1, oy)
    int S, f, fo, fp, Mp, nox, ldx, ldxo, Ny;
    int n2, n1, col1, nmblk, npencils, accumulate;
};

// Both operands of an iteration (four input images, all K taps) are requested one iteration ahead.  Where the
// registers allow, into the other of two register sets, all requests at the top of the iteration (TWO_SETS);
// otherwise into the registers a tap has just released, tap by tap.  The first form is the faster one where it fits
// 256 registers: this kernel runs best with two waves per SIMD (a single wave can keep a matrix core busy; with
// three or four resident waves the same instruction stream was measured up to 1.5 times slower), so registers are
// not what limits it.
template <int RTW, int CTW, int K>
constexpr bool mac_xd_two_sets() { return 12 * RTW * CTW + 4 * K * (RTW + CTW) + 30 <= 250; }

template <int RTW, int CTW, int K>
__device__ __forceinline__ void mac_xd_body(const XdArgs& g, int col0, int ncolblk, int pencil, int sub)
{
    const int colblk = sub % ncolblk, mblk = sub / ncolblk;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int l16 = lane & 15, kk = lane >> 4;
    const int Ct = g.S * g.nox;                              // columns of the pencil: (input of the batch, xo)
    const int m0 = mblk * RTW * 16;
    const int colw = col0 + colblk * 64 * CTW + wave * CTW * 16;     // first column of this wave
    const int f = g.f, Mp = g.Mp;
    const int poz = pencil / g.Ny, poy = pencil - poz * g.Ny;

    floatx4 p1[RTW][CTW], p2[RTW][CTW], p3[RTW][CTW];
#pragma unroll
    for (int r = 0; r < RTW; ++r)
#pragma unroll
        for (int c = 0; c < CTW; ++c) {
            p1[r][c] = floatx4{0.f, 0.f, 0.f, 0.f}; p2[r][c] = p1[r][c]; p3[r][c] = p1[r][c];
        }

    const size_t jstride = (size_t)4 * Mp;              // one step (one tap of one group of four images)
    const size_t istride = (size_t)K * jstride;         // one iteration
    const int nI = g.fp >> 2;
    const float2* Ab = g.A + (size_t)pencil * K * g.fp * Mp + (size_t)kk * Mp + m0 + l16;
    // Lane (kk, l16) supplies, for column tile c and tap a, X2[4*I4 + kk][xo + K-1 - a]: Xc[c] points at x = xo + K-1
    // of row 0 of the lane's input, the taps are constant offsets below it.  Columns beyond Ct are clamped (never
    // stored), rows beyond f are clamped to the last one (their A operands are zero).
    const float2* Xc[CTW];
#pragma unroll
    for (int c = 0; c < CTW; ++c) {
        const int col = min(colw + c * 16 + l16, Ct - 1);
        const int sI = g.S == 1 ? 0 : col / g.nox, xo = col - sI * g.nox;
        Xc[c] = g.X2 + (size_t)sI * f * g.ximg + (size_t)poz * g.xpen + (size_t)poy * g.ldx + xo + (K - 1);
    }
    // Row offset of the group of four images being requested; group 0 first.  Only the last group can hold rows
    // beyond f, so all steps but the one onto the last group are the same for every lane.
    size_t xrow = (size_t)min(kk, f - 1) * g.ximg;
    const size_t xstep = (size_t)4 * g.ximg;
    const size_t xlast = nI >= 2 ? (size_t)(min(4 * (nI - 1) + kk, f - 1) - (4 * (nI - 2) + kk)) * g.ximg : 0;

    // the 3 * RTW * CTW matrix instructions of one tap: three real products per complex one
#define ZNNI_XD_TAP(GG, XX)                                                                                \
    {                                                                                                      \
        float bs_[CTW], as_[RTW];                                                                          \
        _Pragma("unroll") for (int c = 0; c < CTW; ++c) bs_[c] = XX[c].x + XX[c].y;                        \
        _Pragma("unroll") for (int r = 0; r < RTW; ++r) as_[r] = GG[r].x + GG[r].y;                        \
        _Pragma("unroll") for (int r = 0; r < RTW; ++r)                                                    \
            _Pragma("unroll") for (int c = 0; c < CTW; ++c) {                                              \
                p1[r][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(GG[r].x, XX[c].x, p1[r][c], 0, 0, 0);      \
                p2[r][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(GG[r].y, XX[c].y, p2[r][c], 0, 0, 0);      \
                p3[r][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(as_[r], bs_[c], p3[r][c], 0, 0, 0);        \
            }                                                                                              \
    }

    if constexpr (mac_xd_two_sets<RTW, CTW, K>()) {
        float2 Ga[K][RTW], Gb[K][RTW], Xa[K][CTW], Xb[K][CTW];
#pragma unroll
        for (int a = 0; a < K; ++a) {
#pragma unroll
            for (int r = 0; r < RTW; ++r) Ga[a][r] = Ab[(size_t)a * jstride + r * 16];
#pragma unroll
            for (int c = 0; c < CTW; ++c) Xa[a][c] = (Xc[c] + xrow)[-a];
        }
        // One iteration on the operands in (CG, CX) while those of the following one travel into (NG, NX); past the
        // last iteration the A requests read the next pencil or the zeroed padding behind A, the image requests
        // the last group again, and the values are never used.
#define ZNNI_XD_ITER(CG, NG, CX, NX, I4)                                                                   \
    {                                                                                                      \
        const float2* an_ = Ab + (size_t)((I4) + 1) * istride;                                             \
        xrow += (I4) + 2 < nI ? xstep : ((I4) + 2 == nI ? xlast : 0);                                      \
        _Pragma("unroll") for (int a = 0; a < K; ++a) {                                                    \
            _Pragma("unroll") for (int r = 0; r < RTW; ++r) NG[a][r] = an_[(size_t)a * jstride + r * 16];  \
            _Pragma("unroll") for (int c = 0; c < CTW; ++c) NX[a][c] = (Xc[c] + xrow)[-a];                 \
        }                                                                                                  \
        __builtin_amdgcn_sched_barrier(0);                                                                 \
        __builtin_amdgcn_iglp_opt(0);       /* interleave the additions with the matrix instructions */    \
        _Pragma("unroll") for (int a = 0; a < K; ++a) ZNNI_XD_TAP(CG[a], CX[a])                            \
        __builtin_amdgcn_sched_barrier(0);                                                                 \
    }
        int i4 = 0;
        for (; i4 + 2 <= nI; i4 += 2) {
            ZNNI_XD_ITER(Ga, Gb, Xa, Xb, i4)
            ZNNI_XD_ITER(Gb, Ga, Xb, Xa, i4 + 1)
        }
        if (i4 < nI) ZNNI_XD_ITER(Ga, Gb, Xa, Xb, i4)
#undef ZNNI_XD_ITER
    } else {
        // One register set: the operands of tap a of the following iteration are requested right after tap a of
        // this one has been issued, into the registers it has just released.  The requests are issued in the same
        // order in the prologue as in the loop (tap by tap, A operands then image values), so that the wait for
        // tap a's operands can leave everything requested after them in flight.
        float2 G[K][RTW], X[K][CTW];
#pragma unroll
        for (int a = 0; a < K; ++a) {
#pragma unroll
            for (int r = 0; r < RTW; ++r) G[a][r] = Ab[(size_t)a * jstride + r * 16];
#pragma unroll
            for (int c = 0; c < CTW; ++c) X[a][c] = (Xc[c] + xrow)[-a];
            __builtin_amdgcn_sched_barrier(0);
        }
        for (int i4 = 0; i4 < nI; ++i4) {
            const float2* an = Ab + (size_t)(i4 + 1) * istride;
            xrow += i4 + 2 < nI ? xstep : (i4 + 2 == nI ? xlast : 0);
#pragma unroll
            for (int a = 0; a < K; ++a) {
                __builtin_amdgcn_iglp_opt(0);
                ZNNI_XD_TAP(G[a], X[a])
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int r = 0; r < RTW; ++r) G[a][r] = an[(size_t)a * jstride + r * 16];
#pragma unroll
                for (int c = 0; c < CTW; ++c) X[a][c] = (Xc[c] + xrow)[-a];
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
#undef ZNNI_XD_TAP

    // Combine the three partial products (Re = P1 - P2, Im = P3 - P1 - P2) and store.  Accumulator element e of
    // lane l is row 4*(l/16)+e, column l%16: 16 neighbouring lanes write 128 contiguous bytes of a row of Yd.
#pragma unroll
    for (int c = 0; c < CTW; ++c) {
        const int col = colw + c * 16 + l16;
        if (col >= Ct) continue;
        const int sI = g.S == 1 ? 0 : col / g.nox, xo = col - sI * g.nox;
        const int row0 = m0 + 4 * kk;
        float2* y = g.Yd + (size_t)(sI * g.fo + row0) * g.yimg + (size_t)poz * g.ypen + (size_t)poy * g.ldxo + xo;
#pragma unroll
        for (int r = 0; r < RTW; ++r)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float re = p1[r][c][e] - p2[r][c][e];
                float im = p3[r][c][e] - p1[r][c][e] - p2[r][c][e];
                if (row0 + r * 16 + e < g.fo) {
                    float2* dst = y + (size_t)(r * 16 + e) * g.yimg;
                    if (g.accumulate) {
                        const float2 old = *dst;
                        re += old.x;
                        im += old.y;
                    }
                    *dst = make_float2(re, im);
                }
            }
    }
}

// Register budget: two waves per SIMD (up to 256 registers) for the tiles that are bound by the matrix cores;
// the small tiles of narrow layers are bound by memory and keep more waves in flight.
template <int RTW, int K, bool WIDE>
constexpr int mac_xd_min_blocks()
{
    return (RTW >= 3 || (WIDE && RTW >= 2)) ? 2 : 3;
}

// One launch for all of a layer's column blocks: pieces [0, n2*nmblk) of a pencil are 128-wide blocks, the rest
// 64-wide blocks behind them.  WIDE = false leaves the 128-wide path out (row blocks too tall for it).
template <int RTW, int K, bool WIDE>
__global__ __launch_bounds__(256, (mac_xd_min_blocks<RTW, K, WIDE>()))
void k_mac_xd(XdArgs g)
{
    int pencil, sub;
    if (!mac_block((g.n2 + g.n1) * g.nmblk, g.npencils, pencil, sub)) return;
    if constexpr (WIDE) {
        if (sub < g.n2 * g.nmblk) {
            mac_xd_body<RTW, 2, K>(g, 0, g.n2, pencil, sub);
            return;
        }
    }
    mac_xd_body<RTW, 1, K>(g, g.col1, g.n1, pencil, sub - g.n2 * g.nmblk);
}

bool mac_xd_available(const LayerPlan& L)
{
    const int k = L.d.kx;
    return k >= 1 && k <= 9 && !(k == 9 && L.mac_RTW == 5);
}

template <int RTW, int K, bool WIDE>
static znni_status launch_xd(const LayerPlan& L, int accumulate, hipStream_t st)
{
    const Dims& d = L.d;
    XdArgs g;
    g.X2 = L.buf1; g.A = L.A; g.Yd = L.Yt;
    g.ximg = (size_t)d.x2i * d.ldx; g.xpen = (size_t)d.x2o * d.ldx;
    g.yimg = (size_t)d.ydi * d.ldxo; g.ypen = (size_t)d.ydo * d.ldxo;
    g.Ny = d.Ny;
    g.S = L.S; g.f = L.f; g.fo = L.fo; g.fp = L.fp; g.Mp = L.Mp;
    g.nox = d.nox; g.ldx = d.ldx; g.ldxo = d.ldxo;
    // columns (input of the batch, xo): blocks of 128 where the row block leaves room, a 64-wide remainder
    const int Ct = L.S * d.nox;
    // (a remainder of more than 64 columns goes to one more 128-wide block, ragged, rather than to two 64-wide ones:
    // the same column slots, half the reads of the kernel transforms)
    g.n2 = WIDE ? (Ct + 63) / 128 : 0;
    g.n1 = Ct > g.n2 * 128 ? (Ct - g.n2 * 128 + 63) / 64 : 0;
    g.col1 = g.n2 * 128;
    g.nmblk = L.mac_nmblk;
    g.npencils = d.zc * d.Ny;
    g.accumulate = accumulate;
    const int per_pencil = (g.n2 + g.n1) * g.nmblk;
    const long long blocks = (long long)((g.npencils + 7) / 8) * per_pencil * 8;
    k_mac_xd<RTW, K, WIDE><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(g);
    if (hipGetLastError() != hipSuccess) return ZNNI_ERR_HIP;
    return ZNNI_OK;
}

template <int K>
static znni_status launch_xd_tiles(const LayerPlan& L, int accumulate, hipStream_t st)
{
    const bool wide = L.mac_RTW <= 3 && L.S * L.d.nox > 64;
    if (wide) {
        switch (L.mac_RTW) {
            case 1: return launch_xd<1, K, true>(L, accumulate, st);
            case 2: return launch_xd<2, K, true>(L, accumulate, st);
            case 3: return launch_xd<3, K, true>(L, accumulate, st);
        }
    }
    switch (L.mac_RTW) {
        case 1: return launch_xd<1, K, false>(L, accumulate, st);
        case 2: return launch_xd<2, K, false>(L, accumulate, st);
        case 3: return launch_xd<3, K, false>(L, accumulate, st);
        case 4: return launch_xd<4, K, false>(L, accumulate, st);
        case 5: return launch_xd<5, K, false>(L, accumulate, st);
    }
    return ZNNI_ERR_SHAPE;
}

znni_status launch_mac_xd(const LayerPlan& L, int accumulate, hipStream_t st)
{
    if (!mac_xd_available(L)) return ZNNI_ERR_UNSUPPORTED_SIZE;
    switch (L.d.kx) {
        case 1: return launch_xd_tiles<1>(L, accumulate, st);
        case 2: return launch_xd_tiles<2>(L, accumulate, st);
        case 3: return launch_xd_tiles<3>(L, accumulate, st);
        case 4: return launch_xd_tiles<4>(L, accumulate, st);
        case 5: return launch_xd_tiles<5>(L, accumulate, st);
        case 6: return launch_xd_tiles<6>(L, accumulate, st);
        case 7: return launch_xd_tiles<7>(L, accumulate, st);
        case 8: return launch_xd_tiles<8>(L, accumulate, st);
        case 9: return launch_xd_tiles<9>(L, accumulate, st);
    }
    return ZNNI_ERR_SHAPE;
}

}  // namespace znni
