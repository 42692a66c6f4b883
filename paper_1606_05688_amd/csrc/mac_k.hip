// mac_k.hip -- matrix-core multiply-accumulate with the number of kernel taps K known at compile time.
//
// Same computation, data layout and work split as the general kernel in mac.hip (see there and mac_common.h):
//
//     Yt[j][col] = sum_{(i,a)} A(a,i,j) * ( T[a*ox(col)] * X[i][col] ).
//
// With K fixed, one loop iteration covers one group of four input images (i/4) and all K taps, fully unrolled:
// the K twiddles of a lane's columns live in registers for the whole kernel, the image fragment is read once per
// iteration instead of once per step (straight from global memory: no LDS, no barrier), there is no per-step
// bookkeeping, and the A operands and image fragment of the next iteration are requested, into the other of two
// register sets, before the current iteration's arithmetic.
// Every instruction a wave issues costs matrix-core time on this hardware, so per 9*K (or 18*K) matrix
// instructions the iteration carries only the 5 vector instructions per step and column tile that form the
// right operand (complex product and real+imaginary sum), RTW additions per step for the left operand's
// real+imaginary sum, and the A and image loads.
#include "mac_common.h"

namespace znni {

template <int RTW, int CTW, int K>
__device__ __forceinline__ void mac_k_body(const float2* __restrict__ Xt, const float2* __restrict__ A,
                                           float2* __restrict__ Yt, const float2* __restrict__ twg, int N, int S,
                                           int f, int fo, int fp, int Mp, int col0, int ncolblk, int pencil,
                                           int sub, int accumulate)
{
    MacWork w;
    mac_decode<RTW, CTW>(w, Xt, A, Yt, N, S, f, fo, K, fp, Mp, col0, ncolblk, pencil, sub);
    // (A wave whose columns are all padding still runs: letting it return early was measured slower, because the
    // waves of a workgroup sit on fixed SIMDs and the padding waves' SIMDs then idle while the others work.)

    // twiddles of this lane's columns, one per tap
    float2 T[K][CTW];
#pragma unroll
    for (int c = 0; c < CTW; ++c) {
        const int ox = (w.colbase + w.cw0 + c * 16 + w.l16) % N;
        int q = 0;
#pragma unroll
        for (int a = 0; a < K; ++a) {
            T[a][c] = twg[q];
            q += ox;
            q = q >= N ? q - N : q;
        }
    }

    floatx4 p1[RTW][CTW], p2[RTW][CTW], p3[RTW][CTW];
#pragma unroll
    for (int r = 0; r < RTW; ++r)
#pragma unroll
        for (int c = 0; c < CTW; ++c) {
            p1[r][c] = floatx4{0.f, 0.f, 0.f, 0.f}; p2[r][c] = p1[r][c]; p3[r][c] = p1[r][c];
        }

    const size_t jstride = (size_t)4 * Mp;              // one step (one tap of one group of four images)
    const size_t istride = (size_t)K * jstride;         // one iteration

    {
        // The image fragment of a lane -- rows 4*I4 + kk, its own CTW columns -- comes straight from global
        // memory, one iteration ahead like the A operands: no wave reads another wave's columns, so there is
        // nothing to share through LDS, and without the staging a workgroup starts its arithmetic after one
        // memory round trip and never meets a barrier.  Rows beyond f are clamped to the last one (their A
        // operands are zero); columns beyond Ct are clamped too and never stored.
        const int nI = fp >> 2;
        const float2* Ab = w.Ap + (size_t)w.kk * Mp + w.m0 + w.l16;
        const float2* Xc[CTW];
#pragma unroll
        for (int c = 0; c < CTW; ++c) {
            const int col = min(w.colbase + w.cw0 + c * 16 + w.l16, w.Ct - 1);
            const int sI = col / N, ox = col - sI * N;
            Xc[c] = w.Xp + (size_t)sI * f * N + ox;
        }

        // One iteration: image rows 4*I4..4*I4+3, all K taps, A operands in CUR.  First the A operands of the
        // following iteration are requested into NXT (past the last iteration this reads the next pencil or the
        // zeroed padding behind A; the values are never used) and the image fragment of the following
        // iteration into XN.
#define ZNNI_MAC_ITER(CUR, NXT, XC, XN, I4)                                                               \
    {                                                                                                     \
        const float2* an_ = Ab + (size_t)((I4) + 1) * istride;                                            \
        _Pragma("unroll") for (int a = 0; a < K; ++a)                                                     \
            _Pragma("unroll") for (int r = 0; r < RTW; ++r) NXT[a][r] = an_[(size_t)a * jstride + r * 16];\
        const size_t xo_ = (size_t)min(4 * min((I4) + 1, nI - 1) + w.kk, f - 1) * N;                      \
        _Pragma("unroll") for (int c = 0; c < CTW; ++c) XN[c] = Xc[c][xo_];                               \
        __builtin_amdgcn_sched_barrier(0);                                                                \
        __builtin_amdgcn_iglp_opt(0); /* interleave matrix and other instructions: 3-8 % for tall row blocks */ \
        _Pragma("unroll") for (int a = 0; a < K; ++a) {                                                   \
            float2 b_[CTW]; float bs_[CTW];                                                               \
            _Pragma("unroll") for (int c = 0; c < CTW; ++c) {                                             \
                b_[c] = a == 0 ? XC[c] /* T[0] = 1 */                                                     \
                               : make_float2(XC[c].x * T[a][c].x - XC[c].y * T[a][c].y,                   \
                                             XC[c].x * T[a][c].y + XC[c].y * T[a][c].x);                  \
                bs_[c] = b_[c].x + b_[c].y;                                                               \
            }                                                                                             \
            _Pragma("unroll") for (int r = 0; r < RTW; ++r) {                                             \
                const float as_ = CUR[a][r].x + CUR[a][r].y;                                              \
                _Pragma("unroll") for (int c = 0; c < CTW; ++c) {                                         \
                    p1[r][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(CUR[a][r].x, b_[c].x, p1[r][c], 0, 0, 0); \
                    p2[r][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(CUR[a][r].y, b_[c].y, p2[r][c], 0, 0, 0); \
                    p3[r][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(as_, bs_[c], p3[r][c], 0, 0, 0);      \
                }                                                                                         \
            }                                                                                             \
        }                                                                                                 \
        __builtin_amdgcn_sched_barrier(0);                                                                \
    }
        float2 ga[K][RTW], gb[K][RTW], xa[CTW], xb[CTW];
#pragma unroll
        for (int a = 0; a < K; ++a)
#pragma unroll
            for (int r = 0; r < RTW; ++r) ga[a][r] = Ab[(size_t)a * jstride + r * 16];
        {
            const size_t xo0 = (size_t)min(w.kk, f - 1) * N;
#pragma unroll
            for (int c = 0; c < CTW; ++c) xa[c] = Xc[c][xo0];
        }
        int i4 = 0;
        for (; i4 + 2 <= nI; i4 += 2) {
            ZNNI_MAC_ITER(ga, gb, xa, xb, i4)
            ZNNI_MAC_ITER(gb, ga, xb, xa, i4 + 1)
        }
        if (i4 < nI) ZNNI_MAC_ITER(ga, gb, xa, xb, i4)
#undef ZNNI_MAC_ITER
    }
    mac_store<RTW, CTW>(w, p1, p2, p3, N, fo, accumulate);
}

// One launch for all of a layer's column blocks: pieces [0, n2*nmblk) of a pencil are 128-wide blocks, the rest
// 64-wide blocks behind them.  WIDE = false leaves the 128-wide path out (row blocks too tall for it).
// Workgroups per CU the register allocation is held to.  Two instantiations sit a few registers above an
// occupancy step and are pushed below it: three row tiles x 5 taps, wide (171 -> 168 registers, 12 bytes of
// scratch, three waves per SIMD instead of two: 4 % faster on the 320-wide workload) and three row tiles x 2 taps,
// wide (129 -> 128, no scratch).  Wherever the step is further away the spills cost more than the occupancy
// gains (tried: 5 tiles x 5 taps, 5 x 3, 3 x 3 wide: 30 % slower).
template <int RTW, int K, bool WIDE>
constexpr int mac_k_min_blocks()
{
    if (RTW == 3 && K == 5 && WIDE) return 3;
    if (RTW == 3 && K == 2 && WIDE) return 4;
    return (RTW * (WIDE ? 2 : 1) * (K > 5 ? 2 : 1)) <= 3 ? 3 : 2;
}

template <int RTW, int K, bool WIDE>
__global__ __launch_bounds__(256, (mac_k_min_blocks<RTW, K, WIDE>()))
void k_mac_mfma_k(const float2* __restrict__ Xt, const float2* __restrict__ A, float2* __restrict__ Yt,
                  const float2* __restrict__ twg, int N, int S, int f, int fo, int fp, int Mp, int n2, int n1,
                  int col1, int nmblk, int npencils, int accumulate)
{
    int pencil, sub;
    if (!mac_block((n2 + n1) * nmblk, npencils, pencil, sub)) return;
    if constexpr (WIDE) {
        if (sub < n2 * nmblk) {
            mac_k_body<RTW, 2, K>(Xt, A, Yt, twg, N, S, f, fo, fp, Mp, 0, n2, pencil, sub, accumulate);
            return;
        }
    }
    mac_k_body<RTW, 1, K>(Xt, A, Yt, twg, N, S, f, fo, fp, Mp, col1, n1, pencil, sub - n2 * nmblk,
                          accumulate);
}

// 2 to 9 taps (the kernel sizes of the benchmarked networks); the tallest row block with 9 taps would
// spill registers and is left to the general kernel
bool mac_k_available(const LayerPlan& L)
{
    const int k = L.d.kx;
    return k >= 2 && k <= 9 && !(k == 9 && L.mac_RTW == 5);
}

template <int RTW, int K, bool WIDE>
static znni_status launch_k(const LayerPlan& L, int n2, int n1, int accumulate, hipStream_t st)
{
    const int npencils = L.d.zc * L.d.Ny;
    const int per_pencil = (n2 + n1) * L.mac_nmblk;
    const long long blocks = (long long)((npencils + 7) / 8) * per_pencil * 8;
    k_mac_mfma_k<RTW, K, WIDE><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(
        L.buf0, L.A, L.Yt, L.twx, L.d.Nx, L.S, L.f, L.fo, L.fp, L.Mp, n2, n1, L.mac_n2 * 128,
        L.mac_nmblk, npencils, accumulate);
    if (hipGetLastError() != hipSuccess) return ZNNI_ERR_HIP;
    return ZNNI_OK;
}

template <int K>
static znni_status launch_narrow(const LayerPlan& L, int accumulate, hipStream_t st)
{
    switch (L.mac_RTW) {
        case 1: return launch_k<1, K, false>(L, 0, L.mac_n1, accumulate, st);
        case 2: return launch_k<2, K, false>(L, 0, L.mac_n1, accumulate, st);
        case 3: return launch_k<3, K, false>(L, 0, L.mac_n1, accumulate, st);
        case 4: return launch_k<4, K, false>(L, 0, L.mac_n1, accumulate, st);
        case 5: return launch_k<5, K, false>(L, 0, L.mac_n1, accumulate, st);
    }
    return ZNNI_ERR_SHAPE;
}

template <int K>
static znni_status launch_tiles(const LayerPlan& L, int accumulate, hipStream_t st)
{
    if (L.mac_n2 == 0) return launch_narrow<K>(L, accumulate, st);
    // one launch for both block widths (two launches were measured 2 % faster for the multiply-accumulate at the
    // 320-wide workload, because the narrow blocks then run three to a CU; not worth a second kernel per call)
    switch (L.mac_RTW) {
        case 1: return launch_k<1, K, true>(L, L.mac_n2, L.mac_n1, accumulate, st);
        case 2: return launch_k<2, K, true>(L, L.mac_n2, L.mac_n1, accumulate, st);
        case 3: return launch_k<3, K, true>(L, L.mac_n2, L.mac_n1, accumulate, st);
    }
    return ZNNI_ERR_SHAPE;
}

znni_status launch_mac_k(const LayerPlan& L, int accumulate, hipStream_t st)
{
    switch (L.d.kx) {
        case 2: return launch_tiles<2>(L, accumulate, st);
        case 3: return launch_tiles<3>(L, accumulate, st);
        case 4: return launch_tiles<4>(L, accumulate, st);
        case 5: return launch_tiles<5>(L, accumulate, st);
        case 6: return launch_tiles<6>(L, accumulate, st);
        case 7: return launch_tiles<7>(L, accumulate, st);
        case 8: return launch_tiles<8>(L, accumulate, st);
        case 9: return launch_tiles<9>(L, accumulate, st);
    }
    return ZNNI_ERR_SHAPE;
}

}  // namespace znni
