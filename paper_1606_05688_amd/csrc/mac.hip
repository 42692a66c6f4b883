// mac.hip -- pruned kernel transform and the per-bin multiply-accumulate.
//
// Kernel side of the layer (Sections III-A and IV-B-2).  A k^3 kernel zero-padded to N^3 is transformed
// axis by axis, touching only lines that are not all zero: k^2 lines along z, then k*zc lines along y, then
// N*zc lines along x.  With k small each of these one-dimensional transforms of a k-sample line is evaluated
// directly from its k non-zero inputs.  The first two stages are stored (array A, k*N*zc values per kernel
// instead of N*N*zc); the third is evaluated where it is consumed, inside the multiply-accumulate
//
//     Yt[s][j](ox,oy,oz) = sum_i  Wt[j][i](ox,oy,oz) * Xt[s][i](ox,oy,oz),
//     Wt[j][i](ox,oy,oz) = sum_{a<k} A[oz][oy][a][i][j] * exp(-2 pi i a ox / N)
//
// which is the second stage of Algorithm 3 (multiply the f image spectra by the f kernel spectra of output
// image j, accumulate over the f products) without a stored kernel spectrum.  The 1/N^3 of the unnormalised
// transforms is folded into A.
//
// For one (oz,oy) pencil the two sums commute:
//
//     Yt[j][col] = sum_a T[a*ox(col)] * P_a[j][col],     P_a = A_a (Mp x fp)  *  X (fp x columns)
//
// with col = s*N + ox running over all images of the batch: k dense complex matrix products per pencil whose
// left operand does not depend on the column.  That is a contraction, so it runs on the matrix cores
// (v_mfma_f32_16x16x4_f32), each complex product done as three real ones:
//     P1 = Ar Xr, P2 = Ai Xi, P3 = (Ar+Ai)(Xr+Xi);  Re = P1 - P2, Im = P3 - P1 - P2.
#include "znni_internal.h"

namespace znni {

typedef float floatx4 __attribute__((ext_vector_type(4)));

// A1[oz][b][a][i<fp][j<Mp] = sum_c w[j][i][a][b][c] exp(-2 pi i oz c / N); zero where i >= f or j >= fo.
// (j fastest, so the y stage below reads and writes contiguous runs.)
__global__ void k_kprep_z(const float* __restrict__ w, float2* __restrict__ A1, const float2* __restrict__ tw,
                          int N, int f, int fo, int k, int fp, int Mp)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    const int oz = blockIdx.y;
    const int per = k * k * fp * Mp;
    if (idx >= per) return;
    const int j = idx % Mp;
    const int i = (idx / Mp) % fp;
    const int ba = idx / (Mp * fp);
    const int a = ba % k, b = ba / k;
    float2 acc = make_float2(0.f, 0.f);
    if (i < f && j < fo) {
        const float* wr = w + ((((size_t)j * f + i) * k + a) * k + b) * k;
        for (int c = 0; c < k; ++c) acc = caxpy(acc, wr[c], tw[(oz * c) % N]);
    }
    A1[(size_t)oz * per + idx] = acc;
}

// A[oz][oy][a][i<fp][j<Mp] = scale * sum_b A1[oz][b][a][i][j] exp(-2 pi i oy b / N)
// (fp, Mp: f and fo rounded up to the matrix-core tiles; the padding holds zeros).
// One thread produces KPREP_OY consecutive oy for one (a,i,j): each A1 value is loaded once and the twiddle
// index advances by b per oy, so the kernel is bound by its 8-byte stores.
constexpr int KPREP_OY = 8;
__global__ void k_kprep_y(const float2* __restrict__ A1, float2* __restrict__ A, const float2* __restrict__ tw,
                          int N, int k, int per, float scale)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;     // (a, i, j)
    const int oy0 = blockIdx.y * KPREP_OY, oz = blockIdx.z;
    if (idx >= per) return;
    const float2* a1 = A1 + (size_t)oz * k * per + idx;
    float2 acc[KPREP_OY];
#pragma unroll
    for (int o = 0; o < KPREP_OY; ++o) acc[o] = make_float2(0.f, 0.f);
    for (int b = 0; b < k; ++b) {
        const float2 v = a1[(size_t)b * per];
        int q = (int)(((long long)oy0 * b) % N);
        const int step = b % N;
#pragma unroll
        for (int o = 0; o < KPREP_OY; ++o) {
            acc[o] = cadd(acc[o], cmul(v, tw[q]));
            q += step;
            if (q >= N) q -= N;
        }
    }
    float2* d = A + ((size_t)oz * N + oy0) * per + idx;
#pragma unroll
    for (int o = 0; o < KPREP_OY; ++o)
        if (oy0 + o < N) d[(size_t)o * per] = cscale(acc[o], scale);
}

__global__ void k_zero(float2* p, size_t count)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = make_float2(0.f, 0.f);
}

// Plain multiply-accumulate, one workgroup per (oz, oy) pencil, one thread per ox.  Slow and simple; kept as
// a diagnostic path (flag ZNNI_MAC_REFERENCE) the matrix-core kernel can be compared with.
__global__ void k_mac_simple(const float2* __restrict__ Xt, const float2* __restrict__ A, float2* __restrict__ Yt,
                             const float2* __restrict__ tw, int N, int S, int f, int fo, int k, int fp, int Mp)
{
    const size_t pencil = (size_t)blockIdx.y * N + blockIdx.x;
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
                        W = cadd(W, cmul(Ap[(size_t)(a * fp + i) * Mp + j], tw[(a * ox) % N]));
                    acc = cadd(acc, cmul(W, Xp[(size_t)(s * f + i) * N + ox]));
                }
                Yp[(size_t)(s * fo + j) * N + ox] = acc;
            }
    }
}

// Matrix-core multiply-accumulate.
//
// One workgroup = 4 waves = one pencil x one block of NW = 64*CTW columns x one block of 16*RTW output rows.
// Four waves per workgroup put exactly one wave on each of the CU's four SIMDs, which keeps the four matrix
// cores evenly loaded however many workgroups share the CU.  Wave w owns the RTW x CTW tiles (16x16 each) of
// all RTW row tiles in its own 16*CTW columns.  The fp x NW block of image spectra stays in LDS for the whole
// call (in chunks of FC input images if it does not fit); A is streamed from global memory straight into the
// matrix-core operand layout (lane l supplies A[row l%16][k-index l/16]); the four waves of a workgroup read
// the same A values, which the vector L1 serves.
//
// blockIdx is decoded so that the workgroups sharing a pencil's A (different column blocks) and X (different
// row blocks) are neighbours on one XCD: hardware deals consecutive workgroup ids round-robin to the 8 XCDs,
// so id = 8*slot + xcd and consecutive slots of one XCD walk (column block, row block) fastest.
template <int RTW, int CTW, bool TAIL>
__global__ __launch_bounds__(256) void k_mac_mfma(const float2* __restrict__ Xt, const float2* __restrict__ A,
                                                  float2* __restrict__ Yt, const float2* __restrict__ twg,
                                                  int N, int S, int f, int fo, int k, int fp, int Mp, int FC,
                                                  int ncolblk, int nmblk, int npencils)
{
    extern __shared__ float2 lds[];
    constexpr int NW = 64 * CTW;
    float2* tws = lds;              // [N]
    float2* Xs = lds + N;           // [FC + pad][NW]; pad rows are read ahead (4) or, zeroed, by surplus steps (16)

    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int per_pencil = ncolblk * nmblk;
    const int pencil = (slot / per_pencil) * 8 + xcd;
    if (pencil >= npencils) return;
    const int sub = slot % per_pencil;
    const int colblk = sub % ncolblk, mblk = sub / ncolblk;

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int l16 = lane & 15, kk = lane >> 4;
    const int Ct = S * N;                           // columns of the pencil
    const int m0 = mblk * RTW * 16;                 // first output row of this block (Mp is a multiple of 16*RTW)
    const int cw0 = wave * CTW * 16;                // first column of this wave inside the block
    const int colbase = colblk * NW;

    const float2* Xp = Xt + (size_t)pencil * S * f * N;
    const float2* Ap = A + (size_t)pencil * k * fp * Mp;
    float2* Yp = Yt + (size_t)pencil * S * fo * N;

    for (int q = threadIdx.x; q < N; q += 256) tws[q] = twg[q];

    int oxs[CTW];
#pragma unroll
    for (int c = 0; c < CTW; ++c) oxs[c] = (colbase + cw0 + c * 16 + l16) % N;

    floatx4 yr[RTW][CTW], yi[RTW][CTW];
#pragma unroll
    for (int r = 0; r < RTW; ++r)
#pragma unroll
        for (int c = 0; c < CTW; ++c) { yr[r][c] = floatx4{0.f, 0.f, 0.f, 0.f}; yi[r][c] = yr[r][c]; }

    for (int ic0 = 0; ic0 < fp; ic0 += FC) {
        const int fc = min(FC, fp - ic0);           // multiple of 4
        __syncthreads();
        // ---- stage the fc x NW block of image spectra (rows beyond f and columns beyond Ct hold zeros).
        // Loads come from clamped, always valid addresses and are masked by a multiply, so the compiler keeps
        // several of them in flight instead of branching around each one.
        if ((N & 1) == 0) {
            constexpr int HW = NW / 2;              // 16-byte units per row
#pragma unroll 4
            for (int e = threadIdx.x; e < fc * HW; e += 256) {
                const int i = e / HW, c = (e - i * HW) * 2;
                const int gi = ic0 + i, col = colbase + c;
                const float mk = (gi < f && col < Ct) ? 1.f : 0.f;
                const int colc = min(col, Ct - 2), gic = min(gi, f - 1);
                const int sI = colc / N, ox = colc - sI * N;
                const float4 v = *reinterpret_cast<const float4*>(Xp + (size_t)(sI * f + gic) * N + ox);
                *reinterpret_cast<float4*>(Xs + i * NW + c) = make_float4(v.x * mk, v.y * mk, v.z * mk, v.w * mk);
            }
        } else {
            for (int e = threadIdx.x; e < fc * NW; e += 256) {
                const int i = e / NW, c = e - i * NW;
                const int gi = ic0 + i, col = colbase + c;
                float2 v = make_float2(0.f, 0.f);
                if (gi < f && col < Ct) {
                    const int sI = col / N, ox = col - sI * N;
                    v = Xp[(size_t)(sI * f + gi) * N + ox];
                }
                Xs[i * NW + c] = v;
            }
        }
        if (TAIL)       // surplus steps multiply these rows by zero; keep them finite
            for (int e = threadIdx.x; e < 16 * NW; e += 256) Xs[fc * NW + e] = make_float2(0.f, 0.f);
        __syncthreads();

        // ---- k * fc/4 matrix-core steps; step (a, j) uses A[a][ic0 + 4j + kk][m0 + 16r + l16] and rows
        // 4j..4j+3 of the staged block.  Steps run in groups of four.  At the top of a group the A operands of
        // the NEXT group (which may belong to the next a) are requested into a second register set, so they
        // have four steps of matrix-core work to arrive; the image fragments of step j+1 are read from LDS
        // while step j computes.  Addresses only ever advance by constants; the last group of an a may hold
        // surplus steps (fc/4 not a multiple of four), whose A values are real but multiplied by zero, and
        // the request issued by the very last group reads the padding that follows A in the workspace.
        const int nst = fc >> 2, ngr = (nst + 3) >> 2;
        const size_t jstride = (size_t)4 * Mp;
        const float2* Xw = Xs + kk * NW + cw0 + l16;
#define ZNNI_MAC_STEP(AR, XA, XB, MK)                                                                     \
    {                                                                                                     \
        xr += 4 * NW;                                                                                     \
        _Pragma("unroll") for (int c = 0; c < CTW; ++c) XB[c] = xr[c * 16];                               \
        float ax_[RTW], ay_[RTW], as_[RTW];                                                               \
        _Pragma("unroll") for (int r = 0; r < RTW; ++r) {                                                 \
            ax_[r] = TAIL ? AR[r].x * (MK) : AR[r].x;                                                     \
            ay_[r] = TAIL ? AR[r].y * (MK) : AR[r].y;                                                     \
            as_[r] = ax_[r] + ay_[r];                                                                     \
        }                                                                                                 \
        _Pragma("unroll") for (int c = 0; c < CTW; ++c) {                                                 \
            const float xs_ = XA[c].x + XA[c].y;                                                          \
            _Pragma("unroll") for (int r = 0; r < RTW; ++r) {                                             \
                p1[r][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(ax_[r], XA[c].x, p1[r][c], 0, 0, 0);      \
                p2[r][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(ay_[r], XA[c].y, p2[r][c], 0, 0, 0);      \
                p3[r][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(as_[r], xs_, p3[r][c], 0, 0, 0);          \
            }                                                                                             \
        }                                                                                                 \
        __builtin_amdgcn_sched_barrier(0); /* keep this step's LDS reads inside this step */              \
    }
        float2 cur[4][RTW], nxt[4][RTW];
        {
            const float2* a0p = Ap + ((size_t)ic0 + kk) * Mp + m0 + l16;
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int r = 0; r < RTW; ++r) cur[q][r] = a0p[(size_t)q * jstride + r * 16];
        }
        for (int a = 0; a < k; ++a) {
            const float2* Aa = Ap + ((size_t)a * fp + ic0 + kk) * Mp + m0 + l16;
            floatx4 p1[RTW][CTW], p2[RTW][CTW], p3[RTW][CTW];
#pragma unroll
            for (int r = 0; r < RTW; ++r)
#pragma unroll
                for (int c = 0; c < CTW; ++c) {
                    p1[r][c] = floatx4{0.f, 0.f, 0.f, 0.f}; p2[r][c] = p1[r][c]; p3[r][c] = p1[r][c];
                }
            float2 xa[CTW], xb[CTW];
            const float2* xr = Xw;
#pragma unroll
            for (int c = 0; c < CTW; ++c) xa[c] = xr[c * 16];
            for (int g = 0; g < ngr; ++g) {
                // next group: four steps further in this a, or the first four steps of the next a
                const float2* an = (g + 1 < ngr) ? Aa + (size_t)(g + 1) * 4 * jstride : Aa + (size_t)fp * Mp;
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int r = 0; r < RTW; ++r) nxt[q][r] = an[(size_t)q * jstride + r * 16];
                __builtin_amdgcn_sched_barrier(0);      // requests go out before the group's arithmetic
                const int jb = 4 * g;
                const float m1 = jb + 1 < nst ? 1.f : 0.f, m2 = jb + 2 < nst ? 1.f : 0.f,
                            m3 = jb + 3 < nst ? 1.f : 0.f;
                ZNNI_MAC_STEP(cur[0], xa, xb, 1.f)
                ZNNI_MAC_STEP(cur[1], xb, xa, m1)
                ZNNI_MAC_STEP(cur[2], xa, xb, m2)
                ZNNI_MAC_STEP(cur[3], xb, xa, m3)
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int r = 0; r < RTW; ++r) cur[q][r] = nxt[q][r];
            }
#undef ZNNI_MAC_STEP
            // Yt += T[a*ox] * (P1-P2, P3-P1-P2); accumulator element e of lane l is row 4*(l/16)+e, column l%16
#pragma unroll
            for (int c = 0; c < CTW; ++c) {
                const float2 T = tws[(a * oxs[c]) % N];
#pragma unroll
                for (int r = 0; r < RTW; ++r)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float pr = p1[r][c][e] - p2[r][c][e];
                        const float pi = p3[r][c][e] - p1[r][c][e] - p2[r][c][e];
                        yr[r][c][e] += T.x * pr - T.y * pi;
                        yi[r][c][e] += T.x * pi + T.y * pr;
                    }
            }
        }
    }
#pragma unroll
    for (int c = 0; c < CTW; ++c) {
        const int col = colbase + cw0 + c * 16 + l16;
        if (col >= Ct) continue;
        const int s = col / N, ox = col - s * N;
#pragma unroll
        for (int r = 0; r < RTW; ++r)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int row = m0 + r * 16 + 4 * kk + e;
                if (row < fo) Yp[(size_t)(s * fo + row) * N + ox] = make_float2(yr[r][c][e], yi[r][c][e]);
            }
    }
}

#define ZNNI_LAUNCH_CHECK()                         \
    do {                                            \
        if (hipGetLastError() != hipSuccess) return ZNNI_ERR_HIP; \
    } while (0)

znni_status launch_kernel_prep(const LayerPlan& L, const float* w, hipStream_t st)
{
    const int per = L.k * L.fp * L.Mp;
    const int per1 = per * L.k;
    k_kprep_z<<<dim3((per1 + 255) / 256, L.zc), dim3(256), 0, st>>>(w, L.A1, L.tw, L.N, L.f, L.fo, L.k, L.fp,
                                                                    L.Mp);
    ZNNI_LAUNCH_CHECK();
    const float scale = (float)(1.0 / ((double)L.N * L.N * L.N));
    k_kprep_y<<<dim3((per + 255) / 256, (L.N + KPREP_OY - 1) / KPREP_OY, L.zc), dim3(256), 0, st>>>(
        L.A1, L.A, L.tw, L.N, L.k, per, scale);
    ZNNI_LAUNCH_CHECK();
    // the multiply-accumulate reads a little past the last pencil (values multiplied by zero at most)
    const size_t pad = (size_t)(L.fp + 32) * L.Mp;
    k_zero<<<dim3((unsigned)((pad + 255) / 256)), dim3(256), 0, st>>>(L.A + (size_t)L.zc * L.N * per, pad);
    ZNNI_LAUNCH_CHECK();
    return ZNNI_OK;
}

// Tiling of the matrix-core kernel for a layer shape (host only): wave tile RTW x CTW, row padding Mp.
void plan_mac(LayerPlan* L)
{
    const int rt = (L->fo + 15) / 16;                   // 16-row tiles needed
    const int nmblk = (rt + 4) / 5;                     // at most 5 row tiles per wave
    const int RTW = (rt + nmblk - 1) / nmblk;
    L->mac_RTW = RTW;
    L->mac_nmblk = nmblk;
    L->Mp = nmblk * RTW * 16;
    const int Ct = L->S * L->N;
    // two column tiles per wave when the row count leaves room for the accumulators and no column is wasted
    int CTW = 1;
    if (RTW <= 3) {
        const long w1 = (long)((Ct + 63) / 64) * 64, w2 = (long)((Ct + 127) / 128) * 128;
        if (w2 <= w1) CTW = 2;
    }
    L->mac_CTW = CTW;
    const int NW = 64 * CTW;
    L->mac_ncolblk = (Ct + NW - 1) / NW;
    // image-spectrum block kept in LDS: at most ~32 KB so that several workgroups share a CU
    int FC = (32 * 1024) / (NW * (int)sizeof(float2));
    FC &= ~3;
    if (FC < 4) FC = 4;
    if (FC > L->fp) FC = L->fp;
    L->mac_FC = FC;
    L->mac_tail = ((FC >> 2) & 3) != 0 || (((L->fp % FC) >> 2) & 3) != 0;
    L->mac_lds = sizeof(float2) * ((size_t)L->N + (size_t)(FC + (L->mac_tail ? 16 : 4)) * NW);
}

template <int RTW, int CTW, bool TAIL>
static znni_status launch_mac_tt(const LayerPlan& L, hipStream_t st)
{
    const void* fn = (const void*)k_mac_mfma<RTW, CTW, TAIL>;
    if (L.mac_lds > 48 * 1024 &&
        hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)L.mac_lds) != hipSuccess)
        return ZNNI_ERR_HIP;
    const int npencils = L.zc * L.N;
    const int per_pencil = L.mac_ncolblk * L.mac_nmblk;
    const long long blocks = (long long)((npencils + 7) / 8) * per_pencil * 8;
    k_mac_mfma<RTW, CTW, TAIL><<<dim3((unsigned)blocks), dim3(256), L.mac_lds, st>>>(
        L.buf0, L.A, L.buf1, L.tw, L.N, L.S, L.f, L.fo, L.k, L.fp, L.Mp, L.mac_FC, L.mac_ncolblk, L.mac_nmblk,
        npencils);
    ZNNI_LAUNCH_CHECK();
    return ZNNI_OK;
}

template <int RTW, int CTW>
static znni_status launch_mac_t(const LayerPlan& L, hipStream_t st)
{
    return L.mac_tail ? launch_mac_tt<RTW, CTW, true>(L, st) : launch_mac_tt<RTW, CTW, false>(L, st);
}

znni_status launch_mac(const LayerPlan& L, unsigned flags, hipStream_t st)
{
    if (flags & ZNNI_MAC_REFERENCE) {
        k_mac_simple<<<dim3(L.N, L.zc), dim3(256), 0, st>>>(L.buf0, L.A, L.buf1, L.tw, L.N, L.S, L.f, L.fo, L.k,
                                                            L.fp, L.Mp);
        ZNNI_LAUNCH_CHECK();
        return ZNNI_OK;
    }
    switch (L.mac_RTW * 10 + L.mac_CTW) {
        case 11: return launch_mac_t<1, 1>(L, st);
        case 12: return launch_mac_t<1, 2>(L, st);
        case 21: return launch_mac_t<2, 1>(L, st);
        case 22: return launch_mac_t<2, 2>(L, st);
        case 31: return launch_mac_t<3, 1>(L, st);
        case 32: return launch_mac_t<3, 2>(L, st);
        case 41: return launch_mac_t<4, 1>(L, st);
        case 51: return launch_mac_t<5, 1>(L, st);
    }
    return ZNNI_ERR_SHAPE;
}

}  // namespace znni
