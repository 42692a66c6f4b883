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
// (fp, Mp: f and fo rounded up to the matrix-core tile, 4 and 16; the padding holds zeros).
__global__ void k_kprep_y(const float2* __restrict__ A1, float2* __restrict__ A, const float2* __restrict__ tw,
                          int N, int k, int per, float scale)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;     // (a, i, j)
    const int oy = blockIdx.y, oz = blockIdx.z;
    if (idx >= per) return;
    const float2* a1 = A1 + (size_t)oz * k * per + idx;
    float2 acc = make_float2(0.f, 0.f);
    for (int b = 0; b < k; ++b) acc = cadd(acc, cmul(a1[(size_t)b * per], tw[(oy * b) % N]));
    A[((size_t)oz * N + oy) * per + idx] = cscale(acc, scale);
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
// One workgroup = one pencil x one block of NW = 16*NT*CG columns x one block of 16*RG output rows.
// Wave (rg, cg) owns a 16 x (16*NT) tile of Yt.  The fp x NW block of image spectra stays in LDS for the
// whole call (in chunks of FC input images if it does not fit); A is streamed from global memory straight
// into the matrix-core operand layout (lane l supplies A[row l%16][k-index l/16]), every wave of a row
// group reading the same values, which the vector L1 serves.
//
// blockIdx is decoded so that the workgroups sharing a pencil's A (different column blocks) and X (different
// row blocks) are neighbours on one XCD: hardware deals consecutive workgroup ids round-robin to the 8 XCDs,
// so id = 8*slot + xcd and consecutive slots of one XCD walk (column block, row block) fastest.
template <int NT, int CG>
__global__ __launch_bounds__(768) void k_mac_mfma(const float2* __restrict__ Xt, const float2* __restrict__ A,
                                                  float2* __restrict__ Yt, const float2* __restrict__ twg,
                                                  int N, int S, int f, int fo, int k, int fp, int Mp, int FC,
                                                  int RG, int ncolblk, int nmblk, int npencils)
{
    extern __shared__ float2 lds[];
    constexpr int NW = 16 * NT * CG;
    float2* tws = lds;              // [N]
    float2* Xs = lds + N;           // [FC][NW]

    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int per_pencil = ncolblk * nmblk;
    const int pencil = (slot / per_pencil) * 8 + xcd;
    if (pencil >= npencils) return;
    const int sub = slot % per_pencil;
    const int colblk = sub % ncolblk, mblk = sub / ncolblk;

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int rg = wave % RG, cg = wave / RG;
    const int l16 = lane & 15, kk = lane >> 4;
    const int Ct = S * N;                           // columns of the pencil
    const int m0 = (mblk * RG + rg) * 16;           // first output row of this wave (may be >= Mp: idle)
    const bool active = m0 < Mp;
    const int cw0 = cg * NT * 16;                   // first column of this wave inside the block
    const int colbase = colblk * NW;

    const float2* Xp = Xt + (size_t)pencil * S * f * N;
    const float2* Ap = A + (size_t)pencil * k * fp * Mp;
    float2* Yp = Yt + (size_t)pencil * S * fo * N;

    for (int q = threadIdx.x; q < N; q += blockDim.x) tws[q] = twg[q];

    int oxs[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) oxs[t] = (colbase + cw0 + t * 16 + l16) % N;

    floatx4 yr[NT], yi[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) { yr[t] = floatx4{0.f, 0.f, 0.f, 0.f}; yi[t] = yr[t]; }

    for (int ic0 = 0; ic0 < fp; ic0 += FC) {
        const int fc = min(FC, fp - ic0);           // multiple of 4
        __syncthreads();
        // ---- stage the fc x NW block of image spectra (rows beyond f and columns beyond Ct hold zeros).
        // Loads come from clamped, always valid addresses and are masked by a multiply, so the compiler keeps
        // several of them in flight instead of branching around each one.
        if ((N & 1) == 0) {
            constexpr int HW = NW / 2;              // 16-byte units per row
#pragma unroll 4
            for (int e = threadIdx.x; e < fc * HW; e += blockDim.x) {
                const int i = e / HW, c = (e - i * HW) * 2;
                const int gi = ic0 + i, col = colbase + c;
                const float mk = (gi < f && col < Ct) ? 1.f : 0.f;
                const int colc = min(col, Ct - 2), gic = min(gi, f - 1);
                const int sI = colc / N, ox = colc - sI * N;
                const float4 v = *reinterpret_cast<const float4*>(Xp + (size_t)(sI * f + gic) * N + ox);
                *reinterpret_cast<float4*>(Xs + i * NW + c) = make_float4(v.x * mk, v.y * mk, v.z * mk, v.w * mk);
            }
        } else {
            for (int e = threadIdx.x; e < fc * NW; e += blockDim.x) {
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
        __syncthreads();
        if (!active) continue;

        // ---- k * fc/4 matrix-core steps; step (a, j) uses A[a][ic0 + 4j + kk][m0 + l16].  The A operand of
        // step s+4 is requested while step s computes (ring of 4), far enough ahead to cover an HBM miss.
        const int nst = fc >> 2, ST = k * nst;
        const size_t jstride = (size_t)4 * Mp;
        const size_t awrap = (size_t)fp * Mp - (size_t)nst * jstride;      // from the end of one a to the next
        const float2* pp = Ap + (size_t)(ic0 + kk) * Mp + m0 + l16;        // prefetch cursor
        int pj = 0, sp = 0;
        float2 ring[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            ring[d] = make_float2(0.f, 0.f);
            if (sp < ST) {
                ring[d] = *pp;
                pp += jstride; ++sp;
                if (++pj == nst) { pj = 0; pp += awrap; }
            }
        }
        floatx4 p1[NT], p2[NT], p3[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) { p1[t] = floatx4{0.f, 0.f, 0.f, 0.f}; p2[t] = p1[t]; p3[t] = p1[t]; }
        const float2* Xw = Xs + kk * NW + cw0 + l16;
        int cj = 0, ca = 0;
        for (int s0 = 0; s0 < ST; s0 += 4) {
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                if (s0 + d < ST) {
                    const float2 ac = ring[d];
                    if (sp < ST) {
                        ring[d] = *pp;
                        pp += jstride; ++sp;
                        if (++pj == nst) { pj = 0; pp += awrap; }
                    }
                    const float as = ac.x + ac.y;
                    const float2* xr = Xw + cj * 4 * NW;
#pragma unroll
                    for (int t = 0; t < NT; ++t) {
                        const float2 xv = xr[t * 16];
                        p1[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(ac.x, xv.x, p1[t], 0, 0, 0);
                        p2[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(ac.y, xv.y, p2[t], 0, 0, 0);
                        p3[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(as, xv.x + xv.y, p3[t], 0, 0, 0);
                    }
                    if (++cj == nst) {
                        // Yt += T[a*ox] * (P1-P2, P3-P1-P2); accumulator element r of lane l is row 4*(l/16)+r,
                        // column l%16
#pragma unroll
                        for (int t = 0; t < NT; ++t) {
                            const float2 T = tws[(ca * oxs[t]) % N];
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                const float pr = p1[t][r] - p2[t][r];
                                const float pi = p3[t][r] - p1[t][r] - p2[t][r];
                                yr[t][r] += T.x * pr - T.y * pi;
                                yi[t][r] += T.x * pi + T.y * pr;
                            }
                            p1[t] = floatx4{0.f, 0.f, 0.f, 0.f}; p2[t] = p1[t]; p3[t] = p1[t];
                        }
                        cj = 0; ++ca;
                    }
                }
            }
        }
    }
    if (!active) return;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int col = colbase + cw0 + t * 16 + l16;
        if (col >= Ct) continue;
        const int s = col / N, ox = col - s * N;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = m0 + 4 * kk + r;
            if (row < fo) Yp[(size_t)(s * fo + row) * N + ox] = make_float2(yr[t][r], yi[t][r]);
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
    k_kprep_y<<<dim3((per + 255) / 256, L.N, L.zc), dim3(256), 0, st>>>(L.A1, L.A, L.tw, L.N, L.k, per, scale);
    ZNNI_LAUNCH_CHECK();
    return ZNNI_OK;
}

// Tiling of the matrix-core kernel for a layer shape (host only).
void plan_mac(LayerPlan* L)
{
    const int Ct = L->S * L->N;
    static const int cand[6][2] = {{5, 2}, {4, 2}, {5, 1}, {4, 1}, {2, 1}, {1, 1}};   // (NT, CG), widest first
    int best = 0;
    long best_waste = -1;
    for (int c = 0; c < 6; ++c) {
        const int NW = 16 * cand[c][0] * cand[c][1];
        const long waste = (long)((Ct + NW - 1) / NW) * NW - Ct;
        if (best_waste < 0 || waste < best_waste) { best = c; best_waste = waste; }
    }
    L->mac_NT = cand[best][0];
    L->mac_CG = cand[best][1];
    const int NW = 16 * L->mac_NT * L->mac_CG;
    L->mac_ncolblk = (Ct + NW - 1) / NW;
    const int rt = L->Mp / 16;
    const int rgmax = 12 / L->mac_CG;
    L->mac_RG = rt < rgmax ? rt : rgmax;
    L->mac_nmblk = (rt + L->mac_RG - 1) / L->mac_RG;
    // image-spectrum block kept in LDS: at most ~64 KB so two workgroups share a CU
    int FC = (64 * 1024) / (NW * (int)sizeof(float2));
    FC &= ~3;
    if (FC < 4) FC = 4;
    if (FC > L->fp) FC = L->fp;
    L->mac_FC = FC;
    L->mac_lds = sizeof(float2) * ((size_t)L->N + (size_t)FC * NW);
}

template <int NT, int CG>
static znni_status launch_mac_nt(const LayerPlan& L, hipStream_t st)
{
    const void* fn = (const void*)k_mac_mfma<NT, CG>;
    if (L.mac_lds > 48 * 1024 &&
        hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)L.mac_lds) != hipSuccess)
        return ZNNI_ERR_HIP;
    const int npencils = L.zc * L.N;
    const int per_pencil = L.mac_ncolblk * L.mac_nmblk;
    const long long blocks = (long long)((npencils + 7) / 8) * per_pencil * 8;
    k_mac_mfma<NT, CG><<<dim3((unsigned)blocks), dim3(64 * L.mac_RG * CG), L.mac_lds, st>>>(
        L.buf0, L.A, L.buf1, L.tw, L.N, L.S, L.f, L.fo, L.k, L.fp, L.Mp, L.mac_FC, L.mac_RG,
        L.mac_ncolblk, L.mac_nmblk, npencils);
    ZNNI_LAUNCH_CHECK();
    return ZNNI_OK;
}

znni_status launch_mac(const LayerPlan& L, unsigned flags, hipStream_t st)
{
    if (flags & ZNNI_MAC_REFERENCE) {
        k_mac_simple<<<dim3(L.N, L.zc), dim3(256), 0, st>>>(L.buf0, L.A, L.buf1, L.tw, L.N, L.S, L.f, L.fo, L.k,
                                                            L.fp, L.Mp);
        ZNNI_LAUNCH_CHECK();
        return ZNNI_OK;
    }
    switch (L.mac_NT * 10 + L.mac_CG) {
        case 52: return launch_mac_nt<5, 2>(L, st);
        case 42: return launch_mac_nt<4, 2>(L, st);
        case 51: return launch_mac_nt<5, 1>(L, st);
        case 41: return launch_mac_nt<4, 1>(L, st);
        case 21: return launch_mac_nt<2, 1>(L, st);
        default: return launch_mac_nt<1, 1>(L, st);
    }
}

}  // namespace znni
