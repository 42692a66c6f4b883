// mac_common.h -- pieces shared by the matrix-core multiply-accumulate kernels (mac.hip, mac_k.hip).
#pragma once
#include "znni_internal.h"

namespace znni {

typedef float floatx4 __attribute__((ext_vector_type(4)));

// Which part of the output a workgroup and a wave own.
//
// One workgroup = 4 waves = one pencil x one block of NW = 64*CTW columns x one block of 16*RTW output rows.
// Four waves per workgroup put exactly one wave on each of the CU's four SIMDs, which keeps the four matrix
// cores evenly loaded however many workgroups share the CU.  Wave w owns the RTW x CTW tiles (16x16 each) of
// all RTW row tiles in its own 16*CTW columns.
//
// blockIdx is decoded so that the workgroups sharing a pencil's A (different column blocks) and X (different
// row blocks) are neighbours on one XCD: hardware deals consecutive workgroup ids round-robin to the 8 XCDs,
// so id = 8*slot + xcd and consecutive slots of one XCD walk (column block, row block) fastest.  One launch
// covers every column block of every pencil: the 128-wide blocks (two column tiles per wave) and the 64-wide
// blocks that take the remaining columns run as two code paths of the same kernel, so a pencil's A is fetched
// from HBM once and there is no second launch with its own ramp-up and tail.
struct MacWork {
    int pencil, colbase, m0, cw0, l16, kk, Ct;
    const float2* Xp;
    const float2* Ap;
    float2* Yp;
};

// Which pencil this workgroup works on and which of the pencil's (n2 + n1) * nmblk pieces; false = none.
__device__ __forceinline__ bool mac_block(int per_pencil, int npencils, int& pencil, int& sub)
{
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    pencil = (slot / per_pencil) * 8 + xcd;
    sub = slot % per_pencil;
    return pencil < npencils;
}

// Piece `sub` of a run of ncolblk column blocks of width 64*CTW starting at column col0, times nmblk row blocks.
template <int RTW, int CTW>
__device__ __forceinline__ void mac_decode(MacWork& w, const float2* Xt, const float2* A, float2* Yt, int N,
                                           int S, int f, int fo, int k, int fp, int Mp, int col0, int ncolblk,
                                           int pencil, int sub)
{
    w.pencil = pencil;
    const int colblk = sub % ncolblk, mblk = sub / ncolblk;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    w.l16 = lane & 15;
    w.kk = lane >> 4;
    w.Ct = S * N;                                   // columns of the pencil
    w.m0 = mblk * RTW * 16;                         // first output row of the block (Mp is a multiple of 16*RTW)
    w.cw0 = wave * CTW * 16;                        // first column of this wave inside the block
    w.colbase = col0 + colblk * 64 * CTW;
    w.Xp = Xt + (size_t)w.pencil * S * f * N;
    w.Ap = A + (size_t)w.pencil * k * fp * Mp;
    w.Yp = Yt + (size_t)w.pencil * S * fo * N;
}

// Stage rows ic0..ic0+fc of the pencil's image spectra, columns colbase..colbase+NW, into Xs[fc][NW]
// (rows beyond f and columns beyond Ct hold zeros).  Loads come from clamped, always valid addresses and are
// masked by a multiply, so the compiler keeps several of them in flight instead of branching around each one.
// Every thread of the 256-thread block takes part; the caller puts barriers around the call.
template <int NW>
__device__ __forceinline__ void mac_stage_x(float2* Xs, const MacWork& w, int ic0, int fc, int f, int N)
{
    if ((N & 1) == 0) {
        constexpr int HW = NW / 2;                  // 16-byte units per row
#pragma unroll 4
        for (int e = threadIdx.x; e < fc * HW; e += 256) {
            const int i = e / HW, c = (e - i * HW) * 2;
            const int gi = ic0 + i, col = w.colbase + c;
            const float mk = (gi < f && col < w.Ct) ? 1.f : 0.f;
            const int colc = min(col, w.Ct - 2), gic = min(gi, f - 1);
            const int sI = colc / N, ox = colc - sI * N;
            const float4 v = *reinterpret_cast<const float4*>(w.Xp + (size_t)(sI * f + gic) * N + ox);
            *reinterpret_cast<float4*>(Xs + i * NW + c) = make_float4(v.x * mk, v.y * mk, v.z * mk, v.w * mk);
        }
    } else {
        for (int e = threadIdx.x; e < fc * NW; e += 256) {
            const int i = e / NW, c = e - i * NW;
            const int gi = ic0 + i, col = w.colbase + c;
            float2 v = make_float2(0.f, 0.f);
            if (gi < f && col < w.Ct) {
                const int sI = col / N, ox = col - sI * N;
                v = w.Xp[(size_t)(sI * f + gi) * N + ox];
            }
            Xs[i * NW + c] = v;
        }
    }
}

// Combine the three partial products (Re = P1 - P2, Im = P3 - P1 - P2) and store the wave's tiles.
// Accumulator element e of lane l is row 4*(l/16)+e, column l%16.
// accumulate != 0: the result is added to what Yt already holds.
template <int RTW, int CTW>
__device__ __forceinline__ void mac_store(const MacWork& w, const floatx4 (&p1)[RTW][CTW],
                                          const floatx4 (&p2)[RTW][CTW], const floatx4 (&p3)[RTW][CTW], int N,
                                          int fo, int accumulate)
{
#pragma unroll
    for (int c = 0; c < CTW; ++c) {
        const int col = w.colbase + w.cw0 + c * 16 + w.l16;
        if (col >= w.Ct) continue;
        const int sI = col / N, ox = col - sI * N;
        const int row0 = w.m0 + 4 * w.kk;
        float2* y = w.Yp + (size_t)(sI * fo + row0) * N + ox;       // rows advance by N elements
#pragma unroll
        for (int r = 0; r < RTW; ++r)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float re = p1[r][c][e] - p2[r][c][e];
                float im = p3[r][c][e] - p1[r][c][e] - p2[r][c][e];
                if (row0 + r * 16 + e < fo) {
                    float2* dst = y + (size_t)(r * 16 + e) * N;
                    if (accumulate) {
                        const float2 old = *dst;
                        re += old.x;
                        im += old.y;
                    }
                    *dst = make_float2(re, im);
                }
            }
    }
}

// mac_batch.hip: the form for batches, kernel-spectrum values generated once per bin and shared by the S inputs.
bool mac_batch_available(const LayerPlan& L);      // up to 12 taps along x
bool mac_batch_preferred(const LayerPlan& L);
znni_status launch_mac_batch(const LayerPlan& L, int accumulate, hipStream_t st);

// mac_xd.hip: the form for layers whose x axis is not transformed (1 to 9 taps along x).
bool mac_xd_available(const LayerPlan& L);
znni_status launch_mac_xd(const LayerPlan& L, int accumulate, hipStream_t st);

// mac_xb.hip: the same route with the x axis transformed in overlapping blocks of eight (up to 5 taps along x):
// its own second stage of the kernel transform (launch_kprep_yb, after the z stage of mac.hip) and the bytes the
// result takes.
bool mac_xb_available(const LayerPlan& L);
size_t mac_xb_kernel_bytes(const LayerPlan& L);
znni_status launch_kprep_yb(const LayerPlan& L, hipStream_t st);
znni_status launch_mac_xb(const LayerPlan& L, int accumulate, hipStream_t st);

// mac_k.hip: kernels with the number of kernel taps known at compile time (2 to 9).
bool mac_k_available(const LayerPlan& L);
znni_status launch_mac_k(const LayerPlan& L, int accumulate, hipStream_t st);

}  // namespace znni
