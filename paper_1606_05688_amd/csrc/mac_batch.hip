// mac_batch.hip -- per-bin multiply-accumulate for batches (S > 1): each kernel-spectrum value is generated once
// per bin and reused for every input of the batch.
//
//     Yt[s][j](ox) = sum_i Wt[j][i](ox) * Xt[s][i](ox),      Wt[j][i](ox) = sum_{a<k} A(a,i,j) * T[a*ox]
//
// (one (oz,oy) pencil; A = kernel transform after its z and y stages, T[q] = exp(-2 pi i q / Nx); Section III-A's
// last stage followed by the multiply-accumulate of Algorithm 3).  The kernels in mac.hip / mac_k.hip fold T into
// the image operand, which makes their work proportional to k*S: the cheapest form for S = 1, the wrong one for a
// batch.  Here both steps are matrix products on v_mfma_f32_16x16x4_f32, chained through LDS:
//
//   step 1, per input image i:   Wt[j][ox]   = sum_a A[j][a] * T[a][ox]        (16 j  x  k taps  x  16 ox)
//   step 2, per bin ox:          Yt[j][s]   += sum_i Wt[j][i] * Xt[i][s]       (16 j  x  8 i per chunk  x  16 s)
//
// Workgroup = 4 waves = one pencil x 16 consecutive ox x 16 output images x up to 16 inputs of the batch; input
// images are walked in chunks of 8.  Per chunk each wave runs step 1 for two of the eight images and parks real
// and imaginary parts in LDS ([ox][i][j], the order step 2 reads its left operand in); after a barrier each wave
// runs step 2 for four of the sixteen ox.  Step 1's complex products are three real ones (P1 = ar br, P2 = ai bi,
// P3 = (ar+ai)(br+bi)).  The result leaves through LDS so that stores run along ox.
//
// Two kernels, by batch size:
//  * k_mac_batch (more than 8 inputs; with more than 16, eight waves take two tiles of 16 inputs per workgroup, so that
//    a generated kernel-spectrum tile serves 32 inputs: a third of the matrix instructions of the 16-input form
//    regenerate spectra, a fifth of this one's; 64 x 80 -> 80 images of 55^3, 7^3 kernels: 4.96 -> 4.46 ms): the image values of a chunk are staged in LDS ([ox][i][s]) with coalesced
//    loads; step 2 uses three real products per complex one.
//  * k_mac_batch8 (at most 8 inputs): real and imaginary parts sit side by side in the 16 columns of the step-2
//    tile, [Yr | Yi] += Wr [Xr | Xi] + Wi [-Xi | Xr]: two full products instead of three half-empty ones and no
//    combination afterwards.  Lane (i, s) needs Xt[i][s] at the wave's four consecutive ox, 32 contiguous bytes,
//    and loads them straight from global memory one chunk ahead (lanes 8 columns apart share an address), so the
//    image values never touch LDS; the Wt arrays are double-buffered and one barrier per chunk is left.  (With
//    16 different inputs per wave the same direct loads touch 64 cache lines per instruction and were measured
//    13 % slower than staging, so the larger batches keep the staging kernel.)
#include "mac_common.h"

namespace znni {

constexpr int MB_IC = 8;              // input images per chunk
constexpr int MB_WP = 132;            // floats between consecutive ox in the Wt arrays (8*16 + padding)
constexpr int MB_OP = 17;             // float2 between consecutive (j, s) rows of the output tile (16 ox + padding)
constexpr int MB_WB = 2 * 16 * MB_WP; // floats per Wt buffer (real array, then imaginary array)

// (one and two steps are held to 128 registers, four waves per SIMD: 3-7 % faster for 5^3 to 8^3 kernels)
// NS = tiles of 16 inputs per workgroup: 1 (four waves), or 2 (eight waves: waves 0-3 take the first tile, 4-7 the
// second; each generated kernel-spectrum tile then serves 32 inputs and each wave generates one image's share of it
// instead of two)
template <int KS, int NS>      // KS = steps of four taps: (k + 3) / 4, 1 to 3
__global__ __launch_bounds__(256 * NS) __attribute__((amdgpu_waves_per_eu((KS <= 2 ? 4 : 3)))) void k_mac_batch(const float2* __restrict__ Xt, const float2* __restrict__ A,
                                                   float2* __restrict__ Yt, const float2* __restrict__ twg, int N,
                                                   int S, int f, int fo, int k, int fp, int Mp, int noxt, int njt,
                                                   int nsc, int npencils, int accumulate)
{
    // LDS: Wt as two float arrays (real, imaginary) [16 ox][MB_WP], image values float2 [16 ox][XP]; the
    // output tile (float2 [16 j][16 NS s][MB_OP]) reuses the same memory after the last chunk.
    constexpr int NT = 256 * NS, SW = 16 * NS;           // threads, inputs of the workgroup
    constexpr int XP = MB_IC * SW + 1;                   // float2 between consecutive ox in the image array
    constexpr int HPW = 2 / NS;                          // images a wave generates the spectrum tile of, per chunk
    extern __shared__ float lds[];
    float* Wr = lds;
    float* Wi = Wr + 16 * MB_WP;
    float2* Xl = reinterpret_cast<float2*>(Wi + 16 * MB_WP);

    int pencil, sub;
    if (!mac_block(noxt * njt * nsc, npencils, pencil, sub)) return;
    const int oxt = sub % noxt, jt = (sub / noxt) % njt, sc = sub / (noxt * njt);
    const int t = threadIdx.x, wave = t >> 6, lane = t & 63, l16 = lane & 15, kk = lane >> 4;
    const int w4 = wave & 3, sw = wave >> 2;             // group of four bins, tile of 16 inputs
    const int ox0 = oxt * 16, j0 = jt * 16, s0 = sc * SW;
    const float2* Xp = Xt + (size_t)pencil * S * f * N;
    const float2* Ap = A + (size_t)pencil * k * fp * Mp;
    float2* Yp = Yt + (size_t)pencil * S * fo * N;

    // step-1 right operand of this lane: T[a = 4*st + kk][ox = ox0 + l16], zero beyond the last tap
    float tr[KS], ti[KS], ts[KS];
    {
        // index (a * ox) mod N without a division: kk * ox and 4 * ox are below 4 N, later taps add 4 * ox
        const int ox = min(ox0 + l16, N - 1);
        int q = kk * ox, q4 = 4 * ox;
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            q = q >= N ? q - N : q;
            q4 = q4 >= N ? q4 - N : q4;
        }
#pragma unroll
        for (int st = 0; st < KS; ++st) {
            const int a = 4 * st + kk;
            float2 v = make_float2(0.f, 0.f);
            if (a < k) v = twg[q];
            tr[st] = v.x; ti[st] = v.y; ts[st] = v.x + v.y;
            q += q4;
            q = q >= N ? q - N : q;
        }
    }

    // what this thread stages per chunk: eight image values (element e = t + 256 r of [i][s][ox]) and the step-1
    // left operands of its wave's two images; both are requested one chunk ahead and wait in registers
    constexpr int XR = MB_IC * 16 * SW / NT;
    // Inputs, bins and images beyond the tensor are read from clamped (valid, finite) places and need no mask: their
    // products land in tile columns or bins that are never stored, or meet kernel-spectrum values that are zero
    // (the kernel transforms of images in [f, fp) are zero, those beyond are masked in step 1).
    size_t xoff[XR];                                 // offset of (s, ox) inside the pencil, image index excluded
    int xi[XR];
#pragma unroll
    for (int r = 0; r < XR; ++r) {
        const int e = t + NT * r;
        const int oxl = e & 15, s = (e >> 4) % SW;
        xi[r] = e / (16 * SW);
        xoff[r] = (size_t)min(s0 + s, S - 1) * f * N + min(ox0 + oxl, N - 1);
    }
    // step-1 left operands of this wave's two images, ic0 + 2*wave + h: A[(i/4)][a][i%4][j] of the pencil, so a chunk
    // of eight images later is 2 * k * 4 * Mp elements further (32-bit offsets: the shape limits of the layer call
    // see to it).  Images in [fp, fp + 4) of a last half chunk are read where they would lie (the next pencil's
    // first rows, or the zeroed padding behind the last pencil) and masked below.
    int a_off[HPW], a_tap[KS];
#pragma unroll
    for (int h = 0; h < HPW; ++h)
        a_off[h] = (((HPW * wave + h) >> 2) * k * 4 + ((HPW * wave + h) & 3)) * Mp + j0 + l16;
#pragma unroll
    for (int st = 0; st < KS; ++st) a_tap[st] = min(4 * st + kk, k - 1) * 4 * Mp;      // surplus taps meet a zero twiddle
    const int a_chunk = 2 * k * 4 * Mp;
    float2 xreg[XR], areg[HPW][KS];
    auto request = [&](int ic0) {
#pragma unroll
        for (int r = 0; r < XR; ++r) xreg[r] = Xp[xoff[r] + (size_t)min(ic0 + xi[r], f - 1) * N];
        const float2* ac = Ap + (ic0 >> 3) * a_chunk;
#pragma unroll
        for (int h = 0; h < HPW; ++h)
#pragma unroll
            for (int st = 0; st < KS; ++st) areg[h][st] = ac[a_off[h] + a_tap[st]];
    };
    request(0);

    floatx4 p1[4], p2[4], p3[4];                     // step-2 accumulators: ox = ox0 + 4*w4 + q
#pragma unroll
    for (int q = 0; q < 4; ++q) { p1[q] = floatx4{0.f, 0.f, 0.f, 0.f}; p2[q] = p1[q]; p3[q] = p1[q]; }

    for (int ic0 = 0; ic0 < f; ic0 += MB_IC) {
        __syncthreads();                             // the previous chunk has been consumed
        // ---- image values of the chunk: Xl[ox][i][s]
#pragma unroll
        for (int r = 0; r < XR; ++r) {
            const int e = t + NT * r;
            Xl[(e & 15) * XP + (e >> 4)] = xreg[r];
        }
        // ---- step 1 for this wave's images of the chunk
#pragma unroll
        for (int h = 0; h < HPW; ++h) {
            const int il = HPW * wave + h;
            const float mi = ic0 + il < fp ? 1.f : 0.f;
            floatx4 q1 = floatx4{0.f, 0.f, 0.f, 0.f}, q2 = q1, q3 = q1;
#pragma unroll
            for (int st = 0; st < KS; ++st) {
                {
                    const float ar = areg[h][st].x * mi, ai = areg[h][st].y * mi;
                    q1 = __builtin_amdgcn_mfma_f32_16x16x4f32(ar, tr[st], q1, 0, 0, 0);
                    q2 = __builtin_amdgcn_mfma_f32_16x16x4f32(ai, ti[st], q2, 0, 0, 0);
                    q3 = __builtin_amdgcn_mfma_f32_16x16x4f32(ar + ai, ts[st], q3, 0, 0, 0);
                }
            }
            // element e of lane: output image j0 + 4*kk + e, bin ox0 + l16
            float4 wr, wi;
            wr.x = q1[0] - q2[0]; wr.y = q1[1] - q2[1]; wr.z = q1[2] - q2[2]; wr.w = q1[3] - q2[3];
            wi.x = q3[0] - q1[0] - q2[0]; wi.y = q3[1] - q1[1] - q2[1];
            wi.z = q3[2] - q1[2] - q2[2]; wi.w = q3[3] - q1[3] - q2[3];
            const int o = l16 * MB_WP + il * 16 + 4 * kk;
            *reinterpret_cast<float4*>(Wr + o) = wr;
            *reinterpret_cast<float4*>(Wi + o) = wi;
        }
        __syncthreads();
        if (ic0 + MB_IC < f) request(ic0 + MB_IC);   // in flight during step 2
        // ---- step 2 for ox = ox0 + 4*wave + q: left operand Wt[j = l16][i = 4*st + kk], right Xt[i][s = l16]
        // the operands of four images for all four bins first, then their products; the scheduling barriers keep the
        // two groups of a chunk apart, which is what lets the two-step form fit 128 registers without scratch
#pragma unroll
        for (int st = 0; st < MB_IC / 4; ++st) {
            float wr_[4], wi_[4];
            float2 x_[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int oxl = 4 * w4 + q;
                const int o = st * 64 + lane;
                wr_[q] = Wr[oxl * MB_WP + o];
                wi_[q] = Wi[oxl * MB_WP + o];
                x_[q] = Xl[oxl * XP + (4 * st + kk) * SW + 16 * sw + l16];
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float wr = wr_[q], wi = wi_[q];
                const float2 x = x_[q];
                p1[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(wr, x.x, p1[q], 0, 0, 0);
                p2[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(wi, x.y, p2[q], 0, 0, 0);
                p3[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(wr + wi, x.x + x.y, p3[q], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // ---- result through LDS: Ol[j][s][ox]; accumulator element e of lane: j = 4*kk + e, s = l16
    __syncthreads();
    float2* Ol = reinterpret_cast<float2*>(lds);
    {
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                Ol[((4 * kk + e) * SW + 16 * sw + l16) * MB_OP + 4 * w4 + q] =
                    make_float2(p1[q][e] - p2[q][e], p3[q][e] - p1[q][e] - p2[q][e]);
    }
    __syncthreads();
    // thread = (input s, bin oxl) of the tile, walking the tile's output images: one address, then a constant stride
    {
        const int oxl = t & 15, s = t >> 4;
        const int gs = s0 + s, gox = ox0 + oxl;
        if (gs < S && gox < N) {
            float2* dst = Yp + ((size_t)gs * fo + j0) * N + gox;
            const float2* src = Ol + s * MB_OP + oxl;        // s < 16 NS
            const int nj = min(16, fo - j0);
            for (int j = 0; j < nj; ++j) {
                float2 v = src[j * SW * MB_OP];
                if (accumulate) {
                    const float2 old = dst[(size_t)j * N];
                    v.x += old.x;
                    v.y += old.y;
                }
                dst[(size_t)j * N] = v;
            }
        }
    }
}

// (one and two steps are held to 128 registers, four waves per SIMD; the operands of the second product are
// staged four images at a time behind scheduling barriers, as above, and no scratch is needed: 3-7 % faster)
template <int KS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu((KS <= 2 ? 4 : 3)))) void k_mac_batch8(const float2* __restrict__ Xt, const float2* __restrict__ A,
                                                    float2* __restrict__ Yt, const float2* __restrict__ twg, int N,
                                                    int S, int f, int fo, int k, int fp, int Mp, int noxt, int njt,
                                                    int nsc, int npencils, int accumulate)
{
    // LDS: two Wt buffers, each two float arrays (real, imaginary) [16 ox][MB_WP]; the output tile
    // (float2 [16 j][16 s][MB_OP]) reuses the same memory after the last chunk.
    extern __shared__ float lds[];

    int pencil, sub;
    if (!mac_block(noxt * njt * nsc, npencils, pencil, sub)) return;
    const int oxt = sub % noxt, jt = (sub / noxt) % njt, sc = sub / (noxt * njt);
    const int t = threadIdx.x, wave = t >> 6, lane = t & 63, l16 = lane & 15, kk = lane >> 4;
    const int ox0 = oxt * 16, j0 = jt * 16, s0 = sc * 16;
    const float2* Xp = Xt + (size_t)pencil * S * f * N;
    const float2* Ap = A + (size_t)pencil * k * fp * Mp;
    float2* Yp = Yt + (size_t)pencil * S * fo * N;

    // step-1 right operand of this lane: T[a = 4*st + kk][ox = ox0 + l16], zero beyond the last tap
    float tr[KS], ti[KS], ts[KS];
    {
        // index (a * ox) mod N without a division: kk * ox and 4 * ox are below 4 N, later taps add 4 * ox
        const int ox = min(ox0 + l16, N - 1);
        int q = kk * ox, q4 = 4 * ox;
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            q = q >= N ? q - N : q;
            q4 = q4 >= N ? q4 - N : q4;
        }
#pragma unroll
        for (int st = 0; st < KS; ++st) {
            const int a = 4 * st + kk;
            float2 v = make_float2(0.f, 0.f);
            if (a < k) v = twg[q];
            tr[st] = v.x; ti[st] = v.y; ts[st] = v.x + v.y;
            q += q4;
            q = q >= N ? q - N : q;
        }
    }

    // step-2 right operand of this lane: input s = l16 & 7 (columns 0..7 of the tile carry the real parts of
    // s = 0..7, columns 8..15 the imaginary parts), image row ic0 + 4*st + kk, bins ox0 + 4*wave + 0..3 as two
    // 16-byte pairs.  Inputs, image rows and bins beyond the tensor are clamped to valid ones: their
    // products land in tile columns, or meet zero Wt values, or belong to bins that are never stored.
    const bool lowcol = l16 < 8;
    const float2* xs = Xp + (size_t)min(s0 + (l16 & 7), S - 1) * f * N;
    const int oxa = min(ox0 + 4 * wave, N - 2), oxb = min(ox0 + 4 * wave + 2, N - 2);     // N is even
    // (offsets inside an input's images and inside a pencil's kernel transforms fit 32 bits: the shape limits of the
    // layer call see to it)
    const int x_last = (f - 1) * N;
    auto request_x = [&](float4 (&x)[MB_IC / 4][2], int ic0) {
#pragma unroll
        for (int st = 0; st < MB_IC / 4; ++st) {
            const float2* row = xs + min((ic0 + 4 * st + kk) * N, x_last);
            x[st][0] = *reinterpret_cast<const float4*>(row + oxa);
            x[st][1] = *reinterpret_cast<const float4*>(row + oxb);
        }
    };
    // step-1 left operands of this wave's two images, ic0 + 2*wave + h: A[(i/4)][a][i%4][j] of the pencil, so a chunk
    // of eight images later is 2 * k * 4 * Mp elements further.  Images in [fp, fp + 4) of a last half chunk are
    // read where they would lie (the next pencil's first rows, or the zeroed padding behind the last pencil) and
    // masked below.
    int a_off[2], a_tap[KS];
#pragma unroll
    for (int h = 0; h < 2; ++h) a_off[h] = (((2 * wave + h) >> 2) * k * 4 + ((2 * wave + h) & 3)) * Mp + j0 + l16;
#pragma unroll
    for (int st = 0; st < KS; ++st) a_tap[st] = min(4 * st + kk, k - 1) * 4 * Mp;      // surplus taps meet a zero twiddle
    const int a_chunk = 2 * k * 4 * Mp;
    float2 areg[2][KS];
    auto request_a = [&](int ic0) {
        const float2* ac = Ap + (ic0 >> 3) * a_chunk;
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int st = 0; st < KS; ++st) areg[h][st] = ac[a_off[h] + a_tap[st]];
    };

    floatx4 p1[4], p2[4];                            // step-2 accumulators, ox = ox0 + 4*wave + q: p1 collects the
#pragma unroll                                       // Wr products, p2 the Wi products
    for (int q = 0; q < 4; ++q) { p1[q] = floatx4{0.f, 0.f, 0.f, 0.f}; p2[q] = p1[q]; }

    const int nch = (f + MB_IC - 1) / MB_IC;
    float4 xA[MB_IC / 4][2], xB[MB_IC / 4][2];
    request_a(0);
    request_x(xA, 0);

    // One chunk: XC holds its image values; those of the next chunk are requested into XN first.
#define ZNNI_MB_CHUNK(C, XC, XN)                                                                          \
    {                                                                                                     \
        const int ic0 = (C) * MB_IC;                                                                      \
        float* Wr = lds + ((C) & 1) * MB_WB;                                                              \
        float* Wi = Wr + 16 * MB_WP;                                                                      \
        if ((C) + 1 < nch) request_x(XN, ic0 + MB_IC);                                                    \
        /* ---- step 1 for images ic0 + 2*wave, ic0 + 2*wave + 1 */                                       \
        _Pragma("unroll") for (int h = 0; h < 2; ++h) {                                                   \
            const int il = 2 * wave + h;                                                                  \
            const float mi = ic0 + il < fp ? 1.f : 0.f;                                                   \
            floatx4 q1 = floatx4{0.f, 0.f, 0.f, 0.f}, q2 = q1, q3 = q1;                                   \
            _Pragma("unroll") for (int st = 0; st < KS; ++st) {                                            \
                {                                                                                         \
                    const float ar = areg[h][st].x * mi, ai = areg[h][st].y * mi;                         \
                    q1 = __builtin_amdgcn_mfma_f32_16x16x4f32(ar, tr[st], q1, 0, 0, 0);                   \
                    q2 = __builtin_amdgcn_mfma_f32_16x16x4f32(ai, ti[st], q2, 0, 0, 0);                   \
                    q3 = __builtin_amdgcn_mfma_f32_16x16x4f32(ar + ai, ts[st], q3, 0, 0, 0);              \
                }                                                                                         \
            }                                                                                             \
            /* element e of lane: output image j0 + 4*kk + e, bin ox0 + l16 */                            \
            float4 wr, wi;                                                                                \
            wr.x = q1[0] - q2[0]; wr.y = q1[1] - q2[1]; wr.z = q1[2] - q2[2]; wr.w = q1[3] - q2[3];       \
            wi.x = q3[0] - q1[0] - q2[0]; wi.y = q3[1] - q1[1] - q2[1];                                   \
            wi.z = q3[2] - q1[2] - q2[2]; wi.w = q3[3] - q1[3] - q2[3];                                   \
            const int o = l16 * MB_WP + il * 16 + 4 * kk;                                                 \
            *reinterpret_cast<float4*>(Wr + o) = wr;                                                      \
            *reinterpret_cast<float4*>(Wi + o) = wi;                                                      \
        }                                                                                                 \
        if ((C) + 1 < nch) request_a(ic0 + MB_IC);   /* in flight during step 2 */                        \
        /* The only barrier of the chunk.  This buffer was last read in step 2 of chunk C-2, which every */\
        /* wave finished before it arrived at the barrier of chunk C-1.                                  */\
        __syncthreads();                                                                                  \
        /* ---- step 2 for ox = ox0 + 4*wave + q: left operand Wt[j = l16][i = 4*st + kk]; all operands */ \
        /* first, then the products                                                                      */\
        _Pragma("unroll") for (int st = 0; st < MB_IC / 4; ++st) {                                        \
            float wr_[4], wi_[4];                                                                         \
            _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                               \
                const int oxl = 4 * wave + q;                                                             \
                wr_[q] = Wr[oxl * MB_WP + st * 64 + lane];                                                \
                wi_[q] = Wi[oxl * MB_WP + st * 64 + lane];                                                \
            }                                                                                             \
            __builtin_amdgcn_sched_barrier(0);                                                            \
            _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                               \
                const float wr = wr_[q], wi = wi_[q];                                                     \
                const float4 xp = XC[st][q >> 1];                                                         \
                const float2 x = (q & 1) ? make_float2(xp.z, xp.w) : make_float2(xp.x, xp.y);             \
                p1[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(wr, lowcol ? x.x : x.y, p1[q], 0, 0, 0);     \
                p2[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(wi, lowcol ? -x.y : x.x, p2[q], 0, 0, 0);    \
            }                                                                                             \
            __builtin_amdgcn_sched_barrier(0);                                                            \
        }                                                                                                 \
    }
    int c = 0;
    for (; c + 2 <= nch; c += 2) {
        ZNNI_MB_CHUNK(c, xA, xB)
        ZNNI_MB_CHUNK(c + 1, xB, xA)
    }
    if (c < nch) ZNNI_MB_CHUNK(c, xA, xB)
#undef ZNNI_MB_CHUNK

    // ---- result through LDS: Ol[j][s][ox]; accumulator element e of lane: j = 4*kk + e, one component (real for
    // columns 0..7, imaginary for 8..15) of input s = l16 & 7
    __syncthreads();
    float2* Ol = reinterpret_cast<float2*>(lds);
    {
        float* Of = lds;
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                Of[2 * (((4 * kk + e) * 16 + (l16 & 7)) * MB_OP + 4 * wave + q) + (lowcol ? 0 : 1)] =
                    p1[q][e] + p2[q][e];
    }
    __syncthreads();
    // thread = (input s, bin oxl) of the tile, walking the tile's output images: one address, then a constant stride
    {
        const int oxl = t & 15, s = t >> 4;
        const int gs = s0 + s, gox = ox0 + oxl;
        if (gs < S && gox < N) {
            float2* dst = Yp + ((size_t)gs * fo + j0) * N + gox;
            const float2* src = Ol + s * MB_OP + oxl;
            const int nj = min(16, fo - j0);
            for (int j = 0; j < nj; ++j) {
                float2 v = src[j * 16 * MB_OP];
                if (accumulate) {
                    const float2 old = dst[(size_t)j * N];
                    v.x += old.x;
                    v.y += old.y;
                }
                dst[(size_t)j * N] = v;
            }
        }
    }
}

// The batch form generates each kernel-spectrum value once per bin (cost independent of S) and pays one 16-column
// matrix product per 16 inputs; the single-input form pays matrix-core work proportional to k*S.
// (up to 8 inputs: even lengths along x only, the image values are fetched in 16-byte pairs of neighbouring bins)
bool mac_batch_available(const LayerPlan& L) { return L.d.kx <= 12 && (L.S > 8 || (L.d.Nx & 1) == 0); }
// Measured on MI355X (32 -> 32 and 80 -> 80 images, 32^3 .. 128^3): the batch form wins from about k*S = 32 on.
bool mac_batch_preferred(const LayerPlan& L) { return mac_batch_available(L) && L.d.kx * L.S >= 32; }

znni_status launch_mac_batch(const LayerPlan& L, int accumulate, hipStream_t st)
{
    if (!mac_batch_available(L)) return ZNNI_ERR_UNSUPPORTED_SIZE;
    const int N = L.d.Nx;
    // more than 16 inputs: two tiles of 16 inputs per workgroup share each generated kernel-spectrum tile
    const int NS = L.S > 16 ? 2 : 1;
    const size_t lds_main = L.S <= 8 ? sizeof(float) * 2 * MB_WB
                                     : sizeof(float) * MB_WB + sizeof(float2) * 16 * (MB_IC * 16 * NS + 1);
    const size_t lds_out = sizeof(float2) * 16 * 16 * (L.S <= 8 ? 1 : NS) * MB_OP;
    const size_t lds = lds_main > lds_out ? lds_main : lds_out;
    const int noxt = (N + 15) / 16, njt = (L.fo + 15) / 16, nsc = (L.S + 16 * NS - 1) / (16 * NS);
    const int npencils = L.d.zc * L.d.Ny;
    const long long blocks = (long long)((npencils + 7) / 8) * noxt * njt * nsc * 8;
    if (blocks > 0x7fffffffll) return ZNNI_ERR_SHAPE;
    // one instantiation per number of tap steps: the loops over them are straight-line code
    const int ks = (L.d.kx + 3) / 4;
    auto* kernel = L.S <= 8 ? (ks == 1 ? k_mac_batch8<1> : ks == 2 ? k_mac_batch8<2> : k_mac_batch8<3>)
                   : NS == 1 ? (ks == 1 ? k_mac_batch<1, 1> : ks == 2 ? k_mac_batch<2, 1> : k_mac_batch<3, 1>)
                             : (ks == 1 ? k_mac_batch<1, 2> : ks == 2 ? k_mac_batch<2, 2> : k_mac_batch<3, 2>);
    if (lds > 48 * 1024 &&
        hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return ZNNI_ERR_HIP;
    kernel<<<dim3((unsigned)blocks), dim3(L.S > 16 ? 512 : 256), lds, st>>>(L.buf0, L.A, L.Yt, L.twx, N, L.S, L.f, L.fo,
                                                                          L.d.kx, L.fp, L.Mp, noxt, njt, nsc, npencils,
                                                                          accumulate);
    if (hipGetLastError() != hipSuccess) return ZNNI_ERR_HIP;
    return ZNNI_OK;
}

}  // namespace znni
