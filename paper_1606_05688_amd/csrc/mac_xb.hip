// mac_xb.hip -- multiply-accumulate with the x axis transformed in short overlapping blocks.
//
// Where the x axis is not transformed at full length (see mac_xd.hip) the work left along x is, per (oz, oy)
// pencil, a kx-tap valid convolution of every input row with every kernel column, kx complex multiply-adds per
// output.  The convolution theorem (Section III-A) holds for any transform length that is at least the kernel
// length, so the same convolution is done here block by block: a block of XB = 8 consecutive inputs is
// transformed (length-8 transform, in registers), multiplied by the length-8 transform of the kx kernel taps and
// accumulated over the input images, transformed back, and the V = XB - kx + 1 outputs that did not wrap are kept;
// consecutive blocks start V inputs apart ("overlap-save").  That is XB / V complex multiply-adds per output
// instead of kx (2 instead of 5 for five taps), and the kernel transform is complete when it is stored: XB values
// per kernel column, (XB / kx) times the size of the taps themselves, nothing generated on the fly.  Pruning is the
// same idea as in Section III-A: no transform is longer than what the kernel's support asks for.
//
// Per pencil and block-frequency p < XB the accumulation over input images is one dense complex matrix product
//     C_p[j][b] = sum_i  Ah_p[i][j] * D_p[i][b],        D_p[i][b] = sum_t X2[i][b V + t] exp(-2 pi i p t / XB)
// over output images j, blocks b and input images i, done on the matrix cores (v_mfma_f32_16x16x4_f32, three real
// products per complex one, as in mac_k.hip).  Layouts: X2[img][oz][oy][x] and Yd[imgo][oz][oy][xo] as in
// mac_xd.hip; Ah[pencil][ch][p][i % 4][j < Mp][(i / 4) % 2] with ch = i / 8, scaled by 1 / (Ny Nz XB).
//
// Workgroup = 4 waves = one pencil x NB = 16 * CTW blocks x 16 * RTW output images; wave w owns the two block
// frequencies 2w and 2w+1.  Input images go through in chunks of eight: every thread transforms one block of one
// image of the following chunk and leaves the eight results in LDS, laid out as the matrix cores' right operand,
// while the waves multiply the current chunk; one barrier per chunk.  At the end the accumulated block spectra
// change hands through LDS once more (wave = frequency becomes thread = (output image, block)), are transformed
// back, and the valid outputs of each block are stored as one contiguous run.
#include <type_traits>

#include "mac_common.h"

namespace znni {

constexpr int XB = 8;
constexpr float kR8 = 0.70710678118654752440f;

// Length-8 transform in registers, v[t] -> v[p], exp(-2 pi i p t / 8) (INV: conjugate twiddles).
template <bool INV>
__device__ __forceinline__ void fft8(float2* v)
{
    // multiply by -i (forward) or +i (inverse)
    auto rot = [](float2 a) { return INV ? make_float2(-a.y, a.x) : make_float2(a.y, -a.x); };
    const float2 a0 = cadd(v[0], v[4]), a1 = csub(v[0], v[4]), a2 = cadd(v[2], v[6]), a3 = rot(csub(v[2], v[6]));
    const float2 a4 = cadd(v[1], v[5]), a5 = csub(v[1], v[5]), a6 = cadd(v[3], v[7]), a7 = rot(csub(v[3], v[7]));
    const float2 e0 = cadd(a0, a2), e2 = csub(a0, a2), e1 = cadd(a1, a3), e3 = csub(a1, a3);
    const float2 o0 = cadd(a4, a6), o2 = rot(csub(a4, a6));
    float2 o1 = cadd(a5, a7), o3 = csub(a5, a7);
    // o1 *= (1 -+ i)/sqrt2, o3 *= (-1 -+ i)/sqrt2
    o1 = INV ? make_float2((o1.x - o1.y) * kR8, (o1.x + o1.y) * kR8) : make_float2((o1.x + o1.y) * kR8, (o1.y - o1.x) * kR8);
    o3 = INV ? make_float2((-o3.x - o3.y) * kR8, (o3.x - o3.y) * kR8) : make_float2((o3.y - o3.x) * kR8, (-o3.x - o3.y) * kR8);
    v[0] = cadd(e0, o0); v[4] = csub(e0, o0);
    v[1] = cadd(e1, o1); v[5] = csub(e1, o1);
    v[2] = cadd(e2, o2); v[6] = csub(e2, o2);
    v[3] = cadd(e3, o3); v[7] = csub(e3, o3);
}

// ---------------------------------------------------------------------------------------- kernel transform
// Ah[pencil][ch][p<8][kk<4][j<Mp][h<2] = scale * sum_{a<K} exp(-2 pi i a p / 8) sum_{b<ky} A1[oz][b][a][i][j] exp(-2 pi i oy b / Ny),
// i = 8 ch + 4 h + kk; zero where i >= f or j >= fo (A1 holds zeros there, images beyond A1's fp rows are skipped).
// One thread: one (ch, kk, j), both h, KB_OY consecutive oy, all K taps in registers; the two h are stored together.
constexpr int KB_OY = 8;
constexpr int KPREP_TAPS_XB = 64;
template <int K>
__global__ __launch_bounds__(256) void k_kprep_yb(const float2* __restrict__ A1, float2* __restrict__ Ah,
                                                  const float2* __restrict__ tw, int N, int ky, int fp, int Mp, int nch,
                                                  float scale)
{
    extern __shared__ float2 tw2[];                            // [taps of the chunk][KB_OY]
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;     // (ch, kk, j)
    const int oy0 = blockIdx.y * KB_OY, oz = blockIdx.z;
    const int items = nch * 4 * Mp;
    const bool live = idx < items;
    const int j = idx % Mp, kk = (idx / Mp) & 3, ch = idx / (4 * Mp);
    const int per = K * fp * Mp;
    float2 acc[2][K][KB_OY];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int a = 0; a < K; ++a)
#pragma unroll
            for (int o = 0; o < KB_OY; ++o) acc[h][a][o] = make_float2(0.f, 0.f);
    for (int b0 = 0; b0 < ky; b0 += KPREP_TAPS_XB) {
        const int nb = min(KPREP_TAPS_XB, ky - b0);
        if (b0) __syncthreads();
        for (int e = threadIdx.x; e < nb * KB_OY; e += 256) {
            const int c = e / KB_OY, o = e - c * KB_OY;
            tw2[e] = tw[(unsigned)((oy0 + o) * (b0 + c)) % (unsigned)N];
        }
        __syncthreads();
        if (live) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int i = 8 * ch + 4 * h + kk;
                if (i >= fp) continue;
                const float2* a1 = A1 + (size_t)oz * ky * per + (size_t)i * Mp + j;
                for (int b = 0; b < nb; ++b) {
                    const float2* tb = tw2 + b * KB_OY;
#pragma unroll
                    for (int a = 0; a < K; ++a) {
                        const float2 v = a1[(size_t)(b0 + b) * per + (size_t)a * fp * Mp];
#pragma unroll
                        for (int o = 0; o < KB_OY; ++o) acc[h][a][o] = cfma(acc[h][a][o], v, tb[o]);
                    }
                }
            }
        }
    }
    if (!live) return;
    // length-8 transform of the K taps (the other 8 - K inputs are zero and fold away)
#pragma unroll
    for (int o = 0; o < KB_OY; ++o) {
        if (oy0 + o >= N) break;
        const size_t pencil = (size_t)oz * N + oy0 + o;
        float4* d = reinterpret_cast<float4*>(Ah) + ((pencil * nch + ch) * 8 * 4 + kk) * Mp + j;
        float2 s0[XB], s1[XB];
#pragma unroll
        for (int a = 0; a < XB; ++a) {
            s0[a] = a < K ? acc[0][a][o] : make_float2(0.f, 0.f);
            s1[a] = a < K ? acc[1][a][o] : make_float2(0.f, 0.f);
        }
        fft8<false>(s0);
        fft8<false>(s1);
#pragma unroll
        for (int p = 0; p < 8; ++p)
            d[(size_t)p * 4 * Mp] = make_float4(s0[p].x * scale, s0[p].y * scale, s1[p].x * scale, s1[p].y * scale);
    }
}

// The same transform for kernels of up to 5 taps along y (KY a template parameter): a thread keeps the K * KY values
// of A1 of both its images in registers and walks KR_OY consecutive oy with them, so that A1 (460 KB per oz on the
// 48 -> 48 layer with 5^3 kernels) is read from the caches Ny / KR_OY times per call instead of Ny / KB_OY times: with
// 4 oy per thread those reads were as many bytes as the kernel writes (1.74 ms), with 8 1.57 ms.
constexpr int KR_OY = 32;
template <int K, int KY>
__global__ __launch_bounds__(256) void k_kprep_yb_r(const float2* __restrict__ A1, float2* __restrict__ Ah,
                                                    const float2* __restrict__ tw, int N, int fp, int Mp, int nch,
                                                    float scale)
{
    __shared__ float2 tw2[KR_OY][KY];
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;     // (ch, kk, j)
    const int oy0 = blockIdx.y * KR_OY, oz = blockIdx.z;
    const int items = nch * 4 * Mp;
    for (int e = threadIdx.x; e < KR_OY * KY; e += 256) {
        const int o = e / KY, b = e - o * KY;
        tw2[o][b] = tw[(unsigned)((oy0 + o) * b) % (unsigned)N];
    }
    __syncthreads();
    if (idx >= items) return;
    const int j = idx % Mp, kk = (idx / Mp) & 3, ch = idx / (4 * Mp);
    const int per = K * fp * Mp;
    float2 a1v[2][KY][K];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int i = min(8 * ch + 4 * h + kk, fp - 1);
        const float m = 8 * ch + 4 * h + kk < fp ? 1.f : 0.f;          // images beyond A1's rows count as zero
        const float2* a1 = A1 + (size_t)oz * KY * per + (size_t)i * Mp + j;
#pragma unroll
        for (int b = 0; b < KY; ++b)
#pragma unroll
            for (int a = 0; a < K; ++a) {
                const float2 v = a1[(size_t)b * per + (size_t)a * fp * Mp];
                a1v[h][b][a] = make_float2(v.x * m, v.y * m);
            }
    }
    const int no = min(KR_OY, N - oy0);
    float4* d = reinterpret_cast<float4*>(Ah) + ((((size_t)oz * N + oy0) * nch + ch) * 8 * 4 + kk) * Mp + j;
    const size_t d_oy = (size_t)nch * 8 * 4 * Mp;
    for (int o = 0; o < no; ++o, d += d_oy) {
        float2 s[2][XB];
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int a = 0; a < XB; ++a) {
                float2 acc = make_float2(0.f, 0.f);
                if (a < K) {
#pragma unroll
                    for (int b = 0; b < KY; ++b) acc = cfma(acc, a1v[h][b][a < K ? a : 0], tw2[o][b]);
                }
                s[h][a] = acc;
            }
        fft8<false>(s[0]);
        fft8<false>(s[1]);
#pragma unroll
        for (int p = 0; p < 8; ++p)
            d[(size_t)p * 4 * Mp] = make_float4(s[0][p].x * scale, s[0][p].y * scale, s[1][p].x * scale, s[1][p].y * scale);
    }
}

// ---------------------------------------------------------------------------------------- multiply-accumulate
struct XbArgs {
    const float2* X2;
    const float2* Ah;
    float2* Yd;
    size_t ximg, yimg, xpen, ypen;    // as in mac_xd.hip
    int S, f, fo, Mp, nx, nox, ldx, ldxo, Ny, K;
    int nch;                          // chunks of eight input images
    int nblk;                         // blocks along x: ceil(nox / V)
    int n2, n1, blk1, nmblk, npencils, accumulate;
    int m_base;                       // first output-image row of this launch (row blocks of another height before it)
};

template <int RTW, int CTW>
__device__ __forceinline__ void mac_xb_body(float2* lds, const XbArgs& g, int blk0, int ncolblk, int pencil, int sub)
{
    constexpr int NB = 16 * CTW;                // blocks of this workgroup
    const int colblk = sub % ncolblk, mblk = sub / ncolblk;
    const int t = threadIdx.x, wave = t >> 6, lane = t & 63;
    const int l16 = lane & 15, kk = lane >> 4;
    const int m0 = g.m_base + mblk * RTW * 16;
    const int b0 = blk0 + colblk * NB;          // first block of the workgroup
    const int sI = blockIdx.y;
    const int f = g.f, Mp = g.Mp, K = g.K, V = XB - K + 1;
    const int poz = pencil / g.Ny, poy = pencil - poz * g.Ny;

    // ---- this thread's share of the block transforms: block fb of image 4*fh + fkk of each chunk
    // (a compile-time `true` for 32 blocks: all 256 threads transform)
    const bool fft_on = (8 * NB >= 256) ? true : t < 8 * NB;
    const int fb = t % NB, fhk = min(t / NB, 7), fh = fhk >> 2, fkk = fhk & 3;
    const int gb = b0 + fb;                                 // block number along x
    const float2* xrow = g.X2 + (size_t)sI * f * g.ximg + (size_t)poz * g.xpen + (size_t)poy * g.ldx;
    // Inputs beyond the image row (last block of a row whose outputs do not fill it, blocks of the padding behind
    // the last one) are read from the row's last element: they reach discarded outputs only, and any finite
    // value of the data's magnitude does there.
    const int x0 = gb * V;
    // LDS: two buffers Ds[buf][p][kk][b][h]
    float2* const Ds = lds;
    constexpr int DS_BUF = 8 * 4 * NB * 2;
    const int ds_w = (fkk * NB + fb) * 2 + fh;              // + p * 4 * NB * 2

    // ---- this wave's share of the products: frequencies 2*wave, 2*wave+1
    floatx4 p1[2][RTW][CTW], p2[2][RTW][CTW], p3[2][RTW][CTW];
    // A operands: float4 = (h = 0, h = 1) of Ah[pencil][ch][p][kk][j]
    const float4* Ab = reinterpret_cast<const float4*>(g.Ah) +
                       (((size_t)pencil * g.nch * 8 + 2 * wave) * 4 + kk) * Mp + m0 + l16;
    const size_t a_p = (size_t)4 * Mp, a_ch = (size_t)8 * 4 * Mp;
    float4 ac[2][RTW];
#pragma unroll
    for (int pp = 0; pp < 2; ++pp)
#pragma unroll
        for (int r = 0; r < RTW; ++r) ac[pp][r] = Ab[pp * a_p + r * 16];

    // transform of chunk `ch` from the values in xv, results to buffer `buf`
    float2 xv[XB];
    auto load_x = [&](int ch) {
        const float2* xr = xrow + (size_t)min(8 * ch + 4 * fh + fkk, f - 1) * g.ximg;
#pragma unroll
        for (int e = 0; e < XB; ++e) xv[e] = xr[min(x0 + e, g.nx - 1)];
    };
    auto transform_x = [&](int buf) {
        fft8<false>(xv);
        float2* d = Ds + buf * DS_BUF + ds_w;
#pragma unroll
        for (int p = 0; p < XB; ++p) d[p * 4 * NB * 2] = xv[p];
    };

    load_x(0);
    if (fft_on) transform_x(0);
    __syncthreads();

    // One chunk of eight input images.  The first chunk's products start from zero through the instruction's own
    // addend, which spares every wave 288 register moves for clearing the accumulators (1.4 % of the kernel's time).
    auto chunk = [&](int ch, auto first_tag) {
        constexpr bool FIRST = decltype(first_tag)::value;
        const floatx4 zero = floatx4{0.f, 0.f, 0.f, 0.f};
        const int chn = min(ch + 1, g.nch - 1);
        // The next chunk's image values travel during the products below.  Every thread requests them, also those
        // without a transform to do (16 blocks: the upper half repeats the last image's requests), and nothing may
        // move across the fence: inside a branch, the wait for the kernel operands (requested earlier, but counted
        // in order) has to assume the image loads were never issued and ends up waiting for them too; and without
        // the fence the scheduler sinks the loads below the products, right in front of their use.  Either way the
        // loads did not overlap with the products: 7.2 against 6.8 ms on the 320-wide workload.
        load_x(chn);
        __builtin_amdgcn_sched_barrier(0);
        const float4* an = Ab + (size_t)chn * a_ch;
        const float4* Bs = reinterpret_cast<const float4*>(Ds + (ch & 1) * DS_BUF) + ((2 * wave) * 4 + kk) * NB + l16;
#pragma unroll
        for (int pp = 0; pp < 2; ++pp) {
            float4 bv[CTW];
#pragma unroll
            for (int c = 0; c < CTW; ++c) bv[c] = Bs[pp * 4 * NB + c * 16];
            float bs0[CTW], bs1[CTW];
#pragma unroll
            for (int c = 0; c < CTW; ++c) { bs0[c] = bv[c].x + bv[c].y; bs1[c] = bv[c].z + bv[c].w; }
#pragma unroll
            for (int r = 0; r < RTW; ++r) {
                const float4 a = ac[pp][r];
                const float as0 = a.x + a.y, as1 = a.z + a.w;
#pragma unroll
                for (int c = 0; c < CTW; ++c) {
                    p1[pp][r][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, bv[c].x, FIRST ? zero : p1[pp][r][c], 0, 0, 0);
                    p2[pp][r][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, bv[c].y, FIRST ? zero : p2[pp][r][c], 0, 0, 0);
                    p3[pp][r][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(as0, bs0[c], FIRST ? zero : p3[pp][r][c], 0, 0, 0);
                    p1[pp][r][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, bv[c].z, p1[pp][r][c], 0, 0, 0);
                    p2[pp][r][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, bv[c].w, p2[pp][r][c], 0, 0, 0);
                    p3[pp][r][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(as1, bs1[c], p3[pp][r][c], 0, 0, 0);
                }
                ac[pp][r] = an[pp * a_p + r * 16];                // the following chunk's operand, same registers
            }
        }
        if (fft_on && ch + 1 < g.nch) transform_x((ch + 1) & 1);
        __syncthreads();
    };
    chunk(0, std::true_type{});
    for (int ch = 1; ch < g.nch; ++ch) chunk(ch, std::false_type{});

    // ---- block spectra change hands: Ex[p][jl<16][b<NB], one tile of 16 output images at a time
    float2* const Ex = lds;
#pragma unroll
    for (int r = 0; r < RTW; ++r) {
        if (r) __syncthreads();                                    // the previous tile has been read
#pragma unroll
        for (int pp = 0; pp < 2; ++pp)
#pragma unroll
            for (int c = 0; c < CTW; ++c)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float re = p1[pp][r][c][e] - p2[pp][r][c][e];
                    const float im = p3[pp][r][c][e] - p1[pp][r][c][e] - p2[pp][r][c][e];
                    Ex[((2 * wave + pp) * 16 + 4 * kk + e) * NB + c * 16 + l16] = make_float2(re, im);
                }
        __syncthreads();
        for (int q = t; q < 16 * NB; q += 256) {
            const int jl = q / NB, b = q - jl * NB;
            const int jrow = m0 + 16 * r + jl, blk = b0 + b;
            if (jrow >= g.fo || blk >= g.nblk) continue;
            float2 cv[XB];
#pragma unroll
            for (int p = 0; p < XB; ++p) cv[p] = Ex[(p * 16 + jl) * NB + b];
            fft8<true>(cv);
            float2* y = g.Yd + (size_t)(sI * g.fo + jrow) * g.yimg + (size_t)poz * g.ypen + (size_t)poy * g.ldxo +
                        blk * V;
            const int nv = min(V, g.nox - blk * V);
            if (K == 5 && nv == 4 && !g.accumulate) {
                // the common case: four outputs, 32 contiguous bytes at a 32-byte boundary (Yd's rows start on
                // 128-byte boundaries)
                float4* y4 = reinterpret_cast<float4*>(y);
                y4[0] = make_float4(cv[4].x, cv[4].y, cv[5].x, cv[5].y);
                y4[1] = make_float4(cv[6].x, cv[6].y, cv[7].x, cv[7].y);
            } else {
#pragma unroll
                for (int m = 0; m < XB; ++m) {
                    const int v = m - (K - 1);
                    if (v >= 0 && v < nv) {
                        float2 o = cv[m];
                        if (g.accumulate) o = cadd(o, y[v]);
                        y[v] = o;
                    }
                }
            }
        }
    }
}

template <int RTW, bool WIDE>
__global__ __launch_bounds__(256, 2) void k_mac_xb(XbArgs g)
{
    extern __shared__ float2 lds[];
    int pencil, sub;
    if (!mac_block((g.n2 + g.n1) * g.nmblk, g.npencils, pencil, sub)) return;
    if constexpr (WIDE) {
        if (sub < g.n2 * g.nmblk) {
            mac_xb_body<RTW, 2>(lds, g, 0, g.n2, pencil, sub);
            return;
        }
    }
    mac_xb_body<RTW, 1>(lds, g, g.blk1, g.n1, pencil, sub - g.n2 * g.nmblk);
}

// ---------------------------------------------------------------------------------------- host side
// Four or five taps along x (four or five outputs per block of eight: with fewer taps the stored transforms grow by
// more than the products shrink), at least 16 input images (they go through in groups of eight), a batch index that
// fits the launch grid.  Output images go in row blocks of three or two tiles of 16 (the accumulators of two
// frequencies per wave must fit the registers); each row block transforms the image blocks again.
bool mac_xb_available(const LayerPlan& L)
{
    return L.d.kx >= 4 && L.d.kx <= 5 && L.f >= 16 && L.S <= 65535;
}

size_t mac_xb_kernel_bytes(const LayerPlan& L)
{
    const size_t nch = (L.f + 7) / 8;
    return (size_t)L.d.zc * L.d.Ny * nch * 8 * 4 * L.Mp * 2 * sizeof(float2);
}

template <int K, int KY>
static znni_status launch_kprep_yb_r(const LayerPlan& L, hipStream_t st)
{
    const Dims& d = L.d;
    const int nch = (L.f + 7) / 8;
    const int items = nch * 4 * L.Mp;
    const float scale = (float)(1.0 / ((double)d.Ny * d.Nz * XB));
    k_kprep_yb_r<K, KY><<<dim3((items + 255) / 256, (d.Ny + KR_OY - 1) / KR_OY, d.zc), dim3(256), 0, st>>>(
        L.A1, L.A, L.twy, d.Ny, L.fp, L.Mp, nch, scale);
    if (hipGetLastError() != hipSuccess) return ZNNI_ERR_HIP;
    return ZNNI_OK;
}

template <int K>
static znni_status launch_kprep_yb_k(const LayerPlan& L, hipStream_t st)
{
    const Dims& d = L.d;
    switch (d.ky) {                    // up to 5 taps along y: A1 values in registers; more: the general kernel
        case 1: return launch_kprep_yb_r<K, 1>(L, st);
        case 2: return launch_kprep_yb_r<K, 2>(L, st);
        case 3: return launch_kprep_yb_r<K, 3>(L, st);
        case 4: return launch_kprep_yb_r<K, 4>(L, st);
        case 5: return launch_kprep_yb_r<K, 5>(L, st);
    }
    const int nch = (L.f + 7) / 8;
    const int items = nch * 4 * L.Mp;
    const float scale = (float)(1.0 / ((double)d.Ny * d.Nz * XB));
    const int taps = d.ky < KPREP_TAPS_XB ? d.ky : KPREP_TAPS_XB;
    k_kprep_yb<K><<<dim3((items + 255) / 256, (d.Ny + KB_OY - 1) / KB_OY, d.zc), dim3(256),
                    sizeof(float2) * KB_OY * (size_t)taps, st>>>(L.A1, L.A, L.twy, d.Ny, d.ky, L.fp, L.Mp, nch, scale);
    if (hipGetLastError() != hipSuccess) return ZNNI_ERR_HIP;
    return ZNNI_OK;
}

// Second stage of the kernel transform for this route (the first, along z, is the one of mac.hip).
znni_status launch_kprep_yb(const LayerPlan& L, hipStream_t st)
{
    switch (L.d.kx) {
        case 4: return launch_kprep_yb_k<4>(L, st);
        case 5: return launch_kprep_yb_k<5>(L, st);
    }
    return ZNNI_ERR_UNSUPPORTED_SIZE;
}

template <int RTW, bool WIDE>
static znni_status launch_xb(const LayerPlan& L, int accumulate, int m_base, int nmblk, hipStream_t st)
{
    const Dims& d = L.d;
    XbArgs g;
    g.X2 = L.buf1; g.Ah = L.A; g.Yd = L.Yt;
    g.ximg = (size_t)d.x2i * d.ldx; g.xpen = (size_t)d.x2o * d.ldx;
    g.yimg = (size_t)d.ydi * d.ldxo; g.ypen = (size_t)d.ydo * d.ldxo;
    g.S = L.S; g.f = L.f; g.fo = L.fo; g.Mp = L.Mp; g.nx = d.nx; g.nox = d.nox; g.ldx = d.ldx; g.ldxo = d.ldxo;
    g.Ny = d.Ny; g.K = d.kx;
    g.nch = (L.f + 7) / 8;
    const int V = XB - d.kx + 1;
    g.nblk = (d.nox + V - 1) / V;
    // (a remainder of more than 16 blocks goes to one more 32-block tile, ragged, rather than to two 16-block ones)
    g.n2 = WIDE ? (g.nblk + 15) / 32 : 0;
    g.n1 = g.nblk > g.n2 * 32 ? (g.nblk - g.n2 * 32 + 15) / 16 : 0;
    g.blk1 = g.n2 * 32;
    g.nmblk = nmblk;
    g.m_base = m_base;
    g.npencils = d.zc * d.Ny;
    g.accumulate = accumulate;
    const int per_pencil = (g.n2 + g.n1) * g.nmblk;
    const long long blocks = (long long)((g.npencils + 7) / 8) * per_pencil * 8;
    const size_t lds = sizeof(float2) * 2 * 8 * 4 * (WIDE ? 32 : 16) * 2;
    k_mac_xb<RTW, WIDE><<<dim3((unsigned)blocks, (unsigned)L.S), dim3(256), lds, st>>>(g);
    if (hipGetLastError() != hipSuccess) return ZNNI_ERR_HIP;
    return ZNNI_OK;
}

template <bool WIDE>
static znni_status launch_xb_rows(const LayerPlan& L, int accumulate, hipStream_t st)
{
    // the 16-row tiles that hold output images, dealt to row blocks of three tiles, then of two (one tile: one block)
    const int q = (L.fo + 15) / 16;
    if (q == 1) return launch_xb<1, WIDE>(L, accumulate, 0, 1, st);
    const int n2 = q % 3 == 0 ? 0 : (q % 3 == 1 ? 2 : 1), n3 = (q - 2 * n2) / 3;
    znni_status rc = ZNNI_OK;
    if (n3) rc = launch_xb<3, WIDE>(L, accumulate, 0, n3, st);
    if (rc == ZNNI_OK && n2) rc = launch_xb<2, WIDE>(L, accumulate, 48 * n3, n2, st);
    return rc;
}

znni_status launch_mac_xb(const LayerPlan& L, int accumulate, hipStream_t st)
{
    if (!mac_xb_available(L)) return ZNNI_ERR_UNSUPPORTED_SIZE;
    const int V = XB - L.d.kx + 1;
    return (L.d.nox + V - 1) / V > 16 ? launch_xb_rows<true>(L, accumulate, st)
                                       : launch_xb_rows<false>(L, accumulate, st);
}

}  // namespace znni
