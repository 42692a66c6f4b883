// direct.hip -- the convolutional layer by direct convolution (Section IV-A-1), for small kernels and few images.
//
// The layer equation O[s][j] = act(bias[j] + sum_i w[j][i] * I[s][i]) written out per output voxel is one dense
// contraction over the index (i, a, b, c) = (input image, kernel tap):
//
//     O[s][j][x][y][z] = sum_{i,a,b,c} w[j][i][a][b][c] * I[s][i][x+kx-1-a][y+ky-1-b][z+kz-1-c],
//
// a matrix product of the f' x (f kx ky kz) kernel bank with a (f kx ky kz) x (voxels) matrix of shifted image
// values that is never formed: it runs on the matrix cores (v_mfma_f32_16x16x4_f32) with the shifted values read
// from an image tile staged in LDS.  Where the paper's direct algorithm (Algorithm 1) loops over (s, j) in
// parallel and over i serially, convolving whole images, here the parallel unit is a tile of output voxels for
// all output images at once, so every staged input voxel is used by all f' kernels and all taps.
//
// Workgroup = 4 waves = one tile of output voxels of one input s, one block of 16*RTW output images.  Two tile
// shapes: compact, TX x 4 x 32 voxels (TX = 1 or 2), whose staged image tile has the smallest halo, for layers
// with many input images; and long, 1 x TY x 128 (TY = 1 or 2), for layers with so little arithmetic per output
// voxel (first layers: one input image) that the output write is the bound, where it makes stores run along whole
// z rows.  A wave owns CTW column tiles (16 consecutive z each) and all RTW row tiles.  The contraction
// walks input images in chunks of IC (their tiles, with a halo of k-1, are staged in LDS), and inside an image
// the taps in steps of four (tap count padded to a multiple of four with zero weights).  Per step a lane reads
// its tap's offset inside the tile from a small table, one image value per column tile from LDS, and its kernel
// values from a bank rearranged once per call into the operand layout ([i][step][row tile][tap%4][row%16], so
// a wave's load is one 256-byte run).
#include <stdint.h>

#include "znni_internal.h"

namespace znni {

typedef float floatx4_d __attribute__((ext_vector_type(4)));

constexpr int DIRECT_NQ = 12;     // staged voxels per thread and image, at most
// tile shape for CTW column tiles per wave (16 or 8 column tiles per workgroup), compact or long
template <int CTW, bool LONGZ> struct DirectTile {
    static constexpr int TZ = LONGZ ? 128 : 32, ZT = TZ / 16;
    static constexpr int TY = LONGZ ? CTW / 2 : 4;
    static constexpr int TX = LONGZ ? 1 : CTW / 2;
};

struct DirectArgs {
    const float* in;
    const float* Wp;
    const float* bias;
    float* out;
    Dims d;          // image, kernel and output sizes (transform sizes unused)
    int S, f, fo;
    int T4;          // taps per image, rounded up to a multiple of 4
    int RT;          // row tiles of the rearranged bank (16 output images each)
    int IC;          // images per staged chunk
    int ntx, nty, ntz;
    int relu;
    int ty_magic;    // long tiles: 65536 / (rows of the staged tile along y) + 1, for divisions of small numbers
};

// Wp[i][st][rt][kk][r] = w[rt*16 + r][i][tap st*4 + kk], zero beyond fo or beyond the last tap.
__global__ void k_direct_prep(const float* __restrict__ w, float* __restrict__ Wp, int f, int fo, int taps, int T4,
                              int RT, size_t wj_stride, size_t total)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int r = idx & 15, kk = (idx >> 4) & 3;
    size_t q = idx >> 6;
    const int rt = q % RT; q /= RT;
    const int steps = T4 >> 2;
    const int st = q % steps;
    const int i = (int)(q / steps);
    const int j = rt * 16 + r, tap = st * 4 + kk;
    Wp[idx] = (i < f && j < fo && tap < taps) ? w[(size_t)j * wj_stride + (size_t)i * taps + tap] : 0.f;
}

template <int RTW, int CTW, bool LONGZ>
__global__ __launch_bounds__(256) void k_direct(DirectArgs a)
{
    using TL = DirectTile<CTW, LONGZ>;
    constexpr int TX = TL::TX, TY = TL::TY, TZ = TL::TZ, ZT = TL::ZT;
    extern __shared__ float lds[];
    int* delta = reinterpret_cast<int*>(lds);        // [T4]
    float* tile = lds + a.T4;                        // [IC][tilevol]
    const Dims& d = a.d;
    const int t = threadIdx.x, wave = t >> 6, lane = t & 63, l16 = lane & 15, kk = lane >> 4;
    const int TXI = TX + d.kx - 1, TYI = TY + d.ky - 1, TZI = TZ + d.kz - 1;
    const int tilevol = TXI * TYI * TZI;
    const int taps = d.kx * d.ky * d.kz;

    // Tiles that are neighbours in memory go to one XCD, one after the other: hardware deals consecutive workgroup
    // ids round-robin to the 8 XCDs, each with an L2 of its own, and the cache lines that two neighbouring tiles
    // both write part of (rows of an output image are not multiples of 128 bytes) then meet in one L2.
    int tile_id;
    {
        const int nb = gridDim.x, xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        const int per = nb >> 3, rem = nb & 7;
        tile_id = xcd * per + min(xcd, rem) + slot;
    }
    const int tz = tile_id % a.ntz, ty = (tile_id / a.ntz) % a.nty, tx = tile_id / (a.ntz * a.nty);
    const int x0 = tx * TX, y0 = ty * TY, z0 = tz * TZ;
    const int s = blockIdx.y;
    const int rt0 = blockIdx.z * RTW;

    for (int q = t; q < a.T4; q += 256) {
        int dl = 0;
        if (q < taps) {
            const int c = q % d.kz, b = (q / d.kz) % d.ky, aa = q / (d.kz * d.ky);
            dl = ((d.kx - 1 - aa) * TYI + (d.ky - 1 - b)) * TZI + (d.kz - 1 - c);
        }
        delta[q] = dl;
    }
    // staged voxels of this thread (compact tiles): offset inside an image (clamped into it).  Long tiles are
    // staged by rows instead, see below.
    int goff[DIRECT_NQ];
    if constexpr (!LONGZ) {
#pragma unroll
        for (int q = 0; q < DIRECT_NQ; ++q) {
            goff[q] = 0;
            if (256 * q < tilevol) {                 // uniform: small kernels need only the first few
                const int e = min(t + 256 * q, tilevol - 1);
                const int lz = e % TZI, ly = (e / TZI) % TYI, lx = e / (TZI * TYI);
                const int gx = min(x0 + lx, d.nx - 1), gy = min(y0 + ly, d.ny - 1), gz = min(z0 + lz, d.nz - 1);
                goff[q] = (gx * d.ny + gy) * d.nz + gz;
            }
        }
    }
    const int wv = __builtin_amdgcn_readfirstlane(wave);      // wave-uniform, and known to be
    // column tiles of this wave: (tx, ty) pair and 16-voxel piece of the z run
    int voxbase[CTW];
#pragma unroll
    for (int c = 0; c < CTW; ++c) {
        const int ct = wave * CTW + c;
        const int zt = ct % ZT, pair = ct / ZT;
        const int vy = pair % TY, vx = pair / TY;
        voxbase[c] = (vx * TYI + vy) * TZI + zt * 16 + l16;
    }

    floatx4_d acc[RTW][CTW];
#pragma unroll
    for (int r = 0; r < RTW; ++r)
#pragma unroll
        for (int c = 0; c < CTW; ++c) acc[r][c] = floatx4_d{0.f, 0.f, 0.f, 0.f};
    // biases of the output images this lane's accumulator elements belong to (requested now, used at the end)
    float bj[RTW][4];
#pragma unroll
    for (int r = 0; r < RTW; ++r)
#pragma unroll
        for (int e = 0; e < 4; ++e) bj[r][e] = 0.f;
    if (a.bias) {                                    // one uniform branch; output images past the last are not stored
#pragma unroll
        for (int r = 0; r < RTW; ++r) {
            const float* bp = a.bias + min((rt0 + r) * 16 + 4 * kk, a.fo - 1);
            const int left = a.fo - 1 - ((rt0 + r) * 16 + 4 * kk);       // last valid element of this group of four
#pragma unroll
            for (int e = 0; e < 4; ++e) bj[r][e] = bp[max(min(e, left), 0)];
        }
    }

    const size_t nvox = (size_t)d.nx * d.ny * d.nz;
    const int steps = a.T4 >> 2;
    for (int ic0 = 0; ic0 < a.f; ic0 += a.IC) {
        const int icn = min(a.IC, a.f - ic0);
        __syncthreads();                             // the previous chunk has been consumed
        for (int il = 0; il < icn; ++il) {
            const float* img = a.in + ((size_t)s * a.f + ic0 + il) * nvox;
            if constexpr (LONGZ) {
                // a wave per (x, y) row of the tile, lanes along z: the row's address is scalar arithmetic.  (With
                // one or a few input images a voxel offset per thread, computed with divisions, is used too
                // rarely to pay for itself.)
                // Two rows per wave and three runs of 64 per row are requested before the first is written.
                const int nrows = TXI * TYI;
                for (int rg = 0; rg < nrows; rg += 8) {
                    for (int zg = 0; zg < TZI; zg += 192) {
                        float v[2][3];
#pragma unroll
                        for (int ri = 0; ri < 2; ++ri) {
                            const int row = min(rg + 4 * ri + wv, nrows - 1);
                            const int lx = (row * a.ty_magic) >> 16, ly = row - lx * TYI;     // row / TYI
                            const float* src =
                                img + ((size_t)min(x0 + lx, d.nx - 1) * d.ny + min(y0 + ly, d.ny - 1)) * d.nz;
#pragma unroll
                            for (int zi = 0; zi < 3; ++zi)
                                v[ri][zi] = src[min(z0 + min(zg + 64 * zi + lane, TZI - 1), d.nz - 1)];
                        }
#pragma unroll
                        for (int ri = 0; ri < 2; ++ri) {
                            const int row = rg + 4 * ri + wv;
#pragma unroll
                            for (int zi = 0; zi < 3; ++zi) {
                                const int z = zg + 64 * zi + lane;
                                if (row < nrows && z < TZI) tile[il * tilevol + row * TZI + z] = v[ri][zi];
                            }
                        }
                    }
                }
            } else {
                float v[DIRECT_NQ];
#pragma unroll
                for (int q = 0; q < DIRECT_NQ; ++q)
                    if (256 * q < tilevol) v[q] = img[goff[q]];
#pragma unroll
                for (int q = 0; q < DIRECT_NQ; ++q)
                    if (t + 256 * q < tilevol) tile[il * tilevol + t + 256 * q] = v[q];
            }
        }
        __syncthreads();
        // all steps of the chunk in one flat loop; the kernel values of the next step are requested before the
        // matrix instructions of the current one (past the last step this reads the following image's values or
        // the padding behind the bank; they are not used)
        const float* Ab = a.Wp + (((size_t)ic0 * steps) * a.RT + rt0) * 64 + lane;
        const int nst = icn * steps;
        float an[RTW];
#pragma unroll
        for (int r = 0; r < RTW; ++r) an[r] = Ab[r * 64];
        int st = 0, tbase = 0;                       // step inside the image, start of the image's tile
        for (int g = 0; g < nst; ++g) {
            __builtin_amdgcn_iglp_opt(0);            // interleave the loads with the matrix instructions: 3-6 %
            float av[RTW], bv[CTW];
#pragma unroll
            for (int r = 0; r < RTW; ++r) av[r] = an[r];
            const float* nxt = Ab + (size_t)(g + 1) * a.RT * 64;
#pragma unroll
            for (int r = 0; r < RTW; ++r) an[r] = nxt[r * 64];
            const int dl = delta[st * 4 + kk] + tbase;
#pragma unroll
            for (int c = 0; c < CTW; ++c) bv[c] = tile[voxbase[c] + dl];
#pragma unroll
            for (int r = 0; r < RTW; ++r)
#pragma unroll
                for (int c = 0; c < CTW; ++c)
                    acc[r][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[r], bv[c], acc[r][c], 0, 0, 0);
            if (++st == steps) { st = 0; tbase += tilevol; }
        }
    }

    // Result through LDS, one row tile (16 output images) at a time, so that stores run along z:
    // Ol[j<16][pair][z<TZ] (the tile's voxels of one output image are TX*TY runs of TZ voxels).  Accumulator
    // element e of lane l: output image 16*r + 4*(l/16) + e of the block, voxel l%16 of the column tile.
    float* Ol = lds;
    constexpr int NPAIR = TX * TY, OP = NPAIR * TZ + 1;     // floats per output image in the tile (+1: banks)
    const size_t ovox = (size_t)d.nox * d.noy * d.noz;
#pragma unroll
    for (int r = 0; r < RTW; ++r) {
        __syncthreads();
#pragma unroll
        for (int c = 0; c < CTW; ++c) {
            const int ct = wave * CTW + c;
            const int zt = ct % ZT, pair = ct / ZT;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float v = acc[r][c][e] + bj[r][e];
                if (a.relu) v = fmaxf(v, 0.f);
                Ol[(4 * kk + e) * OP + pair * TZ + zt * 16 + l16] = v;
            }
        }
        __syncthreads();
        if constexpr (LONGZ) {
            // A wave per row (output image, x, y) of the tile, lanes along z.  Rows wv, wv + 4, ... are the same
            // (x, y) of every (4 / NPAIR)-th output image: one address per wave, then a constant stride, and all
            // of a wave's values leave LDS before the first store.
            constexpr int RPW = 4 * NPAIR, JS = 4 / NPAIR;       // rows per wave, output images between them
            static_assert(NPAIR == 1 || NPAIR == 2, "long tiles have one or two (x, y) rows");
            const int pair = wv % NPAIR, jl0 = wv / NPAIR;
            const int X = x0 + pair / TY, Y = y0 + pair % TY;
            const int j0 = (rt0 + r) * 16 + jl0;
            const int nrow = (X < d.nox && Y < d.noy) ? (a.fo - j0 + JS - 1) / JS : 0;      // rows to store: i < nrow
            float val[RPW][TZ / 64];
            const float* src = Ol + jl0 * OP + pair * TZ + lane;
#pragma unroll
            for (int i = 0; i < RPW; ++i)
#pragma unroll
                for (int zi = 0; zi < TZ / 64; ++zi) val[i][zi] = src[i * JS * OP + 64 * zi];
            float* dst = a.out + ((size_t)s * a.fo + j0) * ovox + ((size_t)X * d.noy + Y) * d.noz + z0 + lane;
#pragma unroll
            for (int i = 0; i < RPW; ++i) {
#pragma unroll
                for (int zi = 0; zi < TZ / 64; ++zi)
                    if (i < nrow && z0 + lane + 64 * zi < d.noz) dst[64 * zi] = val[i][zi];
                dst += (size_t)JS * ovox;
            }
        } else {
            for (int e = t; e < 16 * NPAIR * TZ; e += 256) {        // lanes along z, then (x, y), then output image
                const int zl = e % TZ, row = e / TZ;
                const int jl = row / NPAIR, pair = row - jl * NPAIR;
                const int j = (rt0 + r) * 16 + jl;
                const int X = x0 + pair / TY, Y = y0 + pair % TY, Z = z0 + zl;
                if (j >= a.fo || X >= d.nox || Y >= d.noy || Z >= d.noz) continue;
                a.out[((size_t)s * a.fo + j) * ovox + ((size_t)X * d.noy + Y) * d.noz + Z] =
                    Ol[jl * OP + pair * TZ + zl];
            }
        }
    }
}

struct DirectPlan {
    Dims d;
    int S, f, fo;
    int taps, T4, RT, RTW, CTW, nmblk, IC;
    bool longz;      // tile shape
    size_t lds, wp_floats, bytes;
};

static znni_status direct_plan(int S, int f, int fo, const int n[3], const int k[3], DirectPlan* P)
{
    if (!n || !k) return ZNNI_ERR_NULL;
    if (S < 1 || f < 1 || fo < 1) return ZNNI_ERR_SHAPE;
    for (int a = 0; a < 3; ++a)
        if (n[a] < 1 || k[a] < 1 || k[a] > n[a]) return ZNNI_ERR_SHAPE;
    if (S > 65535) return ZNNI_ERR_SHAPE;
    if ((long long)n[0] * n[1] * n[2] > (1ll << 31) - 1) return ZNNI_ERR_SHAPE;
    Dims& d = P->d;
    d.nx = n[0]; d.ny = n[1]; d.nz = n[2];
    d.kx = k[0]; d.ky = k[1]; d.kz = k[2];
    d.Nx = d.Ny = d.Nz = 0; d.zc = d.ldy = d.ldx = d.ldo = 0;
    d.nox = n[0] - k[0] + 1; d.noy = n[1] - k[1] + 1; d.noz = n[2] - k[2] + 1;
    P->S = S; P->f = f; P->fo = fo;
    P->taps = k[0] * k[1] * k[2];
    P->T4 = (P->taps + 3) & ~3;
    const int rt = (fo + 15) / 16;
    if (rt <= 4) { P->nmblk = 1; P->RTW = rt; P->CTW = 4; }
    else if (rt == 5) { P->nmblk = 1; P->RTW = 5; P->CTW = 2; }
    else { P->nmblk = (rt + 3) / 4; P->RTW = (rt + P->nmblk - 1) / P->nmblk; P->CTW = 4; }
    P->RT = P->nmblk * P->RTW;
    if (P->nmblk > 65535) return ZNNI_ERR_SHAPE;
    // long tiles when a voxel of output costs little arithmetic (few input images x taps) and the longer halo
    // still fits the staging registers
    const long long vol_long = (long long)k[0] * (P->CTW / 2 + k[1] - 1) * (128 + k[2] - 1);
    P->longz = (long long)f * P->T4 <= 128 && vol_long <= 256 * DIRECT_NQ;
    const int TX = P->longz ? 1 : P->CTW / 2, TY = P->longz ? P->CTW / 2 : 4, TZ = P->longz ? 128 : 32;
    const long long tilevol = (long long)(TX + k[0] - 1) * (TY + k[1] - 1) * (TZ + k[2] - 1);
    if (tilevol > 256 * DIRECT_NQ) return ZNNI_ERR_UNSUPPORTED_SIZE;      // kernel too large for this primitive
    int IC = (int)((48 * 1024 - 4 * P->T4) / (4 * tilevol));
    if (IC < 1) return ZNNI_ERR_UNSUPPORTED_SIZE;
    if (IC > 8) IC = 8;
    if (IC > f) IC = f;
    P->IC = IC;
    P->lds = 4 * ((size_t)P->T4 + (size_t)IC * tilevol);
    const size_t out_tile = 4 * (size_t)16 * (TX * TY * TZ + 1);
    if (out_tile > P->lds) P->lds = out_tile;
    P->wp_floats = (size_t)f * P->T4 * P->RT * 16;
    // + one step of padding: the kernel requests its kernel values one step ahead
    P->bytes = ((P->wp_floats + (size_t)P->RT * 64) * 4 + 255) / 256 * 256;
    return ZNNI_OK;
}

template <int RTW, int CTW, bool LONGZ>
static znni_status launch_direct_s(const DirectArgs& a, const DirectPlan& P, hipStream_t st)
{
    using TL = DirectTile<CTW, LONGZ>;
    DirectArgs b = a;
    b.ntx = (P.d.nox + TL::TX - 1) / TL::TX;
    b.nty = (P.d.noy + TL::TY - 1) / TL::TY;
    b.ntz = (P.d.noz + TL::TZ - 1) / TL::TZ;
    b.ty_magic = 65536 / (TL::TY + P.d.ky - 1) + 1;                       // exact for numerators below 65536 / TYI
    const long long tiles = (long long)b.ntx * b.nty * b.ntz;
    if (tiles > 0x7fffffffll) return ZNNI_ERR_SHAPE;
    if (P.lds > 48 * 1024 &&
        hipFuncSetAttribute((const void*)k_direct<RTW, CTW, LONGZ>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)P.lds) != hipSuccess)
        return ZNNI_ERR_HIP;
    k_direct<RTW, CTW, LONGZ><<<dim3((unsigned)tiles, (unsigned)P.S, (unsigned)P.nmblk), dim3(256), P.lds, st>>>(b);
    if (hipGetLastError() != hipSuccess) return ZNNI_ERR_HIP;
    return ZNNI_OK;
}

template <int RTW, int CTW>
static znni_status launch_direct_t(const DirectArgs& a, const DirectPlan& P, hipStream_t st)
{
    return P.longz ? launch_direct_s<RTW, CTW, true>(a, P, st) : launch_direct_s<RTW, CTW, false>(a, P, st);
}

}  // namespace znni

using namespace znni;

extern "C" {

znni_status znni_conv3d_direct_workspace_v(int S, int f, int fo, const int n[3], const int k[3], size_t* bytes)
{
    if (!bytes) return ZNNI_ERR_NULL;
    DirectPlan P;
    znni_status rc = direct_plan(S, f, fo, n, k, &P);
    if (rc) return rc;
    *bytes = P.bytes;
    return ZNNI_OK;
}

znni_status znni_conv3d_direct_v(int S, int f, int fo, const int n[3], const int k[3], const float* in,
                                 const float* w, const float* bias, float* out, unsigned flags, void* workspace,
                                 size_t workspace_bytes, void* stream)
{
    if (!in || !w || !out || !workspace) return ZNNI_ERR_NULL;
    if (flags & ~(unsigned)ZNNI_RELU) return ZNNI_ERR_FLAGS;
    DirectPlan P;
    znni_status rc = direct_plan(S, f, fo, n, k, &P);
    if (rc) return rc;
    if (((uintptr_t)in | (uintptr_t)w | (uintptr_t)out) & 3u) return ZNNI_ERR_ALIGN;
    if ((uintptr_t)workspace & 255u) return ZNNI_ERR_ALIGN;
    if (workspace_bytes < P.bytes) return ZNNI_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    float* Wp = (float*)workspace;
    const size_t wp_all = P.wp_floats + (size_t)P.RT * 64;        // the look-ahead padding is zeroed too
    k_direct_prep<<<dim3((unsigned)((wp_all + 255) / 256)), dim3(256), 0, st>>>(
        w, Wp, f, fo, P.taps, P.T4, P.RT, (size_t)f * P.taps, wp_all);
    if (hipGetLastError() != hipSuccess) return ZNNI_ERR_HIP;
    DirectArgs a;
    a.in = in; a.Wp = Wp; a.bias = bias; a.out = out;
    a.d = P.d; a.S = S; a.f = f; a.fo = fo;
    a.T4 = P.T4; a.RT = P.RT; a.IC = P.IC;
    a.ntx = a.nty = a.ntz = 0; a.ty_magic = 0;
    a.relu = (flags & ZNNI_RELU) ? 1 : 0;
    switch (P.RTW * 10 + P.CTW) {
        case 14: return launch_direct_t<1, 4>(a, P, st);
        case 24: return launch_direct_t<2, 4>(a, P, st);
        case 34: return launch_direct_t<3, 4>(a, P, st);
        case 44: return launch_direct_t<4, 4>(a, P, st);
        case 52: return launch_direct_t<5, 2>(a, P, st);
    }
    return ZNNI_ERR_SHAPE;
}

}  // extern "C"
