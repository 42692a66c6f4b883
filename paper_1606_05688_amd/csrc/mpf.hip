// mpf.hip -- max pooling and max-pooling fragments (Section VI).
//
// Max-pooling fragmentation with window p = <px,py,pz> produces, for every offset o = (ox,oy,oz) < p, the max
// pooling of the image shifted by o; with n + 1 divisible by p every fragment has m = floor(n/p) voxels per axis.
// Put differently: the sliding maximum M[X][Y][Z] = max of the p-block starting at (X,Y,Z) is needed at every
// position X < px*mx, Y < py*my, Z < pz*mz, and M[X][Y][Z] is voxel (X/px, Y/py, Z/pz) of fragment (X%px, Y%py, Z%pz).
//
// The layer only moves data (4 bytes in, 4 bytes out per voxel), so the kernel is built to read every input voxel
// from HBM once and to write contiguous runs.  A workgroup owns a tile of TY x ZT positions (Y, Z) and marches
// along x: per input plane it stages (TY+py-1) rows of (ZT+pz-1) voxels in LDS (two LDS planes alternate, one
// barrier per plane; the next plane's loads are already in flight), takes the maximum over the py x pz block of
// each position, and keeps the last px plane results of each of its positions in registers; their maximum is
// M[x-px+1][Y][Z].  Positions are numbered so that consecutive lanes hold
// consecutive voxels of one fragment row, so a wave stores contiguous runs.  Re-read overhead: the py-1 halo rows,
// the pz-1 halo columns and the px-1 halo planes per chunk of x.
#include <stdint.h>

#include "znni_internal.h"

namespace znni {

constexpr int MPF_TY = 16;      // Y positions per tile
constexpr int MPF_PMAX = 4;     // largest window per axis
// A tile covers at most ZT = 128 or 256 positions along z (template parameter; 256 or 512 threads): the wider
// tile reads whole rows of images up to 256 voxels wide in one piece, which HBM serves faster than two half rows.

struct MpfArgs {
    int nx, ny, nz;      // image
    int py, pz;          // window (px is a template parameter)
    int mx, my, mz;      // fragment size
    int f;               // images per tuple
    int CT;              // fragment columns per tile (tile covers pz*CT positions along z)
    int nyt, nzt;        // tiles along y and z
    int XC;              // x positions per chunk (a multiple of px)
};

// PX: window along x.  PY, PZ: windows along y and z when known at compile time, 0 = take them from the arguments.
template <int PX, int PY, int PZ, int MPF_ZT>
__global__ __launch_bounds__(2 * MPF_ZT) void k_mpf(const float* __restrict__ in, float* __restrict__ out, MpfArgs a)
{
    constexpr int NT = 2 * MPF_ZT;                                                            // threads
    constexpr int MPF_NP = MPF_TY * MPF_ZT / NT;                                              // positions per thread
    constexpr int MPF_NL = ((MPF_TY + MPF_PMAX - 1) * (MPF_ZT + MPF_PMAX - 1) + NT - 1) / NT; // staged voxels per thread
    constexpr int RAW = (MPF_TY + MPF_PMAX - 1) * (MPF_ZT + MPF_PMAX - 1);
    __shared__ float raw[2][RAW];                        // two planes: one being read, one being filled
    const int t = threadIdx.x;
    const int zt = blockIdx.x % a.nzt, yt = (blockIdx.x / a.nzt) % a.nyt, xc = blockIdx.x / (a.nzt * a.nyt);
    const int img = blockIdx.y;
    const int py = PY ? PY : a.py, pz = PZ ? PZ : a.pz, nz = a.nz;
    const int Yn = py * a.my, Zn = pz * a.mz, Xn = PX * a.mx;
    const int ZT = pz * a.CT;
    const int Y0 = yt * MPF_TY, Z0 = zt * ZT, X0 = xc * a.XC;
    const int TYv = min(MPF_TY, Yn - Y0), ZTv = min(ZT, Zn - Z0);
    const int Xend = min(X0 + a.XC, Xn);                 // positions X0 .. Xend-1, input planes X0 .. Xend+PX-2
    const int rows = TYv + py - 1, W = ZTv + pz - 1;     // staged block of one plane
    const int CTv = ZTv / pz;                            // fragment columns present in this tile

    // ---- staged voxels of this thread: offset inside a plane (clamped to a valid one) and LDS slot
    int goff[MPF_NL], loff[MPF_NL];
#pragma unroll
    for (int i = 0; i < MPF_NL; ++i) {
        const int e = t + NT * i;
        const bool ok = e < rows * W;
        const int ec = ok ? e : 0;
        const int r = ec / W, c = ec - r * W;
        goff[i] = (Y0 + r) * nz + Z0 + c;
        loff[i] = ok ? r * W + c : -1;
    }
    // ---- positions of this thread: LDS slot of the block's first voxel and where the result goes inside its
    // fragment.  Position e = (Yl, oz, c) with c fastest: consecutive lanes hold consecutive voxels of one
    // fragment row.
    int roff[MPF_NP];
    size_t ooff[MPF_NP];
    const size_t fragvox = (size_t)a.mx * a.my * a.mz;
    const int s = img / a.f, i_in = img - s * a.f;
    const int alpha = PX * py * pz;
#pragma unroll
    for (int i = 0; i < MPF_NP; ++i) {
        const int e = t + NT * i;
        const int Yl = e / ZT, rem = e - Yl * ZT;
        const int oz = rem / a.CT, c = rem - oz * a.CT;
        const bool ok = Yl < TYv && c < CTv;
        roff[i] = ok ? Yl * W + oz + pz * c : -1;
        const int Y = Y0 + Yl, oy = Y % py, b = Y / py;
        const int batch0 = s * alpha + oy * pz + oz;             // fragment of offset (0, oy, oz)
        ooff[i] = ((size_t)batch0 * a.f + i_in) * fragvox + (size_t)b * a.mz + (Z0 / pz + c);
    }
    const size_t ox_stride = (size_t)py * pz * a.f * fragvox;   // from fragment (ox, ., .) to (ox+1, ., .)
    const size_t a_stride = (size_t)a.my * a.mz;

    const float* plane = in + ((size_t)img * a.nx + X0) * a.ny * nz;
    const size_t plane_stride = (size_t)a.ny * nz;
    float v[MPF_NL];
#pragma unroll
    for (int i = 0; i < MPF_NL; ++i) v[i] = plane[goff[i]];

    float ring[PX][MPF_NP];
    const int nplanes = Xend - X0 + PX - 1;
    for (int xb = 0; xb < nplanes; xb += PX) {
#pragma unroll
        for (int r = 0; r < PX; ++r) {
            const int xl = xb + r;                       // plane X0 + xl
            if (xl < nplanes) {                          // uniform over the workgroup
                float* cur = raw[xl & 1];                // its readers of two planes ago passed the last barrier
#pragma unroll
                for (int i = 0; i < MPF_NL; ++i)
                    if (loff[i] >= 0) cur[loff[i]] = v[i];
                __syncthreads();
                if (xl + 1 < nplanes) {                  // next plane: loads stay in flight during the arithmetic
                    const float* nxt = plane + (size_t)(xl + 1) * plane_stride;
#pragma unroll
                    for (int i = 0; i < MPF_NL; ++i) v[i] = nxt[goff[i]];
                }
                const int X = max(X0 + xl - (PX - 1), 0);        // results exist from plane PX-1 of the chunk on
                float* obase = out + (size_t)(X % PX) * ox_stride + (size_t)(X / PX) * a_stride;
#pragma unroll
                for (int i = 0; i < MPF_NP; ++i) {       // maximum over the y-z block, then along x
                    if (roff[i] < 0) continue;
                    const float* p = cur + roff[i];
                    float m = p[0];
                    for (int b = 0; b < py; ++b)
                        for (int c = 0; c < pz; ++c) m = fmaxf(m, p[b * W + c]);
                    ring[r][i] = m;
                    if (xl >= PX - 1) {
                        float mm = ring[0][i];
#pragma unroll
                        for (int q = 1; q < PX; ++q) mm = fmaxf(mm, ring[q][i]);
                        obase[ooff[i]] = mm;
                    }
                }
            }
        }
    }
}

// Plain max pooling: one thread per output voxel, lanes along the contiguous axis.
__global__ __launch_bounds__(256) void k_maxpool(const float* __restrict__ in, float* __restrict__ out, int ny,
                                                 int nz, int px, int py, int pz, int mx, int my, int mz)
{
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= mz) return;
    const int b = blockIdx.y % my, a = blockIdx.y / my;
    const size_t img = blockIdx.z;
    const float* src = in + ((img * (size_t)(mx * px) + (size_t)a * px) * ny + (size_t)b * py) * nz + (size_t)c * pz;
    float m = src[0];
    for (int u = 0; u < px; ++u)
        for (int v = 0; v < py; ++v)
            for (int w = 0; w < pz; ++w) m = fmaxf(m, src[((size_t)u * ny + v) * nz + w]);
    out[((img * mx + a) * my + b) * (size_t)mz + c] = m;
}

template <int PX>
static znni_status launch_mpf_t(const float* in, float* out, const MpfArgs& a, int nimg, hipStream_t st)
{
    const int nxc = (PX * a.mx + a.XC - 1) / a.XC;
    const dim3 grid((unsigned)(a.nyt * a.nzt * nxc), (unsigned)nimg);
    const bool wide = a.pz * a.CT > 128;
    if (a.py == PX && a.pz == PX) {    // cubic windows: all three extents known at compile time
        if (wide) k_mpf<PX, PX, PX, 256><<<grid, dim3(512), 0, st>>>(in, out, a);
        else k_mpf<PX, PX, PX, 128><<<grid, dim3(256), 0, st>>>(in, out, a);
    } else {
        if (wide) k_mpf<PX, 0, 0, 256><<<grid, dim3(512), 0, st>>>(in, out, a);
        else k_mpf<PX, 0, 0, 128><<<grid, dim3(256), 0, st>>>(in, out, a);
    }
    if (hipGetLastError() != hipSuccess) return ZNNI_ERR_HIP;
    return ZNNI_OK;
}

static znni_status pool_shape(int S, int f, const int n[3], const int p[3])
{
    if (!n || !p) return ZNNI_ERR_NULL;
    if (S < 1 || f < 1) return ZNNI_ERR_SHAPE;
    for (int d = 0; d < 3; ++d)
        if (n[d] < 1 || p[d] < 1 || p[d] > n[d] || n[d] > 4096) return ZNNI_ERR_SHAPE;
    if ((long long)S * f > 65535) return ZNNI_ERR_SHAPE;
    return ZNNI_OK;
}

}  // namespace znni

using namespace znni;

extern "C" {

znni_status znni_mpf(int S, int f, const int n[3], const int p[3], const float* in, float* out, void* stream)
{
    znni_status rc = pool_shape(S, f, n, p);
    if (rc) return rc;
    if (!in || !out) return ZNNI_ERR_NULL;
    for (int d = 0; d < 3; ++d) {
        if (p[d] > MPF_PMAX) return ZNNI_ERR_UNSUPPORTED_SIZE;
        if (p[d] > 1 && (n[d] + 1) % p[d]) return ZNNI_ERR_SHAPE;
    }
    if (((uintptr_t)in | (uintptr_t)out) & 3u) return ZNNI_ERR_ALIGN;
    MpfArgs a;
    a.nx = n[0]; a.ny = n[1]; a.nz = n[2];
    a.py = p[1]; a.pz = p[2];
    a.mx = n[0] / p[0]; a.my = n[1] / p[1]; a.mz = n[2] / p[2];
    a.f = f;
    if ((long long)S * p[0] * p[1] * p[2] * f > (1ll << 31) - 1) return ZNNI_ERR_SHAPE;
    // fragment columns per tile: 256 positions along z when the image is wider than 128, else 128
    const int zt_max = a.pz * a.mz > 128 ? 256 : 128;
    a.CT = a.mz < zt_max / a.pz ? a.mz : zt_max / a.pz;
    a.nzt = (a.mz + a.CT - 1) / a.CT;
    a.nyt = (a.py * a.my + MPF_TY - 1) / MPF_TY;
    // x positions per chunk: about 32 planes, so the px-1 halo planes cost a few percent and there are enough
    // workgroups to fill the machine
    a.XC = ((32 + p[0] - 1) / p[0]) * p[0];
    hipStream_t st = (hipStream_t)stream;
    switch (p[0]) {
        case 1: return launch_mpf_t<1>(in, out, a, S * f, st);
        case 2: return launch_mpf_t<2>(in, out, a, S * f, st);
        case 3: return launch_mpf_t<3>(in, out, a, S * f, st);
        case 4: return launch_mpf_t<4>(in, out, a, S * f, st);
    }
    return ZNNI_ERR_UNSUPPORTED_SIZE;
}

znni_status znni_maxpool(int S, int f, const int n[3], const int p[3], const float* in, float* out, void* stream)
{
    znni_status rc = pool_shape(S, f, n, p);
    if (rc) return rc;
    if (!in || !out) return ZNNI_ERR_NULL;
    for (int d = 0; d < 3; ++d)
        if (n[d] % p[d]) return ZNNI_ERR_SHAPE;
    if (((uintptr_t)in | (uintptr_t)out) & 3u) return ZNNI_ERR_ALIGN;
    const int mx = n[0] / p[0], my = n[1] / p[1], mz = n[2] / p[2];
    if ((long long)mx * my > 65535) return ZNNI_ERR_SHAPE;
    k_maxpool<<<dim3((unsigned)((mz + 255) / 256), (unsigned)(mx * my), (unsigned)(S * f)), dim3(256), 0,
                (hipStream_t)stream>>>(in, out, n[1], n[2], p[0], p[1], p[2], mx, my, mz);
    if (hipGetLastError() != hipSuccess) return ZNNI_ERR_HIP;
    return ZNNI_OK;
}

}  // extern "C"
