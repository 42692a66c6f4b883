// passes_fast.hip -- the six transform passes for transform lengths N = R1*R2 with both factors small enough
// for an in-register DFT (46 lengths from 8 to 1024, listed in launch_kind).  Same layouts, pruning and results
// as passes.hip.
//
// One workgroup transforms a tile of 16 lines (passes along z: 16 pairs of real lines).  Each line is done in
// two steps.  Step A: thread (line, j < R2) loads the R1 samples j, j+R2, j+2R2, ... straight from HBM into
// registers (16 consecutive j of a line make a 128-byte run), does a length-R1 DFT, multiplies by the
// twiddles w_N^(j q) and parks the result in LDS.  Step B: thread (q < R1, line) picks up the R2 values of
// its q, does a length-R2 DFT and holds outputs q, q+R1, q+2R1, ...; with the line index fastest across
// lanes, the 16 lines of the tile form one 128-byte run per output index, so passes whose output has the next
// axis contiguous store straight from registers.  Passes whose output is contiguous along the transformed
// axis, and the real<->complex passes, go through LDS once more.  Every byte of a tensor is read once and
// written once per pass; LDS sees one exchange per element.
#include "two_step.h"
#include "znni_internal.h"

namespace znni {

// P_FWD_XT: the forward x pass reading the layout the fused z+y kernel leaves, X2'[img][x][oz][oy]: the 16 lines
// of a tile (neighbouring oy) are adjacent elements of every x row, so the pass loads 128-byte runs with the line
// index fastest across lanes (a transposing load instead of the transposing store of the pass before it).
// P_INV_YT: the inverse y pass of layers whose x axis is not transformed, reading Yd[imgo][oz][oy][xo]: the 16 lines
// of a tile (neighbouring xo) are adjacent elements of every oy row -- the same transposing load.
enum PassKind { P_FWD_Z, P_FWD_Y, P_FWD_X, P_INV_X, P_INV_Y, P_INV_Z, P_FWD_XT, P_INV_YT };
constexpr bool pass_loads_transposed(int kind) { return kind == P_FWD_XT || kind == P_INV_YT; }

struct PassArgs {
    const void* src;
    void* dst;
    const float2* tw;      // [N]
    const float* bias;     // inv_z only
    Dims d;
    int nimg, fo, relu;
};

// Inverse x pass: tiles counted over (oz, oy) together?  Measured 9-11 % faster at lengths 56 and 120 (fewer, full
// tiles), but 30 % slower at 100, where the rows of Y2 are padded to whole cache lines and tiles that start
// anywhere in a row make every 128-byte store straddle two lines.
__host__ __device__ inline bool inv_x_flat(const Dims& d) { return d.ldn == d.Ny && d.Ny > 16 && (d.Ny & 15) != 0; }

template <int R1, int R2, int KIND>
__device__ __forceinline__ void pass_body(const PassArgs& a, float2* lds)
{
    using TS = TwoStep<R1, R2>;
    constexpr int N = TS::N, P = TS::P, NTH = TS::NTH;
    float2* tws = lds;
    float2* buf = lds + N;
    // Streaming accesses only where a lane group moves whole 128-byte lines per instruction (R2 = 16 samples of a
    // line in step A): with shorter runs a cache line is shared by several instructions and must stay cached
    // (measured: lengths 48, 100 and 120 lose up to 40 % on the x passes with streaming loads).
    // The first pass does not stream at all: its output is the smallest tensor in flight next to the real input
    // and was measured 5 to 16 % faster with ordinary stores from 128^3 to 320^3 (a tie on the 320-wide workload).
    constexpr bool STREAM = (R2 % 16 == 0) && KIND != P_FWD_Z;
    const int t = threadIdx.x;
    for (int q = t; q < N; q += NTH) tws[q] = a.tw[q];

    const int tile = blockIdx.x, mid = blockIdx.y, img = blockIdx.z;
    const Dims& d = a.d;
    const int zc = d.zc;

    // ---- where the 16 lines of this tile start, how far apart they are, how many exist, how long they are
    const float2* src = nullptr;      // complex passes
    size_t lpitch = 0, epitch = 1;    // from line to line, from element to element
    int nvalid = 0, lin = N;
    if constexpr (KIND == P_FWD_Y) {          // tile: 16 x of one (img, oz); lines along y in X1
        const int x0 = tile * 16, oz = mid;
        src = (const float2*)a.src + (((size_t)img * d.nx + x0) * zc + oz) * d.ldy;
        lpitch = (size_t)zc * d.ldy; nvalid = min(16, d.nx - x0); lin = d.ny;
    } else if constexpr (KIND == P_FWD_XT) {
        // tile: 16 neighbouring (oz, oy) of one img, counted oz * Ny + oy as they lie in X2' and in Xt, so that
        // tiles are full whatever Ny is (mid = 0); element x of line l at x*epitch + l
        const int q0 = tile * 16;
        src = (const float2*)a.src + (size_t)img * d.nx * zc * d.Ny + q0;
        lpitch = 1; epitch = (size_t)zc * d.Ny; nvalid = min(16, zc * d.Ny - q0); lin = d.nx;
    } else if constexpr (KIND == P_FWD_X) {   // tile: 16 oy of one (img, oz); lines along x in X2
        const int oy0 = tile * 16, oz = mid;
        src = (const float2*)a.src + ((size_t)img * d.x2i + (size_t)oz * d.x2o + oy0) * d.ldx;
        lpitch = d.ldx; nvalid = min(16, d.Ny - oy0); lin = d.nx;
    } else if constexpr (KIND == P_INV_X) {
        // tile: 16 oy of one (oz, imgo); or, where rows of Y2 are not padded to whole cache lines anyway and do not
        // divide into tiles, 16 neighbouring (oz, oy) counted oz * Ny + oy as the pencils lie in Yt, so that
        // tiles are full (mid = 0); lines along ox
        const bool flat = inv_x_flat(d);
        const int q0 = flat ? tile * 16 : mid * d.Ny + tile * 16;
        src = (const float2*)a.src + ((size_t)q0 * a.nimg + img) * N;
        lpitch = (size_t)a.nimg * N; nvalid = flat ? min(16, zc * d.Ny - q0) : min(16, d.Ny - tile * 16);
    } else if constexpr (KIND == P_INV_Y) {   // tile: 16 xo of one (imgo, oz); lines along oy, adjacent in Y2
        const int xo0 = tile * 16, oz = mid;
        src = (const float2*)a.src + (((size_t)img * zc + oz) * d.nox + xo0) * d.ldn;
        lpitch = d.ldn; nvalid = min(16, d.nox - xo0);
    } else if constexpr (KIND == P_INV_YT) {  // the same tile in Yd: element oy of line l at oy*ldxo + l
        const int xo0 = tile * 16, oz = mid;
        src = (const float2*)a.src + ((size_t)img * d.ydi + (size_t)oz * d.ydo) * d.ldxo + xo0;
        lpitch = 1; epitch = d.ldxo; nvalid = min(16, d.nox - xo0);
    }

    // ---- step A: loads first (they do not need the twiddle table), then the barrier, then the arithmetic
    // step A thread = (line la, sample offset ja); samples fastest across lanes, except for the transposing load
    constexpr bool LT = pass_loads_transposed(KIND);
    const int ja = LT ? t >> 4 : t % R2, la = LT ? t & 15 : t / R2;
    const bool in_a = t < 16 * R2;
    float2 v[R1];
    // Every load is issued unconditionally from a clamped (always valid, so finite) address and multiplied by
    // a 0/1 mask afterwards: a select would be turned back into a branch around each load, which fences the
    // R1 loads of a thread one by one instead of keeping them all in flight.
    if (in_a) {
        if constexpr (KIND == P_FWD_Z) {
            // two real lines y0+2*la, y0+2*la+1 of one (img, x) ride as real and imaginary part
            const int y0 = tile * 32, x = mid;
            const int ya = y0 + 2 * la;
            const int ny = d.ny, nz = d.nz;
            const float ma = ya < ny ? 1.f : 0.f, mb = ya + 1 < ny ? 1.f : 0.f;
            const float* ra = (const float*)a.src + (((size_t)img * d.nx + x) * ny + min(ya, ny - 1)) * nz;
            const float* rb = (const float*)a.src + (((size_t)img * d.nx + x) * ny + min(ya + 1, ny - 1)) * nz;
#pragma unroll
            for (int m = 0; m < R1; ++m) {
                const int e = ja + R2 * m, ec = min(e, nz - 1);
                const float me = e < nz ? 1.f : 0.f;
                v[m] = make_float2(ra[ec] * (me * ma), rb[ec] * (me * mb));
            }
        } else if constexpr (KIND == P_INV_Z) {
            // filled below, from LDS
        } else {
            const float ml = la < nvalid ? 1.f : 0.f;
            const float2* ls = src + (size_t)min(la, nvalid - 1) * lpitch;
#pragma unroll
            for (int m = 0; m < R1; ++m) {
                const int e = ja + R2 * m;
                const float mk = e < lin ? ml : 0.f;
                const float2 x = ldg<STREAM && (!LT || KIND == P_INV_YT)>(ls + (size_t)min(e, lin - 1) * epitch);
                v[m] = make_float2(x.x * mk, (KIND == P_INV_X || KIND == P_INV_Y || KIND == P_INV_YT) ? -(x.y * mk)
                                                                                                      : x.y * mk);
            }
        }
    }
    if constexpr (KIND == P_INV_Z) {
        // The 32 lines yo0.. of one (imgo, xo) are read from HBM once into LDS: in Y1 they are 32 neighbouring
        // elements (256 bytes) of each of the zc rows.  Thread (ja, la) then assembles Z = A + iB for lines
        // A = yo0+2*la, B = A+1, extended to all N bins by Hermitian symmetry and conjugated for the
        // inverse-by-forward route.
        constexpr int ZC = N / 2 + 1;
        const int yo0 = tile * 32, xo = mid;
        const int rows = min(32, d.noy - yo0);
        const float2* chunk = (const float2*)a.src + (((size_t)img * d.nox + xo) * ZC) * d.ldo + yo0;
        constexpr int ITER = (32 * ZC + NTH - 1) / NTH;
        float2 raw[ITER];
#pragma unroll
        for (int it = 0; it < ITER; ++it) {       // all requests first ...
            const int e = min(t + it * NTH, 32 * ZC - 1);
            const int r = e & 31, o = e >> 5;
            raw[it] = ldg<STREAM>(chunk + (size_t)o * d.ldo + min(r, rows - 1));
        }
#pragma unroll
        for (int it = 0; it < ITER; ++it) {       // ... then the LDS stores, one row of ZC values per line
            const int e = t + it * NTH;
            const int r = e & 31, o = e >> 5;
            const float mk = r < rows ? 1.f : 0.f;
            if (e < 32 * ZC) buf[r * ZC + o] = make_float2(raw[it].x * mk, raw[it].y * mk);
        }
        __syncthreads();
        if (in_a) {
            const float2* ra = buf + (2 * la) * ZC;
            const float2* rb = ra + ZC;
#pragma unroll
            for (int m = 0; m < R1; ++m) {
                const int e = ja + R2 * m;
                const bool direct = e < ZC;
                const int ee = direct ? e : N - e;
                float2 A = ra[ee], B = rb[ee];
                if (!direct) { A = cconj(A); B = cconj(B); }
                v[m] = cconj(cadd(A, mul_pi(B)));
            }
        }
    }
    __syncthreads();                          // twiddle table is in LDS; inverse z: raw lines fully consumed
    if (in_a) TS::step_a(v, la, ja, tws, buf);
    __syncthreads();

    // ---- step B
    const int lb = t & 15, q = t >> 4;        // q < T; only q < R1 has work
    float2 u[R2];
    if (q < R1) TS::step_b(u, lb, q, buf);

    if constexpr (KIND == P_FWD_Y) {
        // X2[img][oz][oy][x0 + lb]
        if (q < R1 && lb < nvalid) {
            float2* o = (float2*)a.dst + ((size_t)img * d.x2i + (size_t)mid * d.x2o) * d.ldx + tile * 16 + lb;
#pragma unroll
            for (int r = 0; r < R2; ++r) stg<STREAM>(o + (size_t)(q + R1 * r) * d.ldx, u[r]);
        }
    } else if constexpr (KIND == P_INV_X) {
        // Y2[imgo][oz][xo][oy], xo = element - (kx-1) in [0, nox); with (oz, oy) counted together the tile's
        // first line by a scalar division, then at most one row further (rows hold more than 16 values)
        if (q < R1 && lb < nvalid) {
            int oz = mid, oy = tile * 16 + lb;
            if (inv_x_flat(d)) {
                const int q0 = tile * 16;
                oz = q0 / d.Ny; oy = q0 - oz * d.Ny + lb;
                if (oy >= d.Ny) { oy -= d.Ny; ++oz; }
            }
            float2* o = (float2*)a.dst + ((size_t)img * zc + oz) * d.nox * d.ldn + oy;
#pragma unroll
            for (int r = 0; r < R2; ++r) {
                const int xo = q + R1 * r - (d.kx - 1);
                if (xo >= 0 && xo < d.nox) stg<STREAM>(o + (size_t)xo * d.ldn, cconj(u[r]));
            }
        }
    } else {
        // second trip through LDS: natural order per line
        __syncthreads();
        if (q < R1) {
#pragma unroll
            for (int r = 0; r < R2; ++r) buf[lb * P + q + R1 * r] = u[r];
        }
        __syncthreads();
        if constexpr (KIND == P_FWD_X || KIND == P_FWD_XT) {
            // Xt[oz][oy0 + l][img][ox]: whole lines, contiguous (P_FWD_XT: mid = 0, oy0 counts oz * Ny + oy)
            const int oy0 = tile * 16;
            for (int l = t / 64; l < nvalid; l += NTH / 64) {
                float2* o = (float2*)a.dst + (((size_t)mid * d.Ny + oy0 + l) * a.nimg + img) * N;
                for (int e = t % 64; e < N; e += 64) stg<STREAM>(o + e, buf[l * P + e]);
            }
        } else if constexpr (KIND == P_INV_Y || KIND == P_INV_YT) {
            // Y1[imgo][xo0 + l][oz][yo]: the valid part of each line, contiguous
            const int xo0 = tile * 16;
            for (int l = t / 64; l < nvalid; l += NTH / 64) {
                float2* o = (float2*)a.dst + (((size_t)img * d.nox + xo0 + l) * zc + mid) * d.ldo;
                const float2* row = buf + l * P + (d.ky - 1);
                for (int e = t % 64; e < d.noy; e += 64) stg<STREAM>(o + e, cconj(row[e]));
            }
        } else if constexpr (KIND == P_FWD_Z) {
            // untangle the two real lines and store X1[img][x][oz][y0 + ll], ll < 32 fastest across lanes
            const int y0 = tile * 32;
            const int ny = d.ny;
            float2* o = (float2*)a.dst + ((size_t)img * d.nx + mid) * zc * d.ldy + y0;
            const int ll = t & 31;
            if (y0 + ll < ny) {
                const float2* row = buf + (ll >> 1) * P;
                for (int oz = t >> 5; oz < zc; oz += NTH / 32) {
                    const float2 z1 = row[oz], z2 = cconj(row[oz ? N - oz : 0]);
                    stg<STREAM>(o + (size_t)oz * d.ldy + ll, (ll & 1) ? cscale(mul_mi(csub(z1, z2)), 0.5f)
                                                               : cscale(cadd(z1, z2), 0.5f));
                }
            }
        } else {   // P_INV_Z: real part -> line 2l, minus imaginary part -> line 2l+1; crop, bias, transfer
            const int yo0 = tile * 32;
            const float bj = a.bias ? a.bias[img % a.fo] : 0.f;
            const int noz = d.noz;
            float* o = (float*)a.dst + (((size_t)img * d.nox + mid) * d.noy + yo0) * noz;
            const int rows = min(32, d.noy - yo0);
            for (int ll = t / 64; ll < rows; ll += NTH / 64) {
                const float2* row = buf + (ll >> 1) * P + (d.kz - 1);
                for (int zo = t % 64; zo < noz; zo += 64) {
                    const float2 c = row[zo];
                    float v = ((ll & 1) ? -c.y : c.x) + bj;
                    if (a.relu) v = fmaxf(v, 0.f);
                    o[(size_t)ll * noz + zo] = v;
                }
            }
        }
    }
}

template <int R1, int R2, int KIND>
__global__ __launch_bounds__(16 * (R1 > R2 ? R1 : R2)) void k_pass(PassArgs a)
{
    extern __shared__ float2 lds[];
    pass_body<R1, R2, KIND>(a, lds);
}

// Lengths from 640 on: the tile's LDS leaves room for one workgroup of 512 threads per CU, two waves per SIMD, and
// the compiler is told so.  (Left to assume more resident waves it holds the kernel to about 90 registers, and from
// 28 samples per thread on it then waits for each pair of loads of the real-to-complex pass before issuing the
// next: 1.6 to 2 TB/s instead of over 4.)
template <int R1, int R2, int KIND>
__global__ __launch_bounds__(16 * (R1 > R2 ? R1 : R2)) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_pass_long(PassArgs a)
{
    extern __shared__ float2 lds[];
    pass_body<R1, R2, KIND>(a, lds);
}

// ------------------------------------------------------------------------------------------- host side
template <int R1, int R2, int KIND>
static znni_status launch_one(const PassArgs& a, dim3 grid, hipStream_t st)
{
    using TS = TwoStep<R1, R2>;
    constexpr bool LONG = TS::LDS_BYTES > 80 * 1024;      // from length 640 on; two tiles of length 576 share a CU
    const void* fn = LONG ? (const void*)k_pass_long<R1, R2, KIND> : (const void*)k_pass<R1, R2, KIND>;
    if (TS::LDS_BYTES > 48 * 1024 &&
        hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, TS::LDS_BYTES) != hipSuccess)
        return ZNNI_ERR_HIP;
    if constexpr (LONG)
        k_pass_long<R1, R2, KIND><<<grid, dim3(TS::NTH), TS::LDS_BYTES, st>>>(a);
    else
        k_pass<R1, R2, KIND><<<grid, dim3(TS::NTH), TS::LDS_BYTES, st>>>(a);
    if (hipGetLastError() != hipSuccess) return ZNNI_ERR_HIP;
    return ZNNI_OK;
}

template <int KIND>
static znni_status launch_kind(int N, const PassArgs& a, dim3 grid, hipStream_t st)
{
    // N = R1 * R2; R2 is even (step B reads its samples in pairs) and 16 where possible (step A then loads
    // 128-byte runs)
    if constexpr (KIND == P_FWD_Z) {
        // the real-to-complex pass loads two rows per thread in step A, 2*R1 values: with R1 above 20 that is more
        // than a wave keeps in flight, so the long lengths are split the other way round
        switch (N) {
            case 336: return launch_one<12, 28, KIND>(a, grid, st);
            case 384: return launch_one<16, 24, KIND>(a, grid, st);
            case 448: return launch_one<16, 28, KIND>(a, grid, st);
            case 480: return launch_one<16, 30, KIND>(a, grid, st);
            case 512: return launch_one<16, 32, KIND>(a, grid, st);
        }
    }
    // Measured exceptions for the x passes of small and medium images (32 -> 32 images, batches of 1.5 GB): the
    // pass that reads the fused kernel's layout is 5 to 12 % faster with the shorter second factor (its stores
    // then stay out of the streaming path), the inverse x pass 7 to 10 % faster with R2 = 16 at 48 and 64.
    if constexpr (KIND == P_FWD_XT) {
        switch (N) {
            case 28: return launch_one<2, 14, KIND>(a, grid, st);
            case 56: return launch_one<4, 14, KIND>(a, grid, st);
            case 80: return launch_one<10, 8, KIND>(a, grid, st);
            case 96: return launch_one<12, 8, KIND>(a, grid, st);
            case 100: return launch_one<5, 20, KIND>(a, grid, st);
            case 112: return launch_one<14, 8, KIND>(a, grid, st);
            case 128: return launch_one<16, 8, KIND>(a, grid, st);
        }
    }
    if constexpr (KIND == P_INV_X) {
        switch (N) {
            case 48: return launch_one<3, 16, KIND>(a, grid, st);
            case 64: return launch_one<4, 16, KIND>(a, grid, st);
        }
    }
    // ... and for larger images (1.5 GB per tensor): 10 to 14 % for the passes listed
    if constexpr (KIND == P_FWD_X) {
        switch (N) {
            case 128: return launch_one<16, 8, KIND>(a, grid, st);
            case 160: return launch_one<8, 20, KIND>(a, grid, st);
        }
    }
    if constexpr (KIND == P_INV_Y || KIND == P_INV_YT) {
        if (N == 128) return launch_one<16, 8, KIND>(a, grid, st);
    }
    if constexpr (KIND == P_FWD_Z || KIND == P_INV_Z) {
        if (N == 200) return launch_one<10, 20, KIND>(a, grid, st);
    }
    switch (N) {
        case 8: return launch_one<2, 4, KIND>(a, grid, st);
        case 10: return launch_one<5, 2, KIND>(a, grid, st);
        case 12: return launch_one<3, 4, KIND>(a, grid, st);
        case 14: return launch_one<7, 2, KIND>(a, grid, st);
        case 16: return launch_one<4, 4, KIND>(a, grid, st);
        case 20: return launch_one<5, 4, KIND>(a, grid, st);
        case 24: return launch_one<3, 8, KIND>(a, grid, st);
        case 28: return launch_one<7, 4, KIND>(a, grid, st);
        case 32: return launch_one<4, 8, KIND>(a, grid, st);
        case 36: return launch_one<9, 4, KIND>(a, grid, st);
        case 40: return launch_one<5, 8, KIND>(a, grid, st);
        case 48: return launch_one<6, 8, KIND>(a, grid, st);
        case 56: return launch_one<7, 8, KIND>(a, grid, st);
        case 64: return launch_one<8, 8, KIND>(a, grid, st);
        case 72: return launch_one<9, 8, KIND>(a, grid, st);
        case 80: return launch_one<5, 16, KIND>(a, grid, st);
        case 84: return launch_one<6, 14, KIND>(a, grid, st);
        case 96: return launch_one<6, 16, KIND>(a, grid, st);
        case 100: return launch_one<10, 10, KIND>(a, grid, st);
        case 112: return launch_one<7, 16, KIND>(a, grid, st);
        case 120: return launch_one<15, 8, KIND>(a, grid, st);
        case 128: return launch_one<8, 16, KIND>(a, grid, st);
        case 144: return launch_one<9, 16, KIND>(a, grid, st);
        case 160: return launch_one<10, 16, KIND>(a, grid, st);
        case 168: return launch_one<12, 14, KIND>(a, grid, st);
        case 192: return launch_one<12, 16, KIND>(a, grid, st);
        case 200: return launch_one<20, 10, KIND>(a, grid, st);
        case 224: return launch_one<14, 16, KIND>(a, grid, st);
        case 240: return launch_one<15, 16, KIND>(a, grid, st);
        case 256: return launch_one<16, 16, KIND>(a, grid, st);
        case 288: return launch_one<18, 16, KIND>(a, grid, st);
        case 320: return launch_one<20, 16, KIND>(a, grid, st);
        case 336: return launch_one<24, 14, KIND>(a, grid, st);
        case 384: return launch_one<24, 16, KIND>(a, grid, st);
        case 400: return launch_one<20, 20, KIND>(a, grid, st);
        case 448: return launch_one<28, 16, KIND>(a, grid, st);
        case 480: return launch_one<30, 16, KIND>(a, grid, st);
        case 512: return launch_one<32, 16, KIND>(a, grid, st);
        // above 512 a tile of 16 lines takes 74 to 139 KB of LDS: from 640 on one workgroup of 512 threads per CU
        case 576: return launch_one<18, 32, KIND>(a, grid, st);
        case 640: return launch_one<20, 32, KIND>(a, grid, st);
        case 720: return launch_one<24, 30, KIND>(a, grid, st);
        case 768: return launch_one<24, 32, KIND>(a, grid, st);
        case 840: return launch_one<28, 30, KIND>(a, grid, st);
        case 896: return launch_one<28, 32, KIND>(a, grid, st);
        case 960: return launch_one<30, 32, KIND>(a, grid, st);
        case 1024: return launch_one<32, 32, KIND>(a, grid, st);
    }
    return ZNNI_ERR_UNSUPPORTED_SIZE;
}

bool fast_pass_available(int N)
{
    switch (N) {
        case 8: case 10: case 12: case 14:
        case 16: case 20: case 24: case 28: case 32: case 36: case 40: case 48: case 56: case 64: case 72: case 80:
        case 84: case 96: case 100: case 112: case 120: case 128: case 144: case 160: case 168: case 192: case 200:
        case 224: case 240: case 256: case 288: case 320: case 336: case 384: case 400: case 448: case 480: case 512:
        case 576: case 640: case 720: case 768: case 840: case 896: case 960: case 1024:
            return true;
    }
    return false;
}

static PassArgs base_args(const LayerPlan& L, const void* src, void* dst, const float2* tw, int nimg)
{
    PassArgs a;
    a.src = src; a.dst = dst; a.tw = tw; a.bias = nullptr;
    a.d = L.d; a.nimg = nimg; a.fo = L.fo; a.relu = 0;
    return a;
}

znni_status launch_fast_fwd_z(const LayerPlan& L, const float* in, hipStream_t st)
{
    const Dims& d = L.d;
    return launch_kind<P_FWD_Z>(d.Nz, base_args(L, in, L.buf0, L.twz, L.nimg), dim3((d.ny + 31) / 32, d.nx, L.nimg),
                                st);
}
znni_status launch_fast_fwd_y(const LayerPlan& L, hipStream_t st)
{
    const Dims& d = L.d;
    return launch_kind<P_FWD_Y>(d.Ny, base_args(L, L.buf0, L.buf1, L.twy, L.nimg),
                                dim3((d.nx + 15) / 16, d.zc, L.nimg), st);
}
znni_status launch_fast_fwd_x(const LayerPlan& L, hipStream_t st)
{
    const Dims& d = L.d;
    return launch_kind<P_FWD_X>(d.Nx, base_args(L, L.buf1, L.buf0, L.twx, L.nimg),
                                dim3((d.Ny + 15) / 16, d.zc, L.nimg), st);
}
znni_status launch_fast_fwd_xt(const LayerPlan& L, hipStream_t st)
{
    const Dims& d = L.d;
    return launch_kind<P_FWD_XT>(d.Nx, base_args(L, L.buf1, L.buf0, L.twx, L.nimg),
                                 dim3((d.zc * d.Ny + 15) / 16, 1, L.nimg), st);
}
znni_status launch_fast_inv_x(const LayerPlan& L, hipStream_t st)
{
    const Dims& d = L.d;
    const dim3 grid = inv_x_flat(d) ? dim3((d.zc * d.Ny + 15) / 16, 1, L.nimgo) : dim3((d.Ny + 15) / 16, d.zc, L.nimgo);
    return launch_kind<P_INV_X>(d.Nx, base_args(L, L.Yt, L.buf0, L.twx, L.nimgo), grid, st);
}
znni_status launch_fast_inv_y(const LayerPlan& L, hipStream_t st)
{
    const Dims& d = L.d;
    return launch_kind<P_INV_Y>(d.Ny, base_args(L, L.buf0, L.buf1, L.twy, L.nimgo),
                                dim3((d.nox + 15) / 16, d.zc, L.nimgo), st);
}
znni_status launch_fast_inv_yt(const LayerPlan& L, hipStream_t st)
{
    const Dims& d = L.d;
    return launch_kind<P_INV_YT>(d.Ny, base_args(L, L.Yt, L.buf1, L.twy, L.nimgo),
                                 dim3((d.nox + 15) / 16, d.zc, L.nimgo), st);
}
znni_status launch_fast_inv_z(const LayerPlan& L, const float* bias, float* out, unsigned flags, hipStream_t st)
{
    const Dims& d = L.d;
    PassArgs a = base_args(L, L.buf1, out, L.twz, L.nimgo);
    a.bias = bias;
    a.relu = (flags & ZNNI_RELU) ? 1 : 0;
    return launch_kind<P_INV_Z>(d.Nz, a, dim3((d.noy + 31) / 32, d.nox, L.nimgo), st);
}

}  // namespace znni
