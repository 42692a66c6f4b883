// fft_core.h -- device-side building blocks of the one-dimensional transforms (gfx950, wave64).
//
// A three-dimensional transform is a sequence of one-dimensional transforms along the three axes
// (Section III-A).  Each pass kernel stages a tile of lines in LDS, transforms every line there, and writes
// the tile back with the next axis made contiguous.  This header holds the part common to all passes:
// small-radix butterflies and a Stockham autosort transform of `nlines` LDS-resident complex lines of any
// length N = 2^a 3^b 5^c 7^d (the size family of Section III-D).
#pragma once
#include <hip/hip_runtime.h>

namespace znni {

constexpr int kMaxStages = 12;

// Radix schedule of one transform length; built on the host, passed to kernels by value.
struct FftPlan {
    int N;                    // transform length n~
    int nstages;
    int radix[kMaxStages];    // product of radix[0..nstages) == N
};

// Streaming (non-temporal) global accesses for tensors that are written once by one kernel and read once by the
// next and are far larger than the caches.  Measured on the 320^3 workload: the middle four transform passes
// gain 2 to 7 % with both, the last only with streaming loads (its unaligned output rows are merged in L2 when
// stored normally); the first pass uses neither (its input lines are touched by several instructions and must
// stay cached, and its stores were faster without at every smaller size).
typedef float znni_v2f __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void st_stream(float2* p, float2 v)
{
    znni_v2f w; w.x = v.x; w.y = v.y;
    __builtin_nontemporal_store(w, reinterpret_cast<znni_v2f*>(p));
}
__device__ __forceinline__ void st_stream(float* p, float v) { __builtin_nontemporal_store(v, p); }
__device__ __forceinline__ float2 ld_stream(const float2* p)
{
    const znni_v2f w = __builtin_nontemporal_load(reinterpret_cast<const znni_v2f*>(p));
    return make_float2(w.x, w.y);
}
__device__ __forceinline__ float ld_stream(const float* p) { return __builtin_nontemporal_load(p); }
template <bool STREAM, typename T>
__device__ __forceinline__ T ldg(const T* p)
{
    if constexpr (STREAM) return ld_stream(p);
    else return *p;
}
template <bool STREAM, typename T>
__device__ __forceinline__ void stg(T* p, T v)
{
    if constexpr (STREAM) st_stream(p, v);
    else *p = v;
}

__device__ __forceinline__ float2 cadd(float2 a, float2 b) { return make_float2(a.x + b.x, a.y + b.y); }
__device__ __forceinline__ float2 csub(float2 a, float2 b) { return make_float2(a.x - b.x, a.y - b.y); }
__device__ __forceinline__ float2 cmul(float2 a, float2 b)
{
    return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
__device__ __forceinline__ float2 cconj(float2 a) { return make_float2(a.x, -a.y); }
// multiply by -i
__device__ __forceinline__ float2 mul_mi(float2 a) { return make_float2(a.y, -a.x); }
// multiply by +i
__device__ __forceinline__ float2 mul_pi(float2 a) { return make_float2(-a.y, a.x); }
__device__ __forceinline__ float2 cscale(float2 a, float s) { return make_float2(a.x * s, a.y * s); }
// a + s*b with real s
__device__ __forceinline__ float2 caxpy(float2 a, float s, float2 b)
{
    return make_float2(fmaf(s, b.x, a.x), fmaf(s, b.y, a.y));
}
// a + b*c, four fused multiply-adds
__device__ __forceinline__ float2 cfma(float2 a, float2 b, float2 c)
{
    return make_float2(fmaf(-b.y, c.y, fmaf(b.x, c.x, a.x)), fmaf(b.y, c.x, fmaf(b.x, c.y, a.y)));
}

// Forward DFTs of length R in registers: v[m] <- sum_t v[t] exp(-2 pi i t m / R).
template <int R> __device__ __forceinline__ void dft(float2* v);

template <> __device__ __forceinline__ void dft<2>(float2* v)
{
    float2 a = v[0], b = v[1];
    v[0] = cadd(a, b);
    v[1] = csub(a, b);
}

template <> __device__ __forceinline__ void dft<3>(float2* v)
{
    const float s60 = 0.86602540378443864676f;
    float2 t = cadd(v[1], v[2]);
    float2 d = mul_mi(cscale(csub(v[1], v[2]), s60));
    float2 m = caxpy(v[0], -0.5f, t);
    v[0] = cadd(v[0], t);
    v[1] = cadd(m, d);
    v[2] = csub(m, d);
}

template <> __device__ __forceinline__ void dft<4>(float2* v)
{
    float2 a = cadd(v[0], v[2]), b = csub(v[0], v[2]);
    float2 c = cadd(v[1], v[3]), d = mul_mi(csub(v[1], v[3]));
    v[0] = cadd(a, c);
    v[1] = cadd(b, d);
    v[2] = csub(a, c);
    v[3] = csub(b, d);
}

template <> __device__ __forceinline__ void dft<5>(float2* v)
{
    const float c1 = 0.30901699437494742410f, c2 = -0.80901699437494742410f;   // cos(2pi/5), cos(4pi/5)
    const float s1 = 0.95105651629515357212f, s2 = 0.58778525229247312917f;    // sin(2pi/5), sin(4pi/5)
    float2 t1 = cadd(v[1], v[4]), t2 = cadd(v[2], v[3]);
    float2 t3 = csub(v[1], v[4]), t4 = csub(v[2], v[3]);
    float2 a1 = caxpy(caxpy(v[0], c1, t1), c2, t2);
    float2 a2 = caxpy(caxpy(v[0], c2, t1), c1, t2);
    float2 b1 = mul_mi(caxpy(cscale(t3, s1), s2, t4));
    float2 b2 = mul_mi(caxpy(cscale(t3, s2), -s1, t4));
    v[0] = cadd(v[0], cadd(t1, t2));
    v[1] = cadd(a1, b1);
    v[4] = csub(a1, b1);
    v[2] = cadd(a2, b2);
    v[3] = csub(a2, b2);
}

template <> __device__ __forceinline__ void dft<7>(float2* v)
{
    const float c[3] = {0.62348980185873353053f, -0.22252093395631440429f, -0.90096886790241912624f};
    const float s[3] = {0.78183148246802980871f, 0.97492791218182360702f, 0.43388373911755812048f};
    float2 p[3], q[3];
    for (int m = 0; m < 3; ++m) {
        p[m] = cadd(v[m + 1], v[6 - m]);
        q[m] = csub(v[m + 1], v[6 - m]);
    }
    float2 x0 = cadd(v[0], cadd(p[0], cadd(p[1], p[2])));
    float2 o[7];
    o[0] = x0;
#pragma unroll
    for (int m = 1; m <= 3; ++m) {
        float2 a = v[0], b = make_float2(0.f, 0.f);
#pragma unroll
        for (int t = 1; t <= 3; ++t) {
            int e = (m * t) % 7;                       // angle index of cos/sin(2 pi e / 7)
            float ce = (e <= 3) ? c[e - 1] : c[6 - e];
            float se = (e <= 3) ? s[e - 1] : -s[6 - e];
            a = caxpy(a, ce, p[t - 1]);
            b = caxpy(b, se, q[t - 1]);
        }
        b = mul_mi(b);
        o[m] = cadd(a, b);
        o[7 - m] = csub(a, b);
    }
#pragma unroll
    for (int m = 0; m < 7; ++m) v[m] = o[m];
}

template <> __device__ __forceinline__ void dft<8>(float2* v)
{
    const float h = 0.70710678118654752440f;
    float2 e[4] = {v[0], v[2], v[4], v[6]};
    float2 o[4] = {v[1], v[3], v[5], v[7]};
    dft<4>(e);
    dft<4>(o);
    o[1] = make_float2((o[1].x + o[1].y) * h, (o[1].y - o[1].x) * h);      // * exp(-i pi/4)
    o[2] = mul_mi(o[2]);                                                    // * exp(-i pi/2)
    o[3] = make_float2((o[3].y - o[3].x) * h, -(o[3].x + o[3].y) * h);     // * exp(-3 i pi/4)
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        v[m] = cadd(e[m], o[m]);
        v[m + 4] = csub(e[m], o[m]);
    }
}

// One Stockham stage of radix R over `nlines` lines of length N stored with stride ld.
// Ns = product of the radices already applied.  tw[q] = exp(-2 pi i q / N).
template <int R>
__device__ __forceinline__ void stockham_stage(const float2* __restrict__ src, float2* __restrict__ dst,
                                               const float2* __restrict__ tw, int nlines, int ld, int N, int Ns)
{
    const int nb = N / R;              // butterflies per line
    const int tws = N / (Ns * R);      // twiddle stride in the length-N table
    const int total = nlines * nb;
    for (int b = threadIdx.x; b < total; b += blockDim.x) {
        const int line = b / nb;
        const int j = b - line * nb;
        const int k = j % Ns;
        const float2* s = src + line * ld + j;
        float2 v[R];
#pragma unroll
        for (int t = 0; t < R; ++t) v[t] = s[t * nb];
        if (Ns > 1) {
#pragma unroll
            for (int t = 1; t < R; ++t) v[t] = cmul(v[t], tw[t * k * tws]);
        }
        dft<R>(v);
        float2* d = dst + line * ld + (j - k) * R + k;
#pragma unroll
        for (int t = 0; t < R; ++t) d[t * Ns] = v[t];
    }
}

// Forward transform of nlines LDS-resident lines.  Input in a; returns the buffer that holds the result
// (a or b).  Every thread of the block must call it; it ends with a barrier.
__device__ __forceinline__ float2* fft_lines(float2* a, float2* b, const float2* tw, int nlines, int ld,
                                             const FftPlan& P)
{
    int Ns = 1;
    for (int st = 0; st < P.nstages; ++st) {
        const int r = P.radix[st];
        switch (r) {
            case 2: stockham_stage<2>(a, b, tw, nlines, ld, P.N, Ns); break;
            case 3: stockham_stage<3>(a, b, tw, nlines, ld, P.N, Ns); break;
            case 4: stockham_stage<4>(a, b, tw, nlines, ld, P.N, Ns); break;
            case 5: stockham_stage<5>(a, b, tw, nlines, ld, P.N, Ns); break;
            case 7: stockham_stage<7>(a, b, tw, nlines, ld, P.N, Ns); break;
            default: stockham_stage<8>(a, b, tw, nlines, ld, P.N, Ns); break;
        }
        __syncthreads();
        float2* t = a; a = b; b = t;
        Ns *= r;
    }
    return a;
}

}  // namespace znni
