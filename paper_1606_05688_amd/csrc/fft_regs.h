// fft_regs.h -- in-register DFTs of composite length with compile-time twiddle factors (gfx950).
//
// Used by the two-step transform passes: a line of length N = R1*R2 is transformed as R2 DFTs of length R1
// followed by R1 DFTs of length R2, each done entirely in the registers of one thread, with a single
// exchange through LDS in between.
#pragma once
#include "fft_core.h"

namespace znni {

// cos / sin of 2*pi*e/R as compile-time constants (Taylor series in double after reduction to [-pi, pi]).
constexpr double kPi = 3.14159265358979323846264338327950288;

constexpr double ct_sin_series(double x)
{
    double term = x, sum = x;
    for (int n = 1; n < 24; ++n) {
        term *= -x * x / ((2.0 * n) * (2.0 * n + 1.0));
        sum += term;
    }
    return sum;
}
constexpr double ct_cos_series(double x)
{
    double term = 1.0, sum = 1.0;
    for (int n = 1; n < 24; ++n) {
        term *= -x * x / ((2.0 * n - 1.0) * (2.0 * n));
        sum += term;
    }
    return sum;
}
constexpr double ct_angle(int e, int R)
{
    int m = ((e % R) + R) % R;
    double t = 2.0 * kPi * (double)m / (double)R;
    return (2 * m > R) ? t - 2.0 * kPi : t;
}
constexpr float ct_cos(int e, int R) { return (float)ct_cos_series(ct_angle(e, R)); }
constexpr float ct_sin(int e, int R) { return (float)ct_sin_series(ct_angle(e, R)); }

// v * exp(-2 pi i E / R) with E, R compile-time; quarter turns cost nothing.
template <int E, int R> __device__ __forceinline__ float2 mul_w(float2 v)
{
    constexpr int m = ((E % R) + R) % R;
    if constexpr (m == 0) return v;
    else if constexpr (4 * m == R) return mul_mi(v);
    else if constexpr (2 * m == R) return make_float2(-v.x, -v.y);
    else if constexpr (4 * m == 3 * R) return mul_pi(v);
    else {
        constexpr float c = ct_cos(m, R), s = ct_sin(m, R);     // exp(-i t) = c - i s
        return make_float2(v.x * c + v.y * s, v.y * c - v.x * s);
    }
}

template <int R> struct Dft;   // Dft<R>::run(v): v[k] <- sum_n v[n] exp(-2 pi i n k / R), natural order

template <> struct Dft<2> { static __device__ __forceinline__ void run(float2* v) { dft<2>(v); } };
template <> struct Dft<3> { static __device__ __forceinline__ void run(float2* v) { dft<3>(v); } };
template <> struct Dft<4> { static __device__ __forceinline__ void run(float2* v) { dft<4>(v); } };
template <> struct Dft<5> { static __device__ __forceinline__ void run(float2* v) { dft<5>(v); } };
template <> struct Dft<7> { static __device__ __forceinline__ void run(float2* v) { dft<7>(v); } };
template <> struct Dft<8> { static __device__ __forceinline__ void run(float2* v) { dft<8>(v); } };

// Cooley-Tukey step inside registers: R = Ra*Rb, input index n = a + Ra*b, output index k = qb + Rb*qa.
template <int Ra, int Rb> struct DftCT {
    template <int A, int QB> static __device__ __forceinline__ void tw_row(float2 (&z)[Ra][Rb])
    {
        if constexpr (QB < Rb) {
            z[A][QB] = mul_w<A * QB, Ra * Rb>(z[A][QB]);
            tw_row<A, QB + 1>(z);
        }
    }
    template <int A> static __device__ __forceinline__ void first(const float2* v, float2 (&z)[Ra][Rb])
    {
        if constexpr (A < Ra) {
#pragma unroll
            for (int b = 0; b < Rb; ++b) z[A][b] = v[A + Ra * b];
            Dft<Rb>::run(z[A]);
            tw_row<A, 0>(z);
            first<A + 1>(v, z);
        }
    }
    static __device__ __forceinline__ void run(float2* v)
    {
        float2 z[Ra][Rb];
        first<0>(v, z);
#pragma unroll
        for (int qb = 0; qb < Rb; ++qb) {
            float2 t[Ra];
#pragma unroll
            for (int a = 0; a < Ra; ++a) t[a] = z[a][qb];
            Dft<Ra>::run(t);
#pragma unroll
            for (int qa = 0; qa < Ra; ++qa) v[qb + Rb * qa] = t[qa];
        }
    }
};

template <> struct Dft<6> { static __device__ __forceinline__ void run(float2* v) { DftCT<2, 3>::run(v); } };
template <> struct Dft<9> { static __device__ __forceinline__ void run(float2* v) { DftCT<3, 3>::run(v); } };
template <> struct Dft<10> { static __device__ __forceinline__ void run(float2* v) { DftCT<2, 5>::run(v); } };
template <> struct Dft<12> { static __device__ __forceinline__ void run(float2* v) { DftCT<3, 4>::run(v); } };
template <> struct Dft<14> { static __device__ __forceinline__ void run(float2* v) { DftCT<2, 7>::run(v); } };
template <> struct Dft<15> { static __device__ __forceinline__ void run(float2* v) { DftCT<3, 5>::run(v); } };
template <> struct Dft<16> { static __device__ __forceinline__ void run(float2* v) { DftCT<4, 4>::run(v); } };
template <> struct Dft<18> { static __device__ __forceinline__ void run(float2* v) { DftCT<2, 9>::run(v); } };
template <> struct Dft<20> { static __device__ __forceinline__ void run(float2* v) { DftCT<4, 5>::run(v); } };
template <> struct Dft<24> { static __device__ __forceinline__ void run(float2* v) { DftCT<3, 8>::run(v); } };
template <> struct Dft<28> { static __device__ __forceinline__ void run(float2* v) { DftCT<4, 7>::run(v); } };
template <> struct Dft<30> { static __device__ __forceinline__ void run(float2* v) { DftCT<5, 6>::run(v); } };
template <> struct Dft<32> { static __device__ __forceinline__ void run(float2* v) { DftCT<4, 8>::run(v); } };

}  // namespace znni
