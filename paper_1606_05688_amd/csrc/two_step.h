// two_step.h -- a line of length N = R1*R2 transformed as two in-register steps with one LDS exchange between them.
#pragma once
#include "fft_regs.h"

namespace znni {

template <int R1, int R2> struct TwoStep {
    static constexpr int N = R1 * R2;
    static constexpr int T = R1 > R2 ? R1 : R2;      // threads per line
    static constexpr int NTH = 16 * T;               // threads per workgroup
    static constexpr int P = N + 2;                  // LDS line pitch (complex); even, so 16-byte reads stay aligned
    static constexpr int LDS_BYTES = (int)sizeof(float2) * (N + 16 * P);

    // Step A on the R1 samples in v (sample m is element j + R2*m of the line), result to LDS.
    static __device__ __forceinline__ void step_a(float2* v, int line, int j, const float2* tws, float2* buf)
    {
        Dft<R1>::run(v);
#pragma unroll
        for (int q = 1; q < R1; ++q) v[q] = cmul(v[q], tws[j * q]);
#pragma unroll
        for (int q = 0; q < R1; ++q) buf[line * P + q * R2 + j] = v[q];
    }
    // Step B for (line, q): u[r] becomes element q + R1*r of the transformed line.
    static __device__ __forceinline__ void step_b(float2* u, int line, int q, const float2* buf)
    {
        const float4* p = reinterpret_cast<const float4*>(buf + line * P + q * R2);
#pragma unroll
        for (int h = 0; h < R2 / 2; ++h) {
            const float4 t = p[h];
            u[2 * h] = make_float2(t.x, t.y);
            u[2 * h + 1] = make_float2(t.z, t.w);
        }
        Dft<R2>::run(u);
    }
};

}  // namespace znni
