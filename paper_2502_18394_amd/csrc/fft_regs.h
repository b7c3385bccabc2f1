// Small DFTs held entirely in one lane's registers.
//
// dft<R, INV>(x) overwrites x[0..R) with X[u] = sum_j x[j] exp(-/+ j 2 pi j u / R)
// (minus sign for INV = false, Eq. 1's convention; plus for INV = true, unscaled),
// outputs in natural order.  R is a power of two up to 32.  After full unrolling
// every array index and every root of unity is a compile-time constant, so the
// arrays live in VGPRs and the constants are instruction literals.
#pragma once
#include "common.h"

namespace spectre {

// cos(m pi/16) for any integer m; the nine distinct magnitudes to 20 digits, the
// rest of the 32nd roots of unity by symmetry.
__host__ __device__ constexpr float cos_pi16(int m) {
    m = m < 0 ? -m : m;
    m %= 32;
    if (m > 16) m = 32 - m;
    const bool neg = m > 8;
    if (neg) m = 16 - m;
    float c = 0.0f;
    switch (m) {
        case 0: c = 1.0f; break;
        case 1: c = 0.98078528040323044913f; break;
        case 2: c = 0.92387953251128675613f; break;
        case 3: c = 0.83146961230254523708f; break;
        case 4: c = 0.70710678118654752440f; break;
        case 5: c = 0.55557023301960222474f; break;
        case 6: c = 0.38268343236508977173f; break;
        case 7: c = 0.19509032201612826785f; break;
        default: c = 0.0f; break;
    }
    return neg ? -c : c;
}
__host__ __device__ constexpr float sin_pi16(int m) { return cos_pi16(m - 8); }

// a * exp(-/+ j 2 pi m/32), m an integer that is constant after unrolling.
template <bool INV>
__host__ __device__ __forceinline__ float2 mul_root32(float2 a, int m) {
    m &= 31;
    if (m == 0) return a;
    if (m == 16) return make_float2(-a.x, -a.y);
    if (m == 8) return INV ? make_float2(-a.y, a.x) : make_float2(a.y, -a.x);
    if (m == 24) return INV ? make_float2(a.y, -a.x) : make_float2(-a.y, a.x);
    const float c = cos_pi16(m);
    const float s = INV ? sin_pi16(m) : -sin_pi16(m);
    return make_float2(a.x * c - a.y * s, a.x * s + a.y * c);
}

template <int R, bool INV>
__host__ __device__ __forceinline__ void dft(float2 (&x)[R]) {
    static_assert(R == 1 || R == 2 || R == 4 || R == 8 || R == 16 || R == 32, "radix");
    if constexpr (R == 1) {
    } else if constexpr (R == 2) {
        float2 a = x[0] + x[1], b = x[0] - x[1];
        x[0] = a;
        x[1] = b;
    } else if constexpr (R == 4) {
        float2 t0 = x[0] + x[2], t1 = x[0] - x[2], t2 = x[1] + x[3], t3 = x[1] - x[3];
        // forward: X1 = t1 - j t3, X3 = t1 + j t3; inverse swaps them
        float2 jt3 = make_float2(-t3.y, t3.x);
        x[0] = t0 + t2;
        x[2] = t0 - t2;
        x[1] = INV ? t1 + jt3 : t1 - jt3;
        x[3] = INV ? t1 - jt3 : t1 + jt3;
    } else {
        // Cooley-Tukey R = 4 * R2: input j = R2*j1 + j2, output u = u1 + 4*u2.
        constexpr int R2 = R / 4;
        float2 y[R];
#pragma unroll
        for (int j2 = 0; j2 < R2; ++j2) {
            float2 t[4];
#pragma unroll
            for (int j1 = 0; j1 < 4; ++j1) t[j1] = x[R2 * j1 + j2];
            dft<4, INV>(t);
#pragma unroll
            for (int u1 = 0; u1 < 4; ++u1) y[R2 * u1 + j2] = mul_root32<INV>(t[u1], j2 * u1 * (32 / R));
        }
#pragma unroll
        for (int u1 = 0; u1 < 4; ++u1) {
            float2 t[R2];
#pragma unroll
            for (int j2 = 0; j2 < R2; ++j2) t[j2] = y[R2 * u1 + j2];
            dft<R2, INV>(t);
#pragma unroll
            for (int u2 = 0; u2 < R2; ++u2) x[u1 + 4 * u2] = t[u2];
        }
    }
}

}  // namespace spectre
