// Small DFTs held entirely in one lane's registers.
//
// dft<R, INV>(x) overwrites x[0..R) with X[u] = sum_j x[j] exp(-/+ j 2 pi j u / R)
// (minus sign for INV = false, Eq. 1's convention; plus for INV = true, unscaled),
// outputs in natural order.  R is a power of two up to 32.  After full unrolling
// every array index and every root of unity is a compile-time constant, so the
// arrays live in VGPRs and the constants are instruction literals.
//
// dft_odd<R, INV> does the same for R = 3, 5, 7 and small_dft<N, INV> for every
// N = M * Q <= 32 with M in {1, 3, 5, 7} and Q a power of two, by the prime-factor
// index maps (M and Q are coprime, so no twiddles arise between the two stages).
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

// ------------------------------------------------------------------------------------------
// odd prime radices: X_0 = x_0 + sum a_j;  X_k, X_{R-k} = (x_0 + sum_j cos(2 pi jk/R) a_j)
//   -/+ j sum_j sin(2 pi jk/R) b_j  with a_j = x_j + x_{R-j}, b_j = x_j - x_{R-j}.
template <int R> struct OddRoots;
template <> struct OddRoots<3> {
    static constexpr float c[1] = {-0.5f};
    static constexpr float s[1] = {0.86602540378443864676f};
};
template <> struct OddRoots<5> {
    static constexpr float c[2] = {0.30901699437494742410f, -0.80901699437494742410f};
    static constexpr float s[2] = {0.95105651629515357212f, 0.58778525229247312917f};
};
template <> struct OddRoots<7> {
    static constexpr float c[3] = {0.62348980185873353053f, -0.22252093395631440429f, -0.90096886790241912624f};
    static constexpr float s[3] = {0.78183148246802980871f, 0.97492791218182360702f, 0.43388373911755812048f};
};

template <int R>
__device__ constexpr float odd_cos(int m) {   // cos(2 pi m / R)
    m %= R;
    if (m == 0) return 1.0f;
    if (m > R / 2) m = R - m;
    return OddRoots<R>::c[m - 1];
}
template <int R>
__device__ constexpr float odd_sin(int m) {   // sin(2 pi m / R)
    m %= R;
    if (m == 0) return 0.0f;
    if (m > R / 2) return -OddRoots<R>::s[R - m - 1];
    return OddRoots<R>::s[m - 1];
}

template <int R, bool INV>
__device__ __forceinline__ void dft_odd(float2 (&x)[R]) {
    constexpr int Hf = R / 2;
    float2 a[Hf], b[Hf];
#pragma unroll
    for (int j = 1; j <= Hf; ++j) {
        a[j - 1] = x[j] + x[R - j];
        b[j - 1] = x[j] - x[R - j];
    }
    float2 x0 = x[0];
    float2 sum = x0;
#pragma unroll
    for (int j = 0; j < Hf; ++j) sum = sum + a[j];
    x[0] = sum;
#pragma unroll
    for (int k = 1; k <= Hf; ++k) {
        float2 cr = x0, si = make_float2(0.f, 0.f);
#pragma unroll
        for (int j = 1; j <= Hf; ++j) {
            const float c = odd_cos<R>(j * k), s = odd_sin<R>(j * k);
            cr.x = fmaf(c, a[j - 1].x, cr.x);
            cr.y = fmaf(c, a[j - 1].y, cr.y);
            si.x = fmaf(s, b[j - 1].x, si.x);
            si.y = fmaf(s, b[j - 1].y, si.y);
        }
        // forward: X_k = cr - j si, X_{R-k} = cr + j si  (j*si = (-si.y, si.x)); inverse swaps
        const float2 jsi = make_float2(-si.y, si.x);
        x[k] = INV ? cr + jsi : cr - jsi;
        x[R - k] = INV ? cr - jsi : cr + jsi;
    }
}

// Odd part of n (n with its factors of two removed), and a^-1 mod m for coprime a, m (1 if m = 1).
__host__ __device__ constexpr int odd_part(int n) { return (n % 2 == 0) ? odd_part(n / 2) : n; }
__host__ __device__ constexpr int inverse_mod(int a, int m) {
    for (int i = 1; i < m; ++i)
        if ((a * i) % m == 1) return i;
    return 1;
}
__host__ __device__ constexpr bool small_dft_supported(int n) {
    return n >= 1 && n <= 32 && (odd_part(n) == 1 || odd_part(n) == 3 || odd_part(n) == 5 || odd_part(n) == 7);
}

// N = M * Q, M odd prime (or 1), Q a power of two.  Prime-factor algorithm: input index
// n = (Q n1 + M n2) mod N, output index k = (Q (Q^-1 mod M) k1 + M (M^-1 mod Q) k2) mod N, so that
// exp(-j 2 pi n k / N) = exp(-j 2 pi n1 k1 / M) exp(-j 2 pi n2 k2 / Q).
template <int N, bool INV>
__device__ __forceinline__ void small_dft(float2 (&x)[N]) {
    static_assert(small_dft_supported(N), "length");
    constexpr int M = odd_part(N), Q = N / M;
    if constexpr (M == 1) {
        dft<N, INV>(x);
    } else if constexpr (Q == 1) {
        dft_odd<N, INV>(x);
    } else {
        constexpr int eM = Q * inverse_mod(Q % M, M), eQ = M * inverse_mod(M % Q, Q);
        float2 y[N];
#pragma unroll
        for (int n1 = 0; n1 < M; ++n1) {
            float2 t[Q];
#pragma unroll
            for (int n2 = 0; n2 < Q; ++n2) t[n2] = x[(Q * n1 + M * n2) % N];
            dft<Q, INV>(t);
#pragma unroll
            for (int k2 = 0; k2 < Q; ++k2) y[n1 * Q + k2] = t[k2];
        }
#pragma unroll
        for (int k2 = 0; k2 < Q; ++k2) {
            float2 t[M];
#pragma unroll
            for (int n1 = 0; n1 < M; ++n1) t[n1] = y[n1 * Q + k2];
            dft_odd<M, INV>(t);
#pragma unroll
            for (int k1 = 0; k1 < M; ++k1) x[(eM * k1 + eQ * k2) % N] = t[k1];
        }
    }
}

}  // namespace spectre
