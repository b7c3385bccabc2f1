// Arbitrary-length mixing through the four-step kernels: chirp-z evaluation of the per-head
// convolution kernel and its embedding in a padded convolution of a four-step length.
#include "mix_chirp.h"

#include <cmath>
#include <complex>
#include <vector>

#include "common.h"
#include "mix_pow2.h"

namespace spectre {

int chirp_padded_length(int L) {
    if (L < 1 || L > 65536) return 0;
    const int need = 2 * L - 1;
    int best = 0;
    for (int N1 : {256, 4096})
        for (int N2 = 1; N2 <= 32; ++N2) {
            const int M = N1 * N2;
            int a, b, c;
            if (M >= need && (best == 0 || M < best) && pow2_split(M, &a, &b, &c)) best = M;
        }
    return best;
}

__global__ __launch_bounds__(256) void k_chirp_pre(const float2 *__restrict__ g, const float2 *__restrict__ w,
                                                   float2 *__restrict__ A, int BH, int L, int nph, size_t total) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int p = (int)(idx % 32);
    const size_t r = idx / 32;
    const int ph = (int)(r % nph), k = (int)(r / nph);
    const int bh = ph * 32 + p, F = L / 2 + 1;
    float2 val = make_float2(0.f, 0.f);
    if (bh < BH) {
        float2 ge;
        if (k == 0 || 2 * k == L) ge = make_float2(g[(size_t)bh * F + k].x, 0.f);
        else if (2 * k < L) ge = g[(size_t)bh * F + k];
        else ge = cconj(g[(size_t)bh * F + (L - k)]);
        val = cmul(ge, w[k]);
    }
    A[idx] = val;
}

__global__ __launch_bounds__(256) void k_chirp_post(const float2 *__restrict__ U, const float2 *__restrict__ w,
                                                    float2 *__restrict__ KK, int L, int M, int nph, size_t total) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const size_t lane = idx % ((size_t)nph * 32);
    const int i = (int)(idx / ((size_t)nph * 32));
    int m = -1;
    if (i < L) m = i;
    else if (i > M - L) m = i - (M - L);
    float kap = 0.f;
    if (m >= 0) {
        const float2 u = U[(size_t)m * nph * 32 + lane], wm = w[m];
        kap = (wm.x * u.x - wm.y * u.y) * (1.0f / (float)L);
    }
    KK[idx] = make_float2(kap, 0.f);
}

__global__ __launch_bounds__(256) void k_chirp_gate(const float2 *__restrict__ scr, float2 *__restrict__ gp, int BH,
                                                    int N1, int N2, int ph0, float scale, size_t total) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int r = (int)(idx % N1);
    const size_t q = idx / N1;
    const int k2 = (int)(q % N2);
    const size_t lh = q / N2;                         // head index within this group of pseudo-heads
    const int phl = (int)(lh / 32), p = (int)(lh % 32);
    const size_t bh = (size_t)ph0 * 32 + lh;
    if (bh >= (size_t)BH) return;
    const float2 z = scr[(((size_t)phl * N2 + k2) * 32 + p) * N1 + r];   // same entry order on both sides
    gp[(bh * N2 + k2) * N1 + r] = make_float2(z.x * scale, z.y * scale);
}

// The same spectra in plain bin order for the in-LDS kernel: g[bh][k] = spectrum bin k = k2 + N2 k1 of pseudo-head
// column (bh / 32, bh % 32), which the forward-only big kernel left at entry big_position(k1) of column k2;
// unscaled (that kernel divides by its length itself).
__global__ __launch_bounds__(256) void k_chirp_gate_plain(const float2 *__restrict__ scr, float2 *__restrict__ g, int BH,
                                                          int F, int N1, int N2, int P, int ph0, size_t total) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int k = (int)(idx % F);
    const size_t lh = idx / F;                        // head index within this group of pseudo-heads
    const int phl = (int)(lh / 32), p = (int)(lh % 32);
    const size_t bh = (size_t)ph0 * 32 + lh;
    if (bh >= (size_t)BH) return;
    const int k2 = k % N2, k1 = k / N2;
    g[bh * F + k] = scr[(((size_t)phl * N2 + k2) * 32 + p) * N1 + big_position(k1, P)];
}

hipError_t launch_chirp_gate_plain(const float2 *scr, float2 *g, int BH, int M, int N1, int N2, int P, int ph0,
                                   int nphl, hipStream_t st) {
    const int F = M / 2 + 1;
    const size_t total = (size_t)nphl * 32 * F;
    k_chirp_gate_plain<<<(unsigned)((total + 255) / 256), 256, 0, st>>>(scr, g, BH, F, N1, N2, P, ph0, total);
    return hipGetLastError();
}

hipError_t launch_chirp_pre(const float2 *g, const float2 *w, float2 *A, int BH, int L, int nph, hipStream_t st) {
    const size_t total = (size_t)L * nph * 32;
    k_chirp_pre<<<(unsigned)((total + 255) / 256), 256, 0, st>>>(g, w, A, BH, L, nph, total);
    return hipGetLastError();
}

hipError_t launch_chirp_post(const float2 *U, const float2 *w, float2 *KK, int L, int M, int nph, hipStream_t st) {
    const size_t total = (size_t)M * nph * 32;
    k_chirp_post<<<(unsigned)((total + 255) / 256), 256, 0, st>>>(U, w, KK, L, M, nph, total);
    return hipGetLastError();
}

hipError_t launch_chirp_gate(const float2 *scr, float2 *gp, int BH, int M, int N1, int N2, int ph0, int nphl,
                             hipStream_t st) {
    const size_t total = (size_t)nphl * 32 * N2 * N1;
    k_chirp_gate<<<(unsigned)((total + 255) / 256), 256, 0, st>>>(scr, gp, BH, N1, N2, ph0, 1.0f / (float)M, total);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------ host tables
// Forward DFT of n = 2^a 3^b 5^c 7^d points (decimation in time, smallest prime factor first), out of place.
// root[j] = exp(-j 2 pi j / top) for the top-level length, of which n is a divisor.
static void fft_host(const std::complex<double> *in, size_t stride, size_t n, std::complex<double> *out,
                     const std::vector<std::complex<double>> &root) {
    if (n == 1) {
        out[0] = in[0];
        return;
    }
    const size_t top = root.size();
    size_t p = 2;
    while (n % p != 0) ++p;
    const size_t m = n / p;
    for (size_t r = 0; r < p; ++r) fft_host(in + r * stride, stride * p, m, out + r * m, root);
    std::complex<double> col[7];
    for (size_t k = 0; k < m; ++k) {
        for (size_t r = 0; r < p; ++r) col[r] = out[r * m + k] * root[(r * k) * (top / n)];
        for (size_t q = 0; q < p; ++q) {
            std::complex<double> acc = col[0];
            for (size_t r = 1; r < p; ++r) acc += col[r] * root[((r * q) % p) * (top / p)];
            out[k + q * m] = acc;
        }
    }
}

void chirp_tables_host(int L, int M, int N1, int N2, int P, float2 *w, float2 *filt) {
    std::vector<std::complex<double>> wd(L), f(M, std::complex<double>(0.0, 0.0));
    for (int n = 0; n < L; ++n) {
        const long long sq = ((long long)n * n) % (2LL * L);       // exact phase index
        wd[n] = std::polar(1.0, M_PI * (double)sq / (double)L);
        w[n] = make_float2((float)wd[n].real(), (float)wd[n].imag());
    }
    std::vector<std::complex<double>> ft(M, std::complex<double>(0.0, 0.0));
    ft[0] = std::conj(wd[0]);
    for (int i = 1; i < L; ++i) ft[i] = ft[M - i] = std::conj(wd[i]);
    std::vector<std::complex<double>> root(M);
    for (int j = 0; j < M; ++j) root[j] = std::polar(1.0, -2.0 * M_PI * (double)j / (double)M);
    fft_host(ft.data(), 1, (size_t)M, f.data(), root);
    for (int k2 = 0; k2 < N2; ++k2)
        for (int r = 0; r < N1; ++r) {
            const int k = k2 + N2 * big_position(r, P);
            filt[(size_t)k2 * N1 + r] = make_float2((float)(f[k].real() / M), (float)(f[k].imag() / M));
        }
}

// Loads this translation unit's code object (the runtime loads them on first use): called by spectre_prepare so
// that no compute call is the first to touch it.
hipError_t load_kernels_mix_chirp() {
    hipFuncAttributes a;
    return hipFuncGetAttributes(&a, reinterpret_cast<const void *>(k_chirp_pre));
}

}  // namespace spectre
