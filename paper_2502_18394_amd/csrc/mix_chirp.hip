// Arbitrary-length mixing through the power-of-two kernels: chirp-z evaluation of the per-head
// convolution kernel and its embedding in a padded power-of-two convolution.
#include "mix_chirp.h"

#include <cmath>
#include <complex>
#include <vector>

#include "common.h"

namespace spectre {

int chirp_padded_length(int L) {
    if (L < 1 || L > 65536) return 0;
    int M = 256;
    while (M < 2 * L - 1) M <<= 1;
    return M <= 131072 ? M : 0;
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
    const int TPC = N1 / 16;
    const int r = (int)(idx % N1);
    const size_t q = idx / N1;
    const int k2 = (int)(q % N2);
    const size_t lh = q / N2;                         // head index within this group of pseudo-heads
    const int phl = (int)(lh / 32), p = (int)(lh % 32);
    const size_t bh = (size_t)ph0 * 32 + lh;
    if (bh >= (size_t)BH) return;
    const int j = r / TPC, tau = r % TPC;
    const float2 z = scr[(((size_t)phl * N2 + k2) * 32 + p) * N1 + 16 * tau + j];
    gp[(bh * N2 + k2) * N1 + r] = make_float2(z.x * scale, z.y * scale);
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
static void fft_host(std::vector<std::complex<double>> &a) {      // in-place radix-2, forward sign
    const size_t n = a.size();
    for (size_t i = 1, j = 0; i < n; ++i) {
        size_t bit = n >> 1;
        for (; j & bit; bit >>= 1) j ^= bit;
        j ^= bit;
        if (i < j) std::swap(a[i], a[j]);
    }
    for (size_t len = 2; len <= n; len <<= 1) {
        std::vector<std::complex<double>> root(len / 2);
        for (size_t m = 0; m < len / 2; ++m) root[m] = std::polar(1.0, -2.0 * M_PI * (double)m / (double)len);
        for (size_t i = 0; i < n; i += len)
            for (size_t m = 0; m < len / 2; ++m) {
                const std::complex<double> u = a[i + m], t = a[i + m + len / 2] * root[m];
                a[i + m] = u + t;
                a[i + m + len / 2] = u - t;
            }
    }
}

static int digit_reverse16_host(int pos, int P) {
    return P == 2 ? (((pos & 15) << 4) | (pos >> 4)) : (((pos & 15) << 8) | (pos & 0xF0) | (pos >> 8));
}

void chirp_tables_host(int L, int M, int N1, int N2, int P, float2 *w, float2 *filt) {
    std::vector<std::complex<double>> wd(L), f(M, std::complex<double>(0.0, 0.0));
    for (int n = 0; n < L; ++n) {
        const long long sq = ((long long)n * n) % (2LL * L);       // exact phase index
        wd[n] = std::polar(1.0, M_PI * (double)sq / (double)L);
        w[n] = make_float2((float)wd[n].real(), (float)wd[n].imag());
    }
    f[0] = std::conj(wd[0]);
    for (int i = 1; i < L; ++i) f[i] = f[M - i] = std::conj(wd[i]);
    fft_host(f);
    const int TPC = N1 / 16;
    for (int k2 = 0; k2 < N2; ++k2)
        for (int r = 0; r < N1; ++r) {
            const int j = r / TPC, tau = r % TPC;
            const int k = k2 + N2 * digit_reverse16_host(16 * tau + j, P);
            filt[(size_t)k2 * N1 + r] = make_float2((float)(f[k].real() / M), (float)(f[k].imag() / M));
        }
}

}  // namespace spectre
