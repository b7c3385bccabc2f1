// Host check of the index maps the cache's window transform and full readout rely on (compiled for the host only):
// the entry order around the column kernel and the pairing of a pair-spectrum bin with its Hermitian partner.
// For every N = N1 * N2 with N1 = 256 or 4096 and N2 <= 32: big_position is a permutation and its own inverse; walking the lines the
// pair <-> half-spectra kernels walk (columns k2, lines q < N1 / 32, 16 entries each, plus the Nyquist bin) touches
// every bin k <= N/2 exactly once and, together with the partners, every entry of every column exactly once.
#include <cstdio>
#include <vector>

#include "mix_pow2.h"

using namespace spectre;

static int check_plan(int N1, int N2, int P) {
    const int N = N1 * N2;
    std::vector<int> seen(N1, 0);
    for (int e = 0; e < N1; ++e) {
        const int b = big_position(e, P);
        if (b < 0 || b >= N1 || big_position(b, P) != e) return 1;
        seen[b] += 1;
    }
    for (int e = 0; e < N1; ++e)
        if (seen[e] != 1) return 2;
    std::vector<int> bins(N / 2 + 1, 0), entries((size_t)N2 * N1, 0);
    for (int k2 = 0; k2 < N2; ++k2)
        for (int q = 0; q < N1 / 32; ++q)
            for (int c = 0; c < 16; ++c) {
                const int e = 16 * q + c;
                const SpectrumPair sp = spectrum_pair(N, N2, P, k2, e);
                if (sp.k < 0 || 2 * sp.k >= N) return 3;                    // lines below N1/2 hold bins below N/2
                if (sp.k2n < 0 || sp.k2n >= N2 || sp.en < 0 || sp.en >= N1) return 4;
                if (sp.k2n + N2 * big_position(sp.en, P) != sp.kn) return 5;  // the partner entry holds the partner bin
                if ((sp.k + sp.kn) % N != 0) return 6;
                bins[sp.k] += 1;
                entries[(size_t)k2 * N1 + e] += 1;
                if (sp.kn != sp.k) entries[(size_t)sp.k2n * N1 + sp.en] += 1;
                // for k2 > 0 the partners of a line are one line, in reverse order
                if (k2 > 0 && (sp.en / 16 != spectrum_pair(N, N2, P, k2, 16 * q).en / 16 ||
                               sp.en % 16 != 15 - c)) return 7;
            }
    bins[N / 2] += 1;                                                          // the Nyquist bin: column 0, bin N1/2
    entries[big_position(N1 / 2, P)] += 1;
    for (int k = 0; k <= N / 2; ++k)
        if (bins[k] != 1) return 8;
    for (size_t i = 0; i < entries.size(); ++i)
        if (entries[i] != 1) return 9;
    return 0;
}

int main() {
    int failures = 0, plans = 0;
    for (int N2 = 1; N2 <= 32; ++N2)                   // every column count a plan can have (a superset of the plans)
        for (int P : {2, 3}) {
            const int N1 = P == 2 ? 256 : 4096;
            const int rc = check_plan(N1, N2, P);
            plans += 1;
            if (rc) {
                std::printf("plan N1=%d N2=%d P=%d: check %d failed\n", N1, N2, P, rc);
                failures += 1;
            }
        }
    std::printf("%d plans, %d failures\n", plans, failures);
    return failures ? 1 : 0;
}
