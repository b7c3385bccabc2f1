// Short-sequence (whole slab in LDS) mixer path: host-side declarations.
#pragma once
#include <hip/hip_runtime.h>

namespace spectre {

constexpr int kSlabMaxL = 2048;

// True if L <= kSlabMaxL and L = 2^a 3^b 5^c 7^d.
bool slab_supported(int L);

// Host: bin_of_pos[p] = the bin held by position p after the forward passes (mixed-radix digit reversal).
void slab_bin_order(int L, int *bin_of_pos);

// out = irfft_L(g * rfft_L(v)) for d = 64; roots = device table [L] of exp(-j 2 pi m / L), bin_of_pos = device
// copy of slab_bin_order(L).  With 0 < rows < L the tensors hold `rows` rows per sequence: v is taken as followed
// by L - rows zero rows and only the first `rows` rows of the result are written.
hipError_t launch_mix_slab(int io, const void *v, const float2 *g, void *out, const float2 *roots,
                           const int *bin_of_pos, int B, int L, int H, hipStream_t st, int rows = 0);

}  // namespace spectre
