// Wavelet refinement (Sec. 3.5): host-side launch declarations.
//
// Reading: orthonormal Haar wavelet, J levels (2^J divides L), one real gate per band and channel
// (band 0 = coarse approximation, band l = details of level l, level 1 the finest).  With one gate
// per band the module collapses to block means:  the projection of a column on the level-l
// approximation space is its mean A_l over aligned blocks of 2^l rows (A_0 = the column), the
// details of level l span A_(l-1) - A_l, hence
//   out = (1 + s_1) v + sum_{l=1}^{J-1} (s_(l+1) - s_l) A_l + (s_0 - s_J) A_J        (J >= 1)
// and out = (1 + s_0) v for J = 0.  No transform is materialised.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace spectre {

constexpr int kWrmTileRows = 256;   // rows of a head handled by one workgroup (levels 1..8 stay on chip)
constexpr int kWrmTileLevels = 8;

struct WrmDev {
    int Hg, d, d_w, levels;
    const float *ln_gamma, *ln_beta;
    float ln_eps;
    const float *W1, *b1, *W2, *b2;
};

// s [B,H,levels+1,d] = MLP(LayerNorm(inv_count * sum_q)).
hipError_t launch_wrm_gates(const double *sum_q, double inv_count, const WrmDev &P, int B, int H, float *s,
                            hipStream_t st);

// Floats of each of the two scratch arrays (tile sums, upper-level corrections); 0 when levels <= 8.
size_t wrm_scratch_floats(int BH, int L, int levels);

// out = v + iDWT(s * DWT(v)) for v, out [B,L,H,64]; io 0 = fp32, 1 = bf16.  out may be v itself.
// bsum (optional, used when levels > 8): sums of blocks of block_rows adjacent rows of v (block_rows divides 256),
// [B*H][L / block_rows][64], emitted by whoever wrote v; then v is not read a second time for the coarse levels.
hipError_t launch_wrm_apply(int io, const void *v, const float *s, void *out, float *tile_sums, float *upper,
                            int B, int L, int H, int levels, hipStream_t st, const float *bsum = nullptr,
                            int block_rows = 0);

// The same module with one gate per wavelet coefficient and channel: s [B,H,L,64] in the analysis' coefficient order
// [a_J | d_J | ... | d_1] (a real Haar analysis, gate, synthesis; same tiling and scratch as above).
hipError_t launch_wrm_apply_coeff(int io, const void *v, const float *s, void *out, float *tile_sums, float *upper,
                                  int B, int L, int H, int levels, hipStream_t st);

}  // namespace spectre
