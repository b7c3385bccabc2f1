// Mixing layer for sequence lengths with no four-step or in-LDS plan (Sec. 3.2 steps 2-4).
//
// By App. B the layer is a circular convolution of every channel with one real kernel per head,
// kappa = irfft_L(gate).  A length-L circular convolution equals the first L outputs of a
// length-M circular convolution (M >= 2L-1 a length the four-step kernels serve) of the zero-padded signal with the
// periodic extension kk of kappa laid out around index 0, so the data go through the
// four-step kernels once, with rfft_M(kk) as their gate.  kappa itself, one sequence per
// head, is an L-point inverse DFT of arbitrary L; it is evaluated by the chirp-z identity
//   exp(+j 2 pi k m / L) = w_k w_m conj(w_{m-k}),  w_n = exp(+j pi n^2 / L)
// which turns it into one more length-M circular convolution, with a fixed chirp filter.
// The heads' gate sequences ride through the same kernels as the 32 channel pairs of
// pseudo-heads (32 heads per pseudo-head, complex fp32 rows).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace spectre {

// Smallest four-step length M >= max(2L-1, 256); 0 if there is none (L > 65536).
int chirp_padded_length(int L);

// A[k][ph][p] = ext(g[bh])[k] * w_k, bh = 32 ph + p (zero for bh >= BH); ext = Hermitian extension
// of the half spectrum with real DC and Nyquist bins.  g [BH, L/2+1], w [L], A [L, nph, 32].
hipError_t launch_chirp_pre(const float2 *g, const float2 *w, float2 *A, int BH, int L, int nph, hipStream_t st);
// kappa[m] = Re(w_m U[m]) / L, laid out as kk over M rows: KK[i] = kappa[i] (i < L),
// kappa[i - (M - L)] (i > M - L), else 0; imaginary parts zero.  U [L, nph, 32], KK [M, nph, 32].
hipError_t launch_chirp_post(const float2 *U, const float2 *w, float2 *KK, int L, int M, int nph, hipStream_t st);
// Forward-transformed pseudo-head columns (scratch layout of the big kernel, pseudo-heads
// ph0 .. ph0+nphl) -> per-head gate planes gp [BH][N2][N1] in the big kernel's register order,
// scaled by 1/M.
hipError_t launch_chirp_gate(const float2 *scr, float2 *gp, int BH, int M, int N1, int N2, int ph0, int nphl,
                             hipStream_t st);

// The same spectra as per-head gates g [BH][M/2+1] in plain bin order, unscaled: the gate argument of the in-LDS
// kernel when it runs the padded convolution (M <= 2048).
hipError_t launch_chirp_gate_plain(const float2 *scr, float2 *g, int BH, int M, int N1, int N2, int P, int ph0,
                                   int nphl, hipStream_t st);

// Host: chirp w [L] and the chirp filter's M-point spectrum in the big kernel's register order
// ([N2][N1], scaled by 1/M), both evaluated in fp64.
void chirp_tables_host(int L, int M, int N1, int N2, int P, float2 *w, float2 *filt);

}  // namespace spectre
