// Four-step transform path (power-of-two lengths and power-of-two lengths times 3, 5 or 7): host-side plan and
// launch declarations.
//
// An L-point transform (L = N1 * N2) of the channel pairs of one head is split the
// four-step way: N2-point DFTs over the far index inside single lanes ("small"
// kernels, which also own all traffic with the caller's [B,L,H,d] tensors), a
// root-of-unity scaling, and N1-point DFTs staged through LDS ("big" kernel,
// which only touches the library's own scratch layout).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace spectre {

struct Pow2Plan {
    int L = 0;            // transform length
    int N1 = 0, N2 = 0;   // L = N1 * N2; N1 = 16^P, N2 <= 32 of the form {1,3,5,7} * 2^a
    int P = 0;
    const float2 *twL = nullptr;   // [L]  exp(-j 2 pi m / L), device
    const float2 *twN1 = nullptr;  // [N1] exp(-j 2 pi m / N1), device
};

// Order of a scratch column of N1 = 16^P entries around the big kernel (all modes, input and output): entry
// j * (N1 / 16) + tau belongs to register j of lane tau.  In time order (input of the forward passes, output of the
// inverse passes) that is sample t1 = entry; in frequency order (output of the forward-only mode, input of the
// inverse-only mode, and the order of the expanded gate) the register holds bin digit_reverse16(16 tau + j), i.e. the
// natural order for P = 2 and, for P = 3, the bin index with its two low base-16 digits exchanged.  The map is its
// own inverse: it gives the entry of a bin and the bin of an entry.
__host__ __device__ inline int big_position(int k1, int P) {
    return P == 2 ? k1 : ((k1 & 0xF00) | ((k1 & 15) << 4) | ((k1 >> 4) & 15));
}

// Where a bin of the N-point pair spectrum (N = N1 * N2) and its Hermitian partner live in the scratch: entry `e` of
// column k2 holds bin k = k2 + N2 * big_position(e); the partner bin kn = (N - k) mod N is entry `en` of column k2n.
// For the 16 entries of a 128-byte line (e = 16 q + c, q < N1 / 32) all k lie below N / 2, and for k2 > 0 the 16
// partners are again one whole line, in reverse order.  Used by the kernels that turn the pair spectrum into the two
// channels' half spectra and back, and checked on the host (every bin of every column exactly once).
struct SpectrumPair {
    int k, kn, k2n, en;
};
__host__ __device__ inline SpectrumPair spectrum_pair(int N, int N2, int P, int k2, int e) {
    SpectrumPair s;
    s.k = k2 + N2 * big_position(e, P);
    s.kn = (N - s.k) % N;
    s.k2n = s.kn % N2;
    s.en = big_position(s.kn / N2, P);
    return s;
}

// Decomposition rule; returns false if L has no such plan.
bool pow2_split(int L, int *N1, int *N2, int *P);

// Launchers (enqueue only).  `pairs` = d/2 must be 32.  All return hipError_t.
//   small_fwd : rows of v (tensor [B, rows, H, d], zero beyond `rows`) -> scratch[bh_local][k2][pair][t1]
//   big       : in-place N1-point transforms on scratch; mode 0 = forward, gate, inverse;
//               1 = forward only; 2 = inverse only.  gp = expanded gate for mode 0, one
//               [N2][N1] block per head from head bh0 on, or (shared_gate) one block for all.
//   small_inv : scratch -> rows [row0, row0 + out_rows) of the inverse transform into
//               out (tensor [B, out_rows, H, d]); with ring_w > 0 instead the out_rows newest
//               entries, oldest first, of a ring buffer in rows ring0 .. ring0+ring_w-1 whose
//               newest entry is row ring0+newest
// scr16 (bf16 rows, big: mode 0 only): the scratch holds each complex number as two bfloat16 in one 32-bit word at
// the same element index (the buffer is used to half its size); all three kernels of a pass must agree on it.
// affine (nbh a multiple of 8; big: mode 0, fp32 scratch): every workgroup of head bh0 + 8 s + x runs on XCD x, and the
// three kernels walk s up, down, up, so that part of the scratch is read from the L2 it was written through.
// ring (pre-fill of an empty cache without memory rows): the rows read are also stored, as fp32 pairs, to row l of head
// bh of ring [B*H][L][32], the cache's value ring buffer.
hipError_t launch_small_fwd(const Pow2Plan &pl, int io, const void *v, float2 *scratch, int rows, int H,
                            int bh0, int nbh, hipStream_t st, bool scr16 = false, bool affine = false,
                            float2 *ring = nullptr);
// wide (mode 0, 4096-point columns, fp32 scratch): 8 instead of 4 columns per workgroup, for calls on two streams.
hipError_t launch_big(const Pow2Plan &pl, float2 *scratch, const float2 *gp, int bh0, int nbh, int mode,
                      hipStream_t st, bool shared_gate = false, bool scr16 = false, bool affine = false,
                      bool wide = false);
// bsum (whole transforms only): sums of the blocks of small_tile_rows(io) adjacent output rows, over the values as
// stored, to bsum [B*H][L / small_tile_rows][32 pairs] - what the wavelet refinement's coarse levels need.
int small_tile_rows(int io);
hipError_t launch_small_inv(const Pow2Plan &pl, int io, const float2 *scratch, void *out, int row0,
                            int out_rows, int H, int bh0, int nbh, hipStream_t st, int ring0 = 0, int ring_w = 0,
                            int newest = 0, bool scr16 = false, bool affine = false, float2 *bsum = nullptr);
// small_fwd with the token projection of Eq. 2 in front: x = the layer input [B, rows, H, 64] as bf16, wpack = the
// heads' value matrices as packed by launch_pack_w (project.h); the projected rows are rounded to bf16 on chip, as
// the separate projection would have stored them, and transformed.  bf16 rows and fp32 scratch only.
hipError_t launch_small_fwd_proj(const Pow2Plan &pl, const void *x, const void *wpack, int Hw, float2 *scratch, int rows,
                                 int H, int bh0, int nbh, hipStream_t st, bool affine = false);
// g [BH, L/2+1] -> gp [BH][N2][N1] in the big kernel's register order, scaled by 1/L and
// extended to all L bins by Hermitian symmetry (real parts only at DC and Nyquist).
hipError_t launch_gate_expand(const Pow2Plan &pl, const float2 *g, float2 *gp, int BH, hipStream_t st);

// One-kernel path for L = 4096 (a whole column fits in LDS): v, out = tensors [B, 4096, H, 64], g = gate
// [B*H, 2049] as the caller passes it, tw4096 = device table of exp(-j 2 pi m / 4096).  No workspace.
bool fused_supported(int L);
hipError_t launch_fused(int io, const void *v, const float2 *g, void *out, const float2 *tw4096, int L, int H, int BH,
                        hipStream_t st);

}  // namespace spectre
