// Prefix-FFT cache kernels: host-side launch declarations (d = 64 channels per head).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace spectre {

hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t st);          // bytes % 16 == 0
hipError_t launch_fill_twiddle(float2 *tw, int N, hipStream_t st);

// Token `ti` of v_new/q_new [B, Tn, H, d] enters ring slot `slot`; delta [B*H*d] receives
// v_t - (evict ? v_old : 0); sum_q, v_buf, q_buf are updated in place.
hipError_t launch_ring_update(int io, const void *v_new, const void *q_new, int Tn, int ti, float *v_buf,
                              float *q_buf, double *sum_q, float *delta, int B, int H, int d, int N, int slot,
                              int evict, hipStream_t st);

// Number of partial-sum chunks the sweep produces per head for F bins.
int sweep_chunks(int F);
// update: Eq. (5) on every bin; read: partial sums of the newest row's readout with gate g.
hipError_t launch_sweep(bool update, bool read, float2 *X, const float *delta, const float2 *tw, const float2 *g,
                        float *partial, int BH, int F, int N, int slot, hipStream_t st);
// Deferred updates (the cache is only read by a decode step; pending rank-one updates are applied in one sweep
// every few steps).  pending [cap][B*H][64] holds the tokens' Delta rows, slots[i] their ring rows.
//   flush: apply all npend pending updates to X;  read: readout partials for the row `slot_new` with gate g;
//   without flush the kappa partials kpart [BH][chunks][32] of the pending tokens are produced as well.
constexpr int kMaxPending = 32;
// Ring-buffer bookkeeping for T <= W tokens appended at once (token i -> slot (s0 + i) mod W behind M0 memory rows,
// evicting when t0 + i >= W); partial [B][ceil(T/256)][H*64] doubles = per-chunk sums of q_new - q_evicted.
// V == nullptr: only the query side (q_buf, partial); the value rows are then written by whoever reads V.
hipError_t launch_ring_append(int io, const void *V, const void *Q, float *v_buf, float *q_buf, double *partial, int B,
                              int T, int H, int N, int M0, int W, int s0, long long t0, hipStream_t st);
hipError_t launch_sweep_lazy(bool flush, bool read, float2 *X, const float *pending, const float2 *tw, const float2 *g,
                             float *partial, float *kpart, int BH, int F, int N, int slot_new, int npend,
                             const int *slots, hipStream_t st);
hipError_t launch_readout_final_lazy(int io, const float *partial, const float *kpart, const float *pending, void *out,
                                     int BH, int F, int npend, hipStream_t st);
// out [B,1,H,d] (io dtype) from the sweep's partial sums.
hipError_t launch_readout_final(int io, const float *partial, void *out, int BH, int F, hipStream_t st);
// Memory rows mem [mem_batch (1 or B), H, Nmem, 64] into rows 0..Nmem-1 of v_buf [B, H, N, 64].
hipError_t launch_set_memory(const float *mem, int mem_batch, float *v_buf, int B, int H, int N, int Nmem,
                             hipStream_t st);
// scratch (complex transforms of channel pairs, big-kernel order) <-> cache rows.
hipError_t launch_untangle(const float2 *scr, float2 *X, int N, int N1, int N2, int P, int bh0, int nbh,
                           hipStream_t st);
hipError_t launch_tangle(const float2 *X, const float2 *g, float2 *scr, int N, int N1, int N2, int P, int bh0,
                         int nbh, hipStream_t st);

}  // namespace spectre
