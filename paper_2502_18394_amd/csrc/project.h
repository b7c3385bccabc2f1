// Token projection kernels: host-side launch declarations (d = 64 channels per head).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace spectre {

// Number of row chunks (= partial column sums per head) for L rows.
int project_chunks(int L);

// v_out (and q_out unless nullptr) = x W per head; partial [B][chunks][H*64] receives the column sums
// of x per row chunk in fp64.  io 0 = fp32, 1 = bf16.  Wq, Wv [Hw, 64, 64] fp32, Hw = H or 1.
hipError_t launch_project(int io, const void *x, const float *Wq, const float *Wv, int Hw, void *v_out, void *q_out,
                          double *partial, int B, int L, int H, hipStream_t st);

// sum_q [B,H,64] = sum_x [B,H,64] times Wq per head, in fp64.
hipError_t launch_project_pooled(const double *sum_x, const float *Wq, int Hw, int B, int H, double *sum_q,
                                 hipStream_t st);

// W [Hw, 64, 64] fp32 -> wpack [Hw][2][512] x 16 bytes (kProjPackBytes per head): the weights in the order the bf16
// matrix instruction takes its B operand, split into two bf16 terms (hi, then lo).
constexpr size_t kProjPackBytes = 2 * 512 * 16;
hipError_t launch_pack_w(const float *W, int Hw, void *wpack, hipStream_t st);

}  // namespace spectre
