// Gate kernels: host-side launch declarations.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace spectre {

constexpr int kPoolRows = 256;   // rows summed by one workgroup of the pooling pass

struct GateDev {                 // device pointers; layout as in the public parameter block
    int Hg, d, d_g, n_fft;
    const float *ln_gamma, *ln_beta;
    float ln_eps;
    const float *W1, *b1, *W2, *b2, *modrelu_bias;
    const float2 *toeplitz;      // [Hg, 2r+1] or nullptr
    int toeplitz_r;
};

// Bytes of the pooling partial sums for query rows [B, L, H, d].
size_t gate_partial_bytes(int B, int L, int H, int d);

// sum_q [B,H,d] (double) = sum over the L rows of q [B,L,H,d]; io 0 = fp32, 1 = bf16.
hipError_t launch_pool(int io, const void *q, double *partial, double *sum_q, int B, int L, int H, int d,
                       hipStream_t st);

// sum [B][row] = sum over chunks of partial [B][nchunks][row], added in a fixed order in fp64.
// sum[b][ch] = (accumulate ? sum[b][ch] : 0) + sum over chunks of partial[b][chunk][ch]
hipError_t launch_pool_final(const double *partial, double *sum, int B, int row, int nchunks, hipStream_t st,
                             bool accumulate = false);

// g [B,H,F] from sum_q; hid is scratch [B,H,d_g]; raw is scratch [B,H,F] complex, only used when
// P.toeplitz is set; phase already reduced modulo n_fft.
hipError_t launch_gate_mlp(const double *sum_q, double inv_count, const GateDev &P, float *hid, float2 *raw,
                           int B, int H, long long phase, float2 *g, hipStream_t st);

}  // namespace spectre
