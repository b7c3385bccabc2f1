// Content-adaptive spectral gate (Sec. 3.2 step 3a, 3c; positional phase of Sec. 3.5;
// Algorithm 1's decode gate) for gfx950.
//
//   pool    : sum of the query rows over positions, accumulated in fp64 in a fixed order
//   hidden  : x = inv_count * sum;  qbar = LayerNorm(x);  hid = GELU(qbar W1 + b1)
//   out     : u = hid W2 + b2 on the matrix cores (fp32 MFMA, the 2F output reals on the
//             32-row side of v_mfma_f32_32x32x2_f32, the (b,h) rows on the 32-column side),
//             with bias, modReLU and the positional phase applied in the epilogue.
#include "gate.h"

#include "common.h"

namespace spectre {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// ------------------------------------------------------------------------------------------
// pool, stage 1: grid (ceil(pairs_per_row/256), nchunks, B).  Lane = one channel pair of the
// [H*d] row; the workgroup sums rows [chunk*R, min(L, chunk*R+R)) in order.
template <typename IO>
__global__ __launch_bounds__(256) void k_pool_partial(const typename IO::pair_t *__restrict__ q,
                                                      double2 *__restrict__ partial, int L, int ppr,
                                                      int R, int nchunks) {
    const int pi = blockIdx.x * 256 + threadIdx.x;
    if (pi >= ppr) return;
    const int chunk = blockIdx.y, b = blockIdx.z;
    const int l0 = chunk * R, l1 = min(L, l0 + R);
    const typename IO::pair_t *src = q + ((size_t)b * L + l0) * ppr + pi;
    double sx = 0.0, sy = 0.0;
    int l = l0;
    for (; l + 4 <= l1; l += 4) {
        float2 a0 = IO::unpack(src[0]), a1 = IO::unpack(src[(size_t)ppr]);
        float2 a2 = IO::unpack(src[2 * (size_t)ppr]), a3 = IO::unpack(src[3 * (size_t)ppr]);
        sx += (double)a0.x; sy += (double)a0.y;
        sx += (double)a1.x; sy += (double)a1.y;
        sx += (double)a2.x; sy += (double)a2.y;
        sx += (double)a3.x; sy += (double)a3.y;
        src += 4 * (size_t)ppr;
    }
    for (; l < l1; ++l) {
        float2 a = IO::unpack(src[0]);
        sx += (double)a.x; sy += (double)a.y;
        src += ppr;
    }
    partial[((size_t)b * nchunks + chunk) * ppr + pi] = make_double2(sx, sy);
}

// pool, stage 2: sum_q[b][ch] = sum over chunks, in chunk order.  One lane per channel.
__global__ __launch_bounds__(256) void k_pool_final(const double *__restrict__ partial,
                                                    double *__restrict__ sum_q, int row, int nchunks,
                                                    int total) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int b = idx / row, ch = idx % row;
    const double *src = partial + (size_t)b * nchunks * row + ch;
    double s = 0.0;
    for (int c = 0; c < nchunks; ++c) s += src[(size_t)c * row];
    sum_q[idx] = s;
}

// ------------------------------------------------------------------------------------------
// hidden: one workgroup per (b, h).  LayerNorm statistics in fp64 (d values), the small
// d x d_g product on the vector units.
__global__ __launch_bounds__(256) void k_gate_hidden(const double *__restrict__ sum_q, double inv_count,
                                                     const float *__restrict__ gamma,
                                                     const float *__restrict__ beta, float eps,
                                                     const float *__restrict__ W1,
                                                     const float *__restrict__ b1, float *__restrict__ hid,
                                                     int H, int Hg, int d, int dg) {
    __shared__ double xs[256];
    __shared__ float qbar[256];
    __shared__ double stat[2];
    const int bh = blockIdx.x, h = bh % H, hp = (Hg == 1) ? 0 : h;
    const int tid = threadIdx.x;
    if (tid < d) xs[tid] = inv_count * sum_q[(size_t)bh * d + tid];
    __syncthreads();
    if (tid == 0) {
        double mean = 0.0, var = 0.0;
        for (int i = 0; i < d; ++i) mean += xs[i];
        mean /= d;
        for (int i = 0; i < d; ++i) var += (xs[i] - mean) * (xs[i] - mean);
        var /= d;
        stat[0] = mean;
        stat[1] = 1.0 / sqrt(var + (double)eps);
    }
    __syncthreads();
    if (tid < d)
        qbar[tid] = (float)((double)gamma[hp * d + tid] * (xs[tid] - stat[0]) * stat[1] + (double)beta[hp * d + tid]);
    __syncthreads();
    if (tid < dg) {
        float a = b1[hp * dg + tid];
        const float *w = W1 + (size_t)hp * d * dg + tid;
        for (int i = 0; i < d; ++i) a = fmaf(qbar[i], w[(size_t)i * dg], a);
        hid[(size_t)bh * dg + tid] = 0.5f * a * (1.0f + erff(a * 0.70710678118654752440f));
    }
}

// ------------------------------------------------------------------------------------------
// out: grid (ceil(2F/128), Hg == 1 ? 1 : H); 4 waves per workgroup, each wave owns 32
// consecutive output reals n (16 complex bins) and walks over the rows in tiles of 32.
// Row r means (b, h): r = b for per-head weights (h = blockIdx.y), r = b*H + h for shared.
//
// v_mfma_f32_32x32x2_f32 operands (lane l): A[i = l%32][k = l/32], B[k = l/32][j = l%32];
// accumulator register v holds D[i = 8*(v/4) + 4*(l/32) + v%4][j = l%32], so a lane owns, for
// its row j, the four reals v%4 = 0..3 = two whole complex bins of every 8-real group.
__global__ __launch_bounds__(256) void k_gate_out(const float *__restrict__ hid, const float *__restrict__ W2,
                                                  const float *__restrict__ b2,
                                                  const float *__restrict__ mbias, float2 *__restrict__ g,
                                                  int B, int H, int Hg, int dg, int F, int n_fft,
                                                  long long phase) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int twoF = 2 * F;
    const int n0 = (blockIdx.x * 4 + wave) * 32;
    if (n0 >= twoF) return;
    const int hsel = blockIdx.y;                     // head of this block when weights are per head
    const int hp = (Hg == 1) ? 0 : hsel;
    const int M = (Hg == 1) ? B * H : B;
    const int li = lane & 31, lk = lane >> 5;
    const int n_a = n0 + li;                         // this lane's A row (output real index)
    const float *w2 = W2 + (size_t)hp * dg * twoF;

    for (int r0 = 0; r0 < M; r0 += 32) {
        const int r = r0 + li;                       // this lane's B column (row of the product)
        const int bh = (Hg == 1) ? r : r * H + hsel;
        const float *hrow = hid + (size_t)bh * dg;
        floatx16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        for (int j0 = 0; j0 < dg; j0 += 16) {
            float a[8], bv[8];
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const int j = j0 + 2 * s + lk;
                a[s] = (j < dg && n_a < twoF) ? w2[(size_t)j * twoF + n_a] : 0.0f;
                bv[s] = (j < dg && r < M) ? hrow[j] : 0.0f;
            }
#pragma unroll
            for (int s = 0; s < 8; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s], bv[s], acc, 0, 0, 0);
        }
        if (r < M) {
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const int n = n0 + 8 * v4 + 4 * lk + 2 * half;   // even: real part index
                    if (n >= twoF) continue;
                    const int k = n >> 1;
                    float re = acc[4 * v4 + 2 * half] + b2[(size_t)hp * twoF + n];
                    float im = acc[4 * v4 + 2 * half + 1] + b2[(size_t)hp * twoF + n + 1];
                    if (mbias) {
                        const float mag = sqrtf(re * re + im * im);
                        const float act = fmaxf(mag + mbias[(size_t)hp * F + k], 0.0f);
                        const float sc = (mag > 0.0f) ? act / mag : 0.0f;
                        re *= sc;
                        im *= sc;
                    }
                    if (phase != 0) {
                        const long long m = ((long long)k * phase) % n_fft;
                        double s, c;
                        sincospi(2.0 * (double)m / (double)n_fft, &s, &c);
                        const float cf = (float)c, sf = (float)s;
                        const float nr = re * cf - im * sf, ni = re * sf + im * cf;
                        re = nr;
                        im = ni;
                    }
                    g[(size_t)bh * F + k] = make_float2(re, im);
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
size_t gate_partial_bytes(int B, int L, int H, int d) {
    const int nchunks = (L + kPoolRows - 1) / kPoolRows;
    return (size_t)B * nchunks * H * d * sizeof(double);
}

hipError_t launch_pool(int io, const void *q, double *partial, double *sum_q, int B, int L, int H, int d,
                       hipStream_t st) {
    const int ppr = H * d / 2;
    const int nchunks = (L + kPoolRows - 1) / kPoolRows;
    dim3 grid((ppr + 255) / 256, nchunks, B);
    if (io)
        k_pool_partial<IoBf16><<<grid, 256, 0, st>>>(static_cast<const uint32_t *>(q),
                                                     reinterpret_cast<double2 *>(partial), L, ppr, kPoolRows, nchunks);
    else
        k_pool_partial<IoF32><<<grid, 256, 0, st>>>(static_cast<const float2 *>(q),
                                                    reinterpret_cast<double2 *>(partial), L, ppr, kPoolRows, nchunks);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int total = B * H * d;
    k_pool_final<<<(total + 255) / 256, 256, 0, st>>>(partial, sum_q, H * d, nchunks, total);
    return hipGetLastError();
}

hipError_t launch_gate_mlp(const double *sum_q, double inv_count, const GateDev &P, float *hid, int B, int H,
                           long long phase, float2 *g, hipStream_t st) {
    k_gate_hidden<<<B * H, 256, 0, st>>>(sum_q, inv_count, P.ln_gamma, P.ln_beta, P.ln_eps, P.W1, P.b1, hid, H,
                                         P.Hg, P.d, P.d_g);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int F = P.n_fft / 2 + 1;
    dim3 grid((2 * F + 127) / 128, P.Hg == 1 ? 1 : H);
    k_gate_out<<<grid, 256, 0, st>>>(hid, P.W2, P.b2, P.modrelu_bias, g, B, H, P.Hg, P.d_g, F, P.n_fft, phase);
    return hipGetLastError();
}

}  // namespace spectre
