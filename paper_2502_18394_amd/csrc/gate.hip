// Content-adaptive spectral gate (Sec. 3.2 step 3a, 3c; positional phase of Sec. 3.5;
// Algorithm 1's decode gate) for gfx950.
//
//   pool    : sum of the query rows over positions, accumulated in fp64 in a fixed order
//   hidden  : x = inv_count * sum;  qbar = LayerNorm(x);  hid = GELU(qbar W1 + b1)
//   out     : u = W2 hid + b2 on the matrix cores (fp32 MFMA, v_mfma_f32_4x4x1_16B_f32: 64
//             output reals x 4 rows per instruction), with bias and modReLU in the epilogue
//   phase   : the positional phase, a separate pass over g, only when a position is given
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

// The same sums with 16-byte loads: a lane owns four adjacent bf16 pairs or two adjacent fp32 pairs, eight rows in
// flight (the order of additions per channel is the row order, as above).  Needs the pairs per row to be a multiple
// of that and a 16-byte aligned tensor.  ppv = row length in 16-byte pieces.
template <bool BF16>
__global__ __launch_bounds__(256) void k_pool_partial_x16(const uint4 *__restrict__ q, double *__restrict__ partial,
                                                          int L, int ppv, int R, int nchunks) {
    constexpr int NCH = BF16 ? 8 : 4;                 // channels per 16 bytes
    const int pi = blockIdx.x * 256 + threadIdx.x;
    if (pi >= ppv) return;
    const int chunk = blockIdx.y, b = blockIdx.z;
    const int l0 = chunk * R, l1 = min(L, l0 + R);
    const uint4 *src = q + ((size_t)b * L + l0) * ppv + pi;
    double s[NCH];
#pragma unroll
    for (int i = 0; i < NCH; ++i) s[i] = 0.0;
    auto add = [&](const uint4 w) {
        if (BF16) {
            const float2 a = IoBf16::unpack(w.x), c = IoBf16::unpack(w.y), e = IoBf16::unpack(w.z), f = IoBf16::unpack(w.w);
            s[0] += (double)a.x; s[1] += (double)a.y; s[2] += (double)c.x; s[3] += (double)c.y;
            s[4 % NCH] += (double)e.x; s[5 % NCH] += (double)e.y; s[6 % NCH] += (double)f.x; s[7 % NCH] += (double)f.y;
        } else {
            s[0] += (double)__uint_as_float(w.x); s[1] += (double)__uint_as_float(w.y);
            s[2] += (double)__uint_as_float(w.z); s[3] += (double)__uint_as_float(w.w);
        }
    };
    typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
    int l = l0;
    for (; l + 8 <= l1; l += 8) {
        uint4 w[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(src + (size_t)i * ppv));
            w[i] = make_uint4(t.x, t.y, t.z, t.w);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) add(w[i]);
        src += 8 * (size_t)ppv;
    }
    for (; l < l1; ++l) {
        add(*src);
        src += ppv;
    }
    double *dst = partial + ((size_t)b * nchunks + chunk) * ((size_t)NCH * ppv) + (size_t)NCH * pi;
#pragma unroll
    for (int i = 0; i < NCH; i += 2) *reinterpret_cast<double2 *>(dst + i) = make_double2(s[i], s[i + 1]);
}

// pool, stage 2: sum_q[b][ch] = sum over chunks.  grid (row/32, B); 256 lanes = 32 channels x 8
// chunk groups; group r adds chunks r, r+8, ... in order, the 8 group sums are then added in order.
__global__ __launch_bounds__(256) void k_pool_final(const double *__restrict__ partial,
                                                    double *__restrict__ sum_q, int row, int nchunks, int accumulate) {
    __shared__ double red[8][32];
    const int lane = threadIdx.x & 31, grp = threadIdx.x >> 5;
    const int ch = blockIdx.x * 32 + lane, b = blockIdx.y;
    double s = 0.0;
    if (ch < row) {
        const double *src = partial + (size_t)b * nchunks * row + ch;
        int c = grp;
        for (; c + 56 < nchunks; c += 64) {       // eight loads in flight, added in the same order
            double t[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) t[i] = src[(size_t)(c + 8 * i) * row];
#pragma unroll
            for (int i = 0; i < 8; ++i) s += t[i];
        }
        for (; c < nchunks; c += 8) s += src[(size_t)c * row];
    }
    red[grp][lane] = s;
    __syncthreads();
    if (grp == 0 && ch < row) {
        double t = red[0][lane];
#pragma unroll
        for (int r = 1; r < 8; ++r) t += red[r][lane];
        sum_q[(size_t)b * row + ch] = accumulate ? sum_q[(size_t)b * row + ch] + t : t;
    }
}

// ------------------------------------------------------------------------------------------
// hidden: one workgroup per (b, h).  LayerNorm statistics in fp64 (d <= 256 values, one per lane: two tree
// reductions in a fixed order), then the small d x d_g product on the vector units with the d terms of an output
// split over 256 / d_g lane groups (fixed split, partial sums added in group order).
__device__ __forceinline__ double block_sum_256(double x, double *red, int lane, int wave) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    if (lane == 0) red[wave] = x;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

__global__ __launch_bounds__(256) void k_gate_hidden(const double *__restrict__ sum_q, double inv_count,
                                                     const float *__restrict__ gamma,
                                                     const float *__restrict__ beta, float eps,
                                                     const float *__restrict__ W1,
                                                     const float *__restrict__ b1, float *__restrict__ hid,
                                                     int H, int Hg, int d, int dg) {
    __shared__ float qbar[256];
    __shared__ float part[256];
    __shared__ double red[8];
    const int bh = blockIdx.x, h = bh % H, hp = (Hg == 1) ? 0 : h;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const double x = (tid < d) ? inv_count * sum_q[(size_t)bh * d + tid] : 0.0;
    const double mean = block_sum_256(x, red, lane, wave) / d;
    const double dev = (tid < d) ? x - mean : 0.0;
    const double var = block_sum_256(dev * dev, red + 4, lane, wave) / d;
    const double rstd = 1.0 / sqrt(var + (double)eps);
    if (tid < d) qbar[tid] = (float)((double)gamma[hp * d + tid] * dev * rstd + (double)beta[hp * d + tid]);
    __syncthreads();
    const int nseg = (dg <= 64) ? 4 : (dg <= 128) ? 2 : 1, cols = 256 / nseg;
    const int jcol = tid % cols, seg = tid / cols;
    const int dseg = (d + nseg - 1) / nseg, i0 = seg * dseg, i1 = (i0 + dseg < d) ? i0 + dseg : d;
    float a = 0.f;
    if (jcol < dg) {
        const float *w = W1 + (size_t)hp * d * dg + jcol;
#pragma unroll 8
        for (int i = i0; i < i1; ++i) a = fmaf(qbar[i], w[(size_t)i * dg], a);
    }
    part[tid] = a;
    __syncthreads();
    if (tid < dg) {
        float t = b1[hp * dg + tid];
        for (int q = 0; q < nseg; ++q) t += part[q * cols + tid];
        hid[(size_t)bh * dg + tid] = 0.5f * t * (1.0f + erff(t * 0.70710678118654752440f));
    }
}

// ------------------------------------------------------------------------------------------
// out: u = W2 hid + b2 on the matrix cores, then modReLU.  W2 is stored [Hg][2F][d_g] (the d_g
// weights of one output real are contiguous), so a tile of 64 consecutive output reals n is one
// contiguous 64*d_g*4-byte block; every wave walks over tiles with a grid stride and streams them.
//
// v_mfma_f32_4x4x1_16B_f32 multiplies 16 independent 4x1 by 1x4 blocks: lane l belongs to block
// l/4; it supplies A_b[i = l%4] and B_b[j = l%4] and receives D_b[i = v][j = l%4] in register v.
// Block b holds output reals n = n0 + 4b + i (so lane l supplies the weight of n = n0 + l for the
// current hidden index, and ends up with two whole complex bins), j is one of four rows (b, h) of
// the product.  Up to 8 row groups (32 rows) are accumulated per pass over W2.
// Row r means (b, h): r = b for per-head weights (head = blockIdx.y), r = b*H + h for shared.
typedef float floatx4 __attribute__((ext_vector_type(4)));
constexpr int kTileStride = 66;   // floats per staged row: 64 + 2, conflict-free for 8-byte row reads
constexpr int kHalfStride = 34;   // same for the 32-wide half rows of the d_g = 64 fast path

template <bool VEC>
__device__ __forceinline__ float4 load4(const float *__restrict__ p, int j, int dg, bool ok) {
    if (VEC) return ok ? *reinterpret_cast<const float4 *>(p + j) : make_float4(0.f, 0.f, 0.f, 0.f);
    float4 v;
    v.x = (ok && j + 0 < dg) ? p[j + 0] : 0.f;
    v.y = (ok && j + 1 < dg) ? p[j + 1] : 0.f;
    v.z = (ok && j + 2 < dg) ? p[j + 2] : 0.f;
    v.w = (ok && j + 3 < dg) ? p[j + 3] : 0.f;
    return v;
}

// four hidden indices of one staged weight row against RG row groups of hidden activations
template <int RG>
__device__ __forceinline__ void gate_mfma4(floatx4 (&acc)[RG], const float *arow, const float *hrow, int dgs) {
    const float2 a01 = *reinterpret_cast<const float2 *>(arow);
    const float2 a23 = *reinterpret_cast<const float2 *>(arow + 2);
#pragma unroll
    for (int q = 0; q < RG; ++q) {
        const float4 bv = *reinterpret_cast<const float4 *>(hrow + 4 * q * dgs);
        acc[q] = __builtin_amdgcn_mfma_f32_4x4x1f32(a01.x, bv.x, acc[q], 0, 0, 0);
        acc[q] = __builtin_amdgcn_mfma_f32_4x4x1f32(a01.y, bv.y, acc[q], 0, 0, 0);
        acc[q] = __builtin_amdgcn_mfma_f32_4x4x1f32(a23.x, bv.z, acc[q], 0, 0, 0);
        acc[q] = __builtin_amdgcn_mfma_f32_4x4x1f32(a23.y, bv.w, acc[q], 0, 0, 0);
    }
}

// 64 consecutive rows of W2 (d_g = 64) as sixteen 16-byte loads per lane: loads 0..7 cover hidden
// indices 0..31 of rows 8s + lane/8, loads 8..15 indices 32..63 (a wave instruction reads 8 half rows
// of 128 B)
__device__ __forceinline__ void gate_load_tile(float4 (&a)[16], const float *__restrict__ w2h, int tile, int lr,
                                               int lc, int twoF) {
#pragma unroll
    for (int s = 0; s < 16; ++s) {
        const int n = tile * 64 + 8 * (s & 7) + lr;
        a[s] = (n < twoF) ? stream_load(reinterpret_cast<const float4 *>(w2h + (size_t)n * 64 + 32 * (s >> 3) + lc))
                          : make_float4(0.f, 0.f, 0.f, 0.f);
    }
}

// modReLU (Sec. 3.2 step 3c) of one bin and its store
__device__ __forceinline__ void gate_store_bin(float2 *dst, float re, float im, bool act_on, float mb) {
    if (act_on) {
        const float mag = sqrtf(re * re + im * im);
        const float act = fmaxf(mag + mb, 0.0f);
        const float sc = (mag > 0.0f) ? act / mag : 0.0f;
        re *= sc;
        im *= sc;
    }
    *dst = make_float2(re, im);
}

template <bool VEC, int RG>   // VEC: d_g % 4 == 0 and 16-byte aligned rows; RG: row groups of 4
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(RG <= 2 ? 4 : 2))) void k_gate_out(const float *__restrict__ hid, const float *__restrict__ W2,
                                                  const float *__restrict__ b2,
                                                  const float *__restrict__ mbias, float2 *__restrict__ g,
                                                  int B, int H, int Hg, int dg, int F, int r_base0) {
    extern __shared__ float hs[];
    const int r_base = r_base0 + 32 * (int)blockIdx.z;   // blockIdx.z: 32-row tile of the rows (sequences)                    // [4*RG][dgs] hidden rows of this pass, zero padded
    const int dgp = (dg + 3) & ~3, dgs = dgp + 4;    // row stride padded against bank conflicts
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int twoF = 2 * F;
    const int hsel = blockIdx.y;                     // head of this block when weights are per head
    const int hp = (Hg == 1) ? 0 : hsel;
    const int M = (Hg == 1) ? B * H : B;
    for (int idx = threadIdx.x; idx < 4 * RG * dgs; idx += 256) {
        const int rr = idx / dgs, j = idx % dgs, r = r_base + rr;
        float v = 0.f;
        if (r < M && j < dg) v = hid[(size_t)((Hg == 1) ? r : r * H + hsel) * dg + j];
        hs[idx] = v;
    }
    __syncthreads();
    const int jrow = lane & 3;
    const int ntiles = (twoF + 63) / 64;
    // per-wave staging tile [64 rows][kTileStride floats]: filled with fully coalesced 16-byte
    // loads (a wave instruction covers 4 whole rows of 64 weights), read back one row per lane
    float *tile_w = hs + 4 * RG * dgs + wave * (64 * ((VEC && dg == 64) ? kHalfStride : kTileStride));
    const float *w2h = W2 + (size_t)hp * twoF * dg;
    if (VEC && dg == 64) {
        // fast path (one 64-wide slab per tile), software pipelined: the next tile's weights and this
        // tile's bias terms are in flight while the matrix cores work on the staged tile
        const int lr = lane >> 3, lc = 4 * (lane & 7);
        const int tstep = gridDim.x * 4;
        int tile = blockIdx.x * 4 + wave;
        float4 a[16];
        if (tile < ntiles) gate_load_tile(a, w2h, tile, lr, lc, twoF);
        for (; tile < ntiles; tile += tstep) {
            floatx4 acc[RG];
#pragma unroll
            for (int q = 0; q < RG; ++q) acc[q] = floatx4{0.f, 0.f, 0.f, 0.f};
            const float *arow = tile_w + lane * kHalfStride;
            const float *hrow = hs + jrow * dgs;
            // first half of the hidden indices through the staging tile
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                float2 *dst = reinterpret_cast<float2 *>(tile_w + (8 * s + lr) * kHalfStride + lc);
                dst[0] = make_float2(a[s].x, a[s].y);
                dst[1] = make_float2(a[s].z, a[s].w);
            }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int jj = 0; jj < 32; jj += 4) gate_mfma4<RG>(acc, arow + jj, hrow + jj, dgs);
            __builtin_amdgcn_wave_barrier();
            // second half; after its copy to LDS the registers are free for the next tile's loads
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                float2 *dst = reinterpret_cast<float2 *>(tile_w + (8 * s + lr) * kHalfStride + lc);
                dst[0] = make_float2(a[8 + s].x, a[8 + s].y);
                dst[1] = make_float2(a[8 + s].z, a[8 + s].w);
            }
            if (tile + tstep < ntiles) gate_load_tile(a, w2h, tile + tstep, lr, lc, twoF);
            const int n4 = tile * 64 + (lane & ~3);
            const bool e_ok = n4 < twoF;                      // twoF is even and n4 a multiple of 4
            const bool e_ok2 = n4 + 2 < twoF;
            float4 bias4 = make_float4(0.f, 0.f, 0.f, 0.f);
            float2 mb2 = make_float2(0.f, 0.f);
            if (e_ok) {
                const float *bp = b2 + (size_t)hp * twoF + n4;
                bias4.x = bp[0]; bias4.y = bp[1];
                if (e_ok2) { bias4.z = bp[2]; bias4.w = bp[3]; }
                if (mbias) {
                    const float *mp = mbias + (size_t)hp * F + (n4 >> 1);
                    mb2.x = mp[0];
                    if (e_ok2) mb2.y = mp[1];
                }
            }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int jj = 0; jj < 32; jj += 4) gate_mfma4<RG>(acc, arow + jj, hrow + 32 + jj, dgs);
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int q = 0; q < RG; ++q) {
                const int r = r_base + 4 * q + jrow;
                if (r >= M || !e_ok) continue;
                const int bh = (Hg == 1) ? r : r * H + hsel;
                gate_store_bin(g + (size_t)bh * F + (n4 >> 1), acc[q][0] + bias4.x, acc[q][1] + bias4.y, mbias != nullptr, mb2.x);
                if (e_ok2)
                    gate_store_bin(g + (size_t)bh * F + (n4 >> 1) + 1, acc[q][2] + bias4.z, acc[q][3] + bias4.w, mbias != nullptr, mb2.y);
            }
        }
        return;
    }
    for (int tile = blockIdx.x * 4 + wave; tile < ntiles; tile += gridDim.x * 4) {
        floatx4 acc[RG];
#pragma unroll
        for (int q = 0; q < RG; ++q) acc[q] = floatx4{0.f, 0.f, 0.f, 0.f};
        for (int j0 = 0; j0 < dgp; j0 += 64) {
            const int width = min(64, dgp - j0);          // hidden indices in this slab, multiple of 4
            const int lpr = width / 4;                     // lanes per row
            const int rows_per_instr = 64 / lpr;
            const int lr = lane / lpr, lc = 4 * (lane % lpr);
            for (int r0 = 0; r0 < 64; r0 += rows_per_instr) {
                const int row = r0 + lr, n = tile * 64 + row;
                if (row < 64) {
                    const float4 v = load4<VEC>(w2h + (size_t)(n < twoF ? n : 0) * dg, j0 + lc, dg, n < twoF);
                    float *dst = tile_w + row * kTileStride + lc;
                    dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
                }
            }
            // LDS operations of one wave complete in issue order, so the reads below see the writes
            // above; the wave barrier only stops the compiler from moving code across this point
            __builtin_amdgcn_wave_barrier();
            const float *arow = tile_w + lane * kTileStride;
            const float *hrow = hs + jrow * dgs + j0;
            for (int jj = 0; jj < width; jj += 4) gate_mfma4<RG>(acc, arow + jj, hrow + jj, dgs);
            __builtin_amdgcn_wave_barrier();
        }
        // epilogue: this lane holds reals n4 .. n4+3 (two bins) of row r for every row group
        const int n4 = tile * 64 + (lane & ~3);
#pragma unroll
        for (int q = 0; q < RG; ++q) {
            const int r = r_base + 4 * q + jrow;
            if (r >= M) continue;
            const int bh = (Hg == 1) ? r : r * H + hsel;
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int nn = n4 + 2 * half;
                if (nn >= twoF) continue;
                const int k = nn >> 1;
                gate_store_bin(g + (size_t)bh * F + k, acc[q][2 * half] + b2[(size_t)hp * twoF + nn],
                               acc[q][2 * half + 1] + b2[(size_t)hp * twoF + nn + 1], mbias != nullptr,
                               mbias ? mbias[(size_t)hp * F + k] : 0.0f);
            }
        }
    }
}

// Toeplitz low-rank update (Sec. 3.2 step 3b) followed by modReLU (step 3c):
//   g_k = act( raw_k + sum_{m=-r..r} t_m raw_{k-m} ),  raw = 0 outside 0..F-1.   One lane per bin.
__global__ __launch_bounds__(256) void k_gate_toeplitz(const float2 *__restrict__ raw, const float2 *__restrict__ taps,
                                                       const float *__restrict__ mbias, float2 *__restrict__ g,
                                                       int H, int Hg, int F, int r, size_t total) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int k = (int)(idx % F);
    const size_t bh = idx / F;
    const int hp = (Hg == 1) ? 0 : (int)(bh % H);
    const float2 *t = taps + (size_t)hp * (2 * r + 1) + r;
    const float2 *row = raw + bh * F;
    float2 acc = row[k];
    for (int m = -r; m <= r; ++m) {
        const int src = k - m;
        if (src < 0 || src >= F) continue;
        const float2 pr = cmul(t[m], row[src]);
        acc.x += pr.x;
        acc.y += pr.y;
    }
    gate_store_bin(g + idx, acc.x, acc.y, mbias != nullptr, mbias ? mbias[(size_t)hp * F + k] : 0.0f);
}

// positional phase: g[bh][k] *= exp(+j 2 pi ((k p) mod n)/n), angle reduced in integers and
// evaluated in fp64.  One lane per gate entry; only launched when p != 0.
__global__ __launch_bounds__(256) void k_gate_phase(float2 *__restrict__ g, int F, int n_fft, long long phase,
                                                    size_t total) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const long long k = (long long)(idx % F);
    const long long m = (k * phase) % n_fft;
    double s, c;
    sincospi(2.0 * (double)m / (double)n_fft, &s, &c);
    const float cf = (float)c, sf = (float)s;
    const float2 v = g[idx];
    g[idx] = make_float2(v.x * cf - v.y * sf, v.x * sf + v.y * cf);
}

// ------------------------------------------------------------------------------------------
// Rows summed by one workgroup of the pooling pass: kPoolRows, halved (down to 16) while the pass would launch
// fewer than about two workgroups per compute unit (short sequences: 8192 rows of 32 heads are only 32 chunks of 256).
static int pool_rows(int B, int L, int H, int d) {
    const long long wide = ((long long)H * d / 8 + 255) / 256;       // workgroups across a row with 16-byte lanes
    int rows = kPoolRows;
    while (rows > 16 && (long long)B * ((L + rows - 1) / rows) * wide < 512) rows /= 2;
    return rows;
}

size_t gate_partial_bytes(int B, int L, int H, int d) {
    const int rows = pool_rows(B, L, H, d);
    const int nchunks = (L + rows - 1) / rows;
    return (size_t)B * nchunks * H * d * sizeof(double);
}

hipError_t launch_pool(int io, const void *q, double *partial, double *sum_q, int B, int L, int H, int d,
                       hipStream_t st) {
    const int ppr = H * d / 2;
    const int rows = pool_rows(B, L, H, d);
    const int nchunks = (L + rows - 1) / rows;
    dim3 grid((ppr + 255) / 256, nchunks, B);
    const bool aligned = (reinterpret_cast<uintptr_t>(q) & 15) == 0;
    if (io && ppr % 4 == 0 && aligned)
        k_pool_partial_x16<true><<<dim3((ppr / 4 + 255) / 256, nchunks, B), 256, 0, st>>>(
            static_cast<const uint4 *>(q), partial, L, ppr / 4, rows, nchunks);
    else if (!io && ppr % 2 == 0 && aligned)
        k_pool_partial_x16<false><<<dim3((ppr / 2 + 255) / 256, nchunks, B), 256, 0, st>>>(
            static_cast<const uint4 *>(q), partial, L, ppr / 2, rows, nchunks);
    else if (io)
        k_pool_partial<IoBf16><<<grid, 256, 0, st>>>(static_cast<const uint32_t *>(q),
                                                     reinterpret_cast<double2 *>(partial), L, ppr, rows, nchunks);
    else
        k_pool_partial<IoF32><<<grid, 256, 0, st>>>(static_cast<const float2 *>(q),
                                                    reinterpret_cast<double2 *>(partial), L, ppr, rows, nchunks);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    k_pool_final<<<dim3((H * d + 31) / 32, B), 256, 0, st>>>(partial, sum_q, H * d, nchunks, 0);
    return hipGetLastError();
}

hipError_t launch_pool_final(const double *partial, double *sum, int B, int row, int nchunks, hipStream_t st,
                             bool accumulate) {
    k_pool_final<<<dim3((row + 31) / 32, B), 256, 0, st>>>(partial, sum, row, nchunks, accumulate ? 1 : 0);
    return hipGetLastError();
}

hipError_t launch_gate_mlp(const double *sum_q, double inv_count, const GateDev &P, float *hid, float2 *raw,
                           int B, int H, long long phase, float2 *g, hipStream_t st) {
    k_gate_hidden<<<B * H, 256, 0, st>>>(sum_q, inv_count, P.ln_gamma, P.ln_beta, P.ln_eps, P.W1, P.b1, hid, H,
                                         P.Hg, P.d, P.d_g);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int F = P.n_fft / 2 + 1;
    const int M = (P.Hg == 1) ? B * H : B;
    const int ntiles = (2 * F + 63) / 64;
    const int gy = P.Hg == 1 ? 1 : H;
    int gx = (4096 + gy - 1) / gy;                 // about 16 workgroups per compute unit in total (1024: 5 % slower)
    if (gx > (ntiles + 3) / 4) gx = (ntiles + 3) / 4;
    {   // shrink the grid to the smallest one with the same number of tiles per wave (no ragged last round)
        const int iters = (ntiles + 4 * gx - 1) / (4 * gx);
        gx = (ntiles + 4 * iters - 1) / (4 * iters);
    }
    dim3 grid(gx, gy);
    const bool vec = (P.d_g % 4 == 0) && (reinterpret_cast<uintptr_t>(P.W2) & 15) == 0;
    const int dgp = (P.d_g + 3) & ~3;
    // with the Toeplitz update the MLP output goes to `raw` un-activated and a second pass finishes it
    const float *out_bias = P.toeplitz ? nullptr : P.modrelu_bias;
    float2 *out_g = P.toeplitz ? raw : g;
    {
        // every 32-row tile of the rows in one launch (grid.z); a single tile takes the narrowest kernel that fits
        const int ntile = (M + 31) / 32;
        const int rows = (ntile > 1) ? 32 : M;
        const int rg = (rows + 3) / 4;            // 1..8 row groups per tile
        const size_t lds = ((size_t)4 * (rg <= 1 ? 1 : rg <= 2 ? 2 : rg <= 4 ? 4 : 8) * (dgp + 4) +
                            4 * 64 * ((vec && P.d_g == 64) ? kHalfStride : kTileStride)) * sizeof(float);
        for (int z0 = 0; z0 < ntile; z0 += 65535) {
            const int nz = (ntile - z0 < 65535) ? ntile - z0 : 65535;
            const dim3 grid3(grid.x, grid.y, nz);
            const int r_base = 32 * z0;
#define SPECTRE_GATE_OUT(V, R) k_gate_out<V, R><<<grid3, 256, lds, st>>>(hid, P.W2, P.b2, out_bias, out_g, B, H, P.Hg, P.d_g, F, r_base)
            if (vec) {
                if (rg <= 1) SPECTRE_GATE_OUT(true, 1); else if (rg <= 2) SPECTRE_GATE_OUT(true, 2);
                else if (rg <= 4) SPECTRE_GATE_OUT(true, 4); else SPECTRE_GATE_OUT(true, 8);
            } else {
                if (rg <= 1) SPECTRE_GATE_OUT(false, 1); else if (rg <= 2) SPECTRE_GATE_OUT(false, 2);
                else if (rg <= 4) SPECTRE_GATE_OUT(false, 4); else SPECTRE_GATE_OUT(false, 8);
            }
#undef SPECTRE_GATE_OUT
            hipError_t e2 = hipGetLastError();
            if (e2 != hipSuccess) return e2;
        }
    }
    const size_t total = (size_t)B * H * F;
    if (P.toeplitz) {
        k_gate_toeplitz<<<(unsigned)((total + 255) / 256), 256, 0, st>>>(raw, P.toeplitz, P.modrelu_bias, g, H, P.Hg, F,
                                                                         P.toeplitz_r, total);
    }
    e = hipGetLastError();
    if (e != hipSuccess || phase == 0) return e;
    k_gate_phase<<<(unsigned)((total + 255) / 256), 256, 0, st>>>(g, F, P.n_fft, phase, total);
    return hipGetLastError();
}

// Loads this translation unit's code object (the runtime loads them on first use): called by spectre_prepare so
// that no compute call is the first to touch it.
hipError_t load_kernels_gate() {
    hipFuncAttributes a;
    return hipFuncGetAttributes(&a, reinterpret_cast<const void *>(k_pool_final));
}

}  // namespace spectre
