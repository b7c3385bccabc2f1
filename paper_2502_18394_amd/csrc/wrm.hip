// Wavelet refinement (Sec. 3.5) for gfx950: level gates and the block-mean form of
// V + iDWT(s * DWT(V)) for the orthonormal Haar wavelet.
#include "wrm.h"

#include "common.h"

namespace spectre {

// ------------------------------------------------------------------------------------------
// gates: one workgroup per (b, h).  LayerNorm statistics in fp64, both layers on the vector units
// (d x d_w and d_w x (J+1) d are tiny).
__global__ __launch_bounds__(256) void k_wrm_gates(const double *__restrict__ sum_q, double inv_count,
                                                   const float *__restrict__ gamma, const float *__restrict__ beta,
                                                   float eps, const float *__restrict__ W1,
                                                   const float *__restrict__ b1, const float *__restrict__ W2,
                                                   const float *__restrict__ b2, float *__restrict__ s, int H, int Hg,
                                                   int d, int dw, int nout) {
    __shared__ double xs[256];
    __shared__ float qbar[256];
    __shared__ float hid[256];
    __shared__ double stat[2];
    // grid (B*H, ceil(nout / 256)): every workgroup repeats the tiny LayerNorm and first layer and emits 256 outputs
    // (the output layer is a chain of d_w dependent loads per output: one workgroup per head left it latency-bound)
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
    if (tid < dw) {
        float a = b1[hp * dw + tid];
        const float *w = W1 + (size_t)hp * d * dw + tid;
        for (int i = 0; i < d; ++i) a = fmaf(qbar[i], w[(size_t)i * dw], a);
        hid[tid] = 0.5f * a * (1.0f + erff(a * 0.70710678118654752440f));
    }
    __syncthreads();
    const int o = blockIdx.y * 256 + tid;
    if (o < nout) {
        float a = b2[(size_t)hp * nout + o];
        const float *w = W2 + (size_t)hp * dw * nout + o;
        for (int j = 0; j < dw; ++j) a = fmaf(hid[j], w[(size_t)j * nout], a);
        s[(size_t)bh * nout + o] = a;
    }
}

// ------------------------------------------------------------------------------------------
// Grids are (H, tiles, B) with the head index fastest: workgroups that run together then read all heads of
// the same rows, i.e. whole contiguous token rows, and spread over every memory channel (one head's
// 128-byte slices alone, 4 KB apart, sit on a fraction of them).
// Row ownership inside a tile of 256 rows: thread (pair p = tid % 32, r = tid / 32) owns the 32
// consecutive rows 32 r .. 32 r + 31 of channel pair p, so a row of a head is one coalesced
// 128 B / 256 B segment across 32 lanes and levels 1..5 never leave the thread's registers.

// tile sums (only needed above level 8): S[bh][tile][c] = sum of the tile's rows.
template <typename IO>
__global__ __launch_bounds__(256) void k_wrm_tile_sums(const typename IO::pair_t *__restrict__ v,
                                                       float2 *__restrict__ S, int L, int H, int ntiles) {
    __shared__ float2 part[8][32];
    const int tid = threadIdx.x, p = tid & 31, r = tid >> 5;
    const int h = blockIdx.x, tile = blockIdx.y, b = blockIdx.z, bh = b * H + h;
    const int row0 = tile * kWrmTileRows + r * 32;
    // all 32 loads are issued before the first use (the raw words are kept; unpacking inside the guarded
    // load would make every load wait for the previous one)
    typename IO::pair_t raw[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        const int l = row0 + i;
        raw[i] = (l < L) ? v[(((size_t)b * L + l) * H + h) * 32 + p] : IO::zero();
    }
    float2 acc = make_float2(0.f, 0.f);
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        const float2 x = IO::unpack(raw[i]);
        acc.x += x.x;
        acc.y += x.y;
    }
    part[r][p] = acc;
    __syncthreads();
    if (r == 0) {
        float2 t = part[0][p];
#pragma unroll
        for (int q = 1; q < 8; ++q) {
            t.x += part[q][p].x;
            t.y += part[q][p].y;
        }
        S[((size_t)bh * ntiles + tile) * 32 + p] = t;
    }
}

// The same sums over whole token rows with 16-byte loads (four bf16 pairs or two fp32 pairs per lane, eight rows
// in flight) for a 16-byte aligned tensor; every tile is full here (the levels that need the sums make L a multiple
// of 512).  The additions follow the order of the kernel above: 32 rows in turn, then the eight partial sums in turn.
template <bool BF16>
__global__ __launch_bounds__(256) void k_wrm_tile_sums_x16(const uint4 *__restrict__ v, float *__restrict__ S, int L,
                                                           int H, int ntiles, int ppv) {
    constexpr int NCH = BF16 ? 8 : 4;                 // channels per 16 bytes
    typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
    const int pi = blockIdx.x * 256 + threadIdx.x;
    if (pi >= ppv) return;
    const int tile = blockIdx.y, b = blockIdx.z;
    const uint4 *src = v + ((size_t)b * L + (size_t)tile * kWrmTileRows) * ppv + pi;
    float tot[NCH];
#pragma unroll 1
    for (int grp = 0; grp < 8; ++grp) {
        float acc[NCH];
#pragma unroll
        for (int c = 0; c < NCH; ++c) acc[c] = 0.f;
#pragma unroll
        for (int i0 = 0; i0 < 32; i0 += 8) {
            u32x4_t w[8];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                w[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(src + (size_t)(i0 + i) * ppv));
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (BF16) {
                    const float2 a = IoBf16::unpack(w[i].x), c = IoBf16::unpack(w[i].y), e = IoBf16::unpack(w[i].z),
                                 f = IoBf16::unpack(w[i].w);
                    acc[0] += a.x; acc[1] += a.y; acc[2] += c.x; acc[3] += c.y;
                    acc[4 % NCH] += e.x; acc[5 % NCH] += e.y; acc[6 % NCH] += f.x; acc[7 % NCH] += f.y;
                } else {
                    acc[0] += __uint_as_float(w[i].x); acc[1] += __uint_as_float(w[i].y);
                    acc[2] += __uint_as_float(w[i].z); acc[3] += __uint_as_float(w[i].w);
                }
            }
        }
#pragma unroll
        for (int c = 0; c < NCH; ++c) tot[c] = (grp == 0) ? acc[c] : tot[c] + acc[c];
        src += (size_t)32 * ppv;
    }
    const int e0 = NCH * pi, h = e0 >> 6, c0 = e0 & 63;
    float *dst = S + (((size_t)b * H + h) * ntiles + tile) * 64 + c0;
#pragma unroll
    for (int c = 0; c < NCH; c += 4) *reinterpret_cast<float4 *>(dst + c) = make_float4(tot[c], tot[c + 1], tot[c + 2], tot[c + 3]);
}

// Tile sums from sums of smaller row blocks that the producer of v emitted on the side (the mixer's store phase):
// S[bh][tile][c] = sum over the tile's 256 / block_rows blocks, in row order.  One lane per (bh, tile, c).
__global__ __launch_bounds__(256) void k_wrm_tile_sums_from_blocks(const float *__restrict__ bsum, float *__restrict__ S,
                                                                   int per_tile, size_t total) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int c = (int)(idx & 63);
    const size_t bt = idx >> 6;                        // (bh, tile)
    const float *src = bsum + bt * per_tile * 64 + c;
    float acc = 0.f;
    for (int i = 0; i < per_tile; ++i) acc += src[(size_t)i * 64];
    S[idx] = acc;
}

// coefficient of the level-l block mean in the closed form above
__device__ __forceinline__ float wrm_coef(const float *__restrict__ sb, int l, int J, int c) {
    return (l < J) ? sb[(l + 1) * 64 + c] - sb[l * 64 + c] : sb[c] - sb[J * 64 + c];
}

// upper levels 9..J: one workgroup per (bh, group of kUpCh channels) builds the pyramid of block sums
// over the tiles in LDS, then walks it top-down accumulating coef_l * A_l; U[bh][tile][c] is the
// sum of those terms for the blocks that contain the tile.  256 lanes = kUpCh channels x kUpLanes tiles.
constexpr int kUpCh = 4, kUpLanes = 256 / kUpCh;
__global__ __launch_bounds__(256) void k_wrm_upper(const float *__restrict__ S, const float *__restrict__ s,
                                                   float *__restrict__ U, int ntiles, int J) {
    extern __shared__ float pyr[];                     // levels 8, 9, ..., J back to back, kUpCh channels each
    const int tid = threadIdx.x, cl = tid % kUpCh, lane = tid / kUpCh;
    const int bh = blockIdx.x, c = blockIdx.y * kUpCh + cl;
    const float *sb = s + (size_t)bh * (J + 1) * 64;
    for (int i = lane; i < ntiles; i += kUpLanes) pyr[i * kUpCh + cl] = S[((size_t)bh * ntiles + i) * 64 + c];
    __syncthreads();
    int off = 0, n = ntiles;
    for (int l = kWrmTileLevels + 1; l <= J; ++l) {    // up: block sums
        const int noff = off + n, nn = n >> 1;
        for (int i = lane; i < nn; i += kUpLanes)
            pyr[(noff + i) * kUpCh + cl] = pyr[(off + 2 * i) * kUpCh + cl] + pyr[(off + 2 * i + 1) * kUpCh + cl];
        __syncthreads();
        off = noff;
        n = nn;
    }
    // down: entry i of level l becomes the correction shared by the rows of its block
    for (int i = lane; i < n; i += kUpLanes) pyr[(off + i) * kUpCh + cl] *= wrm_coef(sb, J, J, c) * exp2f(-(float)J);
    __syncthreads();
    for (int l = J - 1; l > kWrmTileLevels; --l) {
        const int poff = off, nn = n << 1;
        off -= nn;
        const float cf = wrm_coef(sb, l, J, c) * exp2f(-(float)l);
        for (int i = lane; i < nn; i += kUpLanes)
            pyr[(off + i) * kUpCh + cl] = pyr[(off + i) * kUpCh + cl] * cf + pyr[(poff + (i >> 1)) * kUpCh + cl];
        __syncthreads();
        n = nn;
    }
    // now `off` is level 9's offset (= ntiles) and n its length
    for (int i = lane; i < ntiles; i += kUpLanes)
        U[((size_t)bh * ntiles + i) * 64 + c] = pyr[(off + (i >> 1)) * kUpCh + cl];
}

template <typename IO>
__global__ __launch_bounds__(256) void k_wrm_apply(const typename IO::pair_t *__restrict__ v,
                                                   const float *__restrict__ s, const float2 *__restrict__ U,
                                                   typename IO::pair_t *__restrict__ out, int L, int H, int J,
                                                   int ntiles) {
    __shared__ float2 part[8][33];
    const int tid = threadIdx.x, p = tid & 31, r = tid >> 5;
    const int h = blockIdx.x, tile = blockIdx.y, b = blockIdx.z, bh = b * H + h;
    const int row0 = tile * kWrmTileRows + r * 32;
    const float *sb = s + (size_t)bh * (J + 1) * 64;
    const int c0 = 2 * p;

    float2 x[32];
    {   // issue all loads before the first unpack (see k_wrm_tile_sums)
        typename IO::pair_t raw[32];
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            const int l = row0 + i;
            raw[i] = (l < L) ? IO::load_stream(v + (((size_t)b * L + l) * H + h) * 32 + p) : IO::zero();
        }
#pragma unroll
        for (int i = 0; i < 32; ++i) x[i] = IO::unpack(raw[i]);
    }
    // block sums of levels 1..5 inside the thread
    float2 s1[16], s2[8], s3[4], s4[2], s5;
#pragma unroll
    for (int i = 0; i < 16; ++i) s1[i] = x[2 * i] + x[2 * i + 1];
#pragma unroll
    for (int i = 0; i < 8; ++i) s2[i] = s1[2 * i] + s1[2 * i + 1];
#pragma unroll
    for (int i = 0; i < 4; ++i) s3[i] = s2[2 * i] + s2[2 * i + 1];
#pragma unroll
    for (int i = 0; i < 2; ++i) s4[i] = s3[2 * i] + s3[2 * i + 1];
    s5 = s4[0] + s4[1];
    // levels 6..8 across the 8 row groups of the tile
    part[r][p] = s5;
    __syncthreads();
    float2 corr = make_float2(0.f, 0.f);
    if (J > kWrmTileLevels) corr = U[((size_t)bh * ntiles + tile) * 32 + p];
    auto add_level = [&](int l, float2 sum) {       // corr += coef_l * (block sum / 2^l), levels above J carry no term
        if (l <= J) {
            const float sc = exp2f(-(float)l);
            corr.x = fmaf(wrm_coef(sb, l, J, c0) * sc, sum.x, corr.x);
            corr.y = fmaf(wrm_coef(sb, l, J, c0 + 1) * sc, sum.y, corr.y);
        }
    };
    if (J >= 6) {
        float2 q[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) q[i] = part[i][p];
        float2 s8 = ((q[0] + q[1]) + (q[2] + q[3])) + ((q[4] + q[5]) + (q[6] + q[7]));
        const int r4 = r & ~3, r2 = r & ~1;
        float2 s7 = make_float2(0.f, 0.f), s6 = make_float2(0.f, 0.f);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if ((i & ~3) == r4) s7 = s7 + q[i];
            if ((i & ~1) == r2) s6 = s6 + q[i];
        }
        add_level(8, s8);
        add_level(7, s7);
        add_level(6, s6);
    }
    add_level(5, s5);
    // levels 4..1: the correction splits as the blocks halve
    float cf[4][2];
#pragma unroll
    for (int l = 1; l <= 4; ++l) {
        const float sc = exp2f(-(float)l);
        cf[l - 1][0] = (l <= J) ? wrm_coef(sb, l, J, c0) * sc : 0.f;
        cf[l - 1][1] = (l <= J) ? wrm_coef(sb, l, J, c0 + 1) * sc : 0.f;
    }
    const int sidx = (J >= 1) ? 1 : 0;
    const float f0x = 1.0f + sb[sidx * 64 + c0], f0y = 1.0f + sb[sidx * 64 + c0 + 1];
#pragma unroll
    for (int i4 = 0; i4 < 2; ++i4) {
        const float2 c4 = make_float2(fmaf(cf[3][0], s4[i4].x, corr.x), fmaf(cf[3][1], s4[i4].y, corr.y));
#pragma unroll
        for (int j3 = 0; j3 < 2; ++j3) {
            const int i3 = 2 * i4 + j3;
            const float2 c3 = make_float2(fmaf(cf[2][0], s3[i3].x, c4.x), fmaf(cf[2][1], s3[i3].y, c4.y));
#pragma unroll
            for (int j2 = 0; j2 < 2; ++j2) {
                const int i2 = 2 * i3 + j2;
                const float2 c2 = make_float2(fmaf(cf[1][0], s2[i2].x, c3.x), fmaf(cf[1][1], s2[i2].y, c3.y));
#pragma unroll
                for (int j1 = 0; j1 < 2; ++j1) {
                    const int i1 = 2 * i2 + j1;
                    const float2 c1 = make_float2(fmaf(cf[0][0], s1[i1].x, c2.x), fmaf(cf[0][1], s1[i1].y, c2.y));
#pragma unroll
                    for (int j0 = 0; j0 < 2; ++j0) {
                        const int i = 2 * i1 + j0, l = row0 + i;
                        if (l < L) {
                            const float2 y = make_float2(fmaf(f0x, x[i].x, c1.x), fmaf(f0y, x[i].y, c1.y));
                            IO::store_stream(out + (((size_t)b * L + l) * H + h) * 32 + p, IO::pack(y));
                        }
                    }
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// One gate per wavelet coefficient and channel (Sec. 3.5 step b as printed, s in R^(n x d)): a real Haar analysis,
// gate, synthesis.  sc [B*H][L][64] holds the gates in the analysis' coefficient order [a_J | d_J | ... | d_1]: the
// detail of level l of the block of 2^l rows number i sits at position (L >> l) + i, the approximation of the block
// of 2^J rows number i at position i.  With S1, S2 the sums of a block's two halves, its detail coefficient is
// (S1 - S2) / sqrt(2^l) and contributes -/+ gate * (S1 - S2) / 2^l to the rows of its halves; the approximation
// contributes gate * (S1 + S2) / 2^J to all rows of the block.  Same tiling as k_wrm_apply: a lane owns 32
// consecutive rows of a channel pair (levels 1..5 in registers), levels 6..8 cross the 8 row groups of a tile through
// LDS, and levels above 8 arrive as one per-tile constant U (k_wrm_upper_coeff, from the tile sums).
//
// JT = min(J, 6): the levels inside a lane's 32 rows are compile-time (JT <= 5: the analysis stops at level JT and
// the lane also applies the approximation gates of its 32 >> JT blocks); the levels 6..8 are tested at run time.
template <int JT>
__device__ __forceinline__ float2 coeff_gate(const float *__restrict__ sc, size_t pos, int c0, bool valid) {
    return valid ? *reinterpret_cast<const float2 *>(sc + pos * 64 + c0) : make_float2(0.f, 0.f);
}

template <typename IO, int JT>
__global__ __launch_bounds__(256) void k_wrm_coeff(const typename IO::pair_t *__restrict__ v,
                                                   const float *__restrict__ s, const float2 *__restrict__ U,
                                                   typename IO::pair_t *__restrict__ out, int L, int H, int J,
                                                   int ntiles) {
    __shared__ float2 part[8][33];
    const int tid = threadIdx.x, p = tid & 31, r = tid >> 5;
    const int h = blockIdx.x, tile = blockIdx.y, b = blockIdx.z, bh = b * H + h;
    const int row0 = tile * kWrmTileRows + r * 32;
    const float *sc = s + (size_t)bh * L * 64;
    const int c0 = 2 * p;
    constexpr int LV = JT < 5 ? JT : 5;                // detail levels inside the lane

    // every load is issued before the first use: rows, then the gates of the lane's blocks
    typename IO::pair_t raw[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        const int l = row0 + i;
        raw[i] = (l < L) ? IO::load_stream(v + (((size_t)b * L + l) * H + h) * 32 + p) : IO::zero();
    }
    float2 g1[16], g2[8], g3[4], g4[2], g5 = make_float2(0.f, 0.f), ga[JT <= 5 ? (32 >> LV) : 1];
#pragma unroll
    for (int i = 0; i < 16; ++i) g1[i] = (LV >= 1) ? coeff_gate<JT>(sc, (size_t)(L >> 1) + (row0 >> 1) + i, c0, row0 + 2 * i < L) : make_float2(0.f, 0.f);
#pragma unroll
    for (int i = 0; i < 8; ++i) g2[i] = (LV >= 2) ? coeff_gate<JT>(sc, (size_t)(L >> 2) + (row0 >> 2) + i, c0, row0 + 4 * i < L) : make_float2(0.f, 0.f);
#pragma unroll
    for (int i = 0; i < 4; ++i) g3[i] = (LV >= 3) ? coeff_gate<JT>(sc, (size_t)(L >> 3) + (row0 >> 3) + i, c0, row0 + 8 * i < L) : make_float2(0.f, 0.f);
#pragma unroll
    for (int i = 0; i < 2; ++i) g4[i] = (LV >= 4) ? coeff_gate<JT>(sc, (size_t)(L >> 4) + (row0 >> 4) + i, c0, row0 + 16 * i < L) : make_float2(0.f, 0.f);
    if (LV >= 5) g5 = coeff_gate<JT>(sc, (size_t)(L >> 5) + (row0 >> 5), c0, row0 < L);
    if constexpr (JT <= 5) {
#pragma unroll
        for (int i = 0; i < (32 >> LV); ++i) ga[i] = coeff_gate<JT>(sc, (size_t)(row0 >> LV) + i, c0, row0 + (i << LV) < L);
    } else {
        ga[0] = make_float2(0.f, 0.f);
    }
    float2 g6 = make_float2(0.f, 0.f), g7 = g6, g8 = g6, gup = g6;
    if constexpr (JT == 6) {
        const int t0 = tile * kWrmTileRows;
        if (J >= 6) g6 = coeff_gate<JT>(sc, (size_t)(L >> 6) + (row0 >> 6), c0, ((row0 >> 6) << 6) < L);
        if (J >= 7) g7 = coeff_gate<JT>(sc, (size_t)(L >> 7) + (row0 >> 7), c0, ((row0 >> 7) << 7) < L);
        if (J >= 8) g8 = coeff_gate<JT>(sc, (size_t)(L >> 8) + (t0 >> 8), c0, t0 < L);
        if (J <= 8) gup = coeff_gate<JT>(sc, (size_t)(row0 >> J), c0, ((row0 >> J) << J) < L);   // approximation, levels 6..8
    }

    float2 x[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) x[i] = IO::unpack(raw[i]);
    // block sums and gated details of levels 1..5; d_l[i] is what the first half of block i gains and the second loses
    float2 s1[16], s2[8], s3[4], s4[2], s5, d1[16], d2[8], d3[4], d4[2], d5;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        s1[i] = x[2 * i] + x[2 * i + 1];
        d1[i] = make_float2((x[2 * i].x - x[2 * i + 1].x) * 0.5f * g1[i].x, (x[2 * i].y - x[2 * i + 1].y) * 0.5f * g1[i].y);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        s2[i] = s1[2 * i] + s1[2 * i + 1];
        d2[i] = make_float2((s1[2 * i].x - s1[2 * i + 1].x) * 0.25f * g2[i].x, (s1[2 * i].y - s1[2 * i + 1].y) * 0.25f * g2[i].y);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        s3[i] = s2[2 * i] + s2[2 * i + 1];
        d3[i] = make_float2((s2[2 * i].x - s2[2 * i + 1].x) * 0.125f * g3[i].x, (s2[2 * i].y - s2[2 * i + 1].y) * 0.125f * g3[i].y);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        s4[i] = s3[2 * i] + s3[2 * i + 1];
        d4[i] = make_float2((s3[2 * i].x - s3[2 * i + 1].x) * 0.0625f * g4[i].x, (s3[2 * i].y - s3[2 * i + 1].y) * 0.0625f * g4[i].y);
    }
    s5 = s4[0] + s4[1];
    d5 = make_float2((s4[0].x - s4[1].x) * 0.03125f * g5.x, (s4[0].y - s4[1].y) * 0.03125f * g5.y);

    float2 corr = make_float2(0.f, 0.f);               // what every row of the lane's 32 gains from levels >= 6
    if constexpr (JT == 6) {
        part[r][p] = s5;
        __syncthreads();
        if (J > kWrmTileLevels) corr = U[((size_t)bh * ntiles + tile) * 32 + p];
        float2 q[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) q[i] = part[i][p];
        const int r4 = r & ~3, r2 = r & ~1;
        float2 h7a = make_float2(0.f, 0.f), h7b = h7a, h6a = h7a, h6b = h7a;   // halves of the lane's level-7 / level-6 block
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if ((i & ~3) == r4) { if (i & 2) h7b = h7b + q[i]; else h7a = h7a + q[i]; }
            if ((i & ~1) == r2) { if (i & 1) h6b = h6b + q[i]; else h6a = h6a + q[i]; }
        }
        const float2 h8a = (q[0] + q[1]) + (q[2] + q[3]), h8b = (q[4] + q[5]) + (q[6] + q[7]);
        if (J >= 8) {
            const float sg = (r & 4) ? -0.00390625f : 0.00390625f;
            corr.x = fmaf((h8a.x - h8b.x) * sg, g8.x, corr.x);
            corr.y = fmaf((h8a.y - h8b.y) * sg, g8.y, corr.y);
        }
        if (J >= 7) {
            const float sg = (r & 2) ? -0.0078125f : 0.0078125f;
            corr.x = fmaf((h7a.x - h7b.x) * sg, g7.x, corr.x);
            corr.y = fmaf((h7a.y - h7b.y) * sg, g7.y, corr.y);
        }
        if (J >= 6) {
            const float sg = (r & 1) ? -0.015625f : 0.015625f;
            corr.x = fmaf((h6a.x - h6b.x) * sg, g6.x, corr.x);
            corr.y = fmaf((h6a.y - h6b.y) * sg, g6.y, corr.y);
        }
        if (J <= 8) {                                  // the approximation band ends inside the tile
            const float2 blk = (J == 8) ? h8a + h8b : (J == 7) ? h7a + h7b : h6a + h6b;
            const float sc2 = exp2f(-(float)J);
            corr.x = fmaf(blk.x * sc2, gup.x, corr.x);
            corr.y = fmaf(blk.y * sc2, gup.y, corr.y);
        }
    }
    // down the lane's own levels: a block's correction is its parent's, plus or minus the parent's gated detail,
    // plus (at level JT <= 5) its own gated approximation
    auto approx = [&](int level, int i, float2 sum) {  // level == JT <= 5: gated approximation of block i at that level
        const float sc2 = 1.0f / (float)(1 << (level < 0 ? 0 : level));
        return make_float2(sum.x * sc2 * ga[i].x, sum.y * sc2 * ga[i].y);
    };
    float2 c5 = corr;
    if constexpr (JT == 5) c5 = c5 + approx(5, 0, s5);
#pragma unroll
    for (int i4 = 0; i4 < 2; ++i4) {
        float2 c4 = (i4 == 0) ? c5 + d5 : c5 - d5;
        if constexpr (JT == 4) c4 = c4 + approx(4, i4, s4[i4]);
#pragma unroll
        for (int j3 = 0; j3 < 2; ++j3) {
            const int i3 = 2 * i4 + j3;
            float2 c3 = (j3 == 0) ? c4 + d4[i4] : c4 - d4[i4];
            if constexpr (JT == 3) c3 = c3 + approx(3, i3, s3[i3]);
#pragma unroll
            for (int j2 = 0; j2 < 2; ++j2) {
                const int i2 = 2 * i3 + j2;
                float2 c2 = (j2 == 0) ? c3 + d3[i3] : c3 - d3[i3];
                if constexpr (JT == 2) c2 = c2 + approx(2, i2, s2[i2]);
#pragma unroll
                for (int j1 = 0; j1 < 2; ++j1) {
                    const int i1 = 2 * i2 + j1;
                    float2 c1 = (j1 == 0) ? c2 + d2[i2] : c2 - d2[i2];
                    if constexpr (JT == 1) c1 = c1 + approx(1, i1, s1[i1]);
#pragma unroll
                    for (int j0 = 0; j0 < 2; ++j0) {
                        const int i = 2 * i1 + j0, l = row0 + i;
                        float2 c0v = (j0 == 0) ? c1 + d1[i1] : c1 - d1[i1];
                        if constexpr (JT == 0) c0v = c0v + approx(0, i, x[i]);
                        if (l < L) IO::store_stream(out + (((size_t)b * L + l) * H + h) * 32 + p, IO::pack(x[i] + c0v));
                    }
                }
            }
        }
    }
}

// Levels above 8 with per-coefficient gates: one workgroup per (bh, group of kUpCh channels) sums the tiles' sums
// pairwise up to level J in LDS, then walks down: the top blocks start from their gated approximation, a block's two
// children get its correction plus / minus its gated detail.  U[bh][tile][c] = what every row of the tile gains.
__global__ __launch_bounds__(256) void k_wrm_upper_coeff(const float *__restrict__ S, const float *__restrict__ s,
                                                         float *__restrict__ U, int ntiles, int J, int L) {
    extern __shared__ float pyr[];                     // levels 8, 9, ..., J back to back, kUpCh channels each
    const int tid = threadIdx.x, cl = tid % kUpCh, lane = tid / kUpCh;
    const int bh = blockIdx.x, c = blockIdx.y * kUpCh + cl;
    const float *sc = s + (size_t)bh * L * 64 + c;
    for (int i = lane; i < ntiles; i += kUpLanes) pyr[i * kUpCh + cl] = S[((size_t)bh * ntiles + i) * 64 + c];
    __syncthreads();
    int off = 0, n = ntiles;
    for (int l = kWrmTileLevels + 1; l <= J; ++l) {    // up: block sums
        const int noff = off + n, nn = n >> 1;
        for (int i = lane; i < nn; i += kUpLanes)
            pyr[(noff + i) * kUpCh + cl] = pyr[(off + 2 * i) * kUpCh + cl] + pyr[(off + 2 * i + 1) * kUpCh + cl];
        __syncthreads();
        off = noff;
        n = nn;
    }
    for (int i = lane; i < n; i += kUpLanes)            // top: gated approximation, positions 0 .. L/2^J - 1
        pyr[(off + i) * kUpCh + cl] *= sc[(size_t)i * 64] * exp2f(-(float)J);
    __syncthreads();
    for (int l = J; l > kWrmTileLevels; --l) {         // down: children of the level-l blocks
        const int coff = off - 2 * n;
        const float sc2 = exp2f(-(float)l);
        for (int i = lane; i < n; i += kUpLanes) {
            const float par = pyr[(off + i) * kUpCh + cl];
            const float a = pyr[(coff + 2 * i) * kUpCh + cl], bq = pyr[(coff + 2 * i + 1) * kUpCh + cl];
            const float det = (a - bq) * sc2 * sc[((size_t)(L >> l) + i) * 64];
            pyr[(coff + 2 * i) * kUpCh + cl] = par + det;
            pyr[(coff + 2 * i + 1) * kUpCh + cl] = par - det;
        }
        __syncthreads();
        off = coff;
        n <<= 1;
    }
    for (int i = lane; i < ntiles; i += kUpLanes) U[((size_t)bh * ntiles + i) * 64 + c] = pyr[i * kUpCh + cl];
}

// ------------------------------------------------------------------------------------------
hipError_t launch_wrm_gates(const double *sum_q, double inv_count, const WrmDev &P, int B, int H, float *s,
                            hipStream_t st) {
    const int nout = (P.levels + 1) * P.d;
    k_wrm_gates<<<dim3(B * H, (nout + 255) / 256), 256, 0, st>>>(sum_q, inv_count, P.ln_gamma, P.ln_beta, P.ln_eps, P.W1,
                                                                P.b1, P.W2, P.b2, s, H, P.Hg, P.d, P.d_w, nout);
    return hipGetLastError();
}

size_t wrm_scratch_floats(int BH, int L, int levels) {
    if (levels <= kWrmTileLevels) return 0;
    return (size_t)BH * (size_t)(L / kWrmTileRows) * 64;
}

// tile sums S (one pass over v) for the levels above 8; 2^levels divides L there, so L is a multiple of 512
static hipError_t tile_sums_pass(int io, const void *v, float *tile_sums, int B, int L, int H, int ntiles, hipStream_t st) {
    const dim3 grid(H, ntiles, B);
    if ((reinterpret_cast<uintptr_t>(v) & 15) == 0) {
        const int ppv = H * 32 / (io ? 4 : 2);
        const dim3 g16((ppv + 255) / 256, ntiles, B);
        if (io) k_wrm_tile_sums_x16<true><<<g16, 256, 0, st>>>(static_cast<const uint4 *>(v), tile_sums, L, H, ntiles, ppv);
        else k_wrm_tile_sums_x16<false><<<g16, 256, 0, st>>>(static_cast<const uint4 *>(v), tile_sums, L, H, ntiles, ppv);
    } else if (io) k_wrm_tile_sums<IoBf16><<<grid, 256, 0, st>>>(static_cast<const uint32_t *>(v),
                                                          reinterpret_cast<float2 *>(tile_sums), L, H, ntiles);
    else k_wrm_tile_sums<IoF32><<<grid, 256, 0, st>>>(static_cast<const float2 *>(v),
                                                      reinterpret_cast<float2 *>(tile_sums), L, H, ntiles);
    return hipGetLastError();
}

hipError_t launch_wrm_apply(int io, const void *v, const float *s, void *out, float *tile_sums, float *upper,
                            int B, int L, int H, int levels, hipStream_t st, const float *bsum, int block_rows) {
    const int BH = B * H;
    const int ntiles = (L + kWrmTileRows - 1) / kWrmTileRows;
    const dim3 grid(H, ntiles, B);
    if (levels > kWrmTileLevels) {
        hipError_t e;
        if (bsum) {                                    // the producer of v already summed its rows in small blocks
            if (block_rows < 1 || kWrmTileRows % block_rows != 0) return hipErrorInvalidValue;
            const size_t total = (size_t)BH * ntiles * 64;
            k_wrm_tile_sums_from_blocks<<<(unsigned)((total + 255) / 256), 256, 0, st>>>(bsum, tile_sums,
                                                                                         kWrmTileRows / block_rows, total);
            e = hipGetLastError();
        } else {
            e = tile_sums_pass(io, v, tile_sums, B, L, H, ntiles, st);
        }
        if (e != hipSuccess) return e;
        const size_t lds = (size_t)2 * ntiles * kUpCh * sizeof(float);
        if (lds > 48 * 1024) {
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_wrm_upper),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        k_wrm_upper<<<dim3(BH, 64 / kUpCh), 256, lds, st>>>(tile_sums, s, upper, ntiles, levels);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (io) k_wrm_apply<IoBf16><<<grid, 256, 0, st>>>(static_cast<const uint32_t *>(v), s,
                                                      reinterpret_cast<const float2 *>(upper),
                                                      static_cast<uint32_t *>(out), L, H, levels, ntiles);
    else k_wrm_apply<IoF32><<<grid, 256, 0, st>>>(static_cast<const float2 *>(v), s,
                                                  reinterpret_cast<const float2 *>(upper),
                                                  static_cast<float2 *>(out), L, H, levels, ntiles);
    return hipGetLastError();
}

template <typename IO, int JT>
static hipError_t wrm_coeff_t(const void *v, const float *s, const float *upper, void *out, int B, int L, int H, int levels,
                              int ntiles, hipStream_t st) {
    k_wrm_coeff<IO, JT><<<dim3(H, ntiles, B), 256, 0, st>>>(static_cast<const typename IO::pair_t *>(v), s,
                                                           reinterpret_cast<const float2 *>(upper),
                                                           static_cast<typename IO::pair_t *>(out), L, H, levels, ntiles);
    return hipGetLastError();
}

hipError_t launch_wrm_apply_coeff(int io, const void *v, const float *s, void *out, float *tile_sums, float *upper,
                                  int B, int L, int H, int levels, hipStream_t st) {
    const int BH = B * H;
    const int ntiles = (L + kWrmTileRows - 1) / kWrmTileRows;
    if (levels > kWrmTileLevels) {
        hipError_t e = tile_sums_pass(io, v, tile_sums, B, L, H, ntiles, st);
        if (e != hipSuccess) return e;
        const size_t lds = (size_t)2 * ntiles * kUpCh * sizeof(float);
        if (lds > 48 * 1024) {
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_wrm_upper_coeff),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        k_wrm_upper_coeff<<<dim3(BH, 64 / kUpCh), 256, lds, st>>>(tile_sums, s, upper, ntiles, levels, L);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
#define SPECTRE_WRM_JT(JTV) \
    case JTV: return io ? wrm_coeff_t<IoBf16, JTV>(v, s, upper, out, B, L, H, levels, ntiles, st) \
                        : wrm_coeff_t<IoF32, JTV>(v, s, upper, out, B, L, H, levels, ntiles, st);
    switch (levels < 6 ? levels : 6) {
        SPECTRE_WRM_JT(0) SPECTRE_WRM_JT(1) SPECTRE_WRM_JT(2) SPECTRE_WRM_JT(3) SPECTRE_WRM_JT(4) SPECTRE_WRM_JT(5)
        SPECTRE_WRM_JT(6)
        default: return hipErrorInvalidValue;
    }
#undef SPECTRE_WRM_JT
}

// Loads this translation unit's code object (the runtime loads them on first use): called by spectre_prepare so
// that no compute call is the first to touch it.
hipError_t load_kernels_wrm() {
    hipFuncAttributes a;
    return hipFuncGetAttributes(&a, reinterpret_cast<const void *>(k_wrm_upper));
}

}  // namespace spectre
