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
    for (int o = tid; o < nout; o += 256) {
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
hipError_t launch_wrm_gates(const double *sum_q, double inv_count, const WrmDev &P, int B, int H, float *s,
                            hipStream_t st) {
    k_wrm_gates<<<B * H, 256, 0, st>>>(sum_q, inv_count, P.ln_gamma, P.ln_beta, P.ln_eps, P.W1, P.b1, P.W2, P.b2, s,
                                       H, P.Hg, P.d, P.d_w, (P.levels + 1) * P.d);
    return hipGetLastError();
}

size_t wrm_scratch_floats(int BH, int L, int levels) {
    if (levels <= kWrmTileLevels) return 0;
    return (size_t)BH * (size_t)(L / kWrmTileRows) * 64;
}

hipError_t launch_wrm_apply(int io, const void *v, const float *s, void *out, float *tile_sums, float *upper,
                            int B, int L, int H, int levels, hipStream_t st) {
    const int BH = B * H;
    const int ntiles = (L + kWrmTileRows - 1) / kWrmTileRows;
    const dim3 grid(H, ntiles, B);
    if (levels > kWrmTileLevels) {                      // then 2^levels divides L, so L is a multiple of 512
        if ((reinterpret_cast<uintptr_t>(v) & 15) == 0) {
            const int ppv = H * 32 / (io ? 4 : 2);
            const dim3 g16((ppv + 255) / 256, ntiles, B);
            if (io) k_wrm_tile_sums_x16<true><<<g16, 256, 0, st>>>(static_cast<const uint4 *>(v), tile_sums, L, H, ntiles, ppv);
            else k_wrm_tile_sums_x16<false><<<g16, 256, 0, st>>>(static_cast<const uint4 *>(v), tile_sums, L, H, ntiles, ppv);
        } else if (io) k_wrm_tile_sums<IoBf16><<<grid, 256, 0, st>>>(static_cast<const uint32_t *>(v),
                                                              reinterpret_cast<float2 *>(tile_sums), L, H, ntiles);
        else k_wrm_tile_sums<IoF32><<<grid, 256, 0, st>>>(static_cast<const float2 *>(v),
                                                          reinterpret_cast<float2 *>(tile_sums), L, H, ntiles);
        hipError_t e = hipGetLastError();
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

// Loads this translation unit's code object (the runtime loads them on first use): called by spectre_prepare so
// that no compute call is the first to touch it.
hipError_t load_kernels_wrm() {
    hipFuncAttributes a;
    return hipFuncGetAttributes(&a, reinterpret_cast<const void *>(k_wrm_upper));
}

}  // namespace spectre
