// Prefix-FFT cache kernels (Sec. 3.3, Eq. 5, Algorithm 1) for gfx950.
//
// Cache layout: prefix_fft [B*H][F][d] complex64 (a bin's d channels are one contiguous
// 8*d-byte row), ring buffers [B*H][N][d] fp32, sum_q [B*H][d] fp64, twiddle [N] complex64.
// The decode sweep is a pure stream over prefix_fft: each entry is read once, updated by the
// rank-one term of Eq. (5), written once, and (fused) contributes to the newest row's readout.
#include "prefix.h"

#include "common.h"
#include "mix_pow2.h"

namespace spectre {

// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_fill_zero(uint4 *__restrict__ p, size_t n16) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
}

// twiddle[m] = exp(-j 2 pi m / N), evaluated in fp64 and rounded once.
__global__ __launch_bounds__(256) void k_fill_twiddle(float2 *__restrict__ tw, int N) {
    const int m = blockIdx.x * 256 + threadIdx.x;
    if (m >= N) return;
    double s, c;
    sincospi(2.0 * (double)m / (double)N, &s, &c);
    tw[m] = make_float2((float)c, (float)(-s));
}

// ------------------------------------------------------------------------------------------
// ring update for one token (Algorithm 1, DecodeStep: slot, eviction, buffers, running sum).
// One lane per (b, h, c).  v_t, q_t are the rows [B, T, H, d] at position `ti`.
template <typename T>
__device__ __forceinline__ float load_scalar(const T *p, size_t i);
template <>
__device__ __forceinline__ float load_scalar<float>(const float *p, size_t i) { return p[i]; }
template <>
__device__ __forceinline__ float load_scalar<uint16_t>(const uint16_t *p, size_t i) {
    return __uint_as_float((uint32_t)p[i] << 16);
}

template <typename T>
__global__ __launch_bounds__(256) void k_ring_update(const T *__restrict__ v_new, const T *__restrict__ q_new,
                                                     int Tn, int ti, float *__restrict__ v_buf,
                                                     float *__restrict__ q_buf, double *__restrict__ sum_q,
                                                     float *__restrict__ delta, int H, int d, int N, int slot,
                                                     int evict, int total) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int c = idx % d, bh = idx / d, h = bh % H, b = bh / H;
    const size_t src = (((size_t)b * Tn + ti) * H + h) * d + c;
    const size_t ring = ((size_t)bh * N + slot) * d + c;
    const float vn = load_scalar<T>(v_new, src), qn = load_scalar<T>(q_new, src);
    const float vo = evict ? v_buf[ring] : 0.0f, qo = evict ? q_buf[ring] : 0.0f;
    delta[idx] = vn - vo;
    sum_q[idx] += (double)qn - (double)qo;
    v_buf[ring] = vn;
    q_buf[ring] = qn;
}

// ------------------------------------------------------------------------------------------
// sweep over the cache.  grid (ceil(F/KCH), B*H); 256 lanes = 8 bins x 32 lanes, a lane owns
// two adjacent channels (one 16-byte access).  UPDATE: X[k,:] += delta * w_k with
// w_k = twiddle[(k*slot) mod N] (Eq. 5).  READ: partial[bh][chunk][c] = sum over the chunk's
// bins of Re(r_k X[k,c]) with r_k = (c_k/N) g_k conj(w_k), c_k = 1 at DC and Nyquist, else 2
// (the newest row of Cor. B.2's inverse; exp(+j 2 pi k slot/N) = conj(w_k)).
constexpr int kSweepBins = 128;

// (a b) mod N for a, b < N <= 2^17 without 64-bit division.
__device__ __forceinline__ unsigned mul_mod(unsigned a, unsigned b, int N) {
    if ((N & (N - 1)) == 0) return (a * b) & (unsigned)(N - 1);
    return (((a * (b >> 9)) % (unsigned)N) * 512u + a * (b & 511u)) % (unsigned)N;
}

// The per-bin factors w_k and r_k of a chunk are prepared once by its first 128 lanes and kept in LDS; the rows
// then cost one cache access each, four of them in flight per lane.
template <bool UPDATE, bool READ>
__global__ __launch_bounds__(256) void k_sweep(float4 *__restrict__ X, const float *__restrict__ delta,
                                               const float2 *__restrict__ tw, const float2 *__restrict__ g,
                                               float *__restrict__ partial, int F, int N, int slot,
                                               int nchunks) {
    __shared__ float2 red[8][32];
    __shared__ float2 s_w[kSweepBins], s_r[kSweepBins];
    const int lane = threadIdx.x & 31, row = threadIdx.x >> 5;
    const int chunk = blockIdx.x, bh = blockIdx.y;
    const int k0 = chunk * kSweepBins, k1 = min(F, k0 + kSweepBins);
    if (threadIdx.x < kSweepBins) {
        const int k = min(k0 + (int)threadIdx.x, k1 - 1);
        const float2 w = tw[mul_mod((unsigned)k, (unsigned)slot, N)];
        s_w[threadIdx.x] = w;
        if (READ) {
            const float invN = 1.0f / (float)N;
            const float ck = (k == 0 || 2 * k == N) ? invN : 2.0f * invN;
            const float2 r = cmulc(g[(size_t)bh * F + k], w);   // g_k conj(w_k)
            s_r[threadIdx.x] = make_float2(r.x * ck, r.y * ck);
        }
    }
    float2 dl = make_float2(0.f, 0.f);
    if (UPDATE) dl = *reinterpret_cast<const float2 *>(delta + (size_t)bh * 64 + 2 * lane);
    float acc0 = 0.f, acc1 = 0.f;
    float4 *Xp = X + ((size_t)bh * F) * 32 + lane;
    __syncthreads();
    constexpr int kU = 4;
    for (int kk = k0 + row; kk < k1; kk += 8 * kU) {
        float4 x[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) x[u] = stream_load(Xp + (size_t)min(kk + 8 * u, k1 - 1) * 32);
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int k = kk + 8 * u;
            if (k < k1) {
                if (UPDATE) {
                    const float2 w = s_w[k - k0];
                    x[u].x = fmaf(dl.x, w.x, x[u].x);
                    x[u].y = fmaf(dl.x, w.y, x[u].y);
                    x[u].z = fmaf(dl.y, w.x, x[u].z);
                    x[u].w = fmaf(dl.y, w.y, x[u].w);
                    stream_store(Xp + (size_t)k * 32, x[u]);
                }
                if (READ) {
                    const float2 r = s_r[k - k0];
                    acc0 = fmaf(r.x, x[u].x, fmaf(-r.y, x[u].y, acc0));
                    acc1 = fmaf(r.x, x[u].z, fmaf(-r.y, x[u].w, acc1));
                }
            }
        }
    }
    if (READ) {
        red[row][lane] = make_float2(acc0, acc1);
        __syncthreads();
        if (row == 0) {
            float2 s = red[0][lane];
#pragma unroll
            for (int r = 1; r < 8; ++r) {
                s.x += red[r][lane].x;
                s.y += red[r][lane].y;
            }
            *reinterpret_cast<float2 *>(partial + ((size_t)bh * nchunks + chunk) * 64 + 2 * lane) = s;
        }
    }
}

// ------------------------------------------------------------------------------------------
// Deferred updates.  Eq. (5) is linear, so the rank-one updates of the last few tokens need not be applied to
// the cache before it is read: with X = X_stale + sum_i Delta_i w^(k s_i) over the pending tokens i, the newest
// row of irfft(g * X) is the same row for X_stale plus sum_i kappa[(s - s_i) mod N] Delta_i, where
// kappa = irfft(g) is the real convolution kernel of the gate (App. B) and s the newest slot.  A decode step
// then only READS the cache; every `cap` steps one sweep applies all pending updates at once.
//
// k_sweep_lazy (the read-only step), grid and lanes as k_sweep: partial as in k_sweep<false, true> from the stale
// cache, and kpart[bh][chunk][i] = the chunk's share of kappa[(slot_new - slot_i) mod N], accumulated by lane i of
// every bin row (each of the 32 lanes of a row takes one pending token).
// k_flush_mfma (the flush): X[k,:] += sum_i Delta_i tw[(k slot_i) mod N], stored; with READ the readout partials
// are taken from the updated entries.
struct PendingSlots {
    int n;
    int slot[kMaxPending];
};

__device__ __forceinline__ void index_walk(unsigned k_start, unsigned mult, int N, unsigned &m, unsigned &step) {
    if ((N & (N - 1)) == 0) {
        step = (8u * mult) & (unsigned)(N - 1);
        m = (k_start * mult) & (unsigned)(N - 1);
    } else {
        step = (unsigned)((8ull * mult) % (unsigned)N);
        m = (unsigned)(((unsigned long long)k_start * mult) % (unsigned)N);
    }
}

__global__ __launch_bounds__(256) void k_sweep_lazy(const float4 *__restrict__ X, const float2 *__restrict__ tw,
                                                    const float2 *__restrict__ g, float *__restrict__ partial,
                                                    float *__restrict__ kpart, int F, int N, int BH, int slot_new,
                                                    PendingSlots ps, int nchunks) {
    __shared__ float2 red[8][32];
    __shared__ float kred[8][32];
    __shared__ float2 s_r[kSweepBins], s_g[kSweepBins];   // per bin: c_k/N g_k conj(w_k), and c_k/N g_k
    const int lane = threadIdx.x & 31, row = threadIdx.x >> 5;
    const int chunk = blockIdx.x, bh = blockIdx.y;
    const int k0 = chunk * kSweepBins, k1 = min(F, k0 + kSweepBins);
    if (threadIdx.x < kSweepBins) {
        const int k = k0 + threadIdx.x;
        float2 r = make_float2(0.f, 0.f), gc = make_float2(0.f, 0.f);   // bins past the end carry no weight
        if (k < k1) {
            const float invN = 1.0f / (float)N;
            const float ck = (k == 0 || 2 * k == N) ? invN : 2.0f * invN;
            const float2 gk = g[(size_t)bh * F + k];
            const float2 t = cmulc(gk, tw[mul_mod((unsigned)k, (unsigned)slot_new, N)]);   // g_k conj(w_k)
            r = make_float2(t.x * ck, t.y * ck);
            gc = make_float2(gk.x * ck, gk.y * ck);
        }
        s_r[threadIdx.x] = r;
        s_g[threadIdx.x] = gc;
    }
    float acc0 = 0.f, acc1 = 0.f, kacc = 0.f;
    const float4 *Xp = X + ((size_t)bh * F) * 32 + lane;
    // lane i of every bin row follows pending token i: e_k = exp(-j 2 pi k j_i / N), j_i = (slot_new - slot_i)
    // mod N, read from the table at the lane's first bin and advanced by a fixed rotation per step of 8 bins
    // (at most 15 products per chunk: their rounding stays below 1e-6 of a term that is itself a small part of
    // the output)
    const bool has = lane < ps.n;
    const unsigned mult = has ? (unsigned)((slot_new - ps.slot[lane] + N) % N) : 0u;
    unsigned m_item, step_item;
    index_walk((unsigned)(k0 + row), mult, N, m_item, step_item);
    const float2 rot = tw[step_item];
    float2 e = tw[m_item];
    __syncthreads();
    constexpr int kU = 8;
    // kU bin rows per trip, every load of the trip requested up front (addresses clamped into the chunk,
    // rows past its end weighted with zero)
    for (int kk = k0 + row; kk < k1; kk += 8 * kU) {
        float4 x[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) x[u] = stream_load(Xp + (size_t)min(kk + 8 * u, k1 - 1) * 32);
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int kl = min(kk + 8 * u - k0, kSweepBins - 1);
            const bool live = kk + 8 * u < k1;
            const float2 r = live ? s_r[kl] : make_float2(0.f, 0.f);
            const float2 gc = live ? s_g[kl] : make_float2(0.f, 0.f);
            acc0 = fmaf(r.x, x[u].x, fmaf(-r.y, x[u].y, acc0));
            acc1 = fmaf(r.x, x[u].z, fmaf(-r.y, x[u].w, acc1));
            kacc = fmaf(gc.x, e.x, fmaf(gc.y, e.y, kacc));   // c_k/N Re(g_k conj(e_k))
            e = cmul(e, rot);
        }
    }
    if (!has) kacc = 0.f;
    red[row][lane] = make_float2(acc0, acc1);
    kred[row][lane] = kacc;
    __syncthreads();
    if (row == 0) {
        float2 s = red[0][lane];
        float ks = kred[0][lane];
#pragma unroll
        for (int r = 1; r < 8; ++r) {
            s.x += red[r][lane].x;
            s.y += red[r][lane].y;
            ks += kred[r][lane];
        }
        *reinterpret_cast<float2 *>(partial + ((size_t)bh * nchunks + chunk) * 64 + 2 * lane) = s;
        kpart[((size_t)bh * nchunks + chunk) * 32 + lane] = ks;
    }
}

// The flush as a matrix product on the matrix cores.  For one head, X[k, c] += sum_i w_i(k) Delta_i[c] is a
// (bins x pending) by (pending x channels) product, once with Re w and once with Im w.  A wave owns a block of
// 32 bins x 64 channels: four 32x32 accumulators (real and imaginary part for the even and for the odd
// channels, so that a lane's four values of one bin are the 16 contiguous bytes of the cache entry), loaded
// from the cache, advanced by CAP/2 v_mfma_f32_32x32x2f32 each (two pending tokens per instruction) and
// stored back.  Operand layout of that instruction: A[i][k] in lane 32k + i, B[k][j] in lane 32k + j,
// D[8(v/4) + 4(lane/32) + v%4][lane%32] in register v.
// A workgroup takes kFlushChunks chunks of kSweepBins = 4 x 32 bins, one block per wave and chunk; partial as
// in k_sweep.
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kFlushChunks = 8;   // chunks of kSweepBins bins per workgroup

template <bool READ, int CAP>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void k_flush_mfma(
    float4 *__restrict__ X, const float *__restrict__ pending, const float2 *__restrict__ tw,
    const float2 *__restrict__ g, float *__restrict__ partial, int F, int N, int BH, int slot_new, PendingSlots ps,
    int nchunks) {
    static_assert(kSweepBins == 128, "one 32-bin block per wave and chunk");
    __shared__ float2 red[kFlushChunks][4][32];
    const int l = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = l & 31, half = l >> 5;
    const int bh = blockIdx.y;
    const int chunk_end = min(nchunks, ((int)blockIdx.x + 1) * kFlushChunks);

    // operands that do not depend on the block, kept in LDS: the delta of token i at channels 2c and 2c + 1, and
    // the factor's advance over a block's rows, tw[(c slot_i) mod N]; the block's own factor tw[(kb slot_i) mod N]
    // is one address per half wave, so a block costs no scattered table reads
    __shared__ float2 s_dl[CAP][32], s_adv[CAP][32];
    __shared__ int s_slot[CAP];
    if (threadIdx.x < CAP) s_slot[threadIdx.x] = ps.slot[threadIdx.x];
#pragma unroll
    for (int j = 0; j < CAP / 8; ++j) {
        const int i = 8 * j + (threadIdx.x >> 5), c = threadIdx.x & 31;
        float2 dl = make_float2(0.f, 0.f);
        if (i < ps.n) dl = *reinterpret_cast<const float2 *>(pending + ((size_t)i * BH + bh) * 64 + 2 * c);
        s_dl[i][c] = dl;
        s_adv[i][c] = tw[mul_mod((unsigned)c, (unsigned)ps.slot[i], N)];
    }
    __syncthreads();
    // software pipeline: the cache entries and the factors of the next block are requested before the matrix
    // products of the current one start
    // register v of a block <-> bin row 8(v/4) + 4 half + v%4
    float4 xs[16];
    float2 wbl;
    auto request = [&](int chunk) {
        const int kb = chunk * kSweepBins + 32 * wave;
        const int k1 = min(F, chunk * kSweepBins + kSweepBins);
        const float4 *Xp = X + ((size_t)bh * F + kb) * 32 + col;
        // lane i < CAP fetches token i's factor at the block's first bin
        wbl = tw[mul_mod((unsigned)kb, (unsigned)s_slot[l & (CAP - 1)], N)];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = 8 * (v / 4) + 4 * half + (v % 4);
            xs[v] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (kb + r < k1) xs[v] = stream_load(Xp + (size_t)r * 32);
        }
    };
    request(blockIdx.x * kFlushChunks);
    for (int chunk = blockIdx.x * kFlushChunks; chunk < chunk_end; ++chunk) {
        const int kb = chunk * kSweepBins + 32 * wave;
        const int k1 = min(F, chunk * kSweepBins + kSweepBins);
        float4 *Xp = X + ((size_t)bh * F + kb) * 32 + col;
        floatx16 re0, im0, re1, im1;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            re0[v] = xs[v].x;
            im0[v] = xs[v].y;
            re1[v] = xs[v].z;
            im1[v] = xs[v].w;
        }
        const float2 wcur = wbl;
        if (chunk + 1 < chunk_end) request(chunk + 1);
#pragma unroll 2
        for (int s = 0; s < CAP / 2; ++s) {
            // token 2s + half: A = its factor at bin kb + col, B = its delta
            const float2 wb = make_float2(__shfl(wcur.x, 2 * s + half), __shfl(wcur.y, 2 * s + half));
            const float2 adv = s_adv[2 * s + half][col], dl = s_dl[2 * s + half][col];
            const float ar = wb.x * adv.x - wb.y * adv.y, ai = wb.x * adv.y + wb.y * adv.x;
            re0 = __builtin_amdgcn_mfma_f32_32x32x2f32(ar, dl.x, re0, 0, 0, 0);
            im0 = __builtin_amdgcn_mfma_f32_32x32x2f32(ai, dl.x, im0, 0, 0, 0);
            re1 = __builtin_amdgcn_mfma_f32_32x32x2f32(ar, dl.y, re1, 0, 0, 0);
            im1 = __builtin_amdgcn_mfma_f32_32x32x2f32(ai, dl.y, im1, 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = 8 * (v / 4) + 4 * half + (v % 4);
            if (kb + r < k1) stream_store(Xp + (size_t)r * 32, make_float4(re0[v], im0[v], re1[v], im1[v]));
        }
        if (READ) {
            // lane col prepares the readout factor of bin kb + col; the rows a lane holds fetch theirs by shuffle
            const int k = kb + col;
            float rr = 0.f, ri = 0.f;
            if (k < k1) {
                const float invN = 1.0f / (float)N;
                const float ck = (k == 0 || 2 * k == N) ? invN : 2.0f * invN;
                const float2 r = cmulc(g[(size_t)bh * F + k], tw[mul_mod((unsigned)k, (unsigned)slot_new, N)]);
                rr = r.x * ck;
                ri = r.y * ck;
            }
            float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = 8 * (v / 4) + 4 * half + (v % 4);
                const float a = __shfl(rr, r), b = __shfl(ri, r);
                acc0 = fmaf(a, re0[v], fmaf(-b, im0[v], acc0));
                acc1 = fmaf(a, re1[v], fmaf(-b, im1[v], acc1));
            }
            acc0 += __shfl_xor(acc0, 32);
            acc1 += __shfl_xor(acc1, 32);
            if (half == 0) red[chunk - blockIdx.x * kFlushChunks][wave][col] = make_float2(acc0, acc1);
        }
    }
    if (READ) {
        // the four waves' sums of every chunk, added in a fixed order
        __syncthreads();
        const int c = threadIdx.x >> 5, chunk = blockIdx.x * kFlushChunks + c;
        static_assert(kFlushChunks == 8, "one chunk per 32 threads");
        if (chunk < chunk_end) {
            float2 t = red[c][0][col];
#pragma unroll
            for (int w = 1; w < 4; ++w) {
                t.x += red[c][w][col].x;
                t.y += red[c][w][col].y;
            }
            *reinterpret_cast<float2 *>(partial + ((size_t)bh * nchunks + chunk) * 64 + 2 * col) = t;
        }
    }
}

// out[b, 0, h, c] = sum over chunks of partial + sum_i kappa_i Delta_i[c], kappa_i = sum over chunks of kpart.
template <typename IO>
__global__ __launch_bounds__(256) void k_readout_final_lazy(const float *__restrict__ partial,
                                                            const float *__restrict__ kpart,
                                                            const float *__restrict__ pending,
                                                            typename IO::pair_t *__restrict__ out, int nchunks,
                                                            int BH, int npend) {
    __shared__ float2 red[8][32];
    __shared__ float kred[8][32];
    const int p = threadIdx.x & 31, grp = threadIdx.x >> 5, bh = blockIdx.x;
    const float2 *src = reinterpret_cast<const float2 *>(partial + (size_t)bh * nchunks * 64) + p;
    const float *ksrc = kpart + (size_t)bh * nchunks * 32 + p;
    float2 s = make_float2(0.f, 0.f);
    float ks = 0.f;
    int c = grp;
    for (; c + 56 < nchunks; c += 64) {          // eight loads of each kind in flight, added in the same order
        float2 v[8];
        float kv[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            v[i] = src[(size_t)(c + 8 * i) * 32];
            kv[i] = ksrc[(size_t)(c + 8 * i) * 32];
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            s.x += v[i].x;
            s.y += v[i].y;
            ks += kv[i];
        }
    }
    for (; c < nchunks; c += 8) {
        const float2 v = src[(size_t)c * 32];
        s.x += v.x;
        s.y += v.y;
        ks += ksrc[(size_t)c * 32];
    }
    red[grp][p] = s;
    kred[grp][p] = ks;
    __syncthreads();
    if (grp == 0) {
        float kap = kred[0][p];
#pragma unroll
        for (int r = 1; r < 8; ++r) kap += kred[r][p];
        kred[0][p] = kap;                     // kappa of pending token p
    }
    __syncthreads();
    if (grp == 0) {
        float2 t = red[0][p];
#pragma unroll
        for (int r = 1; r < 8; ++r) {
            t.x += red[r][p].x;
            t.y += red[r][p].y;
        }
        for (int i0 = 0; i0 < npend; i0 += 8) {     // eight delta rows in flight
            float2 dlt[8];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                dlt[i] = (i0 + i < npend)
                             ? *reinterpret_cast<const float2 *>(pending + ((size_t)(i0 + i) * BH + bh) * 64 + 2 * p)
                             : make_float2(0.f, 0.f);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (i0 + i < npend) {
                    t.x = fmaf(kred[0][i0 + i], dlt[i].x, t.x);
                    t.y = fmaf(kred[0][i0 + i], dlt[i].y, t.y);
                }
            }
        }
        out[(size_t)bh * 32 + p] = IO::pack(t);
    }
}

// out[b, 0, h, c] = sum over chunks of partial.  One workgroup per head: 256 lanes = 32 channel
// pairs x 8 chunk groups; group r adds chunks r, r+8, ... in order, then the 8 sums in order.
template <typename IO>
__global__ __launch_bounds__(256) void k_readout_final(const float *__restrict__ partial,
                                                       typename IO::pair_t *__restrict__ out, int nchunks) {
    __shared__ float2 red[8][32];
    const int p = threadIdx.x & 31, grp = threadIdx.x >> 5, bh = blockIdx.x;
    const float2 *src = reinterpret_cast<const float2 *>(partial + (size_t)bh * nchunks * 64) + p;
    float2 s = make_float2(0.f, 0.f);
    int c = grp;
    for (; c + 56 < nchunks; c += 64) {          // eight loads in flight, added in the same order
        float2 v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = src[(size_t)(c + 8 * i) * 32];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            s.x += v[i].x;
            s.y += v[i].y;
        }
    }
    for (; c < nchunks; c += 8) {
        const float2 v = src[(size_t)c * 32];
        s.x += v.x;
        s.y += v.y;
    }
    red[grp][p] = s;
    __syncthreads();
    if (grp == 0) {
        float2 t = red[0][p];
#pragma unroll
        for (int r = 1; r < 8; ++r) {
            t.x += red[r][p].x;
            t.y += red[r][p].y;
        }
        out[(size_t)bh * 32 + p] = IO::pack(t);
    }
}

// ------------------------------------------------------------------------------------------
// pre-fill helpers.
// Many tokens appended at once - the prompt on an empty cache (whose ring buffers are all zero), or a long append to
// a cache that already holds some (T <= ring capacity W, so every slot is written at most once): token i of the call goes to ring slot (s0 + i) mod W, evicting what was there when t0 + i >= W (Eq. 5's
// ring-buffer bookkeeping for T tokens at once).  grid (ceil(T / 256), B*H); 256 lanes = 32 channel pairs x 8 row
// lanes; partial[b][chunk][h*64 + c] = the chunk's sum of q_new - q_evicted in fp64 (added to sum_q afterwards).
template <typename IO>
__global__ __launch_bounds__(256) void k_ring_append(const typename IO::pair_t *__restrict__ V,
                                                     const typename IO::pair_t *__restrict__ Q,
                                                     float2 *__restrict__ v_buf, float2 *__restrict__ q_buf,
                                                     double *__restrict__ partial, int T, int H, int N, int M0, int W,
                                                     int s0, long long t0, int nchunks) {
    __shared__ double red[8][64];
    const int p = threadIdx.x & 31, rl = threadIdx.x >> 5;
    const int chunk = blockIdx.x, bh = blockIdx.y, h = bh % H, b = bh / H;
    double sx = 0.0, sy = 0.0;
    const int i_end = min(T, chunk * 256 + 256);
    for (int i0 = chunk * 256 + rl; i0 < i_end; i0 += 64) {          // eight rows per trip, their loads up front
        typename IO::pair_t rv[8], rq[8];
        float2 qo[8];
        size_t ring[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = min(i0 + 8 * u, i_end - 1);               // clamped: rows past the end are not stored
            const int slot = (int)(((long long)s0 + i) % W);
            ring[u] = ((size_t)bh * N + M0 + slot) * 32 + p;
            const size_t src = (((size_t)b * T + i) * H + h) * 32 + p;
            rv[u] = V ? V[src] : IO::zero();
            rq[u] = Q[src];
            qo[u] = (t0 + i >= W) ? q_buf[ring[u]] : make_float2(0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (i0 + 8 * u < i_end) {
                const float2 vn = IO::unpack(rv[u]), qn = IO::unpack(rq[u]);
                sx += (double)qn.x - (double)qo[u].x;
                sy += (double)qn.y - (double)qo[u].y;
                if (V) v_buf[ring[u]] = vn;                          // V == nullptr: the value rows are written elsewhere
                q_buf[ring[u]] = qn;
            }
        }
    }
    red[rl][2 * p] = sx;
    red[rl][2 * p + 1] = sy;
    __syncthreads();
    if (threadIdx.x < 64) {
        double t = red[0][threadIdx.x];
#pragma unroll
        for (int r = 1; r < 8; ++r) t += red[r][threadIdx.x];
        partial[((size_t)b * nchunks + chunk) * (H * 64) + h * 64 + threadIdx.x] = t;
    }
}

// Memory rows (Sec. 3.4): v_buf[bh][m][c] = mem[b or 0][h][m][c], m < Nmem.  One lane per element.
__global__ __launch_bounds__(256) void k_set_memory(const float *__restrict__ mem, float *__restrict__ v_buf, int H,
                                                    int N, int Nmem, int d, int per_batch, size_t total) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int c = (int)(idx % d);
    const size_t r = idx / d;
    const int m = (int)(r % Nmem);
    const size_t bh = r / Nmem;
    const size_t src_bh = per_batch ? bh : bh % H;
    v_buf[(bh * N + m) * d + c] = mem[(src_bh * Nmem + m) * d + c];
}

// Scratch <-> cache rows.  A scratch column (head, k2, pair) is handled in lines of 16 adjacent entries (128 bytes):
// entry e = 16 q + c holds bin k1 = big_position(e), and the lines q < N1 / 32 are exactly the bins k = k2 + N2 k1
// below N / 2.  The partner bin N - k lies in column (N2 - k2) mod N2 and, for k2 > 0, its 16 entries are again one
// line (in reverse order), so a workgroup that owns one line of all 32 pairs touches whole 128-byte lines of the
// scratch and, through an LDS tile, whole 512-byte rows (one bin, 32 pairs) of the cache.  The Nyquist bin
// (k2 = 0, k1 = N1 / 2) is its own partner and is done by a few extra workgroups at the end of the grid.
constexpr int kTileStride = 33;                       // float4 entries per bin row of the LDS tile

__device__ __forceinline__ size_t column_base(int bhl, int k2, int p, int N1, int N2) {
    return (((size_t)bhl * N2 + k2) * 32 + p) * N1;
}

// untangle: the complex transform Z of z = v_even + j v_odd separates into the two real
// channels' half spectra, X_even[k] = (Z_k + conj Z_{N-k})/2, X_odd[k] = (Z_k - conj Z_{N-k})/(2j).
__device__ __forceinline__ float4 untangle_pair(float2 zk, float2 zn) {
    float4 o;
    o.x = 0.5f * (zk.x + zn.x);
    o.y = 0.5f * (zk.y - zn.y);
    o.z = 0.5f * (zk.y + zn.y);
    o.w = -0.5f * (zk.x - zn.x);
    return o;
}

__global__ __launch_bounds__(256) void k_untangle(const float2 *__restrict__ scr, float4 *__restrict__ X,
                                                  int N, int N1, int N2, int P, int bh0, int nbh) {
    __shared__ float4 tile[16 * kTileStride];
    const int F = N / 2 + 1, lines = N1 / 32, tid = threadIdx.x;
    const int main_blocks = nbh * N2 * lines;
    if ((int)blockIdx.x >= main_blocks) {              // Nyquist bins: one lane per (head, pair)
        const int idx = ((int)blockIdx.x - main_blocks) * 256 + tid;
        if (idx >= nbh * 32) return;
        const int p = idx & 31, bhl = idx >> 5;
        const float2 z = scr[column_base(bhl, 0, p, N1, N2) + big_position(N1 / 2, P)];
        X[((size_t)(bh0 + bhl) * F + N / 2) * 32 + p] = untangle_pair(z, z);
        return;
    }
    const int q = blockIdx.x % lines, k2 = (blockIdx.x / lines) % N2, bhl = blockIdx.x / (lines * N2);
    {
        const int c = tid & 15, pl = tid >> 4, e = 16 * q + c;
        const SpectrumPair sp = spectrum_pair(N, N2, P, k2, e);
#pragma unroll
        for (int rr = 0; rr < 2; ++rr) {
            const int p = pl + 16 * rr;
            const float2 zk = scr[column_base(bhl, k2, p, N1, N2) + e];
            const float2 zn = scr[column_base(bhl, sp.k2n, p, N1, N2) + sp.en];
            tile[c * kTileStride + p] = untangle_pair(zk, zn);
        }
    }
    __syncthreads();
    const int p = tid & 31, c0 = tid >> 5;
#pragma unroll
    for (int rr = 0; rr < 2; ++rr) {
        const int c = c0 + 8 * rr;
        const int k = k2 + N2 * big_position(16 * q + c, P);
        X[((size_t)(bh0 + bhl) * F + k) * 32 + p] = tile[c * kTileStride + p];
    }
}

// tangle: the inverse of untangle with the gate applied.  Y_c[k] = g_k X_c[k] for k <= N/2
// (real parts only at DC and Nyquist), Hermitian-extended to k > N/2; Z_k = (Y_even + j Y_odd)/N
// goes to the entry the inverse big kernel reads it from.  The lane that holds bin k < N/2 also produces bin N - k.
__global__ __launch_bounds__(256) void k_tangle(const float4 *__restrict__ X, const float2 *__restrict__ g,
                                                float2 *__restrict__ scr, int N, int N1, int N2, int P, int bh0,
                                                int nbh) {
    __shared__ float4 tile[16 * kTileStride];
    const int F = N / 2 + 1, lines = N1 / 32, tid = threadIdx.x;
    const float s = 1.0f / (float)N;
    const int main_blocks = nbh * N2 * lines;
    if ((int)blockIdx.x >= main_blocks) {              // Nyquist bins
        const int idx = ((int)blockIdx.x - main_blocks) * 256 + tid;
        if (idx >= nbh * 32) return;
        const int p = idx & 31, bhl = idx >> 5;
        const size_t bh = (size_t)(bh0 + bhl);
        const float4 x = X[(bh * F + N / 2) * 32 + p];
        const float2 gk = g[bh * F + N / 2];
        const float2 ya = cmul(gk, make_float2(x.x, x.y)), yb = cmul(gk, make_float2(x.z, x.w));
        scr[column_base(bhl, 0, p, N1, N2) + big_position(N1 / 2, P)] = make_float2(ya.x * s, yb.x * s);
        return;
    }
    const int q = blockIdx.x % lines, k2 = (blockIdx.x / lines) % N2, bhl = blockIdx.x / (lines * N2);
    const size_t bh = (size_t)(bh0 + bhl);
    {
        const int p = tid & 31, c0 = tid >> 5;
#pragma unroll
        for (int rr = 0; rr < 2; ++rr) {
            const int c = c0 + 8 * rr;
            const int k = k2 + N2 * big_position(16 * q + c, P);
            const float4 x = X[(bh * F + k) * 32 + p];
            const float2 gk = g[bh * F + k];
            float2 ya = cmul(gk, make_float2(x.x, x.y)), yb = cmul(gk, make_float2(x.z, x.w));
            if (k == 0) {
                ya.y = 0.f;
                yb.y = 0.f;
            }
            // Z_k = Y_even[k] + j Y_odd[k];  Z_{N-k} = conj(Y_even[k]) + j conj(Y_odd[k])
            tile[c * kTileStride + p] = make_float4((ya.x - yb.y) * s, (ya.y + yb.x) * s, (ya.x + yb.y) * s, (yb.x - ya.y) * s);
        }
    }
    __syncthreads();
    const int c = tid & 15, pl = tid >> 4, e = 16 * q + c;
    const SpectrumPair sp = spectrum_pair(N, N2, P, k2, e);
#pragma unroll
    for (int rr = 0; rr < 2; ++rr) {
        const int p = pl + 16 * rr;
        const float4 v = tile[c * kTileStride + p];
        scr[column_base(bhl, k2, p, N1, N2) + e] = make_float2(v.x, v.y);
        if (sp.kn != sp.k) scr[column_base(bhl, sp.k2n, p, N1, N2) + sp.en] = make_float2(v.z, v.w);
    }
}

// ------------------------------------------------------------------------------------------
hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t st) {
    const size_t n16 = bytes / 16;   // callers pass multiples of 16 bytes
    if (n16 == 0) return hipSuccess;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    k_fill_zero<<<(unsigned)blocks, 256, 0, st>>>(static_cast<uint4 *>(p), n16);
    return hipGetLastError();
}

hipError_t launch_fill_twiddle(float2 *tw, int N, hipStream_t st) {
    k_fill_twiddle<<<(N + 255) / 256, 256, 0, st>>>(tw, N);
    return hipGetLastError();
}

hipError_t launch_ring_update(int io, const void *v_new, const void *q_new, int Tn, int ti, float *v_buf,
                              float *q_buf, double *sum_q, float *delta, int B, int H, int d, int N, int slot,
                              int evict, hipStream_t st) {
    const int total = B * H * d;
    const unsigned grid = (unsigned)((total + 255) / 256);
    if (io)
        k_ring_update<uint16_t><<<grid, 256, 0, st>>>(static_cast<const uint16_t *>(v_new),
                                                     static_cast<const uint16_t *>(q_new), Tn, ti, v_buf, q_buf,
                                                     sum_q, delta, H, d, N, slot, evict, total);
    else
        k_ring_update<float><<<grid, 256, 0, st>>>(static_cast<const float *>(v_new),
                                                  static_cast<const float *>(q_new), Tn, ti, v_buf, q_buf, sum_q,
                                                  delta, H, d, N, slot, evict, total);
    return hipGetLastError();
}

int sweep_chunks(int F) { return (F + kSweepBins - 1) / kSweepBins; }

hipError_t launch_sweep(bool update, bool read, float2 *X, const float *delta, const float2 *tw, const float2 *g,
                        float *partial, int BH, int F, int N, int slot, hipStream_t st) {
    const int nch = sweep_chunks(F);
    dim3 grid(nch, BH);
    float4 *X4 = reinterpret_cast<float4 *>(X);
    if (update && read) k_sweep<true, true><<<grid, 256, 0, st>>>(X4, delta, tw, g, partial, F, N, slot, nch);
    else if (update) k_sweep<true, false><<<grid, 256, 0, st>>>(X4, delta, tw, g, partial, F, N, slot, nch);
    else k_sweep<false, true><<<grid, 256, 0, st>>>(X4, delta, tw, g, partial, F, N, slot, nch);
    return hipGetLastError();
}

hipError_t launch_sweep_lazy(bool flush, bool read, float2 *X, const float *pending, const float2 *tw, const float2 *g,
                             float *partial, float *kpart, int BH, int F, int N, int slot_new, int npend,
                             const int *slots, hipStream_t st) {
    if (npend < 0 || npend > kMaxPending) return hipErrorInvalidValue;
    PendingSlots ps;
    ps.n = npend;
    for (int i = 0; i < kMaxPending; ++i) ps.slot[i] = i < npend ? slots[i] : 0;
    const int nch = sweep_chunks(F);
    dim3 grid(nch, BH);
    float4 *X4 = reinterpret_cast<float4 *>(X);
    if (!flush) {
        k_sweep_lazy<<<grid, 256, 0, st>>>(X4, tw, g, partial, kpart, F, N, BH, slot_new, ps, nch);
        return hipGetLastError();
    }
    const dim3 fgrid((nch + kFlushChunks - 1) / kFlushChunks, BH);
#define SPECTRE_FLUSH(RD, CAPV) \
    k_flush_mfma<RD, CAPV><<<fgrid, 256, 0, st>>>(X4, pending, tw, g, partial, F, N, BH, slot_new, ps, nch)
    if (read) {
        if (npend <= 8) SPECTRE_FLUSH(true, 8); else if (npend <= 16) SPECTRE_FLUSH(true, 16); else SPECTRE_FLUSH(true, 32);
    } else {
        if (npend <= 8) SPECTRE_FLUSH(false, 8); else if (npend <= 16) SPECTRE_FLUSH(false, 16); else SPECTRE_FLUSH(false, 32);
    }
#undef SPECTRE_FLUSH
    return hipGetLastError();
}

hipError_t launch_readout_final_lazy(int io, const float *partial, const float *kpart, const float *pending, void *out,
                                     int BH, int F, int npend, hipStream_t st) {
    const int nch = sweep_chunks(F);
    if (io) k_readout_final_lazy<IoBf16><<<BH, 256, 0, st>>>(partial, kpart, pending, static_cast<uint32_t *>(out), nch, BH, npend);
    else k_readout_final_lazy<IoF32><<<BH, 256, 0, st>>>(partial, kpart, pending, static_cast<float2 *>(out), nch, BH, npend);
    return hipGetLastError();
}

hipError_t launch_readout_final(int io, const float *partial, void *out, int BH, int F, hipStream_t st) {
    if (io) k_readout_final<IoBf16><<<BH, 256, 0, st>>>(partial, static_cast<uint32_t *>(out), sweep_chunks(F));
    else k_readout_final<IoF32><<<BH, 256, 0, st>>>(partial, static_cast<float2 *>(out), sweep_chunks(F));
    return hipGetLastError();
}

hipError_t launch_set_memory(const float *mem, int mem_batch, float *v_buf, int B, int H, int N, int Nmem,
                             hipStream_t st) {
    const size_t total = (size_t)B * H * Nmem * 64;
    k_set_memory<<<(unsigned)((total + 255) / 256), 256, 0, st>>>(mem, v_buf, H, N, Nmem, 64, mem_batch == B ? 1 : 0,
                                                                  total);
    return hipGetLastError();
}

hipError_t launch_ring_append(int io, const void *V, const void *Q, float *v_buf, float *q_buf, double *partial, int B,
                              int T, int H, int N, int M0, int W, int s0, long long t0, hipStream_t st) {
    const int nchunks = (T + 255) / 256;
    const dim3 grid(nchunks, B * H);
    if (io)
        k_ring_append<IoBf16><<<grid, 256, 0, st>>>(static_cast<const uint32_t *>(V), static_cast<const uint32_t *>(Q),
                                                    reinterpret_cast<float2 *>(v_buf), reinterpret_cast<float2 *>(q_buf),
                                                    partial, T, H, N, M0, W, s0, t0, nchunks);
    else
        k_ring_append<IoF32><<<grid, 256, 0, st>>>(static_cast<const float2 *>(V), static_cast<const float2 *>(Q),
                                                   reinterpret_cast<float2 *>(v_buf), reinterpret_cast<float2 *>(q_buf),
                                                   partial, T, H, N, M0, W, s0, t0, nchunks);
    return hipGetLastError();
}

static unsigned tangle_blocks(int N1, int N2, int nbh) { return (unsigned)(nbh * N2 * (N1 / 32) + (nbh * 32 + 255) / 256); }

hipError_t launch_untangle(const float2 *scr, float2 *X, int N, int N1, int N2, int P, int bh0, int nbh,
                           hipStream_t st) {
    if ((long long)nbh * N2 * (N1 / 32) > 0x7ffffff0LL) return hipErrorInvalidValue;
    k_untangle<<<tangle_blocks(N1, N2, nbh), 256, 0, st>>>(scr, reinterpret_cast<float4 *>(X), N, N1, N2, P, bh0, nbh);
    return hipGetLastError();
}

hipError_t launch_tangle(const float2 *X, const float2 *g, float2 *scr, int N, int N1, int N2, int P, int bh0,
                         int nbh, hipStream_t st) {
    if ((long long)nbh * N2 * (N1 / 32) > 0x7ffffff0LL) return hipErrorInvalidValue;
    k_tangle<<<tangle_blocks(N1, N2, nbh), 256, 0, st>>>(reinterpret_cast<const float4 *>(X), g, scr, N, N1, N2, P, bh0,
                                                         nbh);
    return hipGetLastError();
}

// Loads this translation unit's code object (the runtime loads them on first use): called by spectre_prepare so
// that no compute call is the first to touch it.
hipError_t load_kernels_prefix() {
    hipFuncAttributes a;
    return hipFuncGetAttributes(&a, reinterpret_cast<const void *>(k_fill_twiddle));
}

}  // namespace spectre
