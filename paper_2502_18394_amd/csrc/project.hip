// Token projection (Sec. 3.2 step 1, Eq. 2) for gfx950: every head multiplies its own d = 64
// channels of the token rows by its d x d matrices W^(v) and W^(q).
//
// The layer only needs V and the pooled query sum_l q_l, and pooling commutes with the
// projection (sum_l x_l W = (sum_l x_l) W), so the kernel reads X once, writes V, and
// accumulates the column sums of X on the side; sum_q is then one 64 x 64 product per head in
// fp64.  Q itself is written only on request (the Prefix-FFT pre-fill keeps the query rows).
//
// The products run on the matrix cores: a wave owns 32 rows of one head, the 64 input channels are
// the reduction axis, two 32-column blocks the outputs.  fp32 rows use v_mfma_f32_32x32x2_f32, bf16
// rows v_mfma_f32_32x32x16_bf16 with the weights split into two bf16 terms.
#include "project.h"

#include "common.h"

namespace spectre {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kProjRows = 512;    // rows of one head per workgroup (4 tiles of 32 per wave; 1024: 3 % slower, 256: 5 %)
constexpr int kWStride = 65;      // LDS row stride of the weight matrices (floats)
constexpr int kOStride = 66;      // LDS row stride of a wave's output staging tile (floats)

template <typename IO> struct ProjLoad;
template <> struct ProjLoad<IoF32> {   // four consecutive channels of a row
    __device__ static __forceinline__ float4 load(const void *base, size_t elem) {
        return *reinterpret_cast<const float4 *>(static_cast<const float *>(base) + elem);
    }
};
template <> struct ProjLoad<IoBf16> {
    __device__ static __forceinline__ float4 load(const void *base, size_t elem) {
        const uint2 w = *reinterpret_cast<const uint2 *>(static_cast<const uint16_t *>(base) + elem);
        const float2 a = IoBf16::unpack(w.x), b = IoBf16::unpack(w.y);
        return make_float4(a.x, a.y, b.x, b.y);
    }
};

// One 32 x 64 product of the rows held in a[] (lane l: row l%32, channels 8q + 4*(l/32) + {0..3})
// with a 64 x 64 matrix in LDS.  MFMA number m of group q pairs channel 8q + m (lanes 0-31) with
// 8q + 4 + m (lanes 32-63) on both operands.
__device__ __forceinline__ void proj_mfma(const float4 (&a)[8], const float *__restrict__ w_lds, int lane,
                                          floatx16 &acc0, floatx16 &acc1) {
    const int j = lane & 31, half = lane >> 5;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const float av[4] = {a[q].x, a[q].y, a[q].z, a[q].w};
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const float *wr = w_lds + (8 * q + 4 * half + m) * kWStride + j;
            acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(av[m], wr[0], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(av[m], wr[32], acc1, 0, 0, 0);
        }
    }
}

// Accumulator register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4, column l%32 of a block.
// The tile goes through LDS so that rows leave as whole 128-byte (bf16) / 256-byte (fp32) segments.
template <typename IO>
__device__ __forceinline__ void proj_store(const floatx16 &acc0, const floatx16 &acc1, float *__restrict__ stage,
                                           typename IO::pair_t *__restrict__ dst, size_t row_stride_pairs,
                                           int rows_left, int lane) {
    const int j = lane & 31, half = lane >> 5;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int row = 8 * (v / 4) + 4 * half + (v % 4);
        stage[row * kOStride + j] = acc0[v];
        stage[row * kOStride + 32 + j] = acc1[v];
    }
    __builtin_amdgcn_wave_barrier();   // LDS operations of one wave complete in issue order
#pragma unroll
    for (int it = 0; it < 16; ++it) {
        const int row = half + 2 * it;
        const float2 val = *reinterpret_cast<const float2 *>(stage + row * kOStride + 2 * j);
        if (row < rows_left) dst[(size_t)row * row_stride_pairs + j] = IO::pack(val);
    }
    __builtin_amdgcn_wave_barrier();
}

// grid (H, ceil(L / kProjRows), B); 256 lanes.
template <typename IO, bool WANT_Q>
__global__ __launch_bounds__(256) void k_project(const void *__restrict__ x, const float *__restrict__ Wq,
                                                 const float *__restrict__ Wv, int Hw,
                                                 typename IO::pair_t *__restrict__ v_out,
                                                 typename IO::pair_t *__restrict__ q_out,
                                                 double *__restrict__ partial, int L, int H, int nchunks) {
    extern __shared__ float lds_proj[];
    float *wv = lds_proj;                                  // [64][kWStride]
    float *wq = wv + 64 * kWStride;                        // [64][kWStride], only filled when WANT_Q
    float *stage_all = wq + (WANT_Q ? 64 * kWStride : 0);  // 4 x [32][kOStride]; reused for the pooling
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = blockIdx.x, chunk = blockIdx.y, b = blockIdx.z;   // head fastest: whole token rows in flight
    const int hw = (Hw == 1) ? 0 : h;
    for (int idx = tid; idx < 64 * 64; idx += 256) {
        wv[(idx >> 6) * kWStride + (idx & 63)] = Wv[(size_t)hw * 4096 + idx];
        if (WANT_Q) wq[(idx >> 6) * kWStride + (idx & 63)] = Wq[(size_t)hw * 4096 + idx];
    }
    __syncthreads();
    float *stage = stage_all + wave * (32 * kOStride);
    const int i = lane & 31, half = lane >> 5;
    const size_t rsp = (size_t)H * 32;                     // row stride in channel pairs
    float pool[32];
#pragma unroll
    for (int r = 0; r < 32; ++r) pool[r] = 0.f;

    const int row_end = min(L, (chunk + 1) * kProjRows);
    for (int r0 = chunk * kProjRows + wave * 32; r0 < row_end; r0 += 128) {
        const int row = r0 + i;
        float4 a[8];
        const size_t elem = (((size_t)b * L + (row < L ? row : 0)) * H + h) * 64 + 4 * half;
#pragma unroll
        for (int q = 0; q < 8; ++q)
            a[q] = (row < L) ? ProjLoad<IO>::load(x, elem + 8 * q) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            pool[4 * q + 0] += a[q].x;
            pool[4 * q + 1] += a[q].y;
            pool[4 * q + 2] += a[q].z;
            pool[4 * q + 3] += a[q].w;
        }
        const size_t out_pair = (((size_t)b * L + r0) * H + h) * 32;
        floatx16 acc0 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, acc1 = acc0;
        proj_mfma(a, wv, lane, acc0, acc1);
        proj_store<IO>(acc0, acc1, stage, v_out + out_pair, rsp, L - r0, lane);
        if (WANT_Q) {
            floatx16 q0 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, q1 = q0;
            proj_mfma(a, wq, lane, q0, q1);
            proj_store<IO>(q0, q1, stage, q_out + out_pair, rsp, L - r0, lane);
        }
    }
    // column sums of X over this workgroup's rows: lane (i, half) holds channels 8q + 4 half + e in
    // pool[4q + e]; the 32 lanes of a half and the 4 waves are added in a fixed order, in fp64
    __syncthreads();
    float *red = stage_all;                                // [4 waves][64 lanes][33]
#pragma unroll
    for (int r = 0; r < 32; ++r) red[(wave * 64 + lane) * 33 + r] = pool[r];
    __syncthreads();
    if (tid < 64) {
        const int c = tid, q = c >> 3, hf = (c >> 2) & 1, e = c & 3;
        double s = 0.0;
        for (int w = 0; w < 4; ++w)
            for (int l = 0; l < 32; ++l) s += (double)red[(w * 64 + hf * 32 + l) * 33 + 4 * q + e];
        partial[((size_t)b * nchunks + chunk) * (H * 64) + h * 64 + c] = s;
    }
}

// ------------------------------------------------------------------------------------------
// bf16 rows: the inputs are exact in bf16, so the product runs on v_mfma_f32_32x32x16_bf16 with every
// fp32 weight split into two bf16 terms (hi + lo, 16 significant bits together; the third term would
// be below the fp32 accumulation error of a 64-term dot product).  Lane l supplies row l%32 and the 8
// consecutive channels 16 ks + 8 (l/32) .. +7 of k-step ks - one 16-byte load straight from the row.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// weights in B-operand order: [ks][column block][lane][8], lane = (k half, column)
__device__ __forceinline__ void proj_fill_w_bf16(const float *__restrict__ W, uint4 *__restrict__ hi,
                                                 uint4 *__restrict__ lo, int tid) {
    for (int idx = tid; idx < 4 * 2 * 64; idx += 256) {
        const int lane = idx & 63, cb = (idx >> 6) & 1, ks = idx >> 7;
        const int j = cb * 32 + (lane & 31), k0 = 16 * ks + 8 * (lane >> 5);
        bf16x8 h8, l8;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float w = W[(k0 + e) * 64 + j];
            const __bf16 hb = (__bf16)w;
            h8[e] = hb;
            l8[e] = (__bf16)(w - (float)hb);
        }
        hi[idx] = __builtin_bit_cast(uint4, h8);
        lo[idx] = __builtin_bit_cast(uint4, l8);
    }
}

__device__ __forceinline__ void proj_mfma_bf16(const uint4 (&a)[4], const uint4 *__restrict__ hi,
                                               const uint4 *__restrict__ lo, int lane, floatx16 &acc0,
                                               floatx16 &acc1) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        const bf16x8 av = __builtin_bit_cast(bf16x8, a[ks]);
        const bf16x8 h0 = __builtin_bit_cast(bf16x8, hi[(ks * 2 + 0) * 64 + lane]);
        const bf16x8 h1 = __builtin_bit_cast(bf16x8, hi[(ks * 2 + 1) * 64 + lane]);
        const bf16x8 l0 = __builtin_bit_cast(bf16x8, lo[(ks * 2 + 0) * 64 + lane]);
        const bf16x8 l1 = __builtin_bit_cast(bf16x8, lo[(ks * 2 + 1) * 64 + lane]);
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, l0, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, l1, acc1, 0, 0, 0);
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, h0, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, h1, acc1, 0, 0, 0);
    }
}

// grid (H, ceil(L / kProjRows), B); 256 lanes.
template <bool WANT_Q>
__global__ __launch_bounds__(256) void k_project_bf16(const uint16_t *__restrict__ x, const float *__restrict__ Wq,
                                                      const float *__restrict__ Wv, int Hw,
                                                      uint32_t *__restrict__ v_out, uint32_t *__restrict__ q_out,
                                                      double *__restrict__ partial, int L, int H, int nchunks) {
    extern __shared__ float lds_proj[];
    uint4 *wv_hi = reinterpret_cast<uint4 *>(lds_proj);    // 512 x 16 B each
    uint4 *wv_lo = wv_hi + 512;
    uint4 *wq_hi = wv_lo + 512;
    uint4 *wq_lo = wq_hi + 512;
    float *stage_all = reinterpret_cast<float *>(WANT_Q ? wq_lo + 512 : wv_lo + 512);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = blockIdx.x, chunk = blockIdx.y, b = blockIdx.z;   // head fastest: whole token rows in flight
    const int hw = (Hw == 1) ? 0 : h;
    proj_fill_w_bf16(Wv + (size_t)hw * 4096, wv_hi, wv_lo, tid);
    if (WANT_Q) proj_fill_w_bf16(Wq + (size_t)hw * 4096, wq_hi, wq_lo, tid);
    __syncthreads();
    float *stage = stage_all + wave * (32 * kOStride);
    const int i = lane & 31, half = lane >> 5;
    const size_t rsp = (size_t)H * 32;
    float pool[32];
#pragma unroll
    for (int r = 0; r < 32; ++r) pool[r] = 0.f;

    const int row_end = min(L, (chunk + 1) * kProjRows);
    for (int r0 = chunk * kProjRows + wave * 32; r0 < row_end; r0 += 128) {
        const int row = r0 + i;
        uint4 a[4];
        const uint16_t *src = x + (((size_t)b * L + (row < L ? row : 0)) * H + h) * 64 + 8 * half;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            a[ks] = (row < L) ? *reinterpret_cast<const uint4 *>(src + 16 * ks) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const uint32_t w[4] = {a[ks].x, a[ks].y, a[ks].z, a[ks].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float2 p = IoBf16::unpack(w[e]);
                pool[8 * ks + 2 * e] += p.x;
                pool[8 * ks + 2 * e + 1] += p.y;
            }
        }
        const size_t out_pair = (((size_t)b * L + r0) * H + h) * 32;
        floatx16 acc0 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, acc1 = acc0;
        proj_mfma_bf16(a, wv_hi, wv_lo, lane, acc0, acc1);
        proj_store<IoBf16>(acc0, acc1, stage, v_out + out_pair, rsp, L - r0, lane);
        if (WANT_Q) {
            floatx16 q0 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, q1 = q0;
            proj_mfma_bf16(a, wq_hi, wq_lo, lane, q0, q1);
            proj_store<IoBf16>(q0, q1, stage, q_out + out_pair, rsp, L - r0, lane);
        }
    }
    // column sums: lane (i, half) holds channel 16 ks + 8 half + e in pool[8 ks + e]
    __syncthreads();
    float *red = stage_all;
#pragma unroll
    for (int r = 0; r < 32; ++r) red[(wave * 64 + lane) * 33 + r] = pool[r];
    __syncthreads();
    if (tid < 64) {
        const int c = tid, ks = c >> 4, hf = (c >> 3) & 1, e = c & 7;
        double s = 0.0;
        for (int w = 0; w < 4; ++w)
            for (int l = 0; l < 32; ++l) s += (double)red[(w * 64 + hf * 32 + l) * 33 + 8 * ks + e];
        partial[((size_t)b * nchunks + chunk) * (H * 64) + h * 64 + c] = s;
    }
}

// sum_q[b,h,j] = sum_i sum_x[b,h,i] Wq[h,i,j] in fp64.  One workgroup of 64 lanes per (b,h).
__global__ __launch_bounds__(64) void k_project_pooled(const double *__restrict__ sum_x, const float *__restrict__ Wq,
                                                       int Hw, int H, double *__restrict__ sum_q) {
    __shared__ double xs[64];
    const int bh = blockIdx.x, h = bh % H, hw = (Hw == 1) ? 0 : h, j = threadIdx.x;
    xs[j] = sum_x[(size_t)bh * 64 + j];
    __syncthreads();
    double s = 0.0;
    for (int i = 0; i < 64; ++i) s += xs[i] * (double)Wq[(size_t)hw * 4096 + i * 64 + j];
    sum_q[(size_t)bh * 64 + j] = s;
}

int project_chunks(int L) { return (L + kProjRows - 1) / kProjRows; }

size_t project_lds_bytes(bool want_q) {
    const size_t stage = (size_t)4 * 32 * kOStride, red = (size_t)4 * 64 * 33;
    return ((size_t)64 * kWStride * (want_q ? 2 : 1) + (stage > red ? stage : red)) * sizeof(float);
}

template <typename IO, bool WANT_Q>
static hipError_t project_t(const void *x, const float *Wq, const float *Wv, int Hw, void *v_out, void *q_out,
                            double *partial, int B, int L, int H, hipStream_t st) {
    const size_t lds = project_lds_bytes(WANT_Q);
    auto kern = k_project<IO, WANT_Q>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    const int nch = project_chunks(L);
    kern<<<dim3(H, nch, B), dim3(256), lds, st>>>(x, Wq, Wv, Hw, static_cast<typename IO::pair_t *>(v_out),
                                                  static_cast<typename IO::pair_t *>(q_out), partial, L, H, nch);
    return hipGetLastError();
}

hipError_t launch_project(int io, const void *x, const float *Wq, const float *Wv, int Hw, void *v_out, void *q_out,
                          double *partial, int B, int L, int H, hipStream_t st) {
    if (io) {
        const size_t stage = (size_t)4 * 32 * kOStride, red = (size_t)4 * 64 * 33;
        const size_t lds = (size_t)512 * 16 * (q_out ? 4 : 2) + (stage > red ? stage : red) * sizeof(float);
        const int nch = project_chunks(L);
        dim3 grid(H, nch, B);
        if (q_out) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_project_bf16<true>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            k_project_bf16<true><<<grid, 256, lds, st>>>(static_cast<const uint16_t *>(x), Wq, Wv, Hw,
                                                         static_cast<uint32_t *>(v_out), static_cast<uint32_t *>(q_out),
                                                         partial, L, H, nch);
        } else {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_project_bf16<false>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            k_project_bf16<false><<<grid, 256, lds, st>>>(static_cast<const uint16_t *>(x), Wq, Wv, Hw,
                                                          static_cast<uint32_t *>(v_out), nullptr, partial, L, H, nch);
        }
        return hipGetLastError();
    }
    return q_out ? project_t<IoF32, true>(x, Wq, Wv, Hw, v_out, q_out, partial, B, L, H, st)
                 : project_t<IoF32, false>(x, Wq, Wv, Hw, v_out, q_out, partial, B, L, H, st);
}

hipError_t launch_project_pooled(const double *sum_x, const float *Wq, int Hw, int B, int H, double *sum_q,
                                 hipStream_t st) {
    k_project_pooled<<<B * H, 64, 0, st>>>(sum_x, Wq, Hw, H, sum_q);
    return hipGetLastError();
}

}  // namespace spectre
