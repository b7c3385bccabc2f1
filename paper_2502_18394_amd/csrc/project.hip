// Token projection (Sec. 3.2 step 1, Eq. 2) for gfx950: every head multiplies its own d = 64
// channels of the token rows by its d x d matrices W^(v) and W^(q).
//
// The layer only needs V and the pooled query sum_l q_l, and pooling commutes with the
// projection (sum_l x_l W = (sum_l x_l) W), so the kernel reads X once, writes V, and
// accumulates the column sums of X on the side; sum_q is then one 64 x 64 product per head in
// fp64.  Q itself is written only on request (the Prefix-FFT pre-fill keeps the query rows).
//
// The products run on the matrix cores: a wave owns 32 rows of one head, the 64 input channels are
// the reduction axis, two 32-column blocks the outputs.  Both row types use v_mfma_f32_32x32x16_bf16:
// bf16 rows with the weights split into two bf16 terms, fp32 rows with rows and weights split into three.
#include "project.h"

#include "common.h"

namespace spectre {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kProjRows = 512;    // rows of one head per workgroup (4 tiles of 32 per wave; 1024: 3 % slower, 256: 5 %)
constexpr int kOStride = 66;      // LDS row stride of a wave's output staging tile (floats)

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
template <bool WANT_Q, bool MULTI>
__global__ __launch_bounds__(256) void k_project_bf16(const uint16_t *__restrict__ x, const float *__restrict__ Wq,
                                                      const float *__restrict__ Wv, int Hw,
                                                      uint32_t *__restrict__ v_out, uint32_t *__restrict__ q_out,
                                                      double *__restrict__ partial, int L, int H, int nchunks, int B, int bpw) {
    extern __shared__ float lds_proj[];
    uint4 *wv_hi = reinterpret_cast<uint4 *>(lds_proj);    // 512 x 16 B each
    uint4 *wv_lo = wv_hi + 512;
    uint4 *wq_hi = wv_lo + 512;
    uint4 *wq_lo = wq_hi + 512;
    float *stage_all = reinterpret_cast<float *>(WANT_Q ? wq_lo + 512 : wv_lo + 512);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = blockIdx.x, chunk = blockIdx.y;                   // head fastest: whole token rows in flight
    const int hw = (Hw == 1) ? 0 : h;
    proj_fill_w_bf16(Wv + (size_t)hw * 4096, wv_hi, wv_lo, tid);
    if (WANT_Q) proj_fill_w_bf16(Wq + (size_t)hw * 4096, wq_hi, wq_lo, tid);
    __syncthreads();
    float *stage = stage_all + wave * (32 * kOStride);
    const int i = lane & 31, half = lane >> 5;
    const size_t rsp = (size_t)H * 32;
    const int row_end = min(L, (chunk + 1) * kProjRows);
    const int b_first = MULTI ? blockIdx.z * bpw : blockIdx.z;
    const int b_end = MULTI ? min(B, b_first + bpw) : b_first + 1;
    for (int b = b_first; b < b_end; ++b) {            // MULTI (short sequences): several per workgroup, one weight set-up
    float pool[32];
#pragma unroll
    for (int r = 0; r < 32; ++r) pool[r] = 0.f;

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
    __syncthreads();                                       // the staging tiles of the next sequence overlay `red`
    }
}

// ------------------------------------------------------------------------------------------
// fp32 rows on the bf16 matrix instruction: v_mfma_f32_32x32x2_f32 runs at 1/16 of the bf16 rate, which made the
// fp32 projection matrix-core-bound.  Every fp32 value is the exact sum of three bf16 terms up to 2^-27 of itself
// (x1 = bf16(x), x2 = bf16(x - x1), x3 = bf16(x - x1 - x2); the subtractions are exact), so x w is evaluated as the six
// products x1 w1, x1 w2, x2 w1, x1 w3, x2 w2, x3 w1 (each exact in the fp32 accumulator's input precision), smallest
// first; the three dropped products are below 2^-26 |x w|, i.e. below the rounding of the fp32 accumulation.  Six bf16
// instructions of 32 cycles replace sixteen fp32 ones of 64.
__device__ __forceinline__ void proj_fill_w_bf16x3(const float *__restrict__ W, uint4 *__restrict__ w1,
                                                   uint4 *__restrict__ w2, uint4 *__restrict__ w3, int tid) {
    for (int idx = tid; idx < 4 * 2 * 64; idx += 256) {
        const int lane = idx & 63, cb = (idx >> 6) & 1, ks = idx >> 7;
        const int j = cb * 32 + (lane & 31), k0 = 16 * ks + 8 * (lane >> 5);
        bf16x8 t1, t2, t3;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float w = W[(k0 + e) * 64 + j];
            const __bf16 b1 = (__bf16)w;
            const float r1 = w - (float)b1;
            const __bf16 b2 = (__bf16)r1;
            const float r2 = r1 - (float)b2;
            t1[e] = b1;
            t2[e] = b2;
            t3[e] = (__bf16)r2;
        }
        w1[idx] = __builtin_bit_cast(uint4, t1);
        w2[idx] = __builtin_bit_cast(uint4, t2);
        w3[idx] = __builtin_bit_cast(uint4, t3);
    }
}

struct Split3 {
    bf16x8 t1[4], t2[4], t3[4];      // per k-step: the lane's 8 channels as three bf16 terms
};

__device__ __forceinline__ void proj_mfma_split(const Split3 &a, const uint4 *__restrict__ w1,
                                                const uint4 *__restrict__ w2, const uint4 *__restrict__ w3, int lane,
                                                floatx16 &acc0, floatx16 &acc1) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        const int i0 = (ks * 2 + 0) * 64 + lane, i1 = (ks * 2 + 1) * 64 + lane;
        const bf16x8 p0 = __builtin_bit_cast(bf16x8, w1[i0]), p1 = __builtin_bit_cast(bf16x8, w1[i1]);
        const bf16x8 q0 = __builtin_bit_cast(bf16x8, w2[i0]), q1 = __builtin_bit_cast(bf16x8, w2[i1]);
        const bf16x8 r0 = __builtin_bit_cast(bf16x8, w3[i0]), r1 = __builtin_bit_cast(bf16x8, w3[i1]);
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.t1[ks], r0, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.t1[ks], r1, acc1, 0, 0, 0);
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.t3[ks], p0, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.t3[ks], p1, acc1, 0, 0, 0);
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.t2[ks], q0, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.t2[ks], q1, acc1, 0, 0, 0);
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.t1[ks], q0, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.t1[ks], q1, acc1, 0, 0, 0);
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.t2[ks], p0, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.t2[ks], p1, acc1, 0, 0, 0);
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.t1[ks], p0, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.t1[ks], p1, acc1, 0, 0, 0);
    }
}

// grid (H, ceil(L / kProjRows), B); 256 lanes.  Lane l holds row l%32 and channels 16 ks + 8 (l/32) .. +7 of k-step ks.
template <bool WANT_Q, bool MULTI>
__global__ __launch_bounds__(256) void k_project_f32(const float *__restrict__ x, const float *__restrict__ Wq,
                                                     const float *__restrict__ Wv, int Hw,
                                                     float2 *__restrict__ v_out, float2 *__restrict__ q_out,
                                                     double *__restrict__ partial, int L, int H, int nchunks, int B, int bpw) {
    extern __shared__ float lds_proj[];
    uint4 *wv1 = reinterpret_cast<uint4 *>(lds_proj);      // 512 x 16 B each
    uint4 *wv2 = wv1 + 512, *wv3 = wv2 + 512;
    uint4 *wq1 = wv3 + 512, *wq2 = wq1 + 512, *wq3 = wq2 + 512;
    float *stage_all = reinterpret_cast<float *>(WANT_Q ? wq3 + 512 : wv3 + 512);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = blockIdx.x, chunk = blockIdx.y;                   // head fastest: whole token rows in flight
    const int hw = (Hw == 1) ? 0 : h;
    proj_fill_w_bf16x3(Wv + (size_t)hw * 4096, wv1, wv2, wv3, tid);
    if (WANT_Q) proj_fill_w_bf16x3(Wq + (size_t)hw * 4096, wq1, wq2, wq3, tid);
    __syncthreads();
    float *stage = stage_all + wave * (32 * kOStride);
    const int i = lane & 31, half = lane >> 5;
    const size_t rsp = (size_t)H * 32;
    const int row_end = min(L, (chunk + 1) * kProjRows);
    const int b_first = MULTI ? blockIdx.z * bpw : blockIdx.z;
    const int b_end = MULTI ? min(B, b_first + bpw) : b_first + 1;
    for (int b = b_first; b < b_end; ++b) {            // MULTI (short sequences): several per workgroup, one weight set-up
    float pool[32];
#pragma unroll
    for (int r = 0; r < 32; ++r) pool[r] = 0.f;

    for (int r0 = chunk * kProjRows + wave * 32; r0 < row_end; r0 += 128) {
        const int row = r0 + i;
        const float *src = x + (((size_t)b * L + (row < L ? row : 0)) * H + h) * 64 + 8 * half;
        float4 raw[8];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            raw[2 * ks] = (row < L) ? *reinterpret_cast<const float4 *>(src + 16 * ks) : make_float4(0.f, 0.f, 0.f, 0.f);
            raw[2 * ks + 1] = (row < L) ? *reinterpret_cast<const float4 *>(src + 16 * ks + 4) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        Split3 a;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const float xv[8] = {raw[2 * ks].x, raw[2 * ks].y, raw[2 * ks].z, raw[2 * ks].w,
                                 raw[2 * ks + 1].x, raw[2 * ks + 1].y, raw[2 * ks + 1].z, raw[2 * ks + 1].w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                pool[8 * ks + e] += xv[e];
                const __bf16 b1 = (__bf16)xv[e];
                const float r1 = xv[e] - (float)b1;
                const __bf16 b2 = (__bf16)r1;
                const float r2 = r1 - (float)b2;
                a.t1[ks][e] = b1;
                a.t2[ks][e] = b2;
                a.t3[ks][e] = (__bf16)r2;
            }
        }
        const size_t out_pair = (((size_t)b * L + r0) * H + h) * 32;
        floatx16 acc0 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, acc1 = acc0;
        proj_mfma_split(a, wv1, wv2, wv3, lane, acc0, acc1);
        proj_store<IoF32>(acc0, acc1, stage, v_out + out_pair, rsp, L - r0, lane);
        if (WANT_Q) {
            floatx16 q0 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, q1 = q0;
            proj_mfma_split(a, wq1, wq2, wq3, lane, q0, q1);
            proj_store<IoF32>(q0, q1, stage, q_out + out_pair, rsp, L - r0, lane);
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
    __syncthreads();                                       // the staging tiles of the next sequence overlay `red`
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

// The value weights of every head as the matrix instruction's B operand, two bf16 terms per weight, for kernels that
// keep them in registers: wpack [Hw][2 (hi, lo)][4 k-steps x 2 column blocks x 64 lanes] of 16 bytes.
__global__ __launch_bounds__(256) void k_pack_w(const float *__restrict__ W, uint4 *__restrict__ wpack) {
    const int hw = blockIdx.x;
    proj_fill_w_bf16(W + (size_t)hw * 4096, wpack + (size_t)hw * 1024, wpack + (size_t)hw * 1024 + 512, threadIdx.x);
}

hipError_t launch_pack_w(const float *W, int Hw, void *wpack, hipStream_t st) {
    k_pack_w<<<Hw, 256, 0, st>>>(W, static_cast<uint4 *>(wpack));
    return hipGetLastError();
}

int project_chunks(int L) { return (L + kProjRows - 1) / kProjRows; }

// Sequences per workgroup: 1 unless a sequence is a single chunk; then enough of them that the launch is about two
// rounds of workgroups (two fit on a compute unit), so that the weight set-up is shared (3 at B*H = 3072, L = 196:
// 5 % faster than 1; 6 and more are slower again).
static int project_bpw(int B, int L, int H) {
    if (project_chunks(L) > 1) return 1;
    int bpw = (int)(((long long)B * H + 1023) / 1024);
    return bpw < 1 ? 1 : bpw > 16 ? 16 : bpw;
}

hipError_t launch_project(int io, const void *x, const float *Wq, const float *Wv, int Hw, void *v_out, void *q_out,
                          double *partial, int B, int L, int H, hipStream_t st) {
    const int bpw = q_out ? 1 : project_bpw(B, L, H), gz = (B + bpw - 1) / bpw;   // Q rows too: registers are short
    const size_t stage = (size_t)4 * 32 * kOStride, red = (size_t)4 * 64 * 33;
    const size_t terms = io ? 2 : 3;                     // bf16 terms per weight
    const size_t lds = (size_t)512 * 16 * terms * (q_out ? 2 : 1) + (stage > red ? stage : red) * sizeof(float);
    const int nch = project_chunks(L);
    const dim3 grid(H, nch, gz);
#define SPECTRE_PROJECT_LAUNCH(KERN, XT, OT)                                                                  \
    do {                                                                                                      \
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(KERN),                              \
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);             \
        if (e != hipSuccess) return e;                                                                        \
        KERN<<<grid, 256, lds, st>>>(static_cast<const XT *>(x), Wq, Wv, Hw, static_cast<OT *>(v_out),        \
                                     static_cast<OT *>(q_out), partial, L, H, nch, B, bpw);                   \
        return hipGetLastError();                                                                             \
    } while (0)
    const bool multi = bpw > 1;
    if (io) {
        if (q_out) SPECTRE_PROJECT_LAUNCH((k_project_bf16<true, false>), uint16_t, uint32_t);
        else { if (multi) SPECTRE_PROJECT_LAUNCH((k_project_bf16<false, true>), uint16_t, uint32_t);
               else SPECTRE_PROJECT_LAUNCH((k_project_bf16<false, false>), uint16_t, uint32_t); }
    } else {
        if (q_out) SPECTRE_PROJECT_LAUNCH((k_project_f32<true, false>), float, float2);
        else { if (multi) SPECTRE_PROJECT_LAUNCH((k_project_f32<false, true>), float, float2);
               else SPECTRE_PROJECT_LAUNCH((k_project_f32<false, false>), float, float2); }
    }
#undef SPECTRE_PROJECT_LAUNCH
}

hipError_t launch_project_pooled(const double *sum_x, const float *Wq, int Hw, int B, int H, double *sum_q,
                                 hipStream_t st) {
    k_project_pooled<<<B * H, 64, 0, st>>>(sum_x, Wq, Hw, H, sum_q);
    return hipGetLastError();
}

// Loads this translation unit's code object (the runtime loads them on first use): called by spectre_prepare so
// that no compute call is the first to touch it.
hipError_t load_kernels_project() {
    hipFuncAttributes a;
    return hipFuncGetAttributes(&a, reinterpret_cast<const void *>(k_project_pooled));
}

}  // namespace spectre
