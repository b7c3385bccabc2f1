// Four-step transform path of the SPECTRE mixing layer (Sec. 3.2 steps 2-4,
// Eq. 3 and Eq. 4) for gfx950: L = N1 * N2 with N1 = 256 or 4096 and N2 <= 32 of the
// form {1, 3, 5, 7} * 2^a.
//
// Two adjacent channels of a head are transformed together as one complex
// sequence z = v_even + j v_odd.  Because the gate is extended to all L bins by
// Hermitian symmetry (App. B, Thm. B.1), multiplying the complex spectrum of z
// by it and transforming back leaves the two real results in the real and
// imaginary parts, so no split/merge pass is needed and a bf16 channel pair is
// one 32-bit load.
//
// L = N1 * N2, time index t = t1 + N1*t2, frequency index k = k2 + N2*k1:
//   small_fwd : A[t1,k2]  = W_L^(t1 k2) * sum_t2 z[t1 + N1 t2] W_N2^(t2 k2)      (one lane per (t1, pair))
//   big       : Z[k2+N2 k1] = sum_t1 A[t1,k2] W_N1^(t1 k1);  Y = G * Z;  B[t1,k2] = sum_k1 Y W_N1^(-t1 k1)
//   small_inv : out[t1 + N1 t2] = sum_k2 conj(W_L^(t1 k2)) B[t1,k2] W_N2^(-t2 k2)
// with W_n = exp(-j 2 pi / n) and the 1/L of the inverse folded into G.
#include "mix_pow2.h"

#include <type_traits>

#include "fft_regs.h"
#include "internal.h"

namespace spectre {

// Shape of the row kernels' tile: TT = 16 adjacent t1 (128-byte runs in the scratch) times kPairs channel pairs, one
// 128-byte segment of every row: a whole bf16 head row, or one half of an fp32 head row (its two halves go to two
// workgroups, so that rows with 8-byte pairs keep whole 128-byte lines on both sides of the kernel).
// kStride: LDS row stride (in pair_t units) of the [t2][t1_local][pair] staging tile, chosen so that a wave reading
// along t1_local with 16 lanes per pair index hits every bank equally.
template <typename IO> struct RowTile;
template <> struct RowTile<IoBf16> { static constexpr int kPairs = 32, kStride = 36; };
template <> struct RowTile<IoF32> { static constexpr int kPairs = 16, kStride = 18; };
template <typename IO> struct TileStride { static constexpr int value = RowTile<IO>::kStride; };

// ------------------------------------------------------------------------------------------
// Element of the transform scratch: one complex number per channel pair, as two fp32 (the default) or, on request
// for bf16 rows, as two bfloat16 in a 32-bit word (half the bytes of every exchange between the three kernels;
// the arithmetic stays fp32).
struct ScrF32 {
    typedef float2 elem_t;
    __device__ static __forceinline__ float2 get(elem_t e) { return e; }
    __device__ static __forceinline__ elem_t put(float2 v) { return v; }
};
struct ScrBf16 {
    typedef uint32_t elem_t;
    __device__ static __forceinline__ float2 get(elem_t e) { return IoBf16::unpack(e); }
    __device__ static __forceinline__ elem_t put(float2 v) { return IoBf16::pack(v); }
};

// Head-affine placement (aff = heads in the launch, a multiple of 8; 0 = off).  Workgroup ids are dealt round-robin
// to the 8 XCDs, each with its own L2.  Here the per_head workgroups of head 8 * slot + xcd all get ids congruent to
// xcd mod 8, so a head's scratch is written and read through one L2, and the three kernels walk the slots in
// alternating order (row transforms up, column kernel down, inverse row transforms up), so that each starts with
// what its predecessor wrote last.  Pays when a few heads' scratch fits one 4 MB L2 (L <= 8192).
__device__ __forceinline__ void head_affine(int id, int per_head, int aff, bool reverse, int *bhl, int *within) {
    const int xcd = id & 7, idx = id >> 3;
    int slot = idx / per_head;
    *within = idx - slot * per_head;
    if (reverse) slot = aff / 8 - 1 - slot;
    *bhl = 8 * slot + xcd;
}

// exp(-j 2 pi t1 k2 / L) for k2 = 1 .. N2-1.  Only the powers of two are read from the table (five loads instead of
// 31 scattered ones at N2 = 32: the gathers were most of the kernel's cache-line requests).  With k2 = 4a + b the
// others are hi[a] * lo[b], products of at most five table values in all, i.e. within 4 rounding errors of the table
// value; only hi and lo stay in registers, the product is formed where it is used.
template <int N2>
struct SmallTwiddles {
    float2 lo[4], hi[8];
    __device__ __forceinline__ SmallTwiddles(const float2 *__restrict__ twL, int t1) {
        float2 p[5];
#pragma unroll
        for (int e = 0; e < 5; ++e) p[e] = ((1 << e) < N2) ? twL[t1 << e] : make_float2(1.f, 0.f);
        lo[0] = make_float2(1.f, 0.f);
        lo[1] = p[0];
        lo[2] = p[1];
        lo[3] = cmul(p[1], p[0]);
        hi[0] = make_float2(1.f, 0.f);
        hi[1] = p[2];
        hi[2] = p[3];
        hi[3] = cmul(p[3], p[2]);
        hi[4] = p[4];
        hi[5] = cmul(p[4], p[2]);
        hi[6] = cmul(p[4], p[3]);
        hi[7] = cmul(p[4], hi[3]);
    }
    __device__ __forceinline__ float2 operator()(int k2) const {     // k2 a compile-time constant after unrolling
        const int a = k2 >> 2, b = k2 & 3;
        if (a == 0) return lo[b];
        if (b == 0) return hi[a];
        return cmul(hi[a], lo[b]);
    }
};

// small_fwd: grid (N1/TT * 32/PW, nbh); block PW*TT threads, PW = RowTile<IO>::kPairs.  Reads the N2*TT rows
// {t1_0 + r + N1*t2} of one head (PW pairs each, one 128-byte segment per row),
// stages them in LDS, then lane (pair p, t1_local) runs the N2-point DFT over t2.
// ring != nullptr (pre-fill of an empty Prefix-FFT cache): every row read is also copied, as fp32, to row l of head bh
// of the value ring buffer ring [B*H][N1 * N2][32 pairs] - the rows then cross HBM once for both purposes.
template <int N2, int TT, typename IO, typename SC>
__global__ __launch_bounds__(RowTile<IO>::kPairs * TT) void k_small_fwd(const typename IO::pair_t *__restrict__ v,
                                                       typename SC::elem_t *__restrict__ scr,
                                                       const float2 *__restrict__ twL, int rows, int H,
                                                       int N1, int bh0, int aff, float2 *__restrict__ ring) {
    typedef typename IO::pair_t pair_t;
    constexpr int S = TileStride<IO>::value, PW = RowTile<IO>::kPairs, NPART = 32 / PW;
    extern __shared__ unsigned char smem_raw[];
    pair_t *lds = reinterpret_cast<pair_t *>(smem_raw);
    const int tid = threadIdx.x;
    int tile = blockIdx.x, bhl = blockIdx.y;
    if (aff) head_affine(blockIdx.x, N1 / TT * NPART, aff, false, &bhl, &tile);
    const int t1_0 = (tile / NPART) * TT, p0 = (tile % NPART) * PW;
    const int bh = bh0 + bhl, b = bh / H, h = bh % H;
    {
        const int lp = tid % PW, r = tid / PW;
        pair_t val[N2];
#pragma unroll
        for (int t2 = 0; t2 < N2; ++t2) {
            const int l = t1_0 + r + N1 * t2;
            val[t2] = (l < rows) ? IO::load_stream(v + (((size_t)b * rows + l) * H + h) * 32 + p0 + lp) : IO::zero();
        }
#pragma unroll
        for (int t2 = 0; t2 < N2; ++t2) lds[(t2 * TT + r) * S + lp] = val[t2];
        if (ring) {
#pragma unroll
            for (int t2 = 0; t2 < N2; ++t2) {
                const int l = t1_0 + r + N1 * t2;
                if (l < rows) stream_store(ring + ((size_t)bh * N1 * N2 + l) * 32 + p0 + lp, IO::unpack(val[t2]));
            }
        }
    }
    __syncthreads();
    const int tl = tid % TT, p = tid / TT, t1 = t1_0 + tl;
    float2 x[N2];
#pragma unroll
    for (int t2 = 0; t2 < N2; ++t2) x[t2] = IO::unpack(lds[(t2 * TT + tl) * S + p]);
    small_dft<N2, false>(x);
    typename SC::elem_t *dst = scr + (((size_t)bhl * N2) * 32 + p0 + p) * N1 + t1;
    const SmallTwiddles<N2> tw(twL, t1);
#pragma unroll
    for (int k2 = 0; k2 < N2; ++k2) {
        const float2 y = (k2 == 0) ? x[0] : cmul(x[k2], tw(k2));
        dst[(size_t)k2 * 32 * N1] = SC::put(y);
    }
}

// small_fwd with the token projection in front (Sec. 3.2 step 1, Eq. 2, feeding step 2): the workgroup reads rows of
// the layer input X instead of V, multiplies every row by its head's 64 x 64 value matrix on the matrix cores and
// rounds the products to bfloat16 into the same LDS tile the plain kernel fills from memory - the bits the separate
// projection kernel would have stored as V (same instruction, same order of the hi/lo weight terms), which then
// never exist in HBM.  bf16 rows, TT = 16.  wpack: the weights as the B operand (k_pack_w), held in registers.
// A wave takes 32 tile rows at a time (two adjacent t2 of the 16 t1): lane l supplies row l % 32 and the channels
// 16 ks + 8 (l / 32) .. + 7 of k-step ks as one 16-byte LDS read; accumulator register v of lane l is row
// 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32 of a 32-column block, so a channel pair sits in two adjacent lanes:
// even lanes pack the pairs of columns 0..31, odd lanes those of columns 32..63, each fetching the neighbour's half
// with a quad permutation.  The rows a wave overwrites are the ones it has just read, and no other wave touches them.
typedef float floatx16_t __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

template <int N2>
__global__ __launch_bounds__(512) void k_small_fwd_proj(const uint32_t *__restrict__ x, const uint4 *__restrict__ wpack,
                                                        int Hw, float2 *__restrict__ scr,
                                                        const float2 *__restrict__ twL, int rows, int H, int N1,
                                                        int bh0, int aff) {
    constexpr int TT = 16, S = TileStride<IoBf16>::value, NROW = N2 * TT, NGRP = (NROW + 31) / 32;
    extern __shared__ unsigned char smem_raw[];
    uint32_t *lds = reinterpret_cast<uint32_t *>(smem_raw);
    const int tid = threadIdx.x;
    int tile = blockIdx.x, bhl = blockIdx.y;
    if (aff) head_affine(blockIdx.x, N1 / TT, aff, false, &bhl, &tile);
    const int t1_0 = tile * TT;
    const int bh = bh0 + bhl, b = bh / H, h = bh % H;
    {
        const int lp = tid & 31, r = tid >> 5;
        uint32_t val[N2];
#pragma unroll
        for (int t2 = 0; t2 < N2; ++t2) {
            const int l = t1_0 + r + N1 * t2;
            val[t2] = (l < rows) ? IoBf16::load_stream(x + (((size_t)b * rows + l) * H + h) * 32 + lp) : 0u;
        }
#pragma unroll
        for (int t2 = 0; t2 < N2; ++t2) lds[(t2 * TT + r) * S + lp] = val[t2];
    }
    const int lane = tid & 63, wave = tid >> 6, i = lane & 31, half = lane >> 5;
    uint4 whi[8], wlo[8];                              // [ks * 2 + column block]
    {
        const uint4 *wp = wpack + (size_t)((Hw == 1) ? 0 : h) * 1024 + lane;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            whi[e] = wp[e * 64];
            wlo[e] = wp[512 + e * 64];
        }
    }
    __syncthreads();
    for (int g = wave; g < NGRP; g += 8) {
        const int ri = 32 * g + i;
        uint4 a[4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            a[ks] = (ri < NROW) ? *reinterpret_cast<const uint4 *>(lds + ri * S + 8 * ks + 4 * half) : make_uint4(0, 0, 0, 0);
        floatx16_t acc0 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, acc1 = acc0;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const bf16x8_t av = __builtin_bit_cast(bf16x8_t, a[ks]);
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, __builtin_bit_cast(bf16x8_t, wlo[2 * ks]), acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, __builtin_bit_cast(bf16x8_t, wlo[2 * ks + 1]), acc1, 0, 0, 0);
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, __builtin_bit_cast(bf16x8_t, whi[2 * ks]), acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, __builtin_bit_cast(bf16x8_t, whi[2 * ks + 1]), acc1, 0, 0, 0);
        }
        const bool odd = i & 1;
        const int pcol = odd ? 16 + (i >> 1) : (i >> 1);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = 32 * g + 8 * (v / 4) + 4 * half + (v % 4);
            const float n0 = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(acc0[v]), 0xB1, 0xF, 0xF, false));
            const float n1 = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(acc1[v]), 0xB1, 0xF, 0xF, false));
            const float2 pr = odd ? make_float2(n1, acc1[v]) : make_float2(acc0[v], n0);
            if (row < NROW) lds[row * S + pcol] = IoBf16::pack(pr);
        }
    }
    __syncthreads();
    const int tl = tid % TT, p = tid / TT, t1 = t1_0 + tl;
    float2 xv[N2];
#pragma unroll
    for (int t2 = 0; t2 < N2; ++t2) xv[t2] = IoBf16::unpack(lds[(t2 * TT + tl) * S + p]);
    small_dft<N2, false>(xv);
    float2 *dst = scr + (((size_t)bhl * N2) * 32 + p) * N1 + t1;
    const SmallTwiddles<N2> tw(twL, t1);
#pragma unroll
    for (int k2 = 0; k2 < N2; ++k2) {
        const float2 y = (k2 == 0) ? xv[0] : cmul(xv[k2], tw(k2));
        dst[(size_t)k2 * 32 * N1] = y;
    }
}

// small_inv: mirror image.  Rows l of the inverse transform with row0 <= l < row0+out_rows
// are written to row l-row0 of out [B, out_rows, H, d].  With ring_w > 0 the rows are instead
// gathered from a ring buffer that occupies rows ring0 .. ring0+ring_w-1 and whose newest entry
// sits at ring0+newest: the out_rows newest entries are written oldest first.
// bsum != nullptr (mixer followed by the wavelet refinement): the workgroup also emits the sums of the TT adjacent rows
// it writes for every t2, taken over the values as stored (after rounding to the I/O type), to
// bsum [bh][L / TT][32 pairs]; block l / TT covers rows l .. l + TT - 1.  Added in row order.
template <int N2, int TT, typename IO, typename SC>
__global__ __launch_bounds__(RowTile<IO>::kPairs * TT) void k_small_inv(const typename SC::elem_t *__restrict__ scr,
                                                       typename IO::pair_t *__restrict__ out,
                                                       const float2 *__restrict__ twL, int row0,
                                                       int out_rows, int H, int N1, int bh0, int ring0,
                                                       int ring_w, int newest, int aff, float2 *__restrict__ bsum) {
    typedef typename IO::pair_t pair_t;
    constexpr int S = TileStride<IO>::value, PW = RowTile<IO>::kPairs, NPART = 32 / PW;
    extern __shared__ unsigned char smem_raw[];
    pair_t *lds = reinterpret_cast<pair_t *>(smem_raw);
    const int tid = threadIdx.x;
    int tile = blockIdx.x, bhl = blockIdx.y;
    if (aff) head_affine(blockIdx.x, N1 / TT * NPART, aff, false, &bhl, &tile);
    const int t1_0 = (tile / NPART) * TT, p0 = (tile % NPART) * PW;
    const int bh = bh0 + bhl, b = bh / H, h = bh % H;
    {
        const int tl = tid % TT, p = tid / TT, t1 = t1_0 + tl;
        const typename SC::elem_t *src = scr + (((size_t)bhl * N2) * 32 + p0 + p) * N1 + t1;
        typename SC::elem_t raw[N2];
#pragma unroll
        for (int k2 = 0; k2 < N2; ++k2) raw[k2] = src[(size_t)k2 * 32 * N1];
        float2 y[N2];
#pragma unroll
        for (int k2 = 0; k2 < N2; ++k2) y[k2] = SC::get(raw[k2]);
        const SmallTwiddles<N2> tw(twL, t1);
#pragma unroll
        for (int k2 = 1; k2 < N2; ++k2) y[k2] = cmulc(y[k2], tw(k2));
        small_dft<N2, true>(y);
#pragma unroll
        for (int t2 = 0; t2 < N2; ++t2) lds[(t2 * TT + tl) * S + p] = IO::pack(y[t2]);
    }
    __syncthreads();
    const int lp = tid % PW, r = tid / PW;
#pragma unroll
    for (int t2 = 0; t2 < N2; ++t2) {
        const int l = t1_0 + r + N1 * t2;
        int orow = l - row0;
        if (ring_w > 0) {
            int age = newest - (l - ring0);            // 0 = newest entry of the ring
            if (age < 0) age += ring_w;
            orow = (l >= ring0) ? out_rows - 1 - age : -1;
        }
        if (orow >= 0 && orow < out_rows)
            IO::store_stream(out + (((size_t)b * out_rows + orow) * H + h) * 32 + p0 + lp, lds[(t2 * TT + r) * S + lp]);
    }
    if (bsum) {                                        // lane (lp, r) sums the TT rows of t2 = r, r + TT, ...
        for (int t2 = r; t2 < N2; t2 += TT) {
            float2 acc = make_float2(0.f, 0.f);
#pragma unroll
            for (int i = 0; i < TT; ++i) acc = acc + IO::unpack(lds[(t2 * TT + i) * S + lp]);
            bsum[((size_t)bh * (N1 / TT) * N2 + (t1_0 / TT + (N1 / TT) * t2)) * 32 + p0 + lp] = acc;
        }
    }
}

// ------------------------------------------------------------------------------------------
// big: N1 = 16^P points per column, 16 per lane, P radix-16 passes each way with an LDS
// exchange between passes.  Forward passes are decimation in frequency (natural order in,
// base-16 digit-reversed order out), inverse passes undo them in reverse, so the gate is
// applied in digit-reversed order (the expanded gate is stored that way) and no reordering
// pass exists.  Pass q (0-based) has stride S = 16^(P-1-q): lane tau owns positions
// (tau / S) * 16 S + tau % S + S * j, j = 0..15.  LDS positions are padded by one element per
// 16 (p -> p + p/16); for S >= 16 that keeps a lane's 16 positions an arithmetic sequence.
//
// Only the exchange between passes 0 and 1 of a 4096-point column crosses waves; every other
// exchange stays inside a group of 16 lanes that own the same 256-position block, and needs no
// workgroup barrier because the LDS operations of one wave complete in issue order.  The forward
// and the inverse cross-wave exchange share one buffer (35 KB per workgroup, which leaves room on a
// compute unit for a row-transform workgroup of a neighbouring head group running on the other
// stream).  Between the two, lanes only touch the 256-position block they own, so the only extra
// barrier is at the end of a column: the next column's forward write lands on positions that
// slower waves may still be reading for the inverse exchange.
template <int P, int Q>
__device__ __forceinline__ int pad_base(int tau) {
    constexpr int S = 1 << (4 * (P - 1 - Q));
    if (S == 1) return 17 * tau;
    const int p = (tau / S) * (16 * S) + (tau % S);
    return p + (p >> 4);
}
template <int P, int Q>
__device__ constexpr int pad_stride() {
    constexpr int S = 1 << (4 * (P - 1 - Q));
    return S == 1 ? 1 : S + S / 16;
}

// write at pass QFROM's positions, read at pass QTO's.  CROSS: other waves take part.
template <int P, int QFROM, int QTO, bool CROSS>
__device__ __forceinline__ void exchange(float2 (&x)[16], float2 *buf, int tau) {
    float2 *w = buf + pad_base<P, QFROM>(tau);
    const float2 *r = buf + pad_base<P, QTO>(tau);
#pragma unroll
    for (int j = 0; j < 16; ++j) w[j * pad_stride<P, QFROM>()] = x[j];
    if (CROSS) __syncthreads();
    else __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int j = 0; j < 16; ++j) x[j] = r[j * pad_stride<P, QTO>()];
    if (!CROSS) __builtin_amdgcn_wave_barrier();
}

// The same exchange inside a group of 16 lanes without LDS: a 16 x 16 transpose (register j of lane a <-> register
// a of lane j) as four steps, one per index bit m, each swapping the elements whose register bit and lane bit
// differ with the partner lane a ^ m, by DPP moves (rows of 16 lanes are the DPP rows of a wave).  For m = 4, 8 the
// lanes that receive are whole banks of four lanes, so two masked moves per value do the step; for m = 1, 2 the
// partner's value is fetched with a quad permutation and selected per lane.  Pure data movement: results are
// bit-identical to the LDS exchange.
template <int M>
__device__ __forceinline__ void transpose16_step(float (&v)[16], int a) {
#pragma unroll
    for (int j0 = 0; j0 < 16; ++j0) {
        if (j0 & M) continue;
        const int j1 = j0 | M;
        const int lo = __float_as_int(v[j0]), hi = __float_as_int(v[j1]);
        int nlo, nhi;
        if constexpr (M == 8) {          // lanes 8..15 take the partner's hi into lo; lanes 0..7 the partner's lo into hi
            nlo = __builtin_amdgcn_update_dpp(lo, hi, 0x118, 0xF, 0xC, false);   // row_shr:8, banks 2,3
            nhi = __builtin_amdgcn_update_dpp(hi, lo, 0x108, 0xF, 0x3, false);   // row_shl:8, banks 0,1
        } else if constexpr (M == 4) {
            nlo = __builtin_amdgcn_update_dpp(lo, hi, 0x114, 0xF, 0xA, false);   // row_shr:4, banks 1,3
            nhi = __builtin_amdgcn_update_dpp(hi, lo, 0x104, 0xF, 0x5, false);   // row_shl:4, banks 0,2
        } else {
            constexpr int ctrl = (M == 1) ? 0xB1 : 0x4E;                          // quad_perm [1,0,3,2] / [2,3,0,1]
            const int phi = __builtin_amdgcn_update_dpp(0, hi, ctrl, 0xF, 0xF, false);
            const int plo = __builtin_amdgcn_update_dpp(0, lo, ctrl, 0xF, 0xF, false);
            nlo = (a & M) ? phi : lo;
            nhi = (a & M) ? hi : plo;
        }
        v[j0] = __int_as_float(nlo);
        v[j1] = __int_as_float(nhi);
    }
}
__device__ __forceinline__ void transpose16(float2 (&x)[16], int tau) {
    const int a = tau & 15;
    float re[16], im[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) { re[j] = x[j].x; im[j] = x[j].y; }
    transpose16_step<8>(re, a); transpose16_step<8>(im, a);
    transpose16_step<4>(re, a); transpose16_step<4>(im, a);
    transpose16_step<2>(re, a); transpose16_step<2>(im, a);
    transpose16_step<1>(re, a); transpose16_step<1>(im, a);
#pragma unroll
    for (int j = 0; j < 16; ++j) x[j] = make_float2(re[j], im[j]);
}

// SHFL: the exchanges that stay inside 16 lanes go through transpose16 instead of LDS.
template <int P, int MODE, typename SC, bool SHFL = false>
__global__ __launch_bounds__(256) void k_big(typename SC::elem_t *__restrict__ scr, const float2 *__restrict__ gp,
                                             const float2 *__restrict__ twN1, int N2, int ppw, int bh0,
                                             int nplanes_xcd, int g_step, int aff) {
    static_assert(P == 2 || P == 3, "N1 is 256 or 4096");
    constexpr int N1 = 1 << (4 * P), TPC = N1 / 16, CPI = 256 / TPC, COLW = N1 + N1 / 16;
    constexpr bool kCross = (P == 3);                // does the pass 0 <-> 1 exchange span waves?
    extern __shared__ float2 lds_big[];
    const int tid = threadIdx.x, tau = tid % TPC, ci = tid / TPC;
    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  The 32/ppw workgroups
    // that share one (head, k2) plane of the expanded gate are given ids 8 apart, so they run on
    // the same XCD and the plane is fetched into one L2 instead of eight.
    const int groups = 32 / ppw;
    int blk = blockIdx.x;
    if (nplanes_xcd > 0) {
        const int xcd = blk & 7, idx = blk >> 3;
        blk = ((idx / groups) * 8 + xcd) * groups + idx % groups;
    }
    int pg = blk % groups;
    blk /= groups;
    int k2 = blk % N2, bhl = blk / N2;
    if (aff) {                                       // all planes of a head on one XCD, heads walked downwards
        int within;
        head_affine(blockIdx.x, N2 * groups, aff, true, &bhl, &within);
        pg = within % groups;
        k2 = within / groups;
    }
    float2 *buf_f = lds_big + ci * COLW;             // forward exchanges
    float2 *buf_i = buf_f;                           // inverse cross-wave exchange: same buffer

    float2 tw[P - 1][15];
#pragma unroll
    for (int q = 0; q < P - 1; ++q) {
        const int S = 1 << (4 * (P - 1 - q));
        const int i = tau % S, step = N1 / (16 * S);
#pragma unroll
        for (int u = 1; u < 16; ++u) tw[q][u - 1] = twN1[i * u * step];
    }
    float2 G[16];
    if (MODE == 0) {
        const float2 *gsrc = gp + ((size_t)(bh0 + bhl * g_step) * N2 + k2) * N1;   // g_step 0: one gate for all
#pragma unroll
        for (int j = 0; j < 16; ++j) G[j] = gsrc[j * TPC + tau];
    }

    typedef typename SC::elem_t elem_t;
    elem_t *col = scr + (((size_t)bhl * N2 + k2) * 32 + pg * ppw + ci) * N1;
    // entry j * TPC + tau of a column <-> register j of lane tau, on the way in and on the way out, in every mode
    // (so every access of a wave is a contiguous 512-byte run); see big_position() for the bin such an entry holds
    elem_t nx[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) nx[j] = col[tau + TPC * j];
    for (int c = ci; c < ppw; c += CPI) {
        float2 x[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) x[j] = SC::get(nx[j]);
        if (c + CPI < ppw) {                          // next column's loads fly during this one's passes
            const elem_t *ncol = col + (size_t)CPI * N1;
#pragma unroll
            for (int j = 0; j < 16; ++j) nx[j] = ncol[tau + TPC * j];
        }
        if (MODE != 2) {
            dft<16, false>(x);
#pragma unroll
            for (int u = 1; u < 16; ++u) x[u] = cmul(x[u], tw[0][u - 1]);
            if constexpr (SHFL && !kCross) transpose16(x, tau);
            else exchange<P, 0, 1, kCross>(x, buf_f, tau);
            dft<16, false>(x);
            if constexpr (P == 3) {
#pragma unroll
                for (int u = 1; u < 16; ++u) x[u] = cmul(x[u], tw[1][u - 1]);
                if constexpr (SHFL) transpose16(x, tau);
                else exchange<P, 1, 2, false>(x, buf_f, tau);
                dft<16, false>(x);
            }
        }
        if (MODE == 0) {
#pragma unroll
            for (int j = 0; j < 16; ++j) x[j] = cmul(x[j], G[j]);
        }
        if (MODE == 1) {
#pragma unroll
            for (int j = 0; j < 16; ++j) col[tau + TPC * j] = SC::put(x[j]);
            if (kCross) __syncthreads();              // buf_f is rewritten by the next column
        } else {
            dft<16, true>(x);
            if constexpr (P == 3) {
                if constexpr (SHFL) transpose16(x, tau);
                else exchange<P, 2, 1, false>(x, buf_f, tau);
#pragma unroll
                for (int u = 1; u < 16; ++u) x[u] = cmulc(x[u], tw[1][u - 1]);
                dft<16, true>(x);
            }
            if constexpr (SHFL && !kCross) transpose16(x, tau);
            else exchange<P, 1, 0, kCross>(x, buf_i, tau);
#pragma unroll
            for (int u = 1; u < 16; ++u) x[u] = cmulc(x[u], tw[0][u - 1]);
            dft<16, true>(x);
#pragma unroll
            for (int j = 0; j < 16; ++j) col[tau + TPC * j] = SC::put(x[j]);
            if (kCross) __syncthreads();              // the next column's forward write reuses the buffer
        }
        col += (size_t)CPI * N1;
    }
}

// ------------------------------------------------------------------------------------------
// fused: L = 4096.  A column of this length (32 KB as complex fp32) fits in LDS, so the three kernels above and the
// gate expansion collapse into one kernel and the tensor crosses HBM once each way.  A workgroup of 512 lanes owns
// four adjacent channel pairs of one head (16 or 32 contiguous bytes of every row), each column with its own padded
// exchange buffer (4 x 34 KB); its two groups of 256 lanes take two columns each, one after the other, with the big
// kernel's lane layout and register budget.
//   load : all lanes sweep the rows, lane pl = tid % 4 of a row reads pair pl into the buffer of column pl;
//   core : the big kernel's passes (forward, gate, inverse) from and to the column's buffer; register j of lane
//          tau holds bin 256 j + 16 (tau % 16) + tau / 16 after the forward passes (base-16 digit reversal), and
//          the gate is read there directly, Hermitian extension and the 1/L of the inverse transform included;
//   store: the mirror image of the load.
// The eight workgroups of a head share its rows; their ids are 8 apart, so they run on the same XCD and a row is
// fetched into one L2.  (The same construction for L = 8192, two columns per pair, leaves room for only two pairs
// per workgroup, i.e. 8-byte pieces of every row, and measured slower than the three kernels.)
template <typename IO>
__global__ __launch_bounds__(512) void k_fused(const typename IO::pair_t *__restrict__ v,
                                               const float2 *__restrict__ g,
                                               typename IO::pair_t *__restrict__ out,
                                               const float2 *__restrict__ twN1, int H, int BH) {
    typedef typename IO::pair_t pair_t;
    constexpr int P = 3, L = 4096, F = L / 2 + 1, COLW = L + L / 16, PP = 4, WPH = 32 / PP;
    constexpr int RPS = 512 / PP, NS = L / RPS;     // rows per sweep of the workgroup, sweeps
    constexpr int kBatch = 16;                      // sweeps whose loads are in flight together
    extern __shared__ float2 lds_fused[];
    const int tid = threadIdx.x, tau = tid & 255, grp = tid >> 8;
    const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
    const int bh = (idx / WPH) * 8 + xcd, part = idx % WPH;
    if (bh >= BH) return;                           // whole workgroup: the grid is padded to 8 heads
    const int b = bh / H, h = bh % H;
    const int pl = tid % PP, r0 = tid / PP;
    const size_t rs = (size_t)H * 32;
    const size_t off = (((size_t)b * L) * H + h) * 32 + part * PP + pl;

    for (int s0 = 0; s0 < NS; s0 += kBatch) {
        pair_t raw[kBatch];
#pragma unroll
        for (int s = 0; s < kBatch; ++s) raw[s] = v[off + (size_t)(r0 + RPS * (s0 + s)) * rs];
#pragma unroll
        for (int s = 0; s < kBatch; ++s) {
            const int r = r0 + RPS * (s0 + s);
            lds_fused[pl * COLW + r + (r >> 4)] = IO::unpack(raw[s]);
        }
    }
    __syncthreads();

    float2 tw[P - 1][15];
#pragma unroll
    for (int u = 1; u < 16; ++u) {
        tw[0][u - 1] = twN1[tau * u];
        tw[1][u - 1] = twN1[(tau & 15) * 16 * u];
    }
    const float2 *gh = g + (size_t)bh * F;
    const int kbase = 16 * (tau & 15) + (tau >> 4);
    const float scale = 1.0f / (float)L;
#pragma unroll 1
    for (int c = grp; c < PP; c += 2) {
        float2 *buf = lds_fused + c * COLW;
        float2 *own = buf + pad_base<P, 0>(tau);     // the lane's pass-0 positions: rows tau + 256 j
        float2 x[16], G[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int k = 256 * j + kbase;
            G[j] = gh[2 * k <= L ? k : L - k];
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) x[j] = own[j * pad_stride<P, 0>()];
        dft<16, false>(x);
#pragma unroll
        for (int u = 1; u < 16; ++u) x[u] = cmul(x[u], tw[0][u - 1]);
        exchange<P, 0, 1, true>(x, buf, tau);
        dft<16, false>(x);
#pragma unroll
        for (int u = 1; u < 16; ++u) x[u] = cmul(x[u], tw[1][u - 1]);
        exchange<P, 1, 2, false>(x, buf, tau);
        dft<16, false>(x);
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int k = 256 * j + kbase;
            float2 gv = make_float2(G[j].x * scale, G[j].y * scale);
            if (2 * k > L) gv.y = -gv.y;
            if (k == 0 || 2 * k == L) gv.y = 0.0f;
            x[j] = cmul(x[j], gv);
        }
        dft<16, true>(x);
        exchange<P, 2, 1, false>(x, buf, tau);
#pragma unroll
        for (int u = 1; u < 16; ++u) x[u] = cmulc(x[u], tw[1][u - 1]);
        dft<16, true>(x);
        exchange<P, 1, 0, true>(x, buf, tau);
#pragma unroll
        for (int u = 1; u < 16; ++u) x[u] = cmulc(x[u], tw[0][u - 1]);
        dft<16, true>(x);
#pragma unroll
        for (int j = 0; j < 16; ++j) own[j * pad_stride<P, 0>()] = x[j];   // nobody else touches these positions
    }
    __syncthreads();

    for (int s0 = 0; s0 < NS; s0 += kBatch) {
#pragma unroll
        for (int s = 0; s < kBatch; ++s) {
            const int r = r0 + RPS * (s0 + s);
            out[off + (size_t)r * rs] = IO::pack(lds_fused[pl * COLW + r + (r >> 4)]);
        }
    }
}

// ------------------------------------------------------------------------------------------
// gate_expand: g [BH][L/2+1] -> gp [BH][N2][N1] with gp[bh][k2][r] = ext(g)[k2 + N2 * big_position(r)] / L: entry
// r = j * N1/16 + tau of plane k2 is the bin that register j of lane tau of the big kernel holds after the forward
// passes, and ext = Hermitian extension with real DC and Nyquist bins.  Consecutive bins run over k2 first, so a
// workgroup loads runs of N2 consecutive bins and turns them in LDS into runs of consecutive entries of each plane.
//
// N1 = 256, where entry r of a plane is bin k1 = r: a workgroup takes 32 consecutive k1 of one
// head, i.e. 32 N2 consecutive bins, and writes 256-byte runs into each of the N2 planes.  Eight workgroups per head:
// one workgroup per head kept 32 compute units busy for 8 us with a chain of dependent loads and stores (a ninth
// of the whole call at L = 8192).
__global__ __launch_bounds__(256) void k_gate_expand256(const float2 *__restrict__ g, float2 *__restrict__ gp, int L,
                                                        int N2) {
    __shared__ float2 tile[32 * 33];
    const int tid = threadIdx.x, bh = blockIdx.y, F = L / 2 + 1, S = N2 + 1;
    const int k1_0 = blockIdx.x * 32, k0 = k1_0 * N2;
    const float scale = 1.0f / (float)L;
    const float2 *gh = g + (size_t)bh * F;
    for (int m = tid; m < 32 * N2; m += 256) {
        const int k = k0 + m;
        float2 val = gh[2 * k <= L ? k : L - k];
        if (2 * k > L) val.y = -val.y;
        if (k == 0 || 2 * k == L) val.y = 0.0f;
        tile[(m / N2) * S + m % N2] = make_float2(val.x * scale, val.y * scale);
    }
    __syncthreads();
    float2 *dst = gp + (size_t)bh * L + k1_0;
    for (int i = tid; i < 32 * N2; i += 256) {
        const int q = i & 31, k2 = i >> 5;
        dst[(size_t)k2 * 256 + q] = tile[q * S + k2];
    }
}

// N1 = 4096, one workgroup per (head, j, b): entries 256 j + 16 b + a, a = 0..15, of every plane are the bins
// k1 = 256 j + 16 a + b, i.e. 16 chunks of N2 consecutive bins, 16 N2 bins apart.  8192 small workgroups at 32 heads
// (two loads and two stores per lane); 512 workgroups that each walked 8192 bins in four dependent rounds took 18 us
// alone, and the expansion sits in front of the first column kernel of a call.
__global__ __launch_bounds__(256) void k_gate_expand4096(const float2 *__restrict__ g, float2 *__restrict__ gp, int L,
                                                         int N2) {
    __shared__ float2 tile[16 * 33];
    const int tid = threadIdx.x, bh = blockIdx.y, F = L / 2 + 1, S = N2 + 1;
    const int j = blockIdx.x >> 4, b = blockIdx.x & 15;
    const float scale = 1.0f / (float)L;
    const float2 *gh = g + (size_t)bh * F;
    for (int m = tid; m < 16 * N2; m += 256) {
        const int a = m / N2, k2 = m % N2;
        const int k = k2 + N2 * (256 * j + 16 * a + b);
        float2 val = gh[2 * k <= L ? k : L - k];
        if (2 * k > L) val.y = -val.y;
        if (k == 0 || 2 * k == L) val.y = 0.0f;
        tile[a * S + k2] = make_float2(val.x * scale, val.y * scale);
    }
    __syncthreads();
    float2 *dst = gp + (size_t)bh * L + 256 * j + 16 * b;
    for (int i = tid; i < 16 * N2; i += 256) {
        const int a = i & 15, k2 = i >> 4;
        dst[(size_t)k2 * 4096 + a] = tile[a * S + k2];
    }
}

// ------------------------------------------------------------------------------------------
bool pow2_split(int L, int *N1, int *N2, int *P) {
    if (L < 256 || L > 131072) return false;
    const bool by256 = (L % 256 == 0) && small_dft_supported(L / 256);
    const bool by4096 = (L % 4096 == 0) && small_dft_supported(L / 4096);
    // the in-register small transform is the cheaper place for stages, so N2 is made as large as 32 allows
    if (by256) { *N1 = 256; *P = 2; }
    else if (by4096) { *N1 = 4096; *P = 3; }
    else return false;
    *N2 = L / *N1;
    return true;
}

template <typename K>
static hipError_t allow_lds(K kernel, size_t bytes) {
    if (bytes <= 48 * 1024) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

template <int N2, int TT, typename IO, typename SC>
static hipError_t small_fwd_t(const Pow2Plan &pl, const void *v, void *scr_v, int rows, int H, int bh0,
                              int nbh, hipStream_t st, int aff, float2 *ring) {
    const size_t lds = (size_t)N2 * TT * TileStride<IO>::value * sizeof(typename IO::pair_t);
    auto kern = k_small_fwd<N2, TT, IO, SC>;
    typename SC::elem_t *scr = static_cast<typename SC::elem_t *>(scr_v);
    hipError_t e = allow_lds(kern, lds);
    if (e != hipSuccess) return e;
    constexpr int PW = RowTile<IO>::kPairs;
    const int tiles = pl.N1 / TT * (32 / PW);
    const dim3 grid = aff ? dim3(tiles * nbh) : dim3(tiles, nbh);
    kern<<<grid, dim3(PW * TT), lds, st>>>(
        static_cast<const typename IO::pair_t *>(v), scr, pl.twL, rows, H, pl.N1, bh0, aff, ring);
    return hipGetLastError();
}

template <int N2, int TT, typename IO, typename SC>
static hipError_t small_inv_t(const Pow2Plan &pl, const void *scr_v, void *out, int row0, int out_rows,
                              int H, int bh0, int nbh, hipStream_t st, int ring0, int ring_w, int newest, int aff,
                              float2 *bsum) {
    const size_t lds = (size_t)N2 * TT * TileStride<IO>::value * sizeof(typename IO::pair_t);
    auto kern = k_small_inv<N2, TT, IO, SC>;
    const typename SC::elem_t *scr = static_cast<const typename SC::elem_t *>(scr_v);
    hipError_t e = allow_lds(kern, lds);
    if (e != hipSuccess) return e;
    constexpr int PW = RowTile<IO>::kPairs;
    const int tiles = pl.N1 / TT * (32 / PW);
    const dim3 grid = aff ? dim3(tiles * nbh) : dim3(tiles, nbh);
    kern<<<grid, dim3(PW * TT), lds, st>>>(
        scr, static_cast<typename IO::pair_t *>(out), pl.twL, row0, out_rows, H, pl.N1, bh0, ring0, ring_w, newest, aff,
        bsum);
    return hipGetLastError();
}

#define SPECTRE_N2_CASE(FN, N, ...) \
    case N: return io ? (scr16 ? FN<N, 16, IoBf16, ScrBf16>(__VA_ARGS__) : FN<N, 16, IoBf16, ScrF32>(__VA_ARGS__)) \
                      : FN<N, 16, IoF32, ScrF32>(__VA_ARGS__);
#define SPECTRE_DISPATCH_N2(FN, ...)                                         \
    switch (pl.N2) {                                                         \
        SPECTRE_N2_CASE(FN, 1, __VA_ARGS__) SPECTRE_N2_CASE(FN, 2, __VA_ARGS__) SPECTRE_N2_CASE(FN, 3, __VA_ARGS__)    \
        SPECTRE_N2_CASE(FN, 4, __VA_ARGS__) SPECTRE_N2_CASE(FN, 5, __VA_ARGS__) SPECTRE_N2_CASE(FN, 6, __VA_ARGS__)    \
        SPECTRE_N2_CASE(FN, 7, __VA_ARGS__) SPECTRE_N2_CASE(FN, 8, __VA_ARGS__) SPECTRE_N2_CASE(FN, 10, __VA_ARGS__)   \
        SPECTRE_N2_CASE(FN, 12, __VA_ARGS__) SPECTRE_N2_CASE(FN, 14, __VA_ARGS__) SPECTRE_N2_CASE(FN, 16, __VA_ARGS__) \
        SPECTRE_N2_CASE(FN, 20, __VA_ARGS__) SPECTRE_N2_CASE(FN, 24, __VA_ARGS__) SPECTRE_N2_CASE(FN, 28, __VA_ARGS__) \
        SPECTRE_N2_CASE(FN, 32, __VA_ARGS__)                                 \
        default: return hipErrorInvalidValue;                                \
    }

hipError_t launch_small_fwd(const Pow2Plan &pl, int io, const void *v, float2 *scratch, int rows, int H,
                            int bh0, int nbh, hipStream_t st, bool scr16, bool affine, float2 *ring) {
    if (scr16 && !io) return hipErrorInvalidValue;
    if (affine && nbh % 8 != 0) return hipErrorInvalidValue;
    const int aff = affine ? nbh : 0;
    SPECTRE_DISPATCH_N2(small_fwd_t, pl, v, scratch, rows, H, bh0, nbh, st, aff, ring)
}

template <int N2, int TT, typename IO, typename SC>
static hipError_t small_fwd_proj_t(const Pow2Plan &pl, const void *x, const void *wpack, int Hw, void *scr_v, int rows,
                                   int H, int bh0, int nbh, hipStream_t st, int aff) {
    if (!std::is_same<IO, IoBf16>::value || !std::is_same<SC, ScrF32>::value) return hipErrorInvalidValue;
    const size_t lds = (size_t)N2 * 16 * TileStride<IoBf16>::value * sizeof(uint32_t);
    auto kern = k_small_fwd_proj<N2>;
    hipError_t e = allow_lds(kern, lds);
    if (e != hipSuccess) return e;
    const dim3 grid = aff ? dim3(pl.N1 / 16 * nbh) : dim3(pl.N1 / 16, nbh);
    kern<<<grid, dim3(512), lds, st>>>(static_cast<const uint32_t *>(x), static_cast<const uint4 *>(wpack), Hw,
                                       static_cast<float2 *>(scr_v), pl.twL, rows, H, pl.N1, bh0, aff);
    return hipGetLastError();
}

hipError_t launch_small_fwd_proj(const Pow2Plan &pl, const void *x, const void *wpack, int Hw, float2 *scratch, int rows,
                                 int H, int bh0, int nbh, hipStream_t st, bool affine) {
    if (affine && nbh % 8 != 0) return hipErrorInvalidValue;
    const int aff = affine ? nbh : 0;
    const int io = 1;
    const bool scr16 = false;
    SPECTRE_DISPATCH_N2(small_fwd_proj_t, pl, x, wpack, Hw, scratch, rows, H, bh0, nbh, st, aff)
}

int small_tile_rows(int io) { (void)io; return 16; }

hipError_t launch_small_inv(const Pow2Plan &pl, int io, const float2 *scratch, void *out, int row0,
                            int out_rows, int H, int bh0, int nbh, hipStream_t st, int ring0, int ring_w,
                            int newest, bool scr16, bool affine, float2 *bsum) {
    if (scr16 && !io) return hipErrorInvalidValue;
    if (affine && nbh % 8 != 0) return hipErrorInvalidValue;
    if (bsum && (row0 != 0 || out_rows != pl.L || ring_w > 0)) return hipErrorInvalidValue;   // whole transforms only
    const int aff = affine ? nbh : 0;
    SPECTRE_DISPATCH_N2(small_inv_t, pl, scratch, out, row0, out_rows, H, bh0, nbh, st, ring0, ring_w, newest, aff,
                        bsum)
}

template <int P, int MODE, typename SC = ScrF32, bool SHFL = false>
static hipError_t big_t(const Pow2Plan &pl, float2 *scr_v, const float2 *gp, int bh0, int nbh, bool shared_gate,
                        hipStream_t st, int aff = 0, bool wide = false) {
    constexpr int N1 = 1 << (4 * P), TPC = N1 / 16, CPI = 256 / TPC, COLW = N1 + N1 / 16;
    const size_t lds = (size_t)CPI * COLW * sizeof(float2);
    // pairs per workgroup; a multiple of CPI dividing 32.  `wide` (a call whose head groups alternate between two
    // streams): 8 columns per workgroup, so that a group's column kernel is fewer workgroups than the chip has room for
    // and the other stream's row kernels run beside it from its first to its last workgroup (-1.5 % at L = 131072; on
    // one stream the longer workgroups cost 2 %)
    const int ppw = (P == 2) ? 16 : (wide ? 8 : 4);
    auto kern = k_big<P, MODE, SC, SHFL>;
    typename SC::elem_t *scr = reinterpret_cast<typename SC::elem_t *>(scr_v);
    hipError_t e = allow_lds(kern, lds);
    if (e != hipSuccess) return e;
    const unsigned grid = (unsigned)nbh * pl.N2 * (32 / ppw);
    const int planes = nbh * pl.N2;                    // remapping needs the plane count to split 8 ways
    kern<<<dim3(grid), dim3(256), lds, st>>>(scr, gp, pl.twN1, pl.N2, ppw, bh0, planes % 8 == 0 ? planes : 0,
                                             shared_gate ? 0 : 1, aff);
    return hipGetLastError();
}

hipError_t launch_big(const Pow2Plan &pl, float2 *scratch, const float2 *gp, int bh0, int nbh, int mode,
                      hipStream_t st, bool shared_gate, bool scr16, bool affine, bool wide) {
    const bool shfl = option(SPECTRE_OPT_LANE_SHUFFLES) != 0 && mode == 0 && !scr16;
    if (affine) {                                      // the mixer's forward-gate-inverse pass, fp32 scratch
        if (mode != 0 || scr16 || nbh % 8 != 0) return hipErrorInvalidValue;
        if (pl.P == 2) return shfl ? big_t<2, 0, ScrF32, true>(pl, scratch, gp, bh0, nbh, shared_gate, st, nbh)
                                   : big_t<2, 0>(pl, scratch, gp, bh0, nbh, shared_gate, st, nbh);
        if (pl.P == 3) return shfl ? big_t<3, 0, ScrF32, true>(pl, scratch, gp, bh0, nbh, shared_gate, st, nbh)
                                   : big_t<3, 0>(pl, scratch, gp, bh0, nbh, shared_gate, st, nbh);
        return hipErrorInvalidValue;
    }
    if (shfl) {
        if (pl.P == 2) return big_t<2, 0, ScrF32, true>(pl, scratch, gp, bh0, nbh, shared_gate, st);
        if (pl.P == 3) return big_t<3, 0, ScrF32, true>(pl, scratch, gp, bh0, nbh, shared_gate, st);
        return hipErrorInvalidValue;
    }
    if (scr16) {                                       // the mixer's forward-gate-inverse pass only
        if (mode != 0) return hipErrorInvalidValue;
        if (pl.P == 2) return big_t<2, 0, ScrBf16>(pl, scratch, gp, bh0, nbh, shared_gate, st);
        if (pl.P == 3) return big_t<3, 0, ScrBf16>(pl, scratch, gp, bh0, nbh, shared_gate, st);
        return hipErrorInvalidValue;
    }
    if (pl.P == 2) {
        if (mode == 0) return big_t<2, 0>(pl, scratch, gp, bh0, nbh, shared_gate, st);
        if (mode == 1) return big_t<2, 1>(pl, scratch, gp, bh0, nbh, shared_gate, st);
        if (mode == 2) return big_t<2, 2>(pl, scratch, gp, bh0, nbh, shared_gate, st);
    } else if (pl.P == 3) {
        if (mode == 0) return big_t<3, 0>(pl, scratch, gp, bh0, nbh, shared_gate, st, 0, wide);
        if (mode == 1) return big_t<3, 1>(pl, scratch, gp, bh0, nbh, shared_gate, st);
        if (mode == 2) return big_t<3, 2>(pl, scratch, gp, bh0, nbh, shared_gate, st);
    }
    return hipErrorInvalidValue;
}

bool fused_supported(int L) { return L == 4096; }

template <typename IO>
static hipError_t fused_t(const void *v, const float2 *g, void *out, const float2 *twN1, int H, int BH,
                          hipStream_t st) {
    constexpr int COLW = 4096 + 4096 / 16;
    const size_t lds = (size_t)4 * COLW * sizeof(float2);
    auto kern = k_fused<IO>;
    hipError_t e = allow_lds(kern, lds);
    if (e != hipSuccess) return e;
    const long long grid = (long long)((BH + 7) / 8) * 8 * 8;   // heads padded to 8, 8 workgroups per head
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    kern<<<dim3((unsigned)grid), dim3(512), lds, st>>>(static_cast<const typename IO::pair_t *>(v), g,
                                                       static_cast<typename IO::pair_t *>(out), twN1, H, BH);
    return hipGetLastError();
}

hipError_t launch_fused(int io, const void *v, const float2 *g, void *out, const float2 *tw4096, int L, int H, int BH,
                        hipStream_t st) {
    if (!fused_supported(L)) return hipErrorInvalidValue;
    return io ? fused_t<IoBf16>(v, g, out, tw4096, H, BH, st) : fused_t<IoF32>(v, g, out, tw4096, H, BH, st);
}

hipError_t launch_gate_expand(const Pow2Plan &pl, const float2 *g, float2 *gp, int BH, hipStream_t st) {
    if (pl.P != 2 && pl.P != 3) return hipErrorInvalidValue;
    for (int bh0 = 0; bh0 < BH; bh0 += 65535) {         // grid.y limit
        const int n = (BH - bh0 < 65535) ? BH - bh0 : 65535;
        const int F = pl.L / 2 + 1;
        if (pl.P == 2)
            k_gate_expand256<<<dim3(8, n), dim3(256), 0, st>>>(g + (size_t)bh0 * F, gp + (size_t)bh0 * pl.L, pl.L, pl.N2);
        else
            k_gate_expand4096<<<dim3(256, n), dim3(256), 0, st>>>(g + (size_t)bh0 * F, gp + (size_t)bh0 * pl.L, pl.L, pl.N2);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Loads this translation unit's code object (the runtime loads them on first use): called by spectre_prepare so
// that no compute call is the first to touch it.
hipError_t load_kernels_mix_pow2() {
    hipFuncAttributes a;
    return hipFuncGetAttributes(&a, reinterpret_cast<const void *>(k_gate_expand256));
}

}  // namespace spectre
