// Short-sequence path of the SPECTRE mixing layer (Sec. 3.2 steps 2-4, Eq. 3 and Eq. 4):
// one workgroup owns the whole [L, d = 64] slab of one head of one sequence in LDS.
//
// Serves every L <= 512 whose prime factors are in {2, 3, 5, 7} - in particular the
// 14 x 14 = 196 = 4 * 7 * 7 patch grid of the ViT workload and power-of-two lengths
// below 256.  Channel pairs are transformed as complex sequences (see mix_pow2.hip).
// The transform is an in-place mixed-radix decimation-in-frequency FFT: after the last
// forward pass position p holds bin k = reverse(p) (mixed-radix digit reversal), the gate
// is applied in that order from a per-workgroup table, and the inverse passes undo the
// forward ones in reverse, so nothing is ever reordered.
#include "mix_slab.h"

#include <stdlib.h>

#include <vector>

#include "fft_regs.h"
#include "internal.h"

namespace spectre {

template <int R, bool INV>
__device__ __forceinline__ void dft_any(float2 (&x)[R]) {
    small_dft<R, INV>(x);
}

// One in-place pass over all 32 columns of the slab.  n = current sub-transform length,
// S = n / R its stride; roots[m] = exp(-j 2 pi m / L).  Forward: butterfly then twiddle (and
// the gate, when GATE, which makes this the last forward pass).  Inverse: conjugate twiddle then
// inverse butterfly.
// UNIT: n == R, every twiddle is 1 and is skipped.
template <int R, bool INV, bool GATE, bool UNIT, int PP>
__device__ __forceinline__ void slab_pass(float2 *__restrict__ slab, const float2 *__restrict__ roots,
                                          const float2 *__restrict__ gpos, int L, int n, int tid, int nthreads) {
    constexpr int kShift = (PP == 32) ? 5 : (PP == 16) ? 4 : (PP == 8) ? 3 : 2;
    static_assert(PP == 32 || PP == 16 || PP == 8 || PP == 4, "pairs per workgroup");
    const int S = n / R, tstep = L / n;
    const int nb = (L / R) * PP;
    // bi / S by a multiply and shift: exact while bi * S < 2^20 (bi < L/R <= 1024, S <= L/R)
    const unsigned inv_s = ((1u << 20) + (unsigned)S - 1) / (unsigned)S;
    for (int w = tid; w < nb; w += nthreads) {
        const int col = w & (PP - 1), bi = w >> kShift;
        const int blk = (int)(((unsigned)bi * inv_s) >> 20), i = bi - blk * S;
        const int base = blk * n + i;
        float2 x[R];
#pragma unroll
        for (int j = 0; j < R; ++j) x[j] = slab[(base + S * j) * PP + col];
        if (INV && !UNIT) {
#pragma unroll
            for (int u = 1; u < R; ++u) x[u] = cmulc(x[u], roots[i * u * tstep]);
        }
        dft_any<R, INV>(x);
        if (!INV) {
            if (!UNIT) {
#pragma unroll
                for (int u = 1; u < R; ++u) x[u] = cmul(x[u], roots[i * u * tstep]);
            }
            if (GATE) {
#pragma unroll
                for (int u = 0; u < R; ++u) x[u] = cmul(x[u], gpos[base + S * u]);
            }
        }
#pragma unroll
        for (int j = 0; j < R; ++j) slab[(base + S * j) * PP + col] = x[j];
    }
}

template <bool INV, bool GATE, bool UNIT, int PP>
__device__ __forceinline__ void slab_pass_dispatch(int R, float2 *slab, const float2 *roots, const float2 *gpos,
                                                   int L, int n, int tid, int nthreads) {
    switch (R) {
        case 2: slab_pass<2, INV, GATE, UNIT, PP>(slab, roots, gpos, L, n, tid, nthreads); break;
        case 3: slab_pass<3, INV, GATE, UNIT, PP>(slab, roots, gpos, L, n, tid, nthreads); break;
        case 4: slab_pass<4, INV, GATE, UNIT, PP>(slab, roots, gpos, L, n, tid, nthreads); break;
        case 5: slab_pass<5, INV, GATE, UNIT, PP>(slab, roots, gpos, L, n, tid, nthreads); break;
        case 6: slab_pass<6, INV, GATE, UNIT, PP>(slab, roots, gpos, L, n, tid, nthreads); break;
        case 7: slab_pass<7, INV, GATE, UNIT, PP>(slab, roots, gpos, L, n, tid, nthreads); break;
        case 8: slab_pass<8, INV, GATE, UNIT, PP>(slab, roots, gpos, L, n, tid, nthreads); break;
        case 10: slab_pass<10, INV, GATE, UNIT, PP>(slab, roots, gpos, L, n, tid, nthreads); break;
        case 12: slab_pass<12, INV, GATE, UNIT, PP>(slab, roots, gpos, L, n, tid, nthreads); break;
        case 14: slab_pass<14, INV, GATE, UNIT, PP>(slab, roots, gpos, L, n, tid, nthreads); break;
        case 16: slab_pass<16, INV, GATE, UNIT, PP>(slab, roots, gpos, L, n, tid, nthreads); break;
        default: break;
    }
}

struct SlabRadices {
    int count;
    int r[10];
};

// Lengths whose radix list is also known at compile time (it must equal what slab_radices() returns on the host,
// which the launcher checks): the kernel variant for such a length has every LDS offset, stride and twiddle index
// folded into its instructions (55-80 registers instead of 120, no address arithmetic left in the passes).
template <int LC> struct CtRadices;
template <> struct CtRadices<196> { static constexpr int count = 2, r0 = 14, r1 = 14, r2 = 1; };
template <> struct CtRadices<256> { static constexpr int count = 2, r0 = 16, r1 = 16, r2 = 1; };
template <> struct CtRadices<512> { static constexpr int count = 3, r0 = 16, r1 = 16, r2 = 2; };
template <> struct CtRadices<1024> { static constexpr int count = 3, r0 = 16, r1 = 16, r2 = 4; };
template <> struct CtRadices<2048> { static constexpr int count = 3, r0 = 16, r1 = 16, r2 = 8; };

// grid = B*H*(32/PP) workgroups of 256 lanes, PP channel pairs each: a whole head, half a head when rows
// are fp32 (still full 128-byte row segments, half the LDS, twice the workgroups per CU), or as little as
// 4 pairs when there are few heads (then the call is one launch over every compute unit instead of four
// dependent ones) or the sequence is long (the slab must fit in LDS).
// LDS: slab [L][PP] float2, roots [L], gpos [L].
// NT = lanes per workgroup.  LC = 0: the length and its radices are run-time arguments; LC > 0: compile-time
// constants (CtRadices).  For LC = 196 (the 14 x 14 patch grid, radices 14, 14) with NT = 448, PP = 32 the 14 * 32
// butterflies of a pass fill seven waves exactly (224 of 256 lanes with NT = 256, PP = 16) and a lane loads and
// stores exactly 14 rows.
template <typename IO, int PP, int NT = 256, int LC = 0>
__global__ __launch_bounds__(NT) void k_mix_slab(const typename IO::pair_t *__restrict__ v,
                                                 const float2 *__restrict__ g,
                                                 typename IO::pair_t *__restrict__ out,
                                                 const float2 *__restrict__ roots_g,
                                                 const int *__restrict__ bin_of_pos, int L_arg, int H,
                                                 SlabRadices rad, int rows) {
    const int L = LC ? LC : L_arg;
    extern __shared__ float2 lds_slab[];
    float2 *slab = lds_slab;
    float2 *roots = slab + (size_t)L * PP;
    float2 *gpos = roots + L;
    constexpr int kParts = 32 / PP, kRows = NT / PP;       // workgroups per head; rows covered per sweep
    static_assert(NT % PP == 0 && NT % 64 == 0, "whole rows per sweep, whole waves");
    const int tid = threadIdx.x;
    const int bh = blockIdx.x / kParts, part = blockIdx.x % kParts, b = bh / H, h = bh % H;
    const int F = L / 2 + 1;

    // rows l = tid/PP + kRows i.  Sixteen loads are put in flight before any is consumed (all 196 rows of
    // the ViT grid at once for fp32 half heads); the first batch flies while the gate table below is built.
    const int lp_in = tid & (PP - 1), row_in = tid / PP;
    // the tensors hold `rows` <= L rows per sequence; the transform sees them followed by zeros and only the first
    // `rows` rows of the result are kept (zero-padded linear convolution)
    const typename IO::pair_t *src = v + (((size_t)b * rows) * H + h) * 32 + part * PP + lp_in;
    const size_t rs = (size_t)H * 32;
    constexpr int kBatch = 16;
    typename IO::pair_t val[kBatch];
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
        const int l = row_in + kRows * i;
        val[i] = (l < rows) ? src[(size_t)l * rs] : IO::zero();
    }

    // roots of unity and the gate in position order (bin_of_pos[p] = the bin that position p holds after
    // the last forward pass); full-length Hermitian extension, 1/L folded in.  The two dependent loads
    // (bin, then gate) are issued for all of a lane's positions at once: L <= 2048 = 8 * 256.
    {
        constexpr int kPos = ((LC ? LC : kSlabMaxL) + NT - 1) / NT;
        int kbin[kPos];
        float2 gv[kPos], rv[kPos];
#pragma unroll
        for (int i = 0; i < kPos; ++i) {
            const int p = tid + NT * i;
            kbin[i] = (p < L) ? bin_of_pos[p] : 0;
            rv[i] = (p < L) ? roots_g[p] : make_float2(0.f, 0.f);
        }
#pragma unroll
        for (int i = 0; i < kPos; ++i) {
            const int k = kbin[i];
            gv[i] = (tid + NT * i < L) ? g[(size_t)bh * F + (2 * k <= L ? k : L - k)] : make_float2(0.f, 0.f);
        }
        const float sc = 1.0f / (float)L;
#pragma unroll
        for (int i = 0; i < kPos; ++i) {
            const int p = tid + NT * i, k = kbin[i];
            if (p < L) {
                float2 val = gv[i];
                if (2 * k > L) val.y = -val.y;
                if (k == 0 || 2 * k == L) val.y = 0.f;
                roots[p] = rv[i];
                gpos[p] = make_float2(val.x * sc, val.y * sc);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
        const int l = row_in + kRows * i;
        if (l < L) slab[l * PP + lp_in] = IO::unpack(val[i]);
    }
    for (int l0 = row_in + kBatch * kRows; l0 < L; l0 += kBatch * kRows) {
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
            const int l = l0 + kRows * i;
            val[i] = (l < rows) ? src[(size_t)l * rs] : IO::zero();
        }
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
            const int l = l0 + kRows * i;
            if (l < L) slab[l * PP + lp_in] = IO::unpack(val[i]);
        }
    }
    __syncthreads();
    if constexpr (LC != 0) {
        typedef CtRadices<LC> R;
        constexpr int n0 = LC, n1 = n0 / R::r0, n2 = n1 / R::r1;
        static_assert((R::count == 2 && n1 == R::r1) || (R::count == 3 && n2 == R::r2), "radices multiply to LC");
        slab_pass<R::r0, false, false, false, PP>(slab, roots, gpos, LC, n0, tid, NT);
        __syncthreads();
        if constexpr (R::count == 3) {
            slab_pass<R::r1, false, false, false, PP>(slab, roots, gpos, LC, n1, tid, NT);
            __syncthreads();
            slab_pass<R::r2, false, true, true, PP>(slab, roots, gpos, LC, n2, tid, NT);
            __syncthreads();
            slab_pass<R::r2, true, false, true, PP>(slab, roots, gpos, LC, n2, tid, NT);
            __syncthreads();
            slab_pass<R::r1, true, false, false, PP>(slab, roots, gpos, LC, n1, tid, NT);
            __syncthreads();
        } else {
            slab_pass<R::r1, false, true, true, PP>(slab, roots, gpos, LC, n1, tid, NT);
            __syncthreads();
            slab_pass<R::r1, true, false, true, PP>(slab, roots, gpos, LC, n1, tid, NT);
            __syncthreads();
        }
        slab_pass<R::r0, true, false, false, PP>(slab, roots, gpos, LC, n0, tid, NT);
        __syncthreads();
    } else {
        int n = L;
        for (int q = 0; q < rad.count; ++q) {
            if (q == rad.count - 1) slab_pass_dispatch<false, true, true, PP>(rad.r[q], slab, roots, gpos, L, n, tid, NT);
            else slab_pass_dispatch<false, false, false, PP>(rad.r[q], slab, roots, gpos, L, n, tid, NT);
            n /= rad.r[q];
            __syncthreads();
        }
        for (int q = rad.count - 1; q >= 0; --q) {
            n *= rad.r[q];
            if (q == rad.count - 1) slab_pass_dispatch<true, false, true, PP>(rad.r[q], slab, roots, gpos, L, n, tid, NT);
            else slab_pass_dispatch<true, false, false, PP>(rad.r[q], slab, roots, gpos, L, n, tid, NT);
            __syncthreads();
        }
    }
    {
        typename IO::pair_t *dst = out + (((size_t)b * rows) * H + h) * 32 + part * PP + lp_in;
        for (int l = row_in; l < rows; l += kRows) dst[(size_t)l * rs] = IO::pack(slab[l * PP + lp_in]);
    }
}

// ------------------------------------------------------------------------------------------
bool slab_supported(int L) {
    if (L < 2 || L > kSlabMaxL) return false;
    int n = L;
    for (int p : {2, 3, 5, 7})
        while (n % p == 0) n /= p;
    return n == 1;
}

// Fewest passes with radices from {16, 14, 12, 10, 8, 7, 6, 5, 4, 3, 2} (each a power of two times at most one
// of 3, 5, 7, which the in-register transform handles without twiddles); larger radices first.
static int slab_best_count(int n, int *memo) {
    if (n == 1) return 0;
    if (memo[n] != 0) return memo[n];
    int best = 1 << 20;
    for (int r : {16, 14, 12, 10, 8, 7, 6, 5, 4, 3, 2})
        if (n % r == 0) {
            const int c = 1 + slab_best_count(n / r, memo);
            if (c < best) best = c;
        }
    return memo[n] = best;
}

static SlabRadices slab_radices(int L) {
    SlabRadices r;
    r.count = 0;
    std::vector<int> memo((size_t)L + 1, 0);
    int n = L;
    while (n > 1 && r.count < 10) {
        const int want = slab_best_count(n, memo.data());
        if (want >= (1 << 20)) break;                      // not smooth: callers check slab_supported first
        for (int c : {16, 14, 12, 10, 8, 7, 6, 5, 4, 3, 2})
            if (n % c == 0 && 1 + slab_best_count(n / c, memo.data()) == want) {
                r.r[r.count++] = c;
                n /= c;
                break;
            }
    }
    return r;
}

// Position p = sum_q u_q S_q (S_q = stride of pass q) holds bin k = sum_q u_q (R_1 ... R_(q-1)) after the
// forward passes: mixed-radix digit reversal.
void slab_bin_order(int L, int *bin_of_pos) {
    const SlabRadices rad = slab_radices(L);
    for (int p = 0; p < L; ++p) {
        int rem = p, n = L, k = 0, w = 1;
        for (int q = 0; q < rad.count; ++q) {
            const int S = n / rad.r[q];
            const int u = rem / S;
            rem -= u * S;
            k += u * w;
            w *= rad.r[q];
            n = S;
        }
        bin_of_pos[p] = k;
    }
}

template <typename IO, int PP, int NT = 256, int LC = 0>
static hipError_t mix_slab_t(const void *v, const float2 *g, void *out, const float2 *roots, const int *bin_of_pos,
                             int B, int L, int H, int rows, hipStream_t st) {
    const size_t lds = ((size_t)L * PP + 2 * (size_t)L) * sizeof(float2);
    const SlabRadices rad = slab_radices(L);
    auto kern = k_mix_slab<IO, PP, NT, LC>;
    if constexpr (LC != 0) {
        typedef CtRadices<LC> R;
        if (L != LC || rad.count != R::count || rad.r[0] != R::r0 || rad.r[1] != R::r1 ||
            (R::count == 3 && rad.r[2] != R::r2))
            return hipErrorInvalidValue;
    }
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    kern<<<dim3(B * H * (32 / PP)), dim3(NT), lds, st>>>(static_cast<const typename IO::pair_t *>(v), g,
                                                         static_cast<typename IO::pair_t *>(out), roots, bin_of_pos, L, H,
                                                         rad, rows);
    return hipGetLastError();
}

// Pairs per workgroup: as many as leave room for three workgroups per compute unit (slab L*PP + two tables of L
// complex numbers <= 52 KB; measured at B*H = 3072: L = 512 and the padded 197 are 5-24 % faster with 8 pairs than
// with 16, L = 256 bf16 30 % faster with 16 than with 32), no more than keeps every compute unit busy
// (B*H*32/PP >= 256 workgroups), at most a whole head (half a head for fp32 rows).
int slab_pairs_per_workgroup(int io, int BH, int L) {
    int pp = io ? 32 : 16;
    while (pp > 4 && (size_t)L * (pp + 2) * sizeof(float2) > (size_t)52 * 1024) pp /= 2;   // three workgroups per CU
    while (pp > 4 && (long long)BH * (32 / pp) < 256) pp /= 2;
    return pp;
}

hipError_t launch_mix_slab(int io, const void *v, const float2 *g, void *out, const float2 *roots,
                           const int *bin_of_pos, int B, int L, int H, hipStream_t st, int rows) {
    if (rows <= 0) rows = L;
    if (rows > L) return hipErrorInvalidValue;
    const int pp = slab_pairs_per_workgroup(io, B * H, L);
    if ((size_t)L * (pp + 2) * sizeof(float2) > (size_t)160 * 1024) return hipErrorInvalidValue;
    if (L == 196 && pp >= 16 && (long long)B * H >= 512 && option(SPECTRE_OPT_SLAB_COMPILE_TIME) != 0)   // whole heads still fill the chip
        return io ? mix_slab_t<IoBf16, 32, 448, 196>(v, g, out, roots, bin_of_pos, B, L, H, rows, st)
                  : mix_slab_t<IoF32, 32, 448, 196>(v, g, out, roots, bin_of_pos, B, L, H, rows, st);
    const bool ct = option(SPECTRE_OPT_SLAB_COMPILE_TIME) != 0;
#define SPECTRE_SLAB_LEN(PPV, LCV)                                                                          \
    if (ct && L == LCV)                                                                                     \
        return io ? mix_slab_t<IoBf16, PPV, 256, LCV>(v, g, out, roots, bin_of_pos, B, L, H, rows, st)      \
                  : mix_slab_t<IoF32, PPV, 256, LCV>(v, g, out, roots, bin_of_pos, B, L, H, rows, st);
#define SPECTRE_SLAB_CASE(PPV, LENS)                                                                 \
    case PPV:                                                                                       \
        LENS                                                                                        \
        return io ? mix_slab_t<IoBf16, PPV>(v, g, out, roots, bin_of_pos, B, L, H, rows, st)        \
                  : mix_slab_t<IoF32, PPV>(v, g, out, roots, bin_of_pos, B, L, H, rows, st);
    switch (pp) {                       // only the (pairs, length) combinations the rule above can produce
        SPECTRE_SLAB_CASE(4, SPECTRE_SLAB_LEN(4, 256) SPECTRE_SLAB_LEN(4, 512) SPECTRE_SLAB_LEN(4, 1024) SPECTRE_SLAB_LEN(4, 2048))
        SPECTRE_SLAB_CASE(8, SPECTRE_SLAB_LEN(8, 256) SPECTRE_SLAB_LEN(8, 512))
        SPECTRE_SLAB_CASE(16, SPECTRE_SLAB_LEN(16, 256) SPECTRE_SLAB_LEN(16, 512))
        SPECTRE_SLAB_CASE(32, SPECTRE_SLAB_LEN(32, 256))
        default: return hipErrorInvalidValue;
    }
#undef SPECTRE_SLAB_LEN
#undef SPECTRE_SLAB_CASE
}

// Loads this translation unit's code object (the runtime loads them on first use): called by spectre_prepare so
// that no compute call is the first to touch it.
hipError_t load_kernels_mix_slab() {
    hipFuncAttributes a;
    return hipFuncGetAttributes(&a, reinterpret_cast<const void *>((k_mix_slab<IoF32, 4, 256, 0>)));
}

}  // namespace spectre
