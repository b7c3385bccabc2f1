/*
 * spectre.h - C ABI of the MI355X (gfx950) SPECTRE spectral-mixing library.
 *
 * SPECTRE replaces each self-attention head by a frequency-domain mixing head
 * (Sec. 3.2): a real FFT of the value rows along the sequence axis, a
 * multiplication by a content-adaptive complex gate with one entry per
 * frequency bin, and the inverse real FFT.  At decode time a "Prefix-FFT cache"
 * (Sec. 3.3, Algorithm 1) keeps the half spectrum of a sliding window of
 * N_max tokens up to date with one rank-one update per new token.
 *
 * Conventions shared by every entry point
 *   - C linkage, plain pointers and sizes.  Unless a parameter says "host",
 *     every pointer is a DEVICE pointer on the current HIP device.
 *   - Token tensors are row-major [B, L, H, d] (batch, position, head, channel),
 *     dtype SPECTRE_F32 (float) or SPECTRE_BF16 (bfloat16 bit patterns); all
 *     spectra, gates and cache state are fp32 / complex64 ((re, im) float pairs);
 *     bf16 outputs are rounded to nearest even from fp32.
 *   - F = floor(n/2) + 1 is the number of stored bins of an n-point real
 *     transform (App. B, Cor. B.2).  The forward transform is unnormalised
 *     (Eq. 1), the inverse carries 1/n.
 *   - Compute calls only enqueue work on `stream` (a hipStream_t passed as void*, NULL =
 *     the default stream) and return: they never allocate device or pinned memory, never
 *     copy from the host, never create streams or events and never synchronise, so they may
 *     be captured into a HIP graph.  Everything of that kind happens in spectre_prepare
 *     (and in spectre_prefix_init, which calls it): a compute call for a transform length
 *     that has not been prepared on the current device returns SPECTRE_ENOTREADY and
 *     enqueues nothing.  Inputs are never modified; outputs are fully overwritten; results
 *     are bitwise reproducible from run to run.  A long spectre_mix_forward call runs every
 *     other head group on a helper stream of the library's own (default priority, made by
 *     spectre_prepare), forked from and joined back into `stream` with events: to the
 *     caller the call still behaves as work enqueued on `stream`, also under HIP graph
 *     capture.  The library reads no environment variable; spectre_set_option holds the few
 *     tuning switches that exist for measurements, none of which changes a result.
 *   - The caller owns every buffer, including the scratch workspace `ws`, whose
 *     minimum size the matching *_workspace_bytes function returns.  The library
 *     itself only keeps small per-device read-only tables (roots of unity, bin orders)
 *     and a helper stream with three events, created by spectre_prepare and kept until
 *     spectre_shutdown().
 *   - Every function returning int returns a spectre_status; on failure nothing
 *     has been enqueued (argument errors are detected on the host before any
 *     launch) and spectre_last_error() describes the reason.  The library never
 *     aborts or throws.
 *   - Supported shapes.  Mixer and cache: d = 64 channels per head.  Transform
 *     lengths of the mixer: every n <= 2048 whose prime factors are 2, 3, 5 or 7
 *     (196 = 4*7*7 among them) and every n = N1 * N2 with N1 = 256 or 4096 and
 *     N2 <= 32 of the form {1, 3, 5, 7} * 2^a (all powers of two from 256 to 131072,
 *     768, 12288 = 3 * 4096, 98304 = 24 * 4096, ...) have their own kernels; every
 *     other n <= 65536 is computed exactly as well, as a zero-padded power-of-two
 *     convolution (2.5 to 5 times the cost of a power of two of similar size).  The
 *     cache window n = N_mem + N_max is one of the N1 * N2 lengths above.  The gate takes any
 *     d <= 256, d_g <= 256 and any n_fft >= 2.  spectre_length_supported() answers
 *     for the mixer; anything else returns SPECTRE_EUNSUPPORTED.
 */
#ifndef SPECTRE_H
#define SPECTRE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SPECTRE_OK = 0,
    SPECTRE_EINVAL = 1,       /* null pointer, non-positive size, overlapping in/out, bad enum */
    SPECTRE_EUNSUPPORTED = 2, /* valid request this build has no kernel for (length, d, ...)   */
    SPECTRE_EWORKSPACE = 3,   /* ws == NULL or ws_bytes below the *_workspace_bytes figure      */
    SPECTRE_EHIP = 4,         /* a HIP runtime call failed; text in spectre_last_error()        */
    SPECTRE_ENOTREADY = 5     /* spectre_prepare has not been called for this length and device */
} spectre_status;

typedef enum { SPECTRE_F32 = 0, SPECTRE_BF16 = 1 } spectre_dtype;

/* Host string describing the last failure on the calling thread ("" if none). */
const char *spectre_last_error(void);

/* Library version as major*10000 + minor*100 + patch. */
int spectre_version(void);

/* 1 if an n-point transform is available for channel count d, else 0. */
int spectre_length_supported(int n, int d);

/*
 * spectre_prepare - set-up for transform length n (a mixer length L, or a cache window N_mem + N_max)
 * with d channels per head, on the current device: builds the read-only tables every kernel route of
 * that length uses (values computed in fp64 on the host, copied once) and, the first time, the helper
 * stream and its events.  This is the one call that allocates, copies and synchronises; it is
 * idempotent and cheap when there is nothing left to do.  Returns SPECTRE_EUNSUPPORTED when no
 * kernel exists for (n, d).  Not to be called while a stream of the device is being captured.
 */
int spectre_prepare(int n, int d);

/* Frees the per-device tables and helper streams (lengths must be prepared again afterwards).
 * Optional; safe to call more than once. */
void spectre_shutdown(void);

/*
 * Tuning switches for measurements and tests.  Process-wide, host-side, read at every call; they
 * must not change between a *_workspace_bytes query and the call it sizes.  None changes a result
 * (the same arithmetic in the same order; at most which of two kernels of identical arithmetic
 * runs, where tests compare the two).  value < 0 restores the default.
 *   SPECTRE_OPT_LANES              1 keeps every head group of a long spectre_mix_forward call on
 *                                  `stream`; 2 (default) alternates them with the helper stream
 *   SPECTRE_OPT_SCRATCH_MB         total transform scratch in flight, MiB (default 204: sized for
 *                                  the 256 MB memory-side cache)
 *   SPECTRE_OPT_FUSED_4096         0 sends n = 4096 through the three four-step kernels instead of
 *                                  the single kernel it has of its own (default 1)
 *   SPECTRE_OPT_SLAB_COMPILE_TIME  0 makes the in-LDS kernel take its run-time-length form also
 *                                  for the lengths that have a compile-time form (default 1)
 *   SPECTRE_OPT_HEAD_AFFINE        0 switches off the placement of all workgroups of a head on one
 *                                  XCD that four-step lengths up to 12288 use (default 1)
 *   SPECTRE_OPT_LANE_SHUFFLES      1 makes the column kernel of the four-step route exchange values
 *                                  between the 16 lanes of a sub-transform with cross-lane (DPP) moves
 *                                  instead of through LDS (default 0: measured slower or equal)
 *   SPECTRE_OPT_GROUPS             n > 0 splits the heads of a four-step call into n groups of equal
 *                                  size (rounded up to an even count on two lanes), whatever the
 *                                  scratch budget says; 0 (default) sizes the groups by the budget
 */
enum { SPECTRE_OPT_LANES = 0, SPECTRE_OPT_SCRATCH_MB = 1, SPECTRE_OPT_FUSED_4096 = 2,
       SPECTRE_OPT_SLAB_COMPILE_TIME = 3, SPECTRE_OPT_HEAD_AFFINE = 4, SPECTRE_OPT_GROUPS = 5,
       SPECTRE_OPT_LANE_SHUFFLES = 6, SPECTRE_OPT_COUNT_ = 7 };
int spectre_set_option(int which, long value);
long spectre_get_option(int which);

/* ------------------------------------------------------------------------------------------
 * Gate parameters (Sec. 3.2 step 3a and 3c; the same network serves Algorithm 1's decode gate).
 * All arrays are device fp32.  Hg = H gives every head its own network, Hg = 1 shares one across
 * heads (the two parameter budgets of Sec. 3.6).  The MLP's second layer emits 2F reals that are
 * read as F interleaved (re, im) pairs, so its width is tied to the transform length n_fft.  W1 is
 * stored input-major (hid = qbar W1), W2 output-major (row n holds the d_g weights of output real
 * n, the layout torch.nn.Linear keeps), so that the weights of one bin are contiguous.
 */
typedef struct {
    int Hg;                    /* H (per-head weights) or 1 (shared)                          */
    int d;                     /* channels per head                                           */
    int d_g;                   /* hidden width of the MLP, 1..256                             */
    int n_fft;                 /* transform length the gate is for; F = n_fft/2 + 1           */
    const float *ln_gamma;     /* [Hg, d]   LayerNorm scale                                   */
    const float *ln_beta;      /* [Hg, d]   LayerNorm shift                                   */
    float ln_eps;              /* added to the biased variance over the d channels            */
    const float *W1;           /* [Hg, d, d_g]                                                */
    const float *b1;           /* [Hg, d_g]                                                   */
    const float *W2;           /* [Hg, 2F, d_g]   u[n] = sum_j hid[j] W2[n][j] + b2[n]        */
    const float *b2;           /* [Hg, 2F]                                                    */
    const float *modrelu_bias; /* [Hg, F] real bias of modReLU, or NULL to skip the activation */
    const float *toeplitz;     /* complex64 [Hg, 2r+1] taps t_{-r..r} (tap m at index m+r) of the   */
    int toeplitz_r;            /* optional low-rank update of step 3b, or NULL / 0 to skip it       */
} spectre_gate_params;

size_t spectre_gate_workspace_bytes(int B, int L, int H, const spectre_gate_params *P /*host*/);

/*
 * spectre_gate - content-adaptive spectral gate, Sec. 3.2 step 3 (a), (c) and the positional-phase
 * paragraph of Sec. 3.5; Algorithm 1's "LN(sum_q/N_max) -> MLP -> modReLU -> phase" lines.
 *
 *   x      = inv_count * sum over positions of the query rows          (global descriptor)
 *   qbar   = ln_gamma * (x - mean(x)) / sqrt(var(x) + ln_eps) + ln_beta
 *   hid    = GELU(qbar W1 + b1)                 (exact erf form)
 *   u      = W2 hid + b2,   g_k = u[2k] + j u[2k+1],  k = 0..F-1
 *   g     <- g + (t * g),  (t * g)_k = sum_{m=-r..r} t_m g_{k-m} with g = 0 outside 0..F-1
 *                                                      (Sec. 3.2 step 3b; skipped if toeplitz NULL)
 *   g_k   <- max(|g_k| + bias_k, 0) * g_k / |g_k|      (0 where |g_k| = 0; skipped if bias NULL)
 *   g_k   <- g_k * exp(+j 2 pi ((k * phase_pos) mod n_fft) / n_fft)    (skipped if phase_pos = 0)
 *
 *   q            q_is_pooled = 0: query rows [B, L, H, d] of dtype q_dtype (pooled here, in
 *                order-fixed partial sums combined in fp64);
 *                q_is_pooled = 1: the sum itself, double [B, H, d] (q_dtype, L ignored) - this is
 *                the cache's running sum at decode time.
 *   inv_count    1/L for the mixing layer, 1/N_max at decode time (as Algorithm 1 prints it).
 *   P            host pointer to the parameter block (its arrays are device pointers).
 *   phase_pos    scalar position p >= 0 of the phase; 0 = none.
 *   g_out        complex64 [B, H, F], F = P->n_fft/2 + 1.
 */
int spectre_gate(const void *q, int q_is_pooled, spectre_dtype q_dtype, double inv_count,
                 const spectre_gate_params *P /*host*/, int B, int L, int H,
                 long long phase_pos, void *g_out, void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------
 * spectre_project - token projection, Sec. 3.2 step 1 (Eq. 2), per head: every head h multiplies its
 * own d channels of the token rows by its d x d matrices,
 *        V[b, l, h, :] = X[b, l, h, :] W^(v)_h        Q[b, l, h, :] = X[b, l, h, :] W^(q)_h .
 * The mixing layer needs V and only the sum of the query rows; since pooling commutes with the
 * projection the call reads X once, writes V and returns sum_q = (sum_l X[b, l, h, :]) W^(q)_h.
 *
 *   x       [B, L, H, d] of dtype io (d = 64)
 *   Wq, Wv  fp32 [Hw, d, d], input-major (row i, column j: out_j = sum_i x_i W[i][j]); Hw = H or 1
 *   v_out   [B, L, H, d] of dtype io; must not overlap x
 *   q_out   [B, L, H, d] of dtype io, or NULL when the query rows themselves are not needed
 *   sum_q   double [B, H, d], or NULL; ready to be passed to spectre_gate with q_is_pooled = 1
 */
size_t spectre_project_workspace_bytes(int B, int L, int H, int d);
int spectre_project(const void *x, const float *Wq, const float *Wv, int Hw, int B, int L, int H, int d,
                    spectre_dtype io, void *v_out, void *q_out, void *sum_q, void *ws, size_t ws_bytes,
                    void *stream);

/* ------------------------------------------------------------------------------------------
 * Wavelet refinement, Sec. 3.5 steps (a)-(d): out = v + iDWT( s * DWT(v) ) along the sequence axis
 * of every (b, h, channel) column.  The section names neither the wavelet nor the shape of the
 * gates; this library implements the orthonormal Haar wavelet with `levels` = J analysis levels
 * (2^J must divide L) and one real gate per band and channel: s [B, H, J+1, d], band 0 = the
 * coarse approximation (L / 2^J coefficients per column), band l = 1..J the details of level l
 * (level 1 = differences of adjacent rows).  The learned controller that skips the module is the
 * caller's: skipping means not calling.
 *
 * spectre_wrm_gates - step (b): s = W2' GELU(qbar W1 + b1) + b2 with qbar the LayerNorm of the pooled
 * query exactly as in spectre_gate (same q / q_is_pooled / inv_count arguments).
 *   P->W1 [Hg, d, d_w], b1 [Hg, d_w], W2 [Hg, d_w, (J+1)*d] (input-major), b2 [Hg, (J+1)*d],
 *   ln_gamma, ln_beta [Hg, d]; Hg = H or 1; d <= 256, d_w <= 256, levels <= 30.
 *   s_out  float [B, H, J+1, d].
 *
 * spectre_wrm_apply - steps (a), (c), (d) for v, out [B, L, H, d] of dtype io, d = 64.  out may be v
 * itself (in place) but must not overlap it otherwise.  One pass over v when J <= 8; above that one
 * extra read of v (sums of 256-row tiles for the coarse levels).
 */
typedef struct {
    int Hg, d, d_w, levels;
    const float *ln_gamma, *ln_beta;
    float ln_eps;
    const float *W1, *b1, *W2, *b2;
} spectre_wrm_params;

size_t spectre_wrm_gates_workspace_bytes(int B, int L, int H, const spectre_wrm_params *P /*host*/);
int spectre_wrm_gates(const void *q, int q_is_pooled, spectre_dtype q_dtype, double inv_count,
                      const spectre_wrm_params *P /*host*/, int B, int L, int H, void *s_out, void *ws,
                      size_t ws_bytes, void *stream);
size_t spectre_wrm_apply_workspace_bytes(int B, int L, int H, int d, int levels);
int spectre_wrm_apply(const void *v, const void *s, void *out, int B, int L, int H, int d, int levels,
                      spectre_dtype io, void *ws, size_t ws_bytes, void *stream);

/*
 * spectre_wrm_apply_coeff - the same module under the other reading of step (b)'s "s in R^(n x d)": one
 * real gate per wavelet coefficient and channel, handed in by the caller (an MLP that emitted them would
 * hold d_w * n * d weights per head; none is built here).  A real Haar analysis, a multiplication of
 * coefficient i of column (b, h, c) by s[b, h, i, c], the synthesis, and the residual add.
 *   s   float [B, H, L, d], 8-byte aligned, coefficients in the order the analysis produces them, coarse to
 *       fine: [ a_J (L/2^J approximations) | d_J (L/2^J details) | d_(J-1) | ... | d_1 (L/2 details) ];
 *       the detail of level l of the block of 2^l rows number i sits at index (L >> l) + i.
 *   Gates constant over each band give spectre_wrm_apply's result.  Same v / out / levels / workspace
 *   (spectre_wrm_apply_workspace_bytes) rules as spectre_wrm_apply; out may be v, must not overlap s.
 */
int spectre_wrm_apply_coeff(const void *v, const void *s, void *out, int B, int L, int H, int d, int levels,
                            spectre_dtype io, void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------
 * spectre_mix_forward - the mixing layer, Sec. 3.2 steps 2 and 4 (Eq. 3, Eq. 4): for every
 * sequence b, head h and channel c
 *        out[b, :, h, c] = irfft_L( g[b, h, :] * rfft_L( v[b, :, h, c] ) ).
 * The gated DC and Nyquist bins contribute their real parts only (the product is extended by
 * Hermitian symmetry before the inverse, as Cor. B.2's inverse assumes).
 *
 *   v     [B, L, H, d] of dtype io        g    complex64 [B, H, F], F = L/2 + 1
 *   out   [B, L, H, d] of dtype io; must not overlap v (SPECTRE_EINVAL if it does)
 *   ws    scratch of at least spectre_mix_workspace_bytes(B, L, H, d, io) bytes, 256-byte aligned
 */
size_t spectre_mix_workspace_bytes(int B, int L, int H, int d, spectre_dtype io);
int spectre_mix_forward(const void *v, const void *g, void *out, int B, int L, int H, int d,
                        spectre_dtype io, void *ws, size_t ws_bytes, void *stream);

/*
 * spectre_mix_forward_ex - the same call with option flags (flags = 0 is spectre_mix_forward).
 *   SPECTRE_MIX_BF16_SCRATCH   bfloat16 rows on the four-step route only (ignored elsewhere): the
 *        complex numbers that cross between the three kernels of that route are stored as two
 *        bfloat16 instead of two fp32.  The arithmetic stays fp32, the error against the exact
 *        result grows from about 1.7e-3 (the rounding of the output rows) to about 2.9e-3, and a
 *        call at n = 131072 takes about 14 % less time.  The spectrum then no longer exists in
 *        fp32 between the kernels, which is why it has to be asked for.
 */
enum { SPECTRE_MIX_BF16_SCRATCH = 1 };
int spectre_mix_forward_ex(const void *v, const void *g, void *out, int B, int L, int H, int d,
                           spectre_dtype io, unsigned flags, void *ws, size_t ws_bytes, void *stream);

/*
 * spectre_mix_forward_static - spectre_mix_forward for callers that cannot allocate or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments without `ws`, same result to rounding (same kernels; the roots of unity are
 * evaluated on the device in fp64 at every call instead of being taken from spectre_prepare's tables,
 * which can differ in the last bit of a table entry).  All scratch - tables, expanded gate, transform
 * columns - lives in one array of spectre_mix_static_bytes() = 98 MiB that is part of the library's
 * device image: every GPU the library runs on holds it until the process ends.  The call allocates
 * nothing, needs no spectre_prepare, and runs entirely on `stream`.
 *   Limits: four-step lengths only (L = N1 * N2 as above, 256 ... 131072), d = 64, and
 *   B*H*L <= 4 194 304 (32 heads at L = 131072); anything else returns SPECTRE_EUNSUPPORTED.
 *   Every call on a GPU uses that GPU's one array, which keeps the previous call's contents (each
 *   call overwrites what it reads, nothing needs clearing): calls that overlap in time on one GPU -
 *   on different streams, or from different host threads - race and must be serialised by the caller.
 */
size_t spectre_mix_static_bytes(void);
int spectre_mix_forward_static(const void *v, const void *g, void *out, int B, int L, int H, int d,
                               spectre_dtype io, void *stream);

/* ------------------------------------------------------------------------------------------
 * spectre_layer_forward - the whole mixing layer of Sec. 3.2 (steps 1 to 4) and, optionally, the refinement of
 * Sec. 3.5 behind it, in one call; the result is that of the chain
 *     (V, sum_q) = spectre_project(x, Wq, Wv);   g = spectre_gate(sum_q pooled, inv_count = 1/L, phase 0);
 *     out = spectre_mix_forward(V, g);           [ s = spectre_wrm_gates(sum_q, 1/L);  out = spectre_wrm_apply(out, s) ]
 * On the four-step route with bf16 rows the chain's intermediate tensors do not exist: the row transforms read X and
 * project it on the matrix cores on their way in (V is never written or re-read; it is rounded to bf16 on chip exactly
 * as the separate call would have stored it), the pooled query comes from one streaming pass over X, and the
 * refinement's coarse levels use block sums that the mixer's store phase emits instead of a second read of the
 * output.  Other lengths and fp32 rows run the chain as it stands, with V in the workspace.
 *   x, out  [B, L, H, d] of dtype io, 16-byte aligned, not overlapping;  Wq, Wv as in spectre_project
 *   P       gate parameters with P->n_fft == L;   W  refinement parameters, or NULL for none
 */
size_t spectre_layer_workspace_bytes(int B, int L, int H, int d, spectre_dtype io,
                                     const spectre_gate_params *P /*host*/, const spectre_wrm_params *W /*host*/);
int spectre_layer_forward(const void *x, const float *Wq, const float *Wv, int Hw,
                          const spectre_gate_params *P /*host*/, const spectre_wrm_params *W /*host or NULL*/,
                          void *out, int B, int L, int H, int d, spectre_dtype io, void *ws, size_t ws_bytes,
                          void *stream);

/* ------------------------------------------------------------------------------------------
 * Prefix-FFT cache, Sec. 3.3 and Algorithm 1.  One cache serves B*H heads that advance in
 * lock-step (one token counter).  The caller allocates the five device arrays (sizes from
 * spectre_prefix_bytes), fills in the dimensions, and calls spectre_prefix_init once.
 *
 * Persistent memory, Sec. 3.4 (N_mem > 0).  The section's literal concatenation of an N_mem-point and
 * an N_max-point half spectrum is the spectrum of no signal; the reading implemented here: the memory
 * rows M are the first N_mem rows of a window of n = N_mem + N_max rows whose other N_max rows are the
 * ring buffer, the cache is the n-point half spectrum of that window, the gate has F = n/2 + 1 bins and
 * the inverse is n-point.  Memory rows are never evicted and never updated by a decode step, carry no
 * query (they do not enter sum_q; the descriptor's divisor stays 1/N_max), and token t lives in row
 * N_mem + (t mod N_max).  With N_mem = 0 everything below reduces to Sec. 3.3 as printed.
 */
typedef struct {
    int B, H, d;
    int N_max;            /* ring capacity: the live window of Sec. 3.3                          */
    int N_mem;            /* persistent memory rows in front of the ring (0 = none)              */
                          /* n = N_mem + N_max is the transform length, a supported power of two */
    long long t;          /* HOST field: tokens appended so far; advanced by update/step        */
    void *prefix_fft;     /* complex64 [B, H, F, d]: n-point half spectrum of the window, F=n/2+1*/
    void *v_buf;          /* float [B, H, n, d]: memory rows, then the ring of values            */
    void *q_buf;          /* float [B, H, n, d]: zeros, then the ring of queries                 */
    void *sum_q;          /* double [B, H, d]: running sum of the live queries                  */
    void *twiddle;        /* complex64 [n]: exp(-j 2 pi m / n), the pre-cached factors          */
    /* Deferred updates (optional; pending == NULL or pending_cap == 0: every step updates the cache).
     * Eq. 5 is linear, so spectre_prefix_step may leave the rank-one updates of the last tokens pending
     * and only READ the cache: the newest row of irfft(g * X) for X = X_stale + sum_i Delta_i w^(k s_i) is
     * that row for X_stale plus sum_i kappa[(s - s_i) mod n] Delta_i with kappa = irfft(g).  Every
     * pending_cap steps one sweep applies all pending updates.  Outputs are the same up to fp32 rounding;
     * prefix_fft lags behind until spectre_prefix_flush (or the flushing step). */
    void *pending;        /* float [pending_cap, B, H, d]: Delta rows of the pending tokens, or NULL     */
    int pending_cap;      /* 0 .. SPECTRE_MAX_PENDING                                                    */
    int n_pending;        /* HOST field: tokens whose update is pending                                  */
    int pending_slot[32]; /* HOST field: their window rows                                               */
} spectre_prefix_cache;
#define SPECTRE_MAX_PENDING 32

enum { SPECTRE_PREFIX_FFT = 0, SPECTRE_PREFIX_VBUF = 1, SPECTRE_PREFIX_QBUF = 2,
       SPECTRE_PREFIX_SUMQ = 3, SPECTRE_PREFIX_TWIDDLE = 4 };
/* Bytes of cache field `which` (one of the enumerators above) for a window of n = N_mem + N_max
 * rows; 0 on bad arguments. */
size_t spectre_prefix_bytes(int B, int H, int d, int n, int which);

/* Zeroes the state, fills the twiddle table (computed in fp64, rounded once), sets t = 0.  A set-up
 * call: it runs spectre_prepare(N_mem + N_max, d) first, so it may allocate and synchronise. */
int spectre_prefix_init(spectre_prefix_cache *cache /*host*/, void *stream);

/* Applies the pending deferred updates (one sweep over the cache); a no-op when there are none.
 * spectre_prefix_update and spectre_prefix_set_memory flush by themselves; spectre_prefix_readout takes a
 * const cache and returns SPECTRE_EINVAL while updates are pending. */
int spectre_prefix_flush(spectre_prefix_cache *cache /*host*/, void *stream);

/*
 * spectre_prefix_set_memory - Sec. 3.4: lay the memory rows down and transform the window once
 * ("store the transform of the memory once").  Only on an empty cache (t = 0), right after init,
 * for a cache with N_mem > 0.   mem  float [mem_batch, H, N_mem, d], mem_batch = 1 (shared by all
 * sequences) or B.
 */
size_t spectre_prefix_set_memory_workspace_bytes(const spectre_prefix_cache *cache /*host*/);
int spectre_prefix_set_memory(spectre_prefix_cache *cache /*host*/, const float *mem, int mem_batch,
                              void *ws, size_t ws_bytes, void *stream);

/*
 * spectre_prefix_update - append T tokens.  v_new, q_new are [B, T, H, d] of dtype `io`.
 *   cache->t == 0 and T > 1 : pre-fill (Algorithm 1, PreFill): one N_max-point real transform of
 *        the prompt zero-padded at the tail, ring buffers filled, sum_q = sum of the prompt's
 *        queries.  Requires T <= N_max.  (With memory rows: the prompt goes behind them and the
 *        whole window is transformed.)
 *   otherwise : T successive decode updates (Algorithm 1, DecodeStep up to the gate; Eq. 5):
 *        s = N_mem + t mod N_max;  delta = v_t - [t >= N_max] v_buf[s];
 *        prefix_fft[k, :] += delta * exp(-j 2 pi ((k s) mod n)/n)   for every bin k;
 *        sum_q += q_t - [t >= N_max] q_buf[s];  v_buf[s] = v_t;  q_buf[s] = q_t;  t += 1.
 *        The ring buffers and sum_q are updated token by token, in order; the cache itself takes the
 *        rank-one terms of up to SPECTRE_MAX_PENDING tokens in one sweep (their sum, by linearity).
 *        From 160 tokens on (and T <= N_max) the ring buffers are instead brought up to date in one
 *        pass and the window is transformed afresh, as in the pre-fill: the same state, cheaper.
 * On success cache->t has advanced by T.
 */
size_t spectre_prefix_update_workspace_bytes(const spectre_prefix_cache *cache /*host*/, int T,
                                             spectre_dtype io);
int spectre_prefix_update(spectre_prefix_cache *cache /*host*/, const void *v_new, const void *q_new,
                          int T, spectre_dtype io, void *ws, size_t ws_bytes, void *stream);

/*
 * spectre_prefix_readout - Algorithm 1's last three lines, z = irfft_N( g * prefix_fft ).
 *   mode SPECTRE_READ_NEWEST : out [B, 1, H, d] = row N_mem + (t-1) mod N_max of z, the newest token's row,
 *        evaluated as a direct sum over the bins (the O(N_max/2 d) per-step cost Sec. 3.3 quotes);
 *        pass the gate WITHOUT positional phase.
 *   mode SPECTRE_READ_WINDOW : out [B, L', H, d] = rows N_max-L' .. N_max-1 of z, L' = min(t, N_max)
 *        (a full inverse transform).  With a gate built with phase_pos = t these rows are the live
 *        tokens in chronological order, the last one equal to the NEWEST readout.
 *        With memory rows (N_mem > 0) a circular shift would move the pinned rows too: pass the
 *        gate WITHOUT phase; the L' live tokens' rows of z are gathered from their ring slots and
 *        returned oldest first.
 *   g     complex64 [B, H, F], F = n/2 + 1.   Requires t >= 1.
 */
enum { SPECTRE_READ_NEWEST = 0, SPECTRE_READ_WINDOW = 1 };
size_t spectre_prefix_readout_workspace_bytes(const spectre_prefix_cache *cache /*host*/, int mode,
                                              spectre_dtype io);
int spectre_prefix_readout(const spectre_prefix_cache *cache /*host*/, const void *g, int mode,
                           void *out, spectre_dtype io, void *ws, size_t ws_bytes, void *stream);

/*
 * spectre_prefix_step - one fused decode step with the results of
 *   spectre_prefix_update(T = 1), spectre_gate(sum_q, 1/N_max, phase 0), spectre_prefix_readout(NEWEST)
 * but a single sweep over the cache (each cache entry is read once and written once).
 *   v_t, q_t  [B, 1, H, d] of dtype io       out  [B, 1, H, d] of dtype io
 *   P         gate parameters with P->n_fft == n = N_mem + N_max
 */
size_t spectre_prefix_step_workspace_bytes(const spectre_prefix_cache *cache /*host*/,
                                           const spectre_gate_params *P /*host*/);
int spectre_prefix_step(spectre_prefix_cache *cache /*host*/, const void *v_t, const void *q_t,
                        const spectre_gate_params *P /*host*/, void *out, spectre_dtype io,
                        void *ws, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SPECTRE_H */
