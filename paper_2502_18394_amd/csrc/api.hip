// C ABI of the SPECTRE library: argument checks, per-device table cache, launch sequencing.
// Every entry point validates on the host, enqueues on the caller's stream and returns.
#include "../../include/spectre.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <mutex>
#include <string>
#include <utility>
#include <vector>

#include "gate.h"
#include "internal.h"
#include "mix_chirp.h"
#include "mix_slab.h"
#include "prefix.h"
#include "project.h"
#include "wrm.h"

namespace spectre {

static thread_local std::string g_err;

// Process-wide tuning switches (spectre_set_option); none of them changes a result.
static std::atomic<long> g_opt[SPECTRE_OPT_COUNT_];
static const long kOptDefault[SPECTRE_OPT_COUNT_] = {2, 204, 1, 1, 1, 0, 0};
long option(int which) {
    const long v = g_opt[which].load(std::memory_order_relaxed);
    return v > 0 ? v - 1 : kOptDefault[which];       // stored as value + 1 so that zero-initialised = default
}

int fail(int code, const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

int fail_hip(hipError_t e, const char *what) {
    return fail(SPECTRE_EHIP, "%s: %s", what, hipGetErrorString(e));
}

// ---------------------------------------------------------------- per-device tables
// A helper stream on which every other head group of a long mixing call runs, so that the memory-bound
// row kernels of one group overlap the arithmetic-heavy column kernel of the next; default priority.
struct SideLane {
    hipStream_t stream = nullptr;
    hipEvent_t fork = nullptr, join = nullptr, gate = nullptr;
};

struct DeviceTables {
    std::map<int, float2 *> roots;   // n -> device array [n] of exp(-j 2 pi m / n)
    std::map<int, float2 *> chirp;   // L -> device array: chirp [L], then its filter spectrum [M]
    std::map<int, int *> slab_order; // L -> device array [L]: bin held by each position of the in-LDS transform
    std::vector<struct SideLane *> lanes;   // idle helper streams (with their fork/join events)
    int lanes_made = 0;
};
static std::mutex g_mu;
static std::map<int, DeviceTables> g_tables;

static void fill_roots(std::vector<float2> &h, int n) {
    h.resize(n);
    for (int m = 0; m < n; ++m) {
        // exact octant symmetry is not needed: the angle is below 2 pi and evaluated in fp64
        const double a = -2.0 * M_PI * (double)m / (double)n;
        h[m] = make_float2((float)std::cos(a), (float)std::sin(a));
    }
}

// Compute calls look tables up (make = false) and never create them: creating allocates and copies, which only
// spectre_prepare may do.
static int not_ready(const char *what, int n) {
    return fail(SPECTRE_ENOTREADY, "%s for length %d missing on this device: call spectre_prepare first", what, n);
}

int get_roots(int n, const float2 **out, bool make) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    std::lock_guard<std::mutex> lk(g_mu);
    DeviceTables &t = g_tables[dev];
    auto it = t.roots.find(n);
    if (it == t.roots.end()) {
        if (!make) return not_ready("roots of unity", n);
        std::vector<float2> h;
        fill_roots(h, n);
        float2 *d = nullptr;
        e = hipMalloc(reinterpret_cast<void **>(&d), sizeof(float2) * (size_t)n);
        if (e != hipSuccess) return fail_hip(e, "hipMalloc(roots)");
        e = hipMemcpy(d, h.data(), sizeof(float2) * (size_t)n, hipMemcpyHostToDevice);
        if (e != hipSuccess) {
            (void)hipFree(d);
            return fail_hip(e, "hipMemcpy(roots)");
        }
        it = t.roots.emplace(n, d).first;
    }
    *out = it->second;
    return SPECTRE_OK;
}

static int get_slab_order(int L, const int **out, bool make = false) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    std::lock_guard<std::mutex> lk(g_mu);
    DeviceTables &t = g_tables[dev];
    auto it = t.slab_order.find(L);
    if (it == t.slab_order.end()) {
        if (!make) return not_ready("bin order table", L);
        std::vector<int> h((size_t)L);
        slab_bin_order(L, h.data());
        int *d = nullptr;
        e = hipMalloc(reinterpret_cast<void **>(&d), sizeof(int) * h.size());
        if (e != hipSuccess) return fail_hip(e, "hipMalloc(slab order)");
        e = hipMemcpy(d, h.data(), sizeof(int) * h.size(), hipMemcpyHostToDevice);
        if (e != hipSuccess) {
            (void)hipFree(d);
            return fail_hip(e, "hipMemcpy(slab order)");
        }
        it = t.slab_order.emplace(L, d).first;
    }
    *out = it->second;
    return SPECTRE_OK;
}

static void release_lane(int dev, SideLane *l) {
    std::lock_guard<std::mutex> lk(g_mu);
    g_tables[dev].lanes.push_back(l);
}

// Helper lanes are pooled per device: a call takes one for the time it enqueues work and puts it back
// (work already enqueued keeps its order; events may be re-recorded once the waits on them are enqueued).
// *out = nullptr when the pool is empty (not prepared, or other host threads hold the lanes): the call then keeps
// all its groups on the caller's stream.
static int acquire_lane(int *dev_out, SideLane **out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    *dev_out = dev;
    *out = nullptr;
    std::lock_guard<std::mutex> lk(g_mu);
    DeviceTables &t = g_tables[dev];
    if (!t.lanes.empty()) {
        *out = t.lanes.back();
        t.lanes.pop_back();
    }
    return SPECTRE_OK;
}

// One more helper lane for the current device's pool (spectre_prepare: one per call while the pool is empty).
static int make_lane() {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    {
        std::lock_guard<std::mutex> lk(g_mu);
        DeviceTables &t = g_tables[dev];
        if (t.lanes_made > 0 && !t.lanes.empty()) return SPECTRE_OK;
        if (t.lanes_made >= 8) return SPECTRE_OK;
        t.lanes_made += 1;
    }
    SideLane *l = new SideLane;
    e = hipStreamCreateWithFlags(&l->stream, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&l->fork, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&l->join, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&l->gate, hipEventDisableTiming);
    if (e != hipSuccess) {
        if (l->gate) (void)hipEventDestroy(l->gate);
        if (l->join) (void)hipEventDestroy(l->join);
        if (l->fork) (void)hipEventDestroy(l->fork);
        if (l->stream) (void)hipStreamDestroy(l->stream);
        delete l;
        return fail_hip(e, "helper stream");
    }
    release_lane(dev, l);
    return SPECTRE_OK;
}


// Chirp tables of an arbitrary length L (padded length M): *w [L], *filt [M].
static int get_chirp(int L, const Pow2Plan &pl, const float2 **w, const float2 **filt, bool make = false) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    std::lock_guard<std::mutex> lk(g_mu);
    DeviceTables &t = g_tables[dev];
    auto it = t.chirp.find(L);
    if (it == t.chirp.end()) {
        if (!make) return not_ready("chirp table", L);
        std::vector<float2> h((size_t)L + pl.L);
        chirp_tables_host(L, pl.L, pl.N1, pl.N2, pl.P, h.data(), h.data() + L);
        float2 *d = nullptr;
        e = hipMalloc(reinterpret_cast<void **>(&d), sizeof(float2) * h.size());
        if (e != hipSuccess) return fail_hip(e, "hipMalloc(chirp)");
        e = hipMemcpy(d, h.data(), sizeof(float2) * h.size(), hipMemcpyHostToDevice);
        if (e != hipSuccess) {
            (void)hipFree(d);
            return fail_hip(e, "hipMemcpy(chirp)");
        }
        it = t.chirp.emplace(L, d).first;
    }
    *w = it->second;
    *filt = it->second + L;
    return SPECTRE_OK;
}

int get_pow2_plan(int L, Pow2Plan *pl, bool make) {
    int N1, N2, P;
    if (!pow2_split(L, &N1, &N2, &P)) return fail(SPECTRE_EUNSUPPORTED, "no four-step plan for length %d", L);
    pl->L = L; pl->N1 = N1; pl->N2 = N2; pl->P = P;
    int rc = get_roots(L, &pl->twL, make);
    if (rc) return rc;
    return get_roots(N1, &pl->twN1, make);
}

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Appends of at least this many tokens re-transform the window instead of sweeping the cache once per 32 tokens
// (a sweep costs about a quarter of a window transform at the decode benchmark's shape).
constexpr int kAppendRetransform = 160;

// Scratch columns are processed in groups of heads small enough to stay in the memory-side
// cache between the three kernels of a group.
int mix_chunk_heads(int BH, int L, int d) {
    size_t per_head = (size_t)L * (size_t)(d / 2) * sizeof(float2);
    const size_t budget = (size_t)option(SPECTRE_OPT_SCRATCH_MB) << 20;
    size_t n = budget / per_head;
    if (n < 1) n = 1;
    if (n > (size_t)BH) n = (size_t)BH;
    return (int)n;
}

// Long calls run their head groups on two lanes (the caller's stream and a helper stream), each with half the
// scratch budget, when that still leaves at least two groups.  Two lanes get an even number of groups whose sizes
// differ by at most one head (larger ones first), so that both lanes carry the same load and end together.
// `scale` = heads that fit in the scratch bytes of one fp32-scratch head (2 with 16-bit scratch elements).
struct MixGroups {
    int lanes = 1, ngroups = 1, chunk = 1;            // chunk = heads in the largest group
    int BH = 1;
    int size(int group) const {                       // heads in group `group`
        if (lanes == 1) { const int left = BH - group * chunk; return left < chunk ? left : chunk; }
        return BH / ngroups + (group < BH % ngroups ? 1 : 0);
    }
};
static MixGroups mix_groups(int BH, int L, int d, int scale) {
    MixGroups m;
    m.BH = BH;
    const int full = mix_chunk_heads(BH, L, d);
    const int half = full / 2;
    const long forced = option(SPECTRE_OPT_GROUPS);
    if (forced > 0) {                                 // measurement: this many groups of (almost) equal size
        m.ngroups = forced < BH ? (int)forced : BH;
        m.lanes = (option(SPECTRE_OPT_LANES) >= 2 && m.ngroups >= 2) ? 2 : 1;
        if (m.lanes == 2 && (m.ngroups & 1)) m.ngroups += 1;
        m.chunk = (BH + m.ngroups - 1) / m.ngroups;
        if (m.lanes == 1) m.ngroups = (BH + m.chunk - 1) / m.chunk;
        return m;
    }
    if (option(SPECTRE_OPT_LANES) < 2 || full >= BH || half < 1) {
        m.chunk = ((long long)full * scale < BH) ? full * scale : BH;
        m.ngroups = (BH + m.chunk - 1) / m.chunk;
        return m;
    }
    const int cap = half * scale;
    m.lanes = 2;
    m.ngroups = 2 * ((BH + 2 * cap - 1) / (2 * cap));
    m.chunk = (BH + m.ngroups - 1) / m.ngroups;
    return m;
}

// ------------------------------------------------------------------------------------------
// Scratch of spectre_mix_forward_static: one array per GPU in the library's own device image, held until the process
// ends.  Layout: [roots of unity, kStaticTables][expanded gate, kStaticGate][transform scratch, kStaticColumns].
constexpr size_t kStaticTables = (size_t)2 << 20;     // (L + N1) complex64 <= 135168 * 8 bytes
constexpr size_t kStaticGate = (size_t)32 << 20;      // B*H*L complex64: up to 4 Mi bins (32 heads at L = 131072)
constexpr size_t kStaticColumns = (size_t)64 << 20;   // at least one head's columns (32 MiB at L = 131072)
constexpr size_t kStaticBytes = kStaticTables + kStaticGate + kStaticColumns;
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

// `scratch` is only a host-side stand-in for the device array: its device address, different on every GPU, comes
// from hipGetSymbolAddress, once per device with that device current, and is what host code passes on.
static std::map<int, unsigned char *> g_static_ptr;
static int static_scratch(unsigned char **out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    std::lock_guard<std::mutex> lk(g_mu);
    auto it = g_static_ptr.find(dev);
    if (it == g_static_ptr.end()) {
        unsigned char *ptr = nullptr;
        e = hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch));
        if (e != hipSuccess) return fail_hip(e, "hipGetSymbolAddress(scratch)");
        if (!ptr || (reinterpret_cast<uintptr_t>(ptr) & 255)) return fail(SPECTRE_EHIP, "static scratch: bad device address");
        it = g_static_ptr.emplace(dev, ptr).first;
    }
    *out = it->second;
    return SPECTRE_OK;
}

}  // namespace spectre

using namespace spectre;

#pragma GCC visibility push(default)
extern "C" {

const char *spectre_last_error(void) { return g_err.c_str(); }

int spectre_version(void) { return 120; }

// 0 = no kernel, 1 = whole slab in LDS, 2 = four-step power-of-two path, 3 = any other length
// through a padded power-of-two convolution, 4 = four-step path fused into one kernel (L = 4096).
static int mix_route(int BH, int L, int d) {
    if (d != 64) return 0;
    int N1, N2, P;
    const bool p2 = pow2_split(L, &N1, &N2, &P), sl = slab_supported(L);
    // the in-LDS kernel is one launch: it wins when the length has no four-step plan, when there are many short
    // slabs, and when the whole call is small enough to be bound by the four-step path's dependent launches
    if (sl && (!p2 || (L <= 512 && BH >= 256) || (long long)BH * L <= 65536)) return 1;
    if (fused_supported(L) && option(SPECTRE_OPT_FUSED_4096)) return 4;
    if (p2) return 2;
    return chirp_padded_length(L) ? 3 : 0;
}

// Workspace sections of the arbitrary-length route.
struct ChirpLayout {
    int M, nph;
    size_t gp, scr, t1, t2;      // byte sizes
    size_t total() const { return gp + scr + t1 + t2; }
};
static ChirpLayout chirp_layout(int BH, int L, int d) {
    ChirpLayout c;
    c.M = chirp_padded_length(L);
    c.nph = (BH + 31) / 32;
    c.gp = align256((size_t)BH * c.M * sizeof(float2));
    c.scr = align256((size_t)mix_chunk_heads(BH, c.M, d) * c.M * (d / 2) * sizeof(float2));
    c.t1 = align256((size_t)L * c.nph * 32 * sizeof(float2));
    c.t2 = align256((size_t)c.M * c.nph * 32 * sizeof(float2));
    return c;
}

static int mix_chirp(const void *v, const float2 *g, void *out, int B, int L, int H, int d, spectre_dtype io,
                     void *ws, hipStream_t st) {
    const int BH = B * H;
    const ChirpLayout c = chirp_layout(BH, L, d);
    Pow2Plan pl;
    int rc = get_pow2_plan(c.M, &pl);
    if (rc) return rc;
    const float2 *w = nullptr, *filt = nullptr;
    rc = get_chirp(L, pl, &w, &filt);
    if (rc) return rc;
    const float2 *slab_roots = nullptr;
    const int *slab_order = nullptr;
    if (slab_supported(c.M)) {                         // all table look-ups before the first launch
        rc = get_roots(c.M, &slab_roots);
        if (rc) return rc;
        rc = get_slab_order(c.M, &slab_order);
        if (rc) return rc;
    }
    char *base = static_cast<char *>(ws);
    float2 *gp = reinterpret_cast<float2 *>(base);
    float2 *scr = reinterpret_cast<float2 *>(base + c.gp);
    float2 *t1 = reinterpret_cast<float2 *>(base + c.gp + c.scr);
    float2 *t2 = reinterpret_cast<float2 *>(base + c.gp + c.scr + c.t1);
    const int nph = c.nph, phchunk = mix_chunk_heads(nph, c.M, d);

    // per-head convolution kernel kappa = irfft_L(gate), all heads at once as pseudo-head columns
    hipError_t e = launch_chirp_pre(g, w, t1, BH, L, nph, st);
    if (e != hipSuccess) return fail_hip(e, "chirp_pre");
    for (int ph0 = 0; ph0 < nph; ph0 += phchunk) {
        const int n = (nph - ph0 < phchunk) ? nph - ph0 : phchunk;
        e = launch_small_fwd(pl, SPECTRE_F32, t1, scr, L, nph, ph0, n, st);
        if (e != hipSuccess) return fail_hip(e, "small_fwd(chirp)");
        e = launch_big(pl, scr, filt, 0, n, 0, st, true);
        if (e != hipSuccess) return fail_hip(e, "big(chirp)");
        e = launch_small_inv(pl, SPECTRE_F32, scr, t1, 0, L, nph, ph0, n, st);
        if (e != hipSuccess) return fail_hip(e, "small_inv(chirp)");
    }
    // its periodic extension around index 0 of the padded length, transformed: the data pass's gate
    e = launch_chirp_post(t1, w, t2, L, c.M, nph, st);
    if (e != hipSuccess) return fail_hip(e, "chirp_post");
    for (int ph0 = 0; ph0 < nph; ph0 += phchunk) {
        const int n = (nph - ph0 < phchunk) ? nph - ph0 : phchunk;
        e = launch_small_fwd(pl, SPECTRE_F32, t2, scr, c.M, nph, ph0, n, st);
        if (e != hipSuccess) return fail_hip(e, "small_fwd(kernel)");
        e = launch_big(pl, scr, nullptr, 0, n, 1, st);
        if (e != hipSuccess) return fail_hip(e, "big(kernel)");
        // short padded lengths run the data pass as one in-LDS launch, which wants the gate in plain bin order
        e = slab_supported(c.M) ? launch_chirp_gate_plain(scr, gp, BH, c.M, pl.N1, pl.N2, pl.P, ph0, n, st)
                                : launch_chirp_gate(scr, gp, BH, c.M, pl.N1, pl.N2, ph0, n, st);
        if (e != hipSuccess) return fail_hip(e, "chirp_gate");
    }
    if (slab_supported(c.M)) {
        e = launch_mix_slab((int)io, v, gp, out, slab_roots, slab_order, B, c.M, H, st, L);
        if (e != hipSuccess) return fail_hip(e, "mix_slab(padded)");
        return SPECTRE_OK;
    }
    // the data: zero-padded to M, first L rows of the result kept
    const int chunk = mix_chunk_heads(BH, c.M, d);
    for (int bh0 = 0; bh0 < BH; bh0 += chunk) {
        const int nbh = (BH - bh0 < chunk) ? BH - bh0 : chunk;
        e = launch_small_fwd(pl, (int)io, v, scr, L, H, bh0, nbh, st);
        if (e != hipSuccess) return fail_hip(e, "small_fwd");
        e = launch_big(pl, scr, gp, bh0, nbh, 0, st);
        if (e != hipSuccess) return fail_hip(e, "big");
        e = launch_small_inv(pl, (int)io, scr, out, 0, L, H, bh0, nbh, st);
        if (e != hipSuccess) return fail_hip(e, "small_inv");
    }
    return SPECTRE_OK;
}

int spectre_length_supported(int n, int d) { return mix_route(1, n, d) != 0; }

void spectre_shutdown(void) {
    std::lock_guard<std::mutex> lk(g_mu);
    int cur = 0;
    (void)hipGetDevice(&cur);
    for (auto &kv : g_tables) {
        (void)hipSetDevice(kv.first);
        for (auto &r : kv.second.roots) (void)hipFree(r.second);
        for (auto &r : kv.second.chirp) (void)hipFree(r.second);
        for (auto &r : kv.second.slab_order) (void)hipFree(r.second);
        for (SideLane *l : kv.second.lanes) {
            (void)hipStreamSynchronize(l->stream);
            (void)hipEventDestroy(l->fork);
            (void)hipEventDestroy(l->join);
            (void)hipEventDestroy(l->gate);
            (void)hipStreamDestroy(l->stream);
            delete l;
        }
    }
    g_tables.clear();
    (void)hipSetDevice(cur);
}

int spectre_set_option(int which, long value) {
    if (which < 0 || which >= SPECTRE_OPT_COUNT_) return fail(SPECTRE_EINVAL, "set_option: unknown option %d", which);
    if (value >= 0) {
        if (which == SPECTRE_OPT_LANES && (value < 1 || value > 2)) return fail(SPECTRE_EINVAL, "set_option: lanes must be 1 or 2");
        if (which == SPECTRE_OPT_SCRATCH_MB && (value < 1 || value > (1L << 20)))
            return fail(SPECTRE_EINVAL, "set_option: scratch size out of range");
    }
    g_opt[which].store(value < 0 ? 0 : value + 1, std::memory_order_relaxed);
    return SPECTRE_OK;
}

long spectre_get_option(int which) {
    if (which < 0 || which >= SPECTRE_OPT_COUNT_) return -1;
    return option(which);
}

int spectre_prepare(int n, int d) {
    if (n < 1 || d < 1) return fail(SPECTRE_EINVAL, "prepare: non-positive size");
    if (d != 64) return fail(SPECTRE_EUNSUPPORTED, "prepare: d=%d (only 64 is built)", d);
    int N1, N2, P, rc;
    const bool p2 = pow2_split(n, &N1, &N2, &P), sl = slab_supported(n);
    const float2 *r = nullptr;
    const int *o = nullptr;
    Pow2Plan pl;
    if (sl) {
        if ((rc = get_roots(n, &r, true))) return rc;
        if ((rc = get_slab_order(n, &o, true))) return rc;
    }
    if (p2 && (rc = get_pow2_plan(n, &pl, true))) return rc;
    if (fused_supported(n) && (rc = get_roots(4096, &r, true))) return rc;
    if (!sl && !p2) {
        const int M = chirp_padded_length(n);
        if (!M) return fail(SPECTRE_EUNSUPPORTED, "prepare: no kernel for length %d", n);
        if ((rc = get_pow2_plan(M, &pl, true))) return rc;
        const float2 *w = nullptr, *filt = nullptr;
        if ((rc = get_chirp(n, pl, &w, &filt, true))) return rc;
        if (slab_supported(M)) {
            if ((rc = get_roots(M, &r, true))) return rc;
            if ((rc = get_slab_order(M, &o, true))) return rc;
        }
    }
    hipError_t (*const loaders[])() = {load_kernels_mix_pow2, load_kernels_mix_slab, load_kernels_mix_chirp, load_kernels_gate,
                                       load_kernels_prefix, load_kernels_project, load_kernels_wrm};
    for (auto load : loaders) {
        const hipError_t e = load();
        if (e != hipSuccess) return fail_hip(e, "prepare: loading kernels");
    }
    unsigned char *static_base = nullptr;
    if ((rc = static_scratch(&static_base))) return rc;
    return make_lane();
}

size_t spectre_mix_workspace_bytes(int B, int L, int H, int d, spectre_dtype io) {
    (void)io;
    if (B < 1 || L < 2 || H < 1 || d < 2) return 0;
    const int BH = B * H;
    const int route = mix_route(BH, L, d);
    if (route == 0) return 0;
    if (route == 1) return 256;
    if (route == 3) return chirp_layout(BH, L, d).total();
    if (route == 4) return 256;
    const MixGroups m = mix_groups(BH, L, d, 1);
    return align256((size_t)BH * L * sizeof(float2)) + m.lanes * align256((size_t)m.chunk * L * (d / 2) * sizeof(float2));
}

static int check_mix_args(const void *v, const void *g, const void *out, int B, int L, int H, int d, spectre_dtype io,
                          const char *who) {
    if (!v || !g || !out) return fail(SPECTRE_EINVAL, "%s: null pointer", who);
    if (B < 1 || L < 1 || H < 1 || d < 1) return fail(SPECTRE_EINVAL, "%s: non-positive size", who);
    if (io != SPECTRE_F32 && io != SPECTRE_BF16) return fail(SPECTRE_EINVAL, "%s: bad dtype", who);
    if ((long long)B * H > 0x7fffffffLL / 64) return fail(SPECTRE_EUNSUPPORTED, "%s: B*H too large", who);
    const size_t bytes = (size_t)B * L * H * d * (io == SPECTRE_BF16 ? 2 : 4);
    const char *vb = static_cast<const char *>(v), *ob = static_cast<const char *>(out);
    if (vb < ob + bytes && ob < vb + bytes) return fail(SPECTRE_EINVAL, "%s: out overlaps v", who);
    return SPECTRE_OK;
}

// The four-step route: gate expansion, then per head group the row transforms, the column kernel and the inverse
// row transforms.  gp = expanded gate [BH][L]; lane_scr[i] = transform scratch of lane i (lane_bytes each).
// side == nullptr keeps every group on st.
// wpack != nullptr: v is the layer input X and the row transforms project it first (bf16 rows, fp32 scratch);
// bsum != nullptr: the inverse row transforms also emit the sums of their blocks of adjacent rows.
static int mix_four_step(const Pow2Plan &pl, const void *v, const float2 *g, void *out, int BH, int L, int H, int d,
                         spectre_dtype io, float2 *gp, char *scr_base, size_t lane_bytes, const MixGroups &mg,
                         bool scr16, SideLane *side, hipStream_t st, const void *wpack = nullptr, int Hw = 0,
                         float2 *bsum = nullptr) {
    hipError_t e = hipSuccess;
    if (side) {
        // fork: the helper stream starts after everything before this call on the caller's stream.  Its first
        // kernel (row transforms) does not read the gate, so it runs beside the gate expansion; the column kernel
        // that follows waits for the event recorded behind the expansion.
        e = hipEventRecord(side->fork, st);
        if (e == hipSuccess) e = hipStreamWaitEvent(side->stream, side->fork, 0);
        if (e != hipSuccess) return fail_hip(e, "fork to helper stream");
    }
    const char *what = nullptr;
    e = launch_gate_expand(pl, g, gp, BH, st);
    if (e != hipSuccess) what = "gate_expand";
    if (!what && side) {
        e = hipEventRecord(side->gate, st);
        if (e != hipSuccess) what = "event behind the gate expansion";
    }
    bool side_has_gate = false;
    for (int group = 0, bh0 = 0; group < mg.ngroups && !what; ++group) {
        const int nbh = mg.size(group);
        if (nbh < 1) continue;
        const int lane = side ? (group & 1) : 0;
        hipStream_t ls = lane ? side->stream : st;
        float2 *scr = reinterpret_cast<float2 *>(scr_base + (size_t)lane * lane_bytes);
        // short columns (L <= 12288): a head's scratch fits the 4 MB L2 of one XCD, see head_affine() in mix_pow2.hip;
        // measured -7 % at L = 8192, -10 % at 4096 (three kernels), nothing or a loss from 16384 on
        const bool affine = !scr16 && nbh % 8 == 0 && (size_t)L * (d / 2) * sizeof(float2) <= ((size_t)3 << 20) &&
                            option(SPECTRE_OPT_HEAD_AFFINE) != 0;
        e = wpack ? launch_small_fwd_proj(pl, v, wpack, Hw, scr, L, H, bh0, nbh, ls, affine)
                  : launch_small_fwd(pl, (int)io, v, scr, L, H, bh0, nbh, ls, scr16, affine);
        if (e != hipSuccess) { what = "small_fwd"; break; }
        if (lane && !side_has_gate) {
            e = hipStreamWaitEvent(side->stream, side->gate, 0);
            if (e != hipSuccess) { what = "wait for the gate expansion"; break; }
            side_has_gate = true;
        }
        e = launch_big(pl, scr, gp, bh0, nbh, 0, ls, false, scr16, affine, side != nullptr);
        if (e != hipSuccess) { what = "big"; break; }
        e = launch_small_inv(pl, (int)io, scr, out, 0, L, H, bh0, nbh, ls, 0, 0, 0, scr16, affine, bsum);
        if (e != hipSuccess) { what = "small_inv"; break; }
        bh0 += nbh;
    }
    if (side) {
        // join: the caller's stream continues after the helper stream's last kernel (also on a launch error,
        // so that nothing of this call is left running unordered)
        hipError_t ej = hipEventRecord(side->join, side->stream);
        if (ej == hipSuccess) ej = hipStreamWaitEvent(st, side->join, 0);
        if (!what && ej != hipSuccess) {
            e = ej;
            what = "join from helper stream";
        }
    }
    if (what) return fail_hip(e, what);
    return SPECTRE_OK;
}

int spectre_mix_forward_ex(const void *v, const void *g, void *out, int B, int L, int H, int d,
                           spectre_dtype io, unsigned flags, void *ws, size_t ws_bytes, void *stream) {
    int rc = check_mix_args(v, g, out, B, L, H, d, io, "mix_forward");
    if (rc) return rc;
    if (flags & ~(unsigned)SPECTRE_MIX_BF16_SCRATCH) return fail(SPECTRE_EINVAL, "mix_forward: unknown flag bits");
    if (!spectre_length_supported(L, d))
        return fail(SPECTRE_EUNSUPPORTED, "mix_forward: no kernel for L=%d, d=%d", L, d);
    const size_t need = spectre_mix_workspace_bytes(B, L, H, d, io);
    if (!ws || ws_bytes < need)
        return fail(SPECTRE_EWORKSPACE, "mix_forward: workspace %zu < %zu bytes", ws_bytes, need);
    if (reinterpret_cast<uintptr_t>(ws) & 255) return fail(SPECTRE_EINVAL, "mix_forward: ws not 256-byte aligned");

    hipStream_t st = static_cast<hipStream_t>(stream);
    const int BH = B * H;
    const int route = mix_route(BH, L, d);
    if (route == 1) {
        const float2 *roots = nullptr;
        rc = get_roots(L, &roots);
        if (rc) return rc;
        const int *order = nullptr;
        rc = get_slab_order(L, &order);
        if (rc) return rc;
        hipError_t e = launch_mix_slab((int)io, v, static_cast<const float2 *>(g), out, roots, order, B, L, H, st);
        if (e != hipSuccess) return fail_hip(e, "mix_slab");
        return SPECTRE_OK;
    }
    if (route == 3) return mix_chirp(v, static_cast<const float2 *>(g), out, B, L, H, d, io, ws, st);
    if (route == 4) {
        const float2 *tw = nullptr;
        rc = get_roots(4096, &tw);
        if (rc) return rc;
        hipError_t e = launch_fused((int)io, v, static_cast<const float2 *>(g), out, tw, L, H, BH, st);
        if (e != hipSuccess) return fail_hip(e, "fused mixer");
        return SPECTRE_OK;
    }
    Pow2Plan pl;
    rc = get_pow2_plan(L, &pl);
    if (rc) return rc;
    float2 *gp = static_cast<float2 *>(ws);
    char *scr_base = static_cast<char *>(ws) + align256((size_t)BH * L * sizeof(float2));
    // on request, bf16 rows only: complex numbers cross between the three kernels as two bfloat16 instead of two
    // fp32, and twice the heads fit in a lane's scratch
    const bool scr16 = (io == SPECTRE_BF16) && (flags & SPECTRE_MIX_BF16_SCRATCH);
    const MixGroups m1 = mix_groups(BH, L, d, 1);
    const size_t lane_bytes = align256((size_t)m1.chunk * L * (d / 2) * sizeof(float2));   // as the workspace was sized
    MixGroups mg = scr16 ? mix_groups(BH, L, d, 2) : m1;
    if (scr16 && (mg.lanes != m1.lanes || (size_t)mg.chunk * L * (d / 2) * sizeof(uint32_t) > lane_bytes)) mg = m1;
    SideLane *side = nullptr;
    int dev = 0;
    if (mg.lanes == 2) {
        rc = acquire_lane(&dev, &side);
        if (rc) return rc;
    }
    rc = mix_four_step(pl, v, static_cast<const float2 *>(g), out, BH, L, H, d, io, gp, scr_base, lane_bytes, mg, scr16,
                       side, st);
    if (side) release_lane(dev, side);
    return rc;
}

int spectre_mix_forward(const void *v, const void *g, void *out, int B, int L, int H, int d,
                        spectre_dtype io, void *ws, size_t ws_bytes, void *stream) {
    return spectre_mix_forward_ex(v, g, out, B, L, H, d, io, 0u, ws, ws_bytes, stream);
}

size_t spectre_mix_static_bytes(void) { return kStaticBytes; }

int spectre_mix_forward_static(const void *v, const void *g, void *out, int B, int L, int H, int d,
                               spectre_dtype io, void *stream) {
    int rc = check_mix_args(v, g, out, B, L, H, d, io, "mix_forward_static");
    if (rc) return rc;
    int N1, N2, P;
    if (d != 64 || !pow2_split(L, &N1, &N2, &P))
        return fail(SPECTRE_EUNSUPPORTED, "mix_forward_static: only the four-step lengths (256 ... 131072) with d = 64, not L=%d, d=%d", L, d);
    const size_t BH = (size_t)B * H, per_head = (size_t)L * (d / 2) * sizeof(float2);
    if (BH * L * sizeof(float2) > kStaticGate)
        return fail(SPECTRE_EUNSUPPORTED, "mix_forward_static: B*H*L = %zu bins exceeds the built-in scratch (%zu bins)",
                    BH * L, kStaticGate / sizeof(float2));
    if (per_head > kStaticColumns || (size_t)(L + N1) * sizeof(float2) > kStaticTables)
        return fail(SPECTRE_EUNSUPPORTED, "mix_forward_static: L=%d exceeds the built-in scratch", L);
    unsigned char *base = nullptr;
    rc = static_scratch(&base);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // everything the kernels read from the array is written earlier in this same call (tables, gate planes, columns):
    // nothing has to start at zero, and what the previous call left behind is never read
    float2 *twL = reinterpret_cast<float2 *>(base), *twN1 = twL + L;
    float2 *gp = reinterpret_cast<float2 *>(base + kStaticTables);
    char *columns = reinterpret_cast<char *>(base + kStaticTables + kStaticGate);
    hipError_t e = launch_fill_twiddle(twL, L, st);
    if (e == hipSuccess) e = launch_fill_twiddle(twN1, N1, st);
    if (e != hipSuccess) return fail_hip(e, "fill_twiddle");
    Pow2Plan pl;
    pl.L = L; pl.N1 = N1; pl.N2 = N2; pl.P = P; pl.twL = twL; pl.twN1 = twN1;
    MixGroups mg;                                      // one lane, groups of as many heads as the columns area holds
    mg.BH = (int)BH;
    mg.chunk = (int)(kStaticColumns / per_head < BH ? kStaticColumns / per_head : BH);
    mg.ngroups = ((int)BH + mg.chunk - 1) / mg.chunk;
    return mix_four_step(pl, v, static_cast<const float2 *>(g), out, (int)BH, L, H, d, io, gp, columns, 0, mg, false,
                         nullptr, st);
}

// ------------------------------------------------------------------------------------------ gate
static int check_gate_params(const spectre_gate_params *P, int H, const char *who) {
    if (!P) return fail(SPECTRE_EINVAL, "%s: null gate parameters", who);
    if (!(P->Hg == H || P->Hg == 1)) return fail(SPECTRE_EINVAL, "%s: Hg must be H or 1", who);
    if (P->d < 2 || P->d > 256 || (P->d & 1)) return fail(SPECTRE_EUNSUPPORTED, "%s: d=%d not in 2..256 even", who, P->d);
    if (P->d_g < 1 || P->d_g > 256) return fail(SPECTRE_EUNSUPPORTED, "%s: d_g=%d not in 1..256", who, P->d_g);
    if (P->n_fft < 2) return fail(SPECTRE_EINVAL, "%s: n_fft < 2", who);
    if (!P->ln_gamma || !P->ln_beta || !P->W1 || !P->b1 || !P->W2 || !P->b2)
        return fail(SPECTRE_EINVAL, "%s: null parameter array", who);
    if (!(P->ln_eps >= 0.0f)) return fail(SPECTRE_EINVAL, "%s: ln_eps must be >= 0", who);
    if (P->toeplitz && (P->toeplitz_r < 0 || P->toeplitz_r > 64))
        return fail(SPECTRE_EUNSUPPORTED, "%s: toeplitz_r=%d not in 0..64", who, P->toeplitz_r);
    return SPECTRE_OK;
}

static GateDev gate_dev(const spectre_gate_params *P) {
    GateDev g;
    g.Hg = P->Hg; g.d = P->d; g.d_g = P->d_g; g.n_fft = P->n_fft;
    g.ln_gamma = P->ln_gamma; g.ln_beta = P->ln_beta; g.ln_eps = P->ln_eps;
    g.W1 = P->W1; g.b1 = P->b1; g.W2 = P->W2; g.b2 = P->b2; g.modrelu_bias = P->modrelu_bias;
    g.toeplitz = reinterpret_cast<const float2 *>(P->toeplitz);
    g.toeplitz_r = P->toeplitz ? P->toeplitz_r : 0;
    return g;
}

// scratch for the un-activated MLP output, needed only with the Toeplitz update
static size_t gate_raw_bytes(int B, int H, const spectre_gate_params *P) {
    return P->toeplitz ? align256((size_t)B * H * (P->n_fft / 2 + 1) * sizeof(float2)) : 0;
}

size_t spectre_gate_workspace_bytes(int B, int L, int H, const spectre_gate_params *P) {
    if (!P || B < 1 || L < 1 || H < 1 || P->d < 2 || P->d_g < 1) return 0;
    return align256(gate_partial_bytes(B, L, H, P->d)) + align256((size_t)B * H * P->d * sizeof(double)) +
           align256((size_t)B * H * P->d_g * sizeof(float)) + gate_raw_bytes(B, H, P);
}

int spectre_gate(const void *q, int q_is_pooled, spectre_dtype q_dtype, double inv_count,
                 const spectre_gate_params *P, int B, int L, int H, long long phase_pos, void *g_out, void *ws,
                 size_t ws_bytes, void *stream) {
    if (!q || !g_out) return fail(SPECTRE_EINVAL, "gate: null pointer");
    if (B < 1 || H < 1 || (!q_is_pooled && L < 1)) return fail(SPECTRE_EINVAL, "gate: non-positive size");
    if (!q_is_pooled && q_dtype != SPECTRE_F32 && q_dtype != SPECTRE_BF16) return fail(SPECTRE_EINVAL, "gate: bad dtype");
    if (phase_pos < 0) return fail(SPECTRE_EINVAL, "gate: negative phase position");
    if (!(inv_count == inv_count)) return fail(SPECTRE_EINVAL, "gate: inv_count is NaN");
    int rc = check_gate_params(P, H, "gate");
    if (rc) return rc;
    if (q_is_pooled) L = 1;
    if ((long long)B * H * P->d > 0x7fffffffLL) return fail(SPECTRE_EUNSUPPORTED, "gate: B*H*d too large");
    const size_t need = spectre_gate_workspace_bytes(B, L, H, P);
    if (!ws || ws_bytes < need) return fail(SPECTRE_EWORKSPACE, "gate: workspace %zu < %zu bytes", ws_bytes, need);
    if (reinterpret_cast<uintptr_t>(ws) & 255) return fail(SPECTRE_EINVAL, "gate: ws not 256-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *w = static_cast<char *>(ws);
    double *partial = reinterpret_cast<double *>(w);
    w += align256(gate_partial_bytes(B, L, H, P->d));
    double *sum_ws = reinterpret_cast<double *>(w);
    w += align256((size_t)B * H * P->d * sizeof(double));
    float *hid = reinterpret_cast<float *>(w);
    w += align256((size_t)B * H * P->d_g * sizeof(float));
    float2 *raw = reinterpret_cast<float2 *>(w);
    const double *sum_q = static_cast<const double *>(q);
    if (!q_is_pooled) {
        hipError_t e = launch_pool((int)q_dtype, q, partial, sum_ws, B, L, H, P->d, st);
        if (e != hipSuccess) return fail_hip(e, "pool");
        sum_q = sum_ws;
    }
    hipError_t e = launch_gate_mlp(sum_q, inv_count, gate_dev(P), hid, raw, B, H, phase_pos % P->n_fft,
                                   static_cast<float2 *>(g_out), st);
    if (e != hipSuccess) return fail_hip(e, "gate_mlp");
    return SPECTRE_OK;
}

// ------------------------------------------------------------------------------------------ projection
size_t spectre_project_workspace_bytes(int B, int L, int H, int d) {
    if (B < 1 || L < 1 || H < 1 || d != 64) return 0;
    return align256((size_t)B * project_chunks(L) * H * d * sizeof(double)) + align256((size_t)B * H * d * sizeof(double));
}

int spectre_project(const void *x, const float *Wq, const float *Wv, int Hw, int B, int L, int H, int d,
                    spectre_dtype io, void *v_out, void *q_out, void *sum_q, void *ws, size_t ws_bytes, void *stream) {
    if (!x || !Wq || !Wv || !v_out) return fail(SPECTRE_EINVAL, "project: null pointer");
    if (B < 1 || L < 1 || H < 1 || d < 1) return fail(SPECTRE_EINVAL, "project: non-positive size");
    if (io != SPECTRE_F32 && io != SPECTRE_BF16) return fail(SPECTRE_EINVAL, "project: bad dtype");
    if (!(Hw == H || Hw == 1)) return fail(SPECTRE_EINVAL, "project: Hw must be H or 1");
    if (d != 64) return fail(SPECTRE_EUNSUPPORTED, "project: d=%d (only 64 is built)", d);
    if (H > 65535 || B > 65535) return fail(SPECTRE_EUNSUPPORTED, "project: H or B above 65535");
    const size_t bytes = (size_t)B * L * H * d * (io == SPECTRE_BF16 ? 2 : 4);
    const char *xb = static_cast<const char *>(x);
    for (const void *o : {static_cast<const void *>(v_out), static_cast<const void *>(q_out)}) {
        const char *ob = static_cast<const char *>(o);
        if (ob && xb < ob + bytes && ob < xb + bytes) return fail(SPECTRE_EINVAL, "project: output overlaps x");
    }
    if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(v_out) | reinterpret_cast<uintptr_t>(q_out)) & 15)
        return fail(SPECTRE_EINVAL, "project: tensors must be 16-byte aligned");
    const size_t need = spectre_project_workspace_bytes(B, L, H, d);
    if (!ws || ws_bytes < need) return fail(SPECTRE_EWORKSPACE, "project: workspace %zu < %zu bytes", ws_bytes, need);
    if (reinterpret_cast<uintptr_t>(ws) & 255) return fail(SPECTRE_EINVAL, "project: ws not 256-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    double *partial = static_cast<double *>(ws);
    double *sum_x = reinterpret_cast<double *>(static_cast<char *>(ws) +
                                               align256((size_t)B * project_chunks(L) * H * d * sizeof(double)));
    hipError_t e = launch_project((int)io, x, Wq, Wv, Hw, v_out, q_out, partial, B, L, H, st);
    if (e != hipSuccess) return fail_hip(e, "project");
    if (sum_q) {
        e = launch_pool_final(partial, sum_x, B, H * d, project_chunks(L), st);
        if (e != hipSuccess) return fail_hip(e, "pool_final");
        e = launch_project_pooled(sum_x, Wq, Hw, B, H, static_cast<double *>(sum_q), st);
        if (e != hipSuccess) return fail_hip(e, "project_pooled");
    }
    return SPECTRE_OK;
}

// ------------------------------------------------------------------------------------------ wavelet refinement
static int check_wrm_params(const spectre_wrm_params *P, int H, const char *who) {
    if (!P) return fail(SPECTRE_EINVAL, "%s: null parameters", who);
    if (!(P->Hg == H || P->Hg == 1)) return fail(SPECTRE_EINVAL, "%s: Hg must be H or 1", who);
    if (P->d < 1 || P->d > 256) return fail(SPECTRE_EUNSUPPORTED, "%s: d=%d not in 1..256", who, P->d);
    if (P->d_w < 1 || P->d_w > 256) return fail(SPECTRE_EUNSUPPORTED, "%s: d_w=%d not in 1..256", who, P->d_w);
    if (P->levels < 0 || P->levels > 30) return fail(SPECTRE_EINVAL, "%s: levels=%d not in 0..30", who, P->levels);
    if (!P->ln_gamma || !P->ln_beta || !P->W1 || !P->b1 || !P->W2 || !P->b2)
        return fail(SPECTRE_EINVAL, "%s: null parameter array", who);
    if (!(P->ln_eps >= 0.0f)) return fail(SPECTRE_EINVAL, "%s: ln_eps must be >= 0", who);
    return SPECTRE_OK;
}

size_t spectre_wrm_gates_workspace_bytes(int B, int L, int H, const spectre_wrm_params *P) {
    if (!P || B < 1 || L < 1 || H < 1 || P->d < 1) return 0;
    return align256(gate_partial_bytes(B, L, H, P->d)) + align256((size_t)B * H * P->d * sizeof(double));
}

int spectre_wrm_gates(const void *q, int q_is_pooled, spectre_dtype q_dtype, double inv_count,
                      const spectre_wrm_params *P, int B, int L, int H, void *s_out, void *ws, size_t ws_bytes,
                      void *stream) {
    if (!q || !s_out) return fail(SPECTRE_EINVAL, "wrm_gates: null pointer");
    if (B < 1 || H < 1 || (!q_is_pooled && L < 1)) return fail(SPECTRE_EINVAL, "wrm_gates: non-positive size");
    if (!q_is_pooled && q_dtype != SPECTRE_F32 && q_dtype != SPECTRE_BF16)
        return fail(SPECTRE_EINVAL, "wrm_gates: bad dtype");
    if (!(inv_count == inv_count)) return fail(SPECTRE_EINVAL, "wrm_gates: inv_count is NaN");
    int rc = check_wrm_params(P, H, "wrm_gates");
    if (rc) return rc;
    if (q_is_pooled) L = 1;
    if ((long long)B * H * P->d > 0x7fffffffLL) return fail(SPECTRE_EUNSUPPORTED, "wrm_gates: B*H*d too large");
    const size_t need = spectre_wrm_gates_workspace_bytes(B, L, H, P);
    if (!ws || ws_bytes < need) return fail(SPECTRE_EWORKSPACE, "wrm_gates: workspace %zu < %zu bytes", ws_bytes, need);
    if (reinterpret_cast<uintptr_t>(ws) & 255) return fail(SPECTRE_EINVAL, "wrm_gates: ws not 256-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *w = static_cast<char *>(ws);
    double *partial = reinterpret_cast<double *>(w);
    w += align256(gate_partial_bytes(B, L, H, P->d));
    double *sum_ws = reinterpret_cast<double *>(w);
    const double *sum_q = static_cast<const double *>(q);
    if (!q_is_pooled) {
        hipError_t e = launch_pool((int)q_dtype, q, partial, sum_ws, B, L, H, P->d, st);
        if (e != hipSuccess) return fail_hip(e, "pool");
        sum_q = sum_ws;
    }
    WrmDev D;
    D.Hg = P->Hg; D.d = P->d; D.d_w = P->d_w; D.levels = P->levels;
    D.ln_gamma = P->ln_gamma; D.ln_beta = P->ln_beta; D.ln_eps = P->ln_eps;
    D.W1 = P->W1; D.b1 = P->b1; D.W2 = P->W2; D.b2 = P->b2;
    hipError_t e = launch_wrm_gates(sum_q, inv_count, D, B, H, static_cast<float *>(s_out), st);
    if (e != hipSuccess) return fail_hip(e, "wrm_gates");
    return SPECTRE_OK;
}

size_t spectre_wrm_apply_workspace_bytes(int B, int L, int H, int d, int levels) {
    if (B < 1 || L < 1 || H < 1 || d != 64 || levels < 0 || levels > 30) return 0;
    if (levels > 0 && (L % (1LL << levels)) != 0) return 0;
    return 256 + 2 * align256(wrm_scratch_floats(B * H, L, levels) * sizeof(float));
}

int spectre_wrm_apply(const void *v, const void *s, void *out, int B, int L, int H, int d, int levels,
                      spectre_dtype io, void *ws, size_t ws_bytes, void *stream) {
    if (!v || !s || !out) return fail(SPECTRE_EINVAL, "wrm_apply: null pointer");
    if (B < 1 || L < 1 || H < 1 || d < 1) return fail(SPECTRE_EINVAL, "wrm_apply: non-positive size");
    if (io != SPECTRE_F32 && io != SPECTRE_BF16) return fail(SPECTRE_EINVAL, "wrm_apply: bad dtype");
    if (levels < 0 || levels > 30) return fail(SPECTRE_EINVAL, "wrm_apply: levels=%d not in 0..30", levels);
    if (levels > 0 && (L % (1LL << levels)) != 0)
        return fail(SPECTRE_EINVAL, "wrm_apply: 2^%d does not divide L=%d", levels, L);
    if (d != 64) return fail(SPECTRE_EUNSUPPORTED, "wrm_apply: d=%d (only 64 is built)", d);
    if (B > 65535 || (L + kWrmTileRows - 1) / kWrmTileRows > 65535)
        return fail(SPECTRE_EUNSUPPORTED, "wrm_apply: B or L/256 above 65535");
    if (levels > kWrmTileLevels && L > 262144)
        return fail(SPECTRE_EUNSUPPORTED, "wrm_apply: more than 8 levels needs L <= 262144");
    const size_t bytes = (size_t)B * L * H * d * (io == SPECTRE_BF16 ? 2 : 4);
    const char *vb = static_cast<const char *>(v), *ob = static_cast<const char *>(out);
    if (vb != ob && vb < ob + bytes && ob < vb + bytes)
        return fail(SPECTRE_EINVAL, "wrm_apply: out overlaps v without being v");
    const size_t need = spectre_wrm_apply_workspace_bytes(B, L, H, d, levels);
    if (!ws || ws_bytes < need) return fail(SPECTRE_EWORKSPACE, "wrm_apply: workspace %zu < %zu bytes", ws_bytes, need);
    if (reinterpret_cast<uintptr_t>(ws) & 255) return fail(SPECTRE_EINVAL, "wrm_apply: ws not 256-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t part = align256(wrm_scratch_floats(B * H, L, levels) * sizeof(float));
    float *tile_sums = static_cast<float *>(ws);
    float *upper = reinterpret_cast<float *>(static_cast<char *>(ws) + part);
    hipError_t e = launch_wrm_apply((int)io, v, static_cast<const float *>(s), out, tile_sums, upper, B, L, H, levels, st);
    if (e != hipSuccess) return fail_hip(e, "wrm_apply");
    return SPECTRE_OK;
}

int spectre_wrm_apply_coeff(const void *v, const void *s, void *out, int B, int L, int H, int d, int levels,
                            spectre_dtype io, void *ws, size_t ws_bytes, void *stream) {
    if (!v || !s || !out) return fail(SPECTRE_EINVAL, "wrm_apply_coeff: null pointer");
    if (B < 1 || L < 1 || H < 1 || d < 1) return fail(SPECTRE_EINVAL, "wrm_apply_coeff: non-positive size");
    if (io != SPECTRE_F32 && io != SPECTRE_BF16) return fail(SPECTRE_EINVAL, "wrm_apply_coeff: bad dtype");
    if (levels < 0 || levels > 30) return fail(SPECTRE_EINVAL, "wrm_apply_coeff: levels=%d not in 0..30", levels);
    if (levels > 0 && (L % (1LL << levels)) != 0)
        return fail(SPECTRE_EINVAL, "wrm_apply_coeff: 2^%d does not divide L=%d", levels, L);
    if (d != 64) return fail(SPECTRE_EUNSUPPORTED, "wrm_apply_coeff: d=%d (only 64 is built)", d);
    if (B > 65535 || (L + kWrmTileRows - 1) / kWrmTileRows > 65535)
        return fail(SPECTRE_EUNSUPPORTED, "wrm_apply_coeff: B or L/256 above 65535");
    if (levels > kWrmTileLevels && L > 262144)
        return fail(SPECTRE_EUNSUPPORTED, "wrm_apply_coeff: more than 8 levels needs L <= 262144");
    if (reinterpret_cast<uintptr_t>(s) & 7) return fail(SPECTRE_EINVAL, "wrm_apply_coeff: s must be 8-byte aligned");
    const size_t bytes = (size_t)B * L * H * d * (io == SPECTRE_BF16 ? 2 : 4);
    const char *vb = static_cast<const char *>(v), *ob = static_cast<const char *>(out);
    if (vb != ob && vb < ob + bytes && ob < vb + bytes)
        return fail(SPECTRE_EINVAL, "wrm_apply_coeff: out overlaps v without being v");
    const char *sb = static_cast<const char *>(s);
    const size_t sbytes = (size_t)B * L * H * d * sizeof(float);
    if (sb < ob + bytes && ob < sb + sbytes) return fail(SPECTRE_EINVAL, "wrm_apply_coeff: out overlaps s");
    const size_t need = spectre_wrm_apply_workspace_bytes(B, L, H, d, levels);
    if (!ws || ws_bytes < need) return fail(SPECTRE_EWORKSPACE, "wrm_apply_coeff: workspace %zu < %zu bytes", ws_bytes, need);
    if (reinterpret_cast<uintptr_t>(ws) & 255) return fail(SPECTRE_EINVAL, "wrm_apply_coeff: ws not 256-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t part = align256(wrm_scratch_floats(B * H, L, levels) * sizeof(float));
    float *tile_sums = static_cast<float *>(ws);
    float *upper = reinterpret_cast<float *>(static_cast<char *>(ws) + part);
    hipError_t e = launch_wrm_apply_coeff((int)io, v, static_cast<const float *>(s), out, tile_sums, upper, B, L, H, levels, st);
    if (e != hipSuccess) return fail_hip(e, "wrm_apply_coeff");
    return SPECTRE_OK;
}

// ------------------------------------------------------------------------------------------ whole layer
// Workspace sections of spectre_layer_forward.
struct LayerLayout {
    bool fused;                   // projection inside the row transforms (four-step route, bf16 rows)
    bool sums;                    // block sums from the inverse row transforms feed the refinement
    size_t partial, sum_x, sum_q, hid, raw, g, wpack, mix, vbuf, s, wrm, bsum;
    size_t total() const { return partial + sum_x + sum_q + hid + raw + g + wpack + mix + vbuf + s + wrm + bsum; }
};
static LayerLayout layer_layout(int B, int L, int H, int d, spectre_dtype io, const spectre_gate_params *P,
                                const spectre_wrm_params *W) {
    LayerLayout y;
    const size_t BH = (size_t)B * H, esize = (io == SPECTRE_BF16) ? 2 : 4;
    y.fused = (io == SPECTRE_BF16) && mix_route((int)BH, L, d) == 2;
    y.sums = y.fused && W && W->levels > kWrmTileLevels;
    const size_t pool = align256(gate_partial_bytes(B, L, H, d));
    const size_t proj = align256((size_t)B * project_chunks(L) * H * d * sizeof(double));
    y.partial = pool > proj ? pool : proj;
    y.sum_x = y.sum_q = align256(BH * d * sizeof(double));
    y.hid = align256(BH * P->d_g * sizeof(float));
    y.raw = gate_raw_bytes(B, H, P);
    y.g = align256(BH * (size_t)(L / 2 + 1) * sizeof(float2));
    y.wpack = y.fused ? align256((size_t)H * kProjPackBytes) : 0;
    y.mix = align256(spectre_mix_workspace_bytes(B, L, H, d, io));
    y.vbuf = y.fused ? 0 : align256(BH * (size_t)L * d * esize);
    y.s = W ? align256(BH * (size_t)(W->levels + 1) * d * sizeof(float)) : 0;
    y.wrm = W ? align256(spectre_wrm_apply_workspace_bytes(B, L, H, d, W->levels)) : 0;
    y.bsum = y.sums ? align256(BH * (size_t)(L / small_tile_rows((int)io)) * d * sizeof(float)) : 0;
    return y;
}

static int check_layer_args(int B, int L, int H, int d, spectre_dtype io, const spectre_gate_params *P,
                            const spectre_wrm_params *W, const char *who) {
    if (B < 1 || L < 1 || H < 1 || d < 1) return fail(SPECTRE_EINVAL, "%s: non-positive size", who);
    if (io != SPECTRE_F32 && io != SPECTRE_BF16) return fail(SPECTRE_EINVAL, "%s: bad dtype", who);
    if (d != 64) return fail(SPECTRE_EUNSUPPORTED, "%s: d=%d (only 64 is built)", who, d);
    if (H > 65535 || B > 65535) return fail(SPECTRE_EUNSUPPORTED, "%s: H or B above 65535", who);
    if ((long long)B * H > 0x7fffffffLL / 64) return fail(SPECTRE_EUNSUPPORTED, "%s: B*H too large", who);
    int rc = check_gate_params(P, H, who);
    if (rc) return rc;
    if (P->n_fft != L || P->d != d) return fail(SPECTRE_EINVAL, "%s: gate is for n_fft=%d, d=%d", who, P->n_fft, P->d);
    if (!spectre_length_supported(L, d)) return fail(SPECTRE_EUNSUPPORTED, "%s: no kernel for L=%d, d=%d", who, L, d);
    if (W) {
        rc = check_wrm_params(W, H, who);
        if (rc) return rc;
        if (W->d != d) return fail(SPECTRE_EINVAL, "%s: refinement parameters are for d=%d", who, W->d);
        if (W->levels > 0 && (L % (1LL << W->levels)) != 0)
            return fail(SPECTRE_EINVAL, "%s: 2^%d does not divide L=%d", who, W->levels, L);
        if (spectre_wrm_apply_workspace_bytes(B, L, H, d, W->levels) == 0 || (L + kWrmTileRows - 1) / kWrmTileRows > 65535 ||
            (W->levels > kWrmTileLevels && L > 262144))
            return fail(SPECTRE_EUNSUPPORTED, "%s: refinement not available for L=%d, levels=%d", who, L, W->levels);
    }
    return SPECTRE_OK;
}

size_t spectre_layer_workspace_bytes(int B, int L, int H, int d, spectre_dtype io, const spectre_gate_params *P,
                                     const spectre_wrm_params *W) {
    if (!P || check_layer_args(B, L, H, d, io, P, W, "layer_workspace_bytes")) return 0;
    return layer_layout(B, L, H, d, io, P, W).total();
}

int spectre_layer_forward(const void *x, const float *Wq, const float *Wv, int Hw, const spectre_gate_params *P,
                          const spectre_wrm_params *W, void *out, int B, int L, int H, int d, spectre_dtype io,
                          void *ws, size_t ws_bytes, void *stream) {
    if (!x || !Wq || !Wv || !out) return fail(SPECTRE_EINVAL, "layer_forward: null pointer");
    if (!P) return fail(SPECTRE_EINVAL, "layer_forward: null gate parameters");
    int rc = check_layer_args(B, L, H, d, io, P, W, "layer_forward");
    if (rc) return rc;
    if (!(Hw == H || Hw == 1)) return fail(SPECTRE_EINVAL, "layer_forward: Hw must be H or 1");
    const size_t bytes = (size_t)B * L * H * d * (io == SPECTRE_BF16 ? 2 : 4);
    const char *xb = static_cast<const char *>(x), *ob = static_cast<const char *>(out);
    if (xb < ob + bytes && ob < xb + bytes) return fail(SPECTRE_EINVAL, "layer_forward: out overlaps x");
    if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(out)) & 15)
        return fail(SPECTRE_EINVAL, "layer_forward: tensors must be 16-byte aligned");
    const LayerLayout y = layer_layout(B, L, H, d, io, P, W);
    if (!ws || ws_bytes < y.total()) return fail(SPECTRE_EWORKSPACE, "layer_forward: workspace %zu < %zu bytes", ws_bytes, y.total());
    if (reinterpret_cast<uintptr_t>(ws) & 255) return fail(SPECTRE_EINVAL, "layer_forward: ws not 256-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int BH = B * H;
    char *w = static_cast<char *>(ws);
    auto take = [&](size_t n) { char *p0 = w; w += n; return p0; };
    double *partial = reinterpret_cast<double *>(take(y.partial));
    double *sum_x = reinterpret_cast<double *>(take(y.sum_x));
    double *sum_q = reinterpret_cast<double *>(take(y.sum_q));
    float *hid = reinterpret_cast<float *>(take(y.hid));
    float2 *raw = reinterpret_cast<float2 *>(take(y.raw));
    float2 *g = reinterpret_cast<float2 *>(take(y.g));
    void *wpack = take(y.wpack);
    char *mix_ws = take(y.mix);
    void *vbuf = take(y.vbuf);
    float *s_lv = reinterpret_cast<float *>(take(y.s));
    char *wrm_ws = take(y.wrm);
    float2 *bsum = y.sums ? reinterpret_cast<float2 *>(take(y.bsum)) : nullptr;

    // every table look-up before the first launch
    Pow2Plan pl;
    SideLane *side = nullptr;
    int dev = 0;
    MixGroups mg;
    if (y.fused) {
        rc = get_pow2_plan(L, &pl);
        if (rc) return rc;
        mg = mix_groups(BH, L, d, 1);
    } else {
        const float2 *probe = nullptr;                 // the unfused mixer call below looks its tables up itself; make
        const int route = mix_route(BH, L, d);         // sure it cannot fail after the projection has been enqueued
        if (route == 1 || route == 2) rc = get_roots(L, &probe);
        else if (route == 4) rc = get_roots(4096, &probe);
        else rc = get_roots(chirp_padded_length(L), &probe);
        if (rc) return rc;
    }
    hipError_t e;
    if (y.fused) {
        // pooled query: sum_q = (sum_l x_l) W_q (pooling commutes with the projection); the rows of X are read once
        // more by the row transforms, V itself never exists in memory
        e = launch_pool((int)io, x, partial, sum_x, B, L, H, d, st);
        if (e != hipSuccess) return fail_hip(e, "pool(x)");
        e = launch_pack_w(Wv, Hw, wpack, st);
        if (e != hipSuccess) return fail_hip(e, "pack_w");
    } else {
        e = launch_project((int)io, x, Wq, Wv, Hw, vbuf, nullptr, partial, B, L, H, st);
        if (e != hipSuccess) return fail_hip(e, "project");
        e = launch_pool_final(partial, sum_x, B, H * d, project_chunks(L), st);
        if (e != hipSuccess) return fail_hip(e, "pool_final");
    }
    e = launch_project_pooled(sum_x, Wq, Hw, B, H, sum_q, st);
    if (e != hipSuccess) return fail_hip(e, "project_pooled");
    e = launch_gate_mlp(sum_q, 1.0 / (double)L, gate_dev(P), hid, raw, B, H, 0, g, st);
    if (e != hipSuccess) return fail_hip(e, "gate_mlp");
    if (y.fused) {
        float2 *gp = reinterpret_cast<float2 *>(mix_ws);
        char *scr_base = mix_ws + align256((size_t)BH * L * sizeof(float2));
        const size_t lane_bytes = align256((size_t)mg.chunk * L * (d / 2) * sizeof(float2));
        if (mg.lanes == 2) {
            rc = acquire_lane(&dev, &side);
            if (rc) return rc;
        }
        rc = mix_four_step(pl, x, g, out, BH, L, H, d, io, gp, scr_base, lane_bytes, mg, false, side, st, wpack, Hw, bsum);
        if (side) release_lane(dev, side);
        if (rc) return rc;
    } else {
        rc = spectre_mix_forward_ex(vbuf, g, out, B, L, H, d, io, 0u, mix_ws, y.mix, stream);
        if (rc) return rc;
    }
    if (W) {
        WrmDev D;
        D.Hg = W->Hg; D.d = W->d; D.d_w = W->d_w; D.levels = W->levels;
        D.ln_gamma = W->ln_gamma; D.ln_beta = W->ln_beta; D.ln_eps = W->ln_eps;
        D.W1 = W->W1; D.b1 = W->b1; D.W2 = W->W2; D.b2 = W->b2;
        e = launch_wrm_gates(sum_q, 1.0 / (double)L, D, B, H, s_lv, st);
        if (e != hipSuccess) return fail_hip(e, "wrm_gates");
        const size_t part = align256(wrm_scratch_floats(BH, L, W->levels) * sizeof(float));
        float *tile_sums = reinterpret_cast<float *>(wrm_ws);
        float *upper = reinterpret_cast<float *>(wrm_ws + part);
        e = launch_wrm_apply((int)io, out, s_lv, out, tile_sums, upper, B, L, H, W->levels, st,
                             reinterpret_cast<const float *>(bsum), small_tile_rows((int)io));
        if (e != hipSuccess) return fail_hip(e, "wrm_apply");
    }
    return SPECTRE_OK;
}

// ------------------------------------------------------------------------------------------ prefix cache
static bool prefix_length_ok(int N, int d) {
    int N1, N2, P;
    return d == 64 && pow2_split(N, &N1, &N2, &P);
}

// Transform length of a cache: the pinned memory rows followed by the ring (Sec. 3.4).
static inline int window_len(const spectre_prefix_cache *c) { return c->N_max + c->N_mem; }

static int check_cache(const spectre_prefix_cache *c, const char *who) {
    if (!c) return fail(SPECTRE_EINVAL, "%s: null cache", who);
    if (c->B < 1 || c->H < 1 || c->d < 1 || c->N_max < 1 || c->N_mem < 0 || c->N_max > (1 << 30) || c->N_mem > (1 << 30))
        return fail(SPECTRE_EINVAL, "%s: bad cache dimensions", who);
    if (!prefix_length_ok(window_len(c), c->d))
        return fail(SPECTRE_EUNSUPPORTED, "%s: no kernel for N_mem+N_max=%d, d=%d", who, window_len(c), c->d);
    if (!c->prefix_fft || !c->v_buf || !c->q_buf || !c->sum_q || !c->twiddle)
        return fail(SPECTRE_EINVAL, "%s: null cache array", who);
    if (c->t < 0) return fail(SPECTRE_EINVAL, "%s: negative token counter", who);
    if (c->pending_cap < 0 || c->pending_cap > kMaxPending || (c->pending_cap > 0 && !c->pending) ||
        c->n_pending < 0 || c->n_pending > c->pending_cap)
        return fail(SPECTRE_EINVAL, "%s: bad deferred-update fields", who);
    if ((long long)c->B * c->H > 0x7fffffffLL / 64) return fail(SPECTRE_EUNSUPPORTED, "%s: B*H too large", who);
    return SPECTRE_OK;
}

size_t spectre_prefix_bytes(int B, int H, int d, int N_max, int which) {
    if (B < 1 || H < 1 || d < 1 || N_max < 2) return 0;
    if (!prefix_length_ok(N_max, d)) return 0;
    const size_t BH = (size_t)B * H, F = (size_t)N_max / 2 + 1;
    switch (which) {
        case SPECTRE_PREFIX_FFT: return BH * F * d * sizeof(float2);
        case SPECTRE_PREFIX_VBUF:
        case SPECTRE_PREFIX_QBUF: return BH * (size_t)N_max * d * sizeof(float);
        case SPECTRE_PREFIX_SUMQ: return BH * d * sizeof(double);
        case SPECTRE_PREFIX_TWIDDLE: return (size_t)N_max * sizeof(float2);
        default: return 0;
    }
}

int spectre_prefix_init(spectre_prefix_cache *c, void *stream) {
    int rc = check_cache(c, "prefix_init");
    if (rc) return rc;
    rc = spectre_prepare(window_len(c), c->d);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    void *arr[4] = {c->prefix_fft, c->v_buf, c->q_buf, c->sum_q};
    const int which[4] = {SPECTRE_PREFIX_FFT, SPECTRE_PREFIX_VBUF, SPECTRE_PREFIX_QBUF, SPECTRE_PREFIX_SUMQ};
    for (int i = 0; i < 4; ++i) {
        if (reinterpret_cast<uintptr_t>(arr[i]) & 15) return fail(SPECTRE_EINVAL, "prefix_init: cache array not 16-byte aligned");
        hipError_t e = launch_fill_zero(arr[i], spectre_prefix_bytes(c->B, c->H, c->d, window_len(c), which[i]), st);
        if (e != hipSuccess) return fail_hip(e, "fill_zero");
    }
    hipError_t e = launch_fill_twiddle(static_cast<float2 *>(c->twiddle), window_len(c), st);
    if (e != hipSuccess) return fail_hip(e, "fill_twiddle");
    c->t = 0;
    c->n_pending = 0;
    return SPECTRE_OK;
}

int spectre_prefix_flush(spectre_prefix_cache *c, void *stream) {
    int rc = check_cache(c, "prefix_flush");
    if (rc) return rc;
    if (c->n_pending == 0) return SPECTRE_OK;
    const int N = window_len(c), BH = c->B * c->H, F = N / 2 + 1;
    hipError_t e = launch_sweep_lazy(true, false, static_cast<float2 *>(c->prefix_fft), static_cast<const float *>(c->pending),
                                     static_cast<const float2 *>(c->twiddle), nullptr, nullptr, nullptr, BH, F, N, 0,
                                     c->n_pending, c->pending_slot, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail_hip(e, "sweep(flush)");
    c->n_pending = 0;
    return SPECTRE_OK;
}

static size_t scratch_bytes(int BH, int N, int d) {
    return align256((size_t)mix_chunk_heads(BH, N, d) * N * (d / 2) * sizeof(float2));
}

// prefix_fft = n-point half spectra of the rows now in v_buf ([B*H, n, d] fp32, read as B*H sequences of
// one head each); scr holds scratch_bytes(...).
static int transform_window(const spectre_prefix_cache *c, float2 *scr, hipStream_t st) {
    const int N = window_len(c), BH = c->B * c->H;
    Pow2Plan pl;
    int rc = get_pow2_plan(N, &pl);
    if (rc) return rc;
    const int chunk = mix_chunk_heads(BH, N, c->d);
    for (int bh0 = 0; bh0 < BH; bh0 += chunk) {
        const int nbh = (BH - bh0 < chunk) ? BH - bh0 : chunk;
        hipError_t e = launch_small_fwd(pl, SPECTRE_F32, c->v_buf, scr, N, 1, bh0, nbh, st);
        if (e != hipSuccess) return fail_hip(e, "small_fwd(window)");
        e = launch_big(pl, scr, nullptr, bh0, nbh, 1, st);
        if (e != hipSuccess) return fail_hip(e, "big(forward)");
        e = launch_untangle(scr, static_cast<float2 *>(c->prefix_fft), N, pl.N1, pl.N2, pl.P, bh0, nbh, st);
        if (e != hipSuccess) return fail_hip(e, "untangle");
    }
    return SPECTRE_OK;
}

size_t spectre_prefix_update_workspace_bytes(const spectre_prefix_cache *c, int T, spectre_dtype io) {
    (void)io;
    if (!c || T < 1 || c->B < 1 || c->H < 1 || c->d < 2 || c->N_max < 1 || c->N_mem < 0) return 0;
    const int BH = c->B * c->H;
    const int rows = T < kMaxPending ? T : kMaxPending;      // delta rows of one batch of appended tokens
    return align256((size_t)rows * BH * c->d * sizeof(float)) + align256(gate_partial_bytes(c->B, T, c->H, c->d)) +
           scratch_bytes(BH, window_len(c), c->d);
}

int spectre_prefix_update(spectre_prefix_cache *c, const void *v_new, const void *q_new, int T, spectre_dtype io,
                          void *ws, size_t ws_bytes, void *stream) {
    int rc = check_cache(c, "prefix_update");
    if (rc) return rc;
    if (!v_new || !q_new) return fail(SPECTRE_EINVAL, "prefix_update: null pointer");
    if (T < 1) return fail(SPECTRE_EINVAL, "prefix_update: T < 1");
    if (io != SPECTRE_F32 && io != SPECTRE_BF16) return fail(SPECTRE_EINVAL, "prefix_update: bad dtype");
    const size_t need = spectre_prefix_update_workspace_bytes(c, T, io);
    if (!ws || ws_bytes < need) return fail(SPECTRE_EWORKSPACE, "prefix_update: workspace %zu < %zu bytes", ws_bytes, need);
    if (reinterpret_cast<uintptr_t>(ws) & 255) return fail(SPECTRE_EINVAL, "prefix_update: ws not 256-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int B = c->B, H = c->H, d = c->d, N = window_len(c), W = c->N_max, M0 = c->N_mem, BH = B * H, F = N / 2 + 1;
    if (c->t == 0 && T > 1 && T > W) return fail(SPECTRE_EINVAL, "prefix_update: prompt of %d tokens exceeds N_max=%d", T, W);
    Pow2Plan pl;
    rc = get_pow2_plan(N, &pl);                      // every route below may transform the window
    if (rc) return rc;
    // every host-side check has passed: from here on work is enqueued
    rc = spectre_prefix_flush(c, stream);
    if (rc) return rc;
    char *w = static_cast<char *>(ws);
    float *delta = reinterpret_cast<float *>(w);
    w += align256((size_t)(T < kMaxPending ? T : kMaxPending) * BH * d * sizeof(float));
    double *partial = reinterpret_cast<double *>(w);
    w += align256(gate_partial_bytes(B, T, H, d));
    float2 *scr = reinterpret_cast<float2 *>(w);
    float2 *X = static_cast<float2 *>(c->prefix_fft);
    hipError_t e;
    if (c->t == 0 && T > 1) {
        // the ring buffers are all zero on an empty cache (spectre_prefix_init): only the prompt's rows are written,
        // and the same pass sums the queries.  Without memory rows the value rows are read once, by the row transform,
        // which also lays them into the ring buffer; with memory rows the window starts with them and is transformed
        // from the ring buffer as a whole.
        const bool fused_ring = (M0 == 0);
        e = launch_ring_append((int)io, fused_ring ? nullptr : v_new, q_new, static_cast<float *>(c->v_buf),
                               static_cast<float *>(c->q_buf), partial, B, T, H, N, M0, W, 0, 0, st);
        if (e != hipSuccess) return fail_hip(e, "ring_append(prompt)");
        e = launch_pool_final(partial, static_cast<double *>(c->sum_q), B, H * d, (T + 255) / 256, st, false);
        if (e != hipSuccess) return fail_hip(e, "pool_final(prompt)");
        if (!fused_ring) {
            rc = transform_window(c, scr, st);
            if (rc) return rc;
            c->t = T;
            return SPECTRE_OK;
        }
        const int chunk = mix_chunk_heads(BH, N, d);
        for (int bh0 = 0; bh0 < BH; bh0 += chunk) {
            const int nbh = (BH - bh0 < chunk) ? BH - bh0 : chunk;
            e = launch_small_fwd(pl, (int)io, v_new, scr, T, H, bh0, nbh, st, false, false,
                                 static_cast<float2 *>(c->v_buf));
            if (e != hipSuccess) return fail_hip(e, "small_fwd");
            e = launch_big(pl, scr, nullptr, bh0, nbh, 1, st);
            if (e != hipSuccess) return fail_hip(e, "big(forward)");
            e = launch_untangle(scr, X, N, pl.N1, pl.N2, pl.P, bh0, nbh, st);
            if (e != hipSuccess) return fail_hip(e, "untangle");
        }
        c->t = T;
        return SPECTRE_OK;
    }
    if (T == 1) {
        const int slot = M0 + (int)(c->t % W), evict = c->t >= W ? 1 : 0;
        e = launch_ring_update((int)io, v_new, q_new, T, 0, static_cast<float *>(c->v_buf), static_cast<float *>(c->q_buf),
                               static_cast<double *>(c->sum_q), delta, B, H, d, N, slot, evict, st);
        if (e != hipSuccess) return fail_hip(e, "ring_update");
        e = launch_sweep(true, false, X, delta, static_cast<const float2 *>(c->twiddle), nullptr, nullptr, BH, F, N, slot, st);
        if (e != hipSuccess) return fail_hip(e, "sweep(update)");
        c->t += 1;
        return SPECTRE_OK;
    }
    // many tokens (T up to the ring capacity): cheaper than T / 32 sweeps is to bring the ring buffers up to date in
    // one pass and transform the window afresh, as the pre-fill does (the cache IS the transform of the window)
    if (T >= kAppendRetransform && T <= W) {
        const int s0 = (int)(c->t % W);
        e = launch_ring_append((int)io, v_new, q_new, static_cast<float *>(c->v_buf), static_cast<float *>(c->q_buf), partial,
                               B, T, H, N, M0, W, s0, c->t, st);
        if (e != hipSuccess) return fail_hip(e, "ring_append");
        e = launch_pool_final(partial, static_cast<double *>(c->sum_q), B, H * d, (T + 255) / 256, st, true);
        if (e != hipSuccess) return fail_hip(e, "pool_final(append)");
        rc = transform_window(c, scr, st);
        if (rc) return rc;
        c->t += T;
        return SPECTRE_OK;
    }
    // several tokens: Eq. 5 is a sum of rank-one terms, so up to kMaxPending of them go into the cache in ONE sweep
    // (the ring buffers are still updated token by token, in order: a ring shorter than the batch reuses its slots)
    for (int t0 = 0; t0 < T; t0 += kMaxPending) {
        const int nb = (T - t0 < kMaxPending) ? T - t0 : kMaxPending;
        int slots[kMaxPending];
        for (int i = 0; i < nb; ++i) {
            const long long ti = c->t + i;
            const int slot = M0 + (int)(ti % W), evict = ti >= W ? 1 : 0;
            slots[i] = slot;
            e = launch_ring_update((int)io, v_new, q_new, T, t0 + i, static_cast<float *>(c->v_buf),
                                   static_cast<float *>(c->q_buf), static_cast<double *>(c->sum_q),
                                   delta + (size_t)i * BH * d, B, H, d, N, slot, evict, st);
            if (e != hipSuccess) return fail_hip(e, "ring_update");
        }
        e = launch_sweep_lazy(true, false, X, delta, static_cast<const float2 *>(c->twiddle), nullptr, nullptr, nullptr, BH,
                              F, N, 0, nb, slots, st);
        if (e != hipSuccess) return fail_hip(e, "sweep(batch update)");
        c->t += nb;                                    // the counter follows the spectrum, batch by batch
    }
    return SPECTRE_OK;
}

size_t spectre_prefix_set_memory_workspace_bytes(const spectre_prefix_cache *c) {
    if (!c || c->B < 1 || c->H < 1 || c->d < 2 || c->N_max < 1 || c->N_mem < 0) return 0;
    return scratch_bytes(c->B * c->H, window_len(c), c->d);
}

int spectre_prefix_set_memory(spectre_prefix_cache *c, const float *mem, int mem_batch, void *ws, size_t ws_bytes,
                              void *stream) {
    int rc = check_cache(c, "prefix_set_memory");
    if (rc) return rc;
    if (!mem) return fail(SPECTRE_EINVAL, "prefix_set_memory: null pointer");
    if (c->N_mem < 1) return fail(SPECTRE_EINVAL, "prefix_set_memory: the cache has no memory rows (N_mem = 0)");
    if (c->t != 0) return fail(SPECTRE_EINVAL, "prefix_set_memory: only on an empty cache (t = 0), right after init");
    if (mem_batch != 1 && mem_batch != c->B) return fail(SPECTRE_EINVAL, "prefix_set_memory: mem_batch must be 1 or B");
    const size_t need = spectre_prefix_set_memory_workspace_bytes(c);
    if (!ws || ws_bytes < need) return fail(SPECTRE_EWORKSPACE, "prefix_set_memory: workspace %zu < %zu bytes", ws_bytes, need);
    if (reinterpret_cast<uintptr_t>(ws) & 255) return fail(SPECTRE_EINVAL, "prefix_set_memory: ws not 256-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    Pow2Plan pl;
    rc = get_pow2_plan(window_len(c), &pl);            // the look-up transform_window repeats: fail before any launch
    if (rc) return rc;
    hipError_t e = launch_set_memory(mem, mem_batch, static_cast<float *>(c->v_buf), c->B, c->H, window_len(c), c->N_mem, st);
    if (e != hipSuccess) return fail_hip(e, "set_memory");
    return transform_window(c, static_cast<float2 *>(ws), st);
}

size_t spectre_prefix_readout_workspace_bytes(const spectre_prefix_cache *c, int mode, spectre_dtype io) {
    (void)io;
    if (!c || c->B < 1 || c->H < 1 || c->d < 2 || c->N_max < 1 || c->N_mem < 0) return 0;
    const int BH = c->B * c->H, F = window_len(c) / 2 + 1;
    if (mode == SPECTRE_READ_NEWEST) return align256((size_t)BH * sweep_chunks(F) * c->d * sizeof(float));
    if (mode == SPECTRE_READ_WINDOW) return scratch_bytes(BH, window_len(c), c->d);
    return 0;
}

int spectre_prefix_readout(const spectre_prefix_cache *c, const void *g, int mode, void *out, spectre_dtype io,
                           void *ws, size_t ws_bytes, void *stream) {
    int rc = check_cache(c, "prefix_readout");
    if (rc) return rc;
    if (!g || !out) return fail(SPECTRE_EINVAL, "prefix_readout: null pointer");
    if (mode != SPECTRE_READ_NEWEST && mode != SPECTRE_READ_WINDOW) return fail(SPECTRE_EINVAL, "prefix_readout: bad mode");
    if (io != SPECTRE_F32 && io != SPECTRE_BF16) return fail(SPECTRE_EINVAL, "prefix_readout: bad dtype");
    if (c->t < 1) return fail(SPECTRE_EINVAL, "prefix_readout: cache is empty");
    if (c->n_pending > 0)
        return fail(SPECTRE_EINVAL, "prefix_readout: %d deferred updates pending, call spectre_prefix_flush first", c->n_pending);
    const size_t need = spectre_prefix_readout_workspace_bytes(c, mode, io);
    if (!ws || ws_bytes < need) return fail(SPECTRE_EWORKSPACE, "prefix_readout: workspace %zu < %zu bytes", ws_bytes, need);
    if (reinterpret_cast<uintptr_t>(ws) & 255) return fail(SPECTRE_EINVAL, "prefix_readout: ws not 256-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int B = c->B, H = c->H, d = c->d, N = window_len(c), W = c->N_max, M0 = c->N_mem, BH = B * H, F = N / 2 + 1;
    float2 *X = static_cast<float2 *>(c->prefix_fft);
    const float2 *gg = static_cast<const float2 *>(g);
    hipError_t e;
    if (mode == SPECTRE_READ_NEWEST) {
        float *partial = static_cast<float *>(ws);
        const int slot = M0 + (int)((c->t - 1) % W);
        e = launch_sweep(false, true, X, nullptr, static_cast<const float2 *>(c->twiddle), gg, partial, BH, F, N, slot, st);
        if (e != hipSuccess) return fail_hip(e, "sweep(read)");
        e = launch_readout_final((int)io, partial, out, BH, F, st);
        if (e != hipSuccess) return fail_hip(e, "readout_final");
        return SPECTRE_OK;
    }
    Pow2Plan pl;
    rc = get_pow2_plan(N, &pl);
    if (rc) return rc;
    float2 *scr = static_cast<float2 *>(ws);
    const int Lw = (int)(c->t < W ? c->t : W);
    const int chunk = mix_chunk_heads(BH, N, d);
    for (int bh0 = 0; bh0 < BH; bh0 += chunk) {
        const int nbh = (BH - bh0 < chunk) ? BH - bh0 : chunk;
        e = launch_tangle(X, gg, scr, N, pl.N1, pl.N2, pl.P, bh0, nbh, st);
        if (e != hipSuccess) return fail_hip(e, "tangle");
        e = launch_big(pl, scr, nullptr, bh0, nbh, 2, st);
        if (e != hipSuccess) return fail_hip(e, "big(inverse)");
        // with memory rows the live tokens are gathered from their ring slots, oldest first
        if (M0 > 0) e = launch_small_inv(pl, (int)io, scr, out, 0, Lw, H, bh0, nbh, st, M0, W, (int)((c->t - 1) % W));
        else e = launch_small_inv(pl, (int)io, scr, out, N - Lw, Lw, H, bh0, nbh, st);
        if (e != hipSuccess) return fail_hip(e, "small_inv");
    }
    return SPECTRE_OK;
}

size_t spectre_prefix_step_workspace_bytes(const spectre_prefix_cache *c, const spectre_gate_params *P) {
    if (!c || !P || c->B < 1 || c->H < 1 || c->d < 2 || c->N_max < 1 || c->N_mem < 0 || P->d_g < 1) return 0;
    const int BH = c->B * c->H, F = window_len(c) / 2 + 1;
    return align256((size_t)BH * c->d * sizeof(float)) + align256((size_t)BH * P->d_g * sizeof(float)) +
           align256((size_t)BH * F * sizeof(float2)) + align256((size_t)BH * sweep_chunks(F) * c->d * sizeof(float)) +
           align256((size_t)BH * sweep_chunks(F) * 32 * sizeof(float)) + gate_raw_bytes(c->B, c->H, P);
}

int spectre_prefix_step(spectre_prefix_cache *c, const void *v_t, const void *q_t, const spectre_gate_params *P,
                        void *out, spectre_dtype io, void *ws, size_t ws_bytes, void *stream) {
    int rc = check_cache(c, "prefix_step");
    if (rc) return rc;
    if (!v_t || !q_t || !out) return fail(SPECTRE_EINVAL, "prefix_step: null pointer");
    if (io != SPECTRE_F32 && io != SPECTRE_BF16) return fail(SPECTRE_EINVAL, "prefix_step: bad dtype");
    rc = check_gate_params(P, c->H, "prefix_step");
    if (rc) return rc;
    if (P->n_fft != window_len(c) || P->d != c->d)
        return fail(SPECTRE_EINVAL, "prefix_step: gate is for n_fft=%d, d=%d", P->n_fft, P->d);
    const size_t need = spectre_prefix_step_workspace_bytes(c, P);
    if (!ws || ws_bytes < need) return fail(SPECTRE_EWORKSPACE, "prefix_step: workspace %zu < %zu bytes", ws_bytes, need);
    if (reinterpret_cast<uintptr_t>(ws) & 255) return fail(SPECTRE_EINVAL, "prefix_step: ws not 256-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int B = c->B, H = c->H, d = c->d, N = window_len(c), W = c->N_max, M0 = c->N_mem, BH = B * H, F = N / 2 + 1;
    char *w = static_cast<char *>(ws);
    float *delta = reinterpret_cast<float *>(w);
    w += align256((size_t)BH * d * sizeof(float));
    float *hid = reinterpret_cast<float *>(w);
    w += align256((size_t)BH * P->d_g * sizeof(float));
    float2 *g = reinterpret_cast<float2 *>(w);
    w += align256((size_t)BH * F * sizeof(float2));
    float *partial = reinterpret_cast<float *>(w);
    w += align256((size_t)BH * sweep_chunks(F) * d * sizeof(float));
    float *kpart = reinterpret_cast<float *>(w);
    w += align256((size_t)BH * sweep_chunks(F) * 32 * sizeof(float));
    float2 *raw = reinterpret_cast<float2 *>(w);
    const int slot = M0 + (int)(c->t % W), evict = c->t >= W ? 1 : 0;
    const bool lazy = c->pending_cap > 0;
    if (lazy) delta = static_cast<float *>(c->pending) + (size_t)c->n_pending * BH * d;   // this token's pending row
    hipError_t e = launch_ring_update((int)io, v_t, q_t, 1, 0, static_cast<float *>(c->v_buf), static_cast<float *>(c->q_buf),
                                      static_cast<double *>(c->sum_q), delta, B, H, d, N, slot, evict, st);
    if (e != hipSuccess) return fail_hip(e, "ring_update");
    e = launch_gate_mlp(static_cast<const double *>(c->sum_q), 1.0 / (double)W, gate_dev(P), hid, raw, B, H, 0, g, st);
    if (e != hipSuccess) return fail_hip(e, "gate_mlp");
    if (lazy) {
        // the ring buffers and sum_q are already updated; from here on the token counts as appended
        c->pending_slot[c->n_pending] = slot;
        c->n_pending += 1;
        c->t += 1;
        const float *pend = static_cast<const float *>(c->pending);
        const float2 *tw = static_cast<const float2 *>(c->twiddle);
        if (c->n_pending == c->pending_cap) {          // the list is full: apply everything, read the updated cache
            e = launch_sweep_lazy(true, true, static_cast<float2 *>(c->prefix_fft), pend, tw, g, partial, kpart, BH, F, N,
                                  slot, c->n_pending, c->pending_slot, st);
            if (e != hipSuccess) return fail_hip(e, "sweep(flush+read)");
            c->n_pending = 0;
            e = launch_readout_final((int)io, partial, out, BH, F, st);
        } else {                                       // read the stale cache, add the pending tokens' share
            e = launch_sweep_lazy(false, true, static_cast<float2 *>(c->prefix_fft), pend, tw, g, partial, kpart, BH, F, N,
                                  slot, c->n_pending, c->pending_slot, st);
            if (e != hipSuccess) return fail_hip(e, "sweep(read)");
            e = launch_readout_final_lazy((int)io, partial, kpart, pend, out, BH, F, c->n_pending, st);
        }
        if (e != hipSuccess) return fail_hip(e, "readout_final");
        return SPECTRE_OK;
    }
    e = launch_sweep(true, true, static_cast<float2 *>(c->prefix_fft), delta, static_cast<const float2 *>(c->twiddle), g,
                     partial, BH, F, N, slot, st);
    if (e != hipSuccess) return fail_hip(e, "sweep(update+read)");
    e = launch_readout_final((int)io, partial, out, BH, F, st);
    if (e != hipSuccess) return fail_hip(e, "readout_final");
    c->t += 1;
    return SPECTRE_OK;
}

}  // extern "C"
#pragma GCC visibility pop
