// C ABI of the SPECTRE library: argument checks, per-device table cache, launch sequencing.
// Every entry point validates on the host, enqueues on the caller's stream and returns.
#include "../../include/spectre.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <mutex>
#include <string>
#include <utility>
#include <vector>

#include "internal.h"

namespace spectre {

static thread_local std::string g_err;

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
struct DeviceTables {
    std::map<int, float2 *> roots;   // n -> device array [n] of exp(-j 2 pi m / n)
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

int get_roots(int n, const float2 **out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    std::lock_guard<std::mutex> lk(g_mu);
    DeviceTables &t = g_tables[dev];
    auto it = t.roots.find(n);
    if (it == t.roots.end()) {
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

int get_pow2_plan(int L, Pow2Plan *pl) {
    int N1, N2, P;
    if (!pow2_split(L, &N1, &N2, &P)) return fail(SPECTRE_EUNSUPPORTED, "no power-of-two plan for length %d", L);
    pl->L = L; pl->N1 = N1; pl->N2 = N2; pl->P = P;
    int rc = get_roots(L, &pl->twL);
    if (rc) return rc;
    return get_roots(N1, &pl->twN1);
}

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Scratch columns are processed in groups of heads small enough to stay in the memory-side
// cache between the three kernels of a group.
int mix_chunk_heads(int BH, int L, int d) {
    size_t per_head = (size_t)L * (size_t)(d / 2) * sizeof(float2);
    size_t budget = (size_t)64 << 20;
    if (const char *e = getenv("SPECTRE_CHUNK_MB")) {
        long mb = atol(e);
        if (mb > 0) budget = (size_t)mb << 20;
    }
    size_t n = budget / per_head;
    if (n < 1) n = 1;
    if (n > (size_t)BH) n = (size_t)BH;
    return (int)n;
}

}  // namespace spectre

using namespace spectre;

#pragma GCC visibility push(default)
extern "C" {

const char *spectre_last_error(void) { return g_err.c_str(); }

int spectre_version(void) { return 100; }

int spectre_length_supported(int n, int d) {
    if (d != 64) return 0;
    int N1, N2, P;
    return pow2_split(n, &N1, &N2, &P) ? 1 : 0;
}

void spectre_shutdown(void) {
    std::lock_guard<std::mutex> lk(g_mu);
    int cur = 0;
    (void)hipGetDevice(&cur);
    for (auto &kv : g_tables) {
        (void)hipSetDevice(kv.first);
        for (auto &r : kv.second.roots) (void)hipFree(r.second);
    }
    g_tables.clear();
    (void)hipSetDevice(cur);
}

size_t spectre_mix_workspace_bytes(int B, int L, int H, int d, spectre_dtype io) {
    (void)io;
    if (B < 1 || L < 2 || H < 1 || d < 2) return 0;
    if (!spectre_length_supported(L, d)) return 0;
    const int BH = B * H;
    const int chunk = mix_chunk_heads(BH, L, d);
    return align256((size_t)BH * L * sizeof(float2)) + align256((size_t)chunk * L * (d / 2) * sizeof(float2));
}

int spectre_mix_forward(const void *v, const void *g, void *out, int B, int L, int H, int d,
                        spectre_dtype io, void *ws, size_t ws_bytes, void *stream) {
    if (!v || !g || !out) return fail(SPECTRE_EINVAL, "mix_forward: null pointer");
    if (B < 1 || L < 1 || H < 1 || d < 1) return fail(SPECTRE_EINVAL, "mix_forward: non-positive size");
    if (io != SPECTRE_F32 && io != SPECTRE_BF16) return fail(SPECTRE_EINVAL, "mix_forward: bad dtype");
    if ((long long)B * H > 0x7fffffffLL / 64) return fail(SPECTRE_EUNSUPPORTED, "mix_forward: B*H too large");
    const size_t bytes = (size_t)B * L * H * d * (io == SPECTRE_BF16 ? 2 : 4);
    const char *vb = static_cast<const char *>(v), *ob = static_cast<const char *>(out);
    if (vb < ob + bytes && ob < vb + bytes) return fail(SPECTRE_EINVAL, "mix_forward: out overlaps v");
    if (!spectre_length_supported(L, d))
        return fail(SPECTRE_EUNSUPPORTED, "mix_forward: no kernel for L=%d, d=%d", L, d);
    const size_t need = spectre_mix_workspace_bytes(B, L, H, d, io);
    if (!ws || ws_bytes < need)
        return fail(SPECTRE_EWORKSPACE, "mix_forward: workspace %zu < %zu bytes", ws_bytes, need);
    if (reinterpret_cast<uintptr_t>(ws) & 255) return fail(SPECTRE_EINVAL, "mix_forward: ws not 256-byte aligned");

    Pow2Plan pl;
    int rc = get_pow2_plan(L, &pl);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int BH = B * H;
    float2 *gp = static_cast<float2 *>(ws);
    float2 *scr = reinterpret_cast<float2 *>(static_cast<char *>(ws) + align256((size_t)BH * L * sizeof(float2)));
    hipError_t e = launch_gate_expand(pl, static_cast<const float2 *>(g), gp, BH, st);
    if (e != hipSuccess) return fail_hip(e, "gate_expand");
    const int chunk = mix_chunk_heads(BH, L, d);
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

}  // extern "C"
#pragma GCC visibility pop
