// Host-side declarations shared by the translation units of the library.
#pragma once
#include <hip/hip_runtime.h>

#include "../../include/spectre.h"
#include "mix_pow2.h"

namespace spectre {

// Record a message for spectre_last_error() and return `code`.
int fail(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
int fail_hip(hipError_t e, const char *what);

// Current value of a tuning switch (spectre_set_option), `which` one of the SPECTRE_OPT_* enumerators.
long option(int which);

// Device table [n] of exp(-j 2 pi m / n), values computed in fp64.  make = false (every compute call): look the
// table up, SPECTRE_ENOTREADY if spectre_prepare has not built it on this device; make = true: build it if missing.
int get_roots(int n, const float2 **out, bool make = false);
int get_pow2_plan(int L, Pow2Plan *pl, bool make = false);

// One per translation unit with kernels: make the runtime load its code object now (spectre_prepare).
hipError_t load_kernels_mix_pow2();
hipError_t load_kernels_mix_slab();
hipError_t load_kernels_mix_chirp();
hipError_t load_kernels_gate();
hipError_t load_kernels_prefix();
hipError_t load_kernels_project();
hipError_t load_kernels_wrm();

}  // namespace spectre
