// Host-side declarations shared by the translation units of the library.
#pragma once
#include <hip/hip_runtime.h>

#include "mix_pow2.h"

namespace spectre {

// Record a message for spectre_last_error() and return `code`.
int fail(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
int fail_hip(hipError_t e, const char *what);

// Device table [n] of exp(-j 2 pi m / n), built in fp64 on first use per device.
int get_roots(int n, const float2 **out);
int get_pow2_plan(int L, Pow2Plan *pl);

}  // namespace spectre
