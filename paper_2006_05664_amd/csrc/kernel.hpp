// hipRTC instantiation of a kernel template under one configuration, module loading,
// launch and hipEvent timing.
#pragma once

#include <string>
#include <vector>

#include <hip/hip_runtime.h>

#include "op.hpp"

struct opevo_kernel {
    opevo_plan plan;
    double flops = 0.0;
    std::string tmpl, defines, name;
    std::vector<char> code;        // gfx950 code object from hipRTC
    size_t zero_bytes = 0;         // > 0: the output is cleared before every launch (split reduction)
    hipModule_t module = nullptr;  // loaded on first launch
    hipFunction_t fn = nullptr;
    int scratch_bytes = 0;         // private scratch per lane the compiler used (known once loaded)
};

namespace opevo {

// Source text of a template by name (generated at build time from csrc/templates/*.hip).
const char *template_source(const char *name);

int build_kernel(const opevo_op &op, int variant, const int32_t *cfg, opevo_kernel **out, double *compile_ms);
// Loads the module on first use; with refuse_spills a kernel that uses private scratch memory is
// answered with OPEVO_E_INVALID (it is never launched).
int load_kernel(opevo_kernel *k, bool refuse_spills = true);
int launch_kernel(opevo_kernel *k, const void *a, const void *b, void *c, hipStream_t stream,
                  unsigned long long *ctl = nullptr);
// timeout_ms > 0 arms the deadline of the scalar template: a launch still running after that
// long winds down and the call returns OPEVO_E_INVALID.
int time_kernel(opevo_kernel *k, const void *a, const void *b, void *c, hipStream_t stream,
                int warmup, double warmup_ms, int launches_per_sample, int samples, double timeout_ms,
                double *median_ms, double *samples_ms);
// Deadline control block (device memory, one per device, library-owned).
int deadline_ctl(unsigned long long **ctl);
int deadline_arm(unsigned long long *ctl, double timeout_ms, hipStream_t stream);
int deadline_expired(unsigned long long *ctl, hipStream_t stream, bool *expired);
// Clears n floats at p (16-byte aligned) with a small kernel on `stream`.
int zero_f32(float *p, int64_t n, hipStream_t stream);
int hip_fail(hipError_t e, const char *what);

}  // namespace opevo

namespace opevo {
int compare_f32(const float *c, const float *ref, int64_t n, const int *rows, int64_t row_len,
                hipStream_t stream, double *max_scaled, double *rel_fro);
}
