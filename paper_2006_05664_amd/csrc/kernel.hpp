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
    // Members whose kernel reads re-laid-out operands.  Every launch first runs one pre-pass kernel on
    // the same stream that writes them into `workspace` (allocated when the module is loaded).
    //   prepass 1 (Conv2d, channels last): [kernel tensor as [Cout][Hk*Wk][Cin]] [256 bytes of zeros]
    //             [image as [B][H*W][Cin]]; the kernel's second pointer is the block of zeros.
    //   prepass 2 (MatMul): the second operand transposed to [N][K].
    int prepass = 0;
    int64_t pp_batches0 = 0, pp_rows0 = 0, pp_cols0 = 0;   // second operand: out[b][c][r] = in[b][r][c]
    int64_t pp_batches1 = 0, pp_rows1 = 0, pp_cols1 = 0;   // first operand (Conv2d only)
    void *workspace = nullptr;
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
// out[b][c][r] = in[b][r][c] for up to two batched matrices of 16-bit elements in one launch on
// `stream` (the second is skipped if in1 is NULL).
int transpose_16(const void *in0, void *out0, int64_t batches0, int64_t rows0, int64_t cols0,
                 const void *in1, void *out1, int64_t batches1, int64_t rows1, int64_t cols1, hipStream_t stream);
int hip_fail(hipError_t e, const char *what);

}  // namespace opevo

namespace opevo {
int compare_f32(const float *c, const float *ref, int64_t n, const int *rows, int64_t row_len,
                hipStream_t stream, double *max_scaled, double *rel_fro);
}
