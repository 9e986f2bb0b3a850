// hipRTC instantiation, module loading, launch and timing: the evaluation f(x) of one trial
// (Sec. 1, Sec. 3: compile the device code under configuration x, run it, measure TFLOP/s).
#include "kernel.hpp"

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstring>
#include <new>
#include <sstream>

#include "pool.hpp"

namespace opevo {

int hip_fail(hipError_t e, const char *what)
{
    return fail(OPEVO_E_HIP, "%s: %s", what, hipGetErrorString(e));
}

#define HIP_TRY(call)                                             \
    do {                                                          \
        hipError_t e_ = (call);                                   \
        if (e_ != hipSuccess) return hip_fail(e_, #call);         \
    } while (0)

int build_kernel(const opevo_op &op, int variant, const int32_t *cfg, opevo_kernel **out, double *compile_ms)
{
    Decoded d;
    if (int rc = decode(op, variant, cfg, d)) return rc;
    if (d.plan.status != OPEVO_OK) return fail(OPEVO_E_INVALID, "invalid configuration: %s", d.plan.reason);
    const auto t0 = std::chrono::steady_clock::now();
    CompileResult r = pool_compile(d.tmpl, d.defines);
    if (r.status != OPEVO_OK)
        return fail(r.status, "hipRTC failed for [%s]: %s", d.defines.c_str(), r.log.c_str());
    opevo_kernel *k = new (std::nothrow) opevo_kernel;
    if (!k) return fail(OPEVO_E_ARG, "out of memory");
    k->code = std::move(r.code);
    k->plan = d.plan;
    k->flops = op.flops();
    k->tmpl = d.tmpl;
    k->defines = d.defines;
    k->name = d.kernel_name;
    if (compile_ms)
        *compile_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
    *out = k;
    return OPEVO_OK;
}

int load_kernel(opevo_kernel *k)
{
    if (k->fn) return OPEVO_OK;
    HIP_TRY(hipModuleLoadData(&k->module, k->code.data()));
    hipError_t e = hipModuleGetFunction(&k->fn, k->module, k->name.c_str());
    if (e != hipSuccess) {
        (void)hipModuleUnload(k->module);
        k->module = nullptr; k->fn = nullptr;
        return hip_fail(e, "hipModuleGetFunction");
    }
    if (k->plan.lds_bytes > 32768) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(k->fn),
                                hipFuncAttributeMaxDynamicSharedMemorySize, k->plan.lds_bytes);
        if (e != hipSuccess && k->plan.lds_bytes > 65536) return hip_fail(e, "hipFuncSetAttribute(max dynamic LDS)");
        (void)hipGetLastError();
    }
    return OPEVO_OK;
}

int launch_kernel(opevo_kernel *k, const void *a, const void *b, void *c, hipStream_t stream,
                  unsigned long long *ctl)
{
    if (int rc = load_kernel(k)) return rc;
    void *args[] = {(void *)&a, (void *)&b, (void *)&c, (void *)&ctl};
    HIP_TRY(hipModuleLaunchKernel(k->fn, k->plan.grid[0], k->plan.grid[1], k->plan.grid[2],
                                  k->plan.block, 1, 1, k->plan.lds_bytes, stream, args, nullptr));
    return OPEVO_OK;
}

int time_kernel(opevo_kernel *k, const void *a, const void *b, void *c, hipStream_t stream,
                int warmup, int launches_per_sample, int samples, double timeout_ms,
                double *median_ms, double *samples_ms)
{
    if (samples < 1) return fail(OPEVO_E_ARG, "kernel_time: samples must be >= 1");
    if (int rc = load_kernel(k)) return rc;
    unsigned long long *ctl = nullptr;
    if (timeout_ms > 0.0 && k->plan.path == 0)
        if (int rc = deadline_ctl(&ctl)) return rc;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    HIP_TRY(hipEventCreate(&e0));
    hipError_t e = hipEventCreate(&e1);
    if (e != hipSuccess) { (void)hipEventDestroy(e0); return hip_fail(e, "hipEventCreate"); }
    int rc = OPEVO_OK;
    std::vector<double> ms(samples, 0.0);
    // n back-to-back launches between two events on the caller's stream -> ms per launch
    auto timed = [&](int n, double *out_ms) -> int {
        if (ctl)
            if (int r2 = deadline_arm(ctl, timeout_ms, stream)) return r2;
        hipError_t err = hipEventRecord(e0, stream);
        if (err != hipSuccess) return hip_fail(err, "hipEventRecord");
        for (int i = 0; i < n; ++i)
            if (int r2 = launch_kernel(k, a, b, c, stream, ctl)) return r2;
        err = hipEventRecord(e1, stream);
        if (err != hipSuccess) return hip_fail(err, "hipEventRecord");
        err = hipEventSynchronize(e1);
        if (err != hipSuccess) return hip_fail(err, "hipEventSynchronize (kernel fault?)");
        float t = 0.f;
        err = hipEventElapsedTime(&t, e0, e1);
        if (err != hipSuccess) return hip_fail(err, "hipEventElapsedTime");
        *out_ms = double(t) / n;
        if (ctl) {
            bool expired = false;
            if (int r2 = deadline_expired(ctl, stream, &expired)) return r2;
            if (expired) return fail(OPEVO_E_INVALID, "trial exceeded its %.0f ms deadline", timeout_ms);
        }
        return OPEVO_OK;
    };
    do {
        // the first launch doubles as warm-up and as the estimate that sizes a sample
        double first = 0.0;
        if ((rc = timed(1, &first))) break;
        if (first >= 50.0) {   // slow member: one launch is measurement enough
            for (int s = 0; s < samples; ++s) ms[s] = first;
            break;
        }
        for (int i = 1; i < warmup && rc == OPEVO_OK; ++i) rc = launch_kernel(k, a, b, c, stream, ctl);
        if (rc) break;
        int n = launches_per_sample;
        if (n <= 0) {   // long enough that event resolution and launch gaps do not dominate
            n = int(std::ceil(0.2 / std::max(first, 1e-4)));
            n = std::max(1, std::min(n, 2000));
        }
        for (int s = 0; s < samples && rc == OPEVO_OK; ++s) rc = timed(n, &ms[s]);
    } while (0);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc) return rc;
    if (samples_ms) std::memcpy(samples_ms, ms.data(), sizeof(double) * samples);
    std::sort(ms.begin(), ms.end());
    if (median_ms) *median_ms = (samples % 2) ? ms[samples / 2] : 0.5 * (ms[samples / 2 - 1] + ms[samples / 2]);
    return OPEVO_OK;
}

}  // namespace opevo

using namespace opevo;

extern "C" {

int opevo_kernel_build(const opevo_op *op, int variant, const int32_t *cfg, opevo_kernel **out, double *compile_ms)
{
    if (!op || !cfg || !out) return fail(OPEVO_E_ARG, "kernel_build: NULL argument");
    *out = nullptr;
    return build_kernel(*op, variant, cfg, out, compile_ms);
}

int opevo_kernel_destroy(opevo_kernel *k)
{
    if (!k) return OPEVO_OK;
    if (k->module) (void)hipModuleUnload(k->module);
    delete k;
    return OPEVO_OK;
}

int opevo_kernel_code_size(const opevo_kernel *k, size_t *bytes)
{
    if (!k || !bytes) return fail(OPEVO_E_ARG, "kernel_code_size: NULL argument");
    *bytes = k->code.size();
    return OPEVO_OK;
}

int opevo_kernel_resources(opevo_kernel *k, int *vgprs, int *sgprs, int *spill_bytes, int *static_lds)
{
    if (!k) return fail(OPEVO_E_ARG, "kernel_resources: NULL argument");
    if (int rc = load_kernel(k)) return rc;
    int v = 0;
    if (vgprs) { HIP_TRY(hipFuncGetAttribute(&v, HIP_FUNC_ATTRIBUTE_NUM_REGS, k->fn)); *vgprs = v; }
    if (sgprs) *sgprs = -1;   // not reported by the runtime
    if (spill_bytes) { HIP_TRY(hipFuncGetAttribute(&v, HIP_FUNC_ATTRIBUTE_LOCAL_SIZE_BYTES, k->fn)); *spill_bytes = v; }
    if (static_lds) { HIP_TRY(hipFuncGetAttribute(&v, HIP_FUNC_ATTRIBUTE_SHARED_SIZE_BYTES, k->fn)); *static_lds = v; }
    return OPEVO_OK;
}

int opevo_kernel_launch(opevo_kernel *k, const void *a, const void *b, void *c, void *stream)
{
    if (!k || !a || !b || !c) return fail(OPEVO_E_ARG, "kernel_launch: NULL argument");
    return launch_kernel(k, a, b, c, static_cast<hipStream_t>(stream));
}

int opevo_kernel_time(opevo_kernel *k, const void *a, const void *b, void *c, void *stream,
                      int warmup, int launches_per_sample, int samples, double timeout_ms,
                      double *median_ms, double *samples_ms)
{
    if (!k || !a || !b || !c) return fail(OPEVO_E_ARG, "kernel_time: NULL argument");
    return time_kernel(k, a, b, c, static_cast<hipStream_t>(stream), warmup, launches_per_sample, samples,
                       timeout_ms, median_ms, samples_ms);
}

}  // extern "C"
