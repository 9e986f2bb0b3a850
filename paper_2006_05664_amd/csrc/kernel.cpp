// hipRTC instantiation, module loading, launch and timing: the evaluation f(x) of one trial
// (Sec. 1, Sec. 3: compile the device code under configuration x, run it, measure TFLOP/s).
#include "kernel.hpp"

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstring>
#include <new>
#include <sstream>

#include "code_cache.hpp"
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
    const std::string key = code_cache_key(d.tmpl, d.defines);
    CompileResult r;
    const bool cached = code_cache_get(key, r.code);
    if (!cached) r = pool_compile(d.tmpl, d.defines);
    if (r.status == OPEVO_E_INVALID)
        return fail(r.status, "invalid configuration: %s [%s]", r.log.c_str(), d.kernel_name.c_str());
    if (r.status != OPEVO_OK)
        return fail(r.status, "hipRTC failed for [%s]: %s", d.defines.c_str(), r.log.c_str());
    // A direct-to-LDS member whose K loop did not unroll compiles into a code object of hundreds of
    // KiB (register arrays indexed through select chains); fully unrolled ones take about 20 KiB.
    // The decoder's size rule should already have kept such members away from this template; one
    // that slips through is never launched.
    if (d.plan.path == 3 && r.code.size() > (128u << 10))
        return fail(OPEVO_E_INVALID, "direct-to-LDS template did not unroll (code object of %zu bytes) [%s]",
                    r.code.size(), d.defines.c_str());
    if (!cached) code_cache_put(key, r.code);
    opevo_kernel *k = new (std::nothrow) opevo_kernel;
    if (!k) return fail(OPEVO_E_ARG, "out of memory");
    k->code = std::move(r.code);
    k->plan = d.plan;
    k->flops = op.flops();
    k->tmpl = d.tmpl;
    k->defines = d.defines;
    k->name = d.kernel_name;
    k->zero_bytes = size_t(d.zero_bytes);
    k->prepass = d.prepass;
    if (d.prepass == 1) {          // image [B][Cin][H*W] -> [B][H*W][Cin]; kernel tensor [Cout][Cin][Hk*Wk] -> [Cout][Hk*Wk][Cin]
        k->pp_batches0 = op.nimg; k->pp_rows0 = op.cin; k->pp_cols0 = op.hin * op.win;
        k->pp_batches1 = op.M; k->pp_rows1 = op.cin; k->pp_cols1 = op.hk * op.wk;
    } else if (d.prepass == 2) {   // B [K][N] -> [N][K]
        k->pp_batches0 = op.batch; k->pp_rows0 = op.K; k->pp_cols0 = op.N;
    }
    if (compile_ms)
        *compile_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
    *out = k;
    return OPEVO_OK;
}

int load_kernel(opevo_kernel *k, bool refuse_spills)
{
    if (!k->fn) {
        HIP_TRY(hipModuleLoadData(&k->module, k->code.data()));
        hipError_t e = hipModuleGetFunction(&k->fn, k->module, k->name.c_str());
        if (e != hipSuccess) {
            (void)hipModuleUnload(k->module);
            k->module = nullptr; k->fn = nullptr;
            return hip_fail(e, "hipModuleGetFunction");
        }
        int scratch_bytes = 0;
        e = hipFuncGetAttribute(&scratch_bytes, HIP_FUNC_ATTRIBUTE_LOCAL_SIZE_BYTES, k->fn);
        k->scratch_bytes = e == hipSuccess ? scratch_bytes : 0;
        (void)hipGetLastError();
        if (k->plan.path != 3 && k->plan.lds_bytes > 32768) {
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(k->fn),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, k->plan.lds_bytes);
            if (e != hipSuccess && k->plan.lds_bytes > 65536) return hip_fail(e, "hipFuncSetAttribute(max dynamic LDS)");
            (void)hipGetLastError();
        }
    }
    if (k->prepass && !k->workspace) {
        const size_t bytes1 = (size_t(k->pp_batches1 * k->pp_rows1 * k->pp_cols1) * 2 + 255) / 256 * 256;
        const size_t bytes0 = size_t(k->pp_batches0 * k->pp_rows0 * k->pp_cols0) * 2;
        HIP_TRY(hipMalloc(&k->workspace, bytes1 + 256 + bytes0));
        hipError_t e = hipMemset(static_cast<char *>(k->workspace) + bytes1, 0, 256);   // the block of zeros padded taps are read from
        if (e != hipSuccess) return hip_fail(e, "hipMemset(workspace zeros)");
    }
    // A member whose kernel needs private scratch memory (register spills) is not run, on any
    // template.  The direct-to-LDS template counts its own outstanding loads (s_waitcnt vmcnt(n)):
    // spill stores would sit on the same counter and may complete out of order with loads, so a
    // count could be reached while a slab is still in flight.  On the register-staged template one
    // spilling member (all 512 registers in use, 20 bytes of scratch) once failed the parity gate
    // with 4 wrong rows in every 128 while its sibling with other spill choices was right; why is
    // not established (the template is not cleared by that, nor is the compiler blamed).  Spilling
    // members are slow in any case; they score as invalid (fitness 0) and stay a regression case
    // of the GPU tests (either refused or right).
    if (refuse_spills && k->scratch_bytes > 0)
        return fail(OPEVO_E_INVALID, "member spills %d bytes of registers per lane", k->scratch_bytes);
    return OPEVO_OK;
}

int launch_kernel(opevo_kernel *k, const void *a, const void *b, void *c, hipStream_t stream,
                  unsigned long long *ctl)
{
    if (int rc = load_kernel(k)) return rc;
    // members whose workgroups add partial sums into the output start from a cleared output
    if (k->zero_bytes)
        if (int rc = zero_f32(static_cast<float *>(c), int64_t(k->zero_bytes / 4), stream)) return rc;
    if (k->prepass) {
        const size_t bytes1 = (size_t(k->pp_batches1 * k->pp_rows1 * k->pp_cols1) * 2 + 255) / 256 * 256;
        char *ws = static_cast<char *>(k->workspace);
        void *first = ws, *zeros = ws + bytes1, *second = ws + bytes1 + 256;
        if (int rc = transpose_16(b, second, k->pp_batches0, k->pp_rows0, k->pp_cols0,
                                  k->prepass == 1 ? a : nullptr, first, k->pp_batches1, k->pp_rows1, k->pp_cols1, stream))
            return rc;
        if (k->prepass == 1) { a = first; b = zeros; }   // Conv2d: a = kernel tensor, b = zeros followed by the image
        else b = second;
    }
    void *args[] = {(void *)&a, (void *)&b, (void *)&c, (void *)&ctl};
    // the direct-to-LDS template declares its stages statically; the others take dynamic LDS
    const unsigned dyn_lds = k->plan.path == 3 ? 0u : unsigned(k->plan.lds_bytes);
    HIP_TRY(hipModuleLaunchKernel(k->fn, k->plan.grid[0], k->plan.grid[1], k->plan.grid[2],
                                  k->plan.block, 1, 1, dyn_lds, stream, args, nullptr));
    return OPEVO_OK;
}

int time_kernel(opevo_kernel *k, const void *a, const void *b, void *c, hipStream_t stream,
                int warmup, double warmup_ms, int launches_per_sample, int samples, double timeout_ms,
                double *median_ms, double *samples_ms)
{
    if (samples < 1) return fail(OPEVO_E_ARG, "kernel_time: samples must be >= 1");
    if (int rc = load_kernel(k)) return rc;
    unsigned long long *ctl = nullptr;
    // the scalar template and folded members of the register-staged templates honour a deadline (the direct-to-LDS
    // and LDS-resident-patch templates have no folded members)
    if (timeout_ms > 0.0 && k->plan.path != 3 && k->plan.path != 5)
        if (int rc = deadline_ctl(&ctl)) return rc;
    // samples + 1 events: the samples run back to back, without a host round trip (and an idle
    // GPU) between them; only the first, estimating launch is followed by a synchronisation
    std::vector<hipEvent_t> ev(size_t(samples) + 1, nullptr);
    int rc = OPEVO_OK;
    for (auto &e : ev) {
        hipError_t err = hipEventCreate(&e);
        if (err != hipSuccess) { rc = hip_fail(err, "hipEventCreate"); break; }
    }
    std::vector<double> ms(samples, 0.0);
    auto elapsed = [&](hipEvent_t a0, hipEvent_t a1, int n, double *out_ms) -> int {
        float t = 0.f;
        hipError_t err = hipEventElapsedTime(&t, a0, a1);
        if (err != hipSuccess) return hip_fail(err, "hipEventElapsedTime");
        *out_ms = double(t) / n;
        return OPEVO_OK;
    };
    auto check_deadline = [&]() -> int {
        if (!ctl) return OPEVO_OK;
        bool expired = false;
        if (int r2 = deadline_expired(ctl, stream, &expired)) return r2;
        if (expired) return fail(OPEVO_E_INVALID, "trial exceeded its %.0f ms deadline", timeout_ms);
        return OPEVO_OK;
    };
#define EV_TRY(call)                                                        \
    do {                                                                    \
        hipError_t err_ = (call);                                           \
        if (err_ != hipSuccess) { rc = hip_fail(err_, #call); break; }      \
    } while (0)
    do {
        if (rc) break;
        // the first launch doubles as warm-up and as the estimate that sizes a sample
        double first = 0.0;
        if (ctl && (rc = deadline_arm(ctl, timeout_ms, stream))) break;
        EV_TRY(hipEventRecord(ev[0], stream));
        if ((rc = launch_kernel(k, a, b, c, stream, ctl))) break;
        EV_TRY(hipEventRecord(ev[1], stream));
        EV_TRY(hipEventSynchronize(ev[1]));
        if ((rc = elapsed(ev[0], ev[1], 1, &first))) break;
        if ((rc = check_deadline())) break;
        if (first >= 20.0) {   // slow member (25 times the time of the fastest kernels of the largest workload): one launch is measurement enough
            for (int s = 0; s < samples; ++s) ms[s] = first;
            break;
        }
        int n = launches_per_sample;
        if (n <= 0) {   // long enough that event resolution and launch gaps do not dominate
            n = int(std::ceil(0.2 / std::max(first, 1e-4)));
            n = std::max(1, std::min(n, 2000));
        }
        // warm-up: at least `warmup` launches and at least warmup_ms of GPU time, so that the
        // clocks have ramped up before the first sample (they take tens of ms after idling)
        int n_warm = std::max(0, warmup - 1);
        if (warmup_ms > 0.0) n_warm = std::max(n_warm, std::min(4000, int(std::ceil(warmup_ms / std::max(first, 1e-4))) - 1));
        // deadline for everything that follows (warm-ups and all samples together)
        if (ctl && (rc = deadline_arm(ctl, timeout_ms * (double(samples) * n + n_warm + 1), stream))) break;
        for (int i = 0; i < n_warm && rc == OPEVO_OK; ++i) rc = launch_kernel(k, a, b, c, stream, ctl);
        if (rc) break;
        EV_TRY(hipEventRecord(ev[0], stream));
        for (int s = 0; s < samples && rc == OPEVO_OK; ++s) {
            for (int i = 0; i < n && rc == OPEVO_OK; ++i) rc = launch_kernel(k, a, b, c, stream, ctl);
            if (rc) break;
            hipError_t err = hipEventRecord(ev[s + 1], stream);
            if (err != hipSuccess) rc = hip_fail(err, "hipEventRecord");
        }
        if (rc) break;
        hipError_t err = hipEventSynchronize(ev[samples]);
        if (err != hipSuccess) { rc = hip_fail(err, "hipEventSynchronize (kernel fault?)"); break; }
        for (int s = 0; s < samples && rc == OPEVO_OK; ++s) rc = elapsed(ev[s], ev[s + 1], n, &ms[s]);
        if (rc) break;
        rc = check_deadline();
    } while (0);
#undef EV_TRY
    for (auto &e : ev)
        if (e) (void)hipEventDestroy(e);
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
    if (k->workspace) (void)hipFree(k->workspace);
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
    if (int rc = load_kernel(k, false)) return rc;   // figures of a spilling member can still be read
    int v = 0;
    if (vgprs) { HIP_TRY(hipFuncGetAttribute(&v, HIP_FUNC_ATTRIBUTE_NUM_REGS, k->fn)); *vgprs = v; }
    if (sgprs) *sgprs = -1;   // not reported by the runtime
    if (spill_bytes) { HIP_TRY(hipFuncGetAttribute(&v, HIP_FUNC_ATTRIBUTE_LOCAL_SIZE_BYTES, k->fn)); *spill_bytes = v; }
    if (static_lds) { HIP_TRY(hipFuncGetAttribute(&v, HIP_FUNC_ATTRIBUTE_SHARED_SIZE_BYTES, k->fn)); *static_lds = v; }
    return OPEVO_OK;
}

int opevo_mfma_ceiling(int in_dtype, int random_data, void *stream_, double *tflops)
{
    return opevo_mfma_ceiling_atom(in_dtype, random_data, 32, stream_, tflops);
}

int opevo_mfma_ceiling_atom(int in_dtype, int random_data, int atom, void *stream_, double *tflops)
{
    if (!tflops || (in_dtype != OPEVO_BF16 && in_dtype != OPEVO_F16))
        return fail(OPEVO_E_ARG, "mfma_ceiling: bf16 or fp16 only");
    if (atom != 16 && atom != 32) return fail(OPEVO_E_ARG, "mfma_ceiling: atom must be 16 (16x16x32) or 32 (32x32x16)");
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const int blocks = 2048, iters = 2048;
    std::ostringstream d;
    d << "-DKERNEL_NAME=opevo_mfma_peak -DIN_DTYPE=" << in_dtype << " -DITERS=" << iters
      << " -DOP=0 -DBATCH_INNER=1 -DPEAK_ATOM=" << atom;
    CompileResult r = pool_compile("mfma_peak", d.str());
    if (r.status != OPEVO_OK) return fail(r.status, "hipRTC failed for the MFMA ceiling kernel: %s", r.log.c_str());
    opevo_kernel k;
    k.code = std::move(r.code);
    k.name = "opevo_mfma_peak";
    std::memset(&k.plan, 0, sizeof k.plan);
    k.plan.path = 1;
    k.plan.grid[0] = blocks; k.plan.grid[1] = 1; k.plan.grid[2] = 1;
    k.plan.block = 256;
    void *buf = nullptr;
    const size_t in_elems = 6 * 256 * 8, in_bytes = in_elems * 2, out_bytes = size_t(blocks) * 256 * 4;
    HIP_TRY(hipMalloc(&buf, in_bytes + out_bytes));
    int rc = OPEVO_OK;
    double ms = 0.0;
    hipError_t e = hipMemsetAsync(buf, 0, in_bytes + out_bytes, stream);
    if (e != hipSuccess) rc = hip_fail(e, "hipMemsetAsync");
    if (!rc && random_data) {
        // uniform values in (-1, 1): random sign, exponent and mantissa bits, as a workload's operands have
        std::vector<uint16_t> host(in_elems);
        Rng rng(0x5eed);
        for (auto &h : host) {
            const float v = float(rng.next_double() * 2.0 - 1.0);
            if (in_dtype == OPEVO_BF16) {
                uint32_t u;
                std::memcpy(&u, &v, 4);
                h = uint16_t((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
            } else {
                const _Float16 f = _Float16(v);
                std::memcpy(&h, &f, 2);
            }
        }
        e = hipMemcpyAsync(buf, host.data(), in_bytes, hipMemcpyHostToDevice, stream);
        if (e == hipSuccess) e = hipStreamSynchronize(stream);
        if (e != hipSuccess) rc = hip_fail(e, "hipMemcpyAsync");
    }
    if (!rc)
        rc = time_kernel(&k, buf, buf, static_cast<char *>(buf) + in_bytes, stream, 3, 40.0, 4, 5, 0.0, &ms, nullptr);
    if (k.module) (void)hipModuleUnload(k.module);
    (void)hipFree(buf);
    if (rc) return rc;
    *tflops = double(blocks) * 4.0 * 8.0 * iters * 32768.0 / (ms * 1e-3) * 1e-12;
    return OPEVO_OK;
}

int opevo_kernel_launch(opevo_kernel *k, const void *a, const void *b, void *c, void *stream)
{
    if (!k || !a || !b || !c) return fail(OPEVO_E_ARG, "kernel_launch: NULL argument");
    return launch_kernel(k, a, b, c, static_cast<hipStream_t>(stream));
}

int opevo_kernel_time(opevo_kernel *k, const void *a, const void *b, void *c, void *stream,
                      int warmup, double warmup_ms, int launches_per_sample, int samples, double timeout_ms,
                      double *median_ms, double *samples_ms)
{
    if (!k || !a || !b || !c) return fail(OPEVO_E_ARG, "kernel_time: NULL argument");
    return time_kernel(k, a, b, c, static_cast<hipStream_t>(stream), warmup, warmup_ms, launches_per_sample, samples,
                       timeout_ms, median_ms, samples_ms);
}

}  // extern "C"
