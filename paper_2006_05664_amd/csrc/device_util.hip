// Precompiled device helpers of the harness.
//
// Parity gate: compares a trial's fp32 output with a reference tensor on the device.
//   max_scaled = max_i |c_i - ref_i| / (|ref_i| + 1),   rel_fro = ||c - ref||_F / ||ref||_F.
// Any NaN in c makes max_scaled infinite, so a broken kernel can never pass.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <mutex>
#include <vector>

#include "kernel.hpp"

// Partials of opevo_compare_f32_static: device memory that exists from the moment the code object
// is loaded, one copy per GPU, so that entry point never allocates.  In host code this name is
// only a handle for hipGetSymbolAddress; the address it yields (static_scratch() below) is what
// kernels and copies are given.
static __device__ __align__(256) double scratch[3 * 1024];   // 3 doubles per workgroup of compare_partial (kBlocks)

namespace {

typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kBlocks = 1024;
static_assert(sizeof(scratch) == sizeof(double) * 3 * kBlocks, "scratch holds one triple per workgroup");
constexpr int kThreads = 256;

// rows == NULL: c and ref are both n elements.  rows != NULL: ref holds n = n_rows * row_len
// elements, the rows rows[0..n_rows) of c viewed as a matrix with row_len columns.
__global__ __launch_bounds__(kThreads)
void compare_partial(const float *__restrict__ c, const float *__restrict__ ref, long n,
                     const int *__restrict__ rows, long row_len, double *__restrict__ part)
{
    double mx = 0.0, se = 0.0, sr = 0.0;
    for (long i = (long)blockIdx.x * kThreads + threadIdx.x; i < n; i += (long)gridDim.x * kThreads) {
        const long ci = rows ? (long)rows[i / row_len] * row_len + i % row_len : i;
        const double r = ref[i], d = (double)c[ci] - r;
        const double s = fabs(d) / (fabs(r) + 1.0);
        mx = (s <= mx) ? mx : (s == s ? s : INFINITY);   // NaN -> inf
        se += d * d;
        sr += r * r;
    }
    __shared__ double smx[kThreads], sse[kThreads], ssr[kThreads];
    smx[threadIdx.x] = mx; sse[threadIdx.x] = se; ssr[threadIdx.x] = sr;
    __syncthreads();
    for (int s = kThreads / 2; s > 0; s >>= 1) {
        if (threadIdx.x < s) {
            smx[threadIdx.x] = fmax(smx[threadIdx.x], smx[threadIdx.x + s]);
            sse[threadIdx.x] += sse[threadIdx.x + s];
            ssr[threadIdx.x] += ssr[threadIdx.x + s];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        part[blockIdx.x * 3 + 0] = smx[0];
        part[blockIdx.x * 3 + 1] = sse[0];
        part[blockIdx.x * 3 + 2] = ssr[0];
    }
}

// Finishes a comparison on the device: folds the per-workgroup partials in workgroup order (the
// order the host-side fold of compare_f32 uses, so both give the same bits) and writes
// result[0] = max_scaled, result[1] = rel_fro.
__global__ void compare_finish(const double *__restrict__ part, int blocks, double *__restrict__ result)
{
    double mx = 0.0, se = 0.0, sr = 0.0;
    for (int b = 0; b < blocks; ++b) {
        mx = fmax(mx, part[b * 3 + 0]);
        se += part[b * 3 + 1];
        sr += part[b * 3 + 2];
    }
    result[0] = mx;
    result[1] = sr > 0.0 ? sqrt(se / sr) : (se > 0.0 ? INFINITY : 0.0);
}

// Deadline control block of the scalar template: {start tick, allowed ticks, expired flag}.
__global__ void stamp_deadline(unsigned long long *ctl, unsigned long long ticks)
{
    ctl[0] = wall_clock64();
    ctl[1] = ticks;
    ctl[2] = 0;
}

// Clears n_vec4 16-byte words: the output of a member whose workgroups add partial sums into it.
// A kernel rather than hipMemsetAsync, so that a caller may record launches into a HIP graph.
__global__ __launch_bounds__(256) void zero_words(f32x4_t *p, long n_vec4)
{
    const f32x4_t z = {0.f, 0.f, 0.f, 0.f};
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n_vec4; i += (long)gridDim.x * 256) p[i] = z;
}
__global__ void zero_tail(float *p, int n)
{
    if ((int)threadIdx.x < n) p[threadIdx.x] = 0.f;
}

std::mutex g_ws_mutex;
double *g_ws[64] = {nullptr};   // one workspace per device, kept until the process ends
double *g_static_ws[64] = {nullptr};   // device address of `scratch` on each device
unsigned long long *g_ctl[64] = {nullptr};
double g_ticks_per_ms[64] = {0.0};

}  // namespace

namespace opevo {

int compare_f32(const float *c, const float *ref, int64_t n, const int *rows, int64_t row_len,
                hipStream_t stream, double *max_scaled, double *rel_fro)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= 64) return fail(OPEVO_E_HIP, "device index %d out of range", dev);
    double *ws;
    {
        std::lock_guard<std::mutex> lock(g_ws_mutex);
        if (!g_ws[dev]) {
            e = hipMalloc(&g_ws[dev], sizeof(double) * 3 * kBlocks);
            if (e != hipSuccess) return hip_fail(e, "hipMalloc(compare workspace)");
        }
        ws = g_ws[dev];
    }
    int blocks = int(std::min<int64_t>(kBlocks, (n + kThreads - 1) / kThreads));
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(compare_partial, dim3(blocks), dim3(kThreads), 0, stream, c, ref, (long)n, rows,
                       (long)row_len, ws);
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "compare_partial launch");
    std::vector<double> host(size_t(3) * blocks);
    e = hipMemcpyAsync(host.data(), ws, sizeof(double) * 3 * blocks, hipMemcpyDeviceToHost, stream);
    if (e != hipSuccess) return hip_fail(e, "hipMemcpyAsync");
    e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return hip_fail(e, "hipStreamSynchronize");
    double mx = 0.0, se = 0.0, sr = 0.0;
    for (int b = 0; b < blocks; ++b) {
        mx = std::fmax(mx, host[b * 3 + 0]);
        se += host[b * 3 + 1];
        sr += host[b * 3 + 2];
    }
    if (max_scaled) *max_scaled = mx;
    if (rel_fro) *rel_fro = sr > 0.0 ? std::sqrt(se / sr) : (se > 0.0 ? INFINITY : 0.0);
    return OPEVO_OK;
}

// Device address of this device's copy of `scratch` (looked up once per device, with that device current).
static int static_scratch(double **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= 64) return fail(OPEVO_E_HIP, "device index %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    if (!g_static_ws[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return hip_fail(e, "hipGetSymbolAddress(compare scratch)");
        g_static_ws[dev] = static_cast<double *>(p);
    }
    *out = g_static_ws[dev];
    return OPEVO_OK;
}

int compare_f32_static(const float *c, const float *ref, int64_t n, hipStream_t stream, double *result_dev)
{
    double *ws = nullptr;
    if (int rc = static_scratch(&ws)) return rc;
    int blocks = int(std::min<int64_t>(kBlocks, (n + kThreads - 1) / kThreads));
    if (blocks < 1) blocks = 1;
    // every workgroup overwrites its own three partials and the fold reads only those `blocks`
    // triples, so nothing left in the array by an earlier call is ever read: no clearing needed
    hipLaunchKernelGGL(compare_partial, dim3(blocks), dim3(kThreads), 0, stream, c, ref, (long)n,
                       (const int *)nullptr, 1L, ws);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "compare_partial launch");
    hipLaunchKernelGGL(compare_finish, dim3(1), dim3(1), 0, stream, (const double *)ws, blocks, result_dev);
    e = hipGetLastError();
    return e == hipSuccess ? OPEVO_OK : hip_fail(e, "compare_finish launch");
}

int deadline_ctl(unsigned long long **ctl)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= 64) return fail(OPEVO_E_HIP, "device index %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    if (!g_ctl[dev]) {
        int khz = 0;
        e = hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev);
        if (e != hipSuccess || khz <= 0) khz = 100000;   // 100 MHz constant clock
        g_ticks_per_ms[dev] = double(khz);
        e = hipMalloc(&g_ctl[dev], 4 * sizeof(unsigned long long));
        if (e != hipSuccess) return hip_fail(e, "hipMalloc(deadline control)");
    }
    *ctl = g_ctl[dev];
    return OPEVO_OK;
}

int zero_f32(float *p, int64_t n, hipStream_t stream)
{
    if (n <= 0) return OPEVO_OK;
    if (reinterpret_cast<uintptr_t>(p) % 16 != 0) return fail(OPEVO_E_ARG, "output pointer is not 16-byte aligned");
    const long n4 = long(n / 4);
    if (n4 > 0) {
        const long want = (n4 + 255) / 256;
        const unsigned blocks = unsigned(want < 2048 ? want : 2048);
        hipLaunchKernelGGL(zero_words, dim3(blocks), dim3(256), 0, stream, reinterpret_cast<f32x4_t *>(p), n4);
    }
    if (n % 4) hipLaunchKernelGGL(zero_tail, dim3(1), dim3(64), 0, stream, p + n4 * 4, int(n % 4));
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? OPEVO_OK : hip_fail(e, "zero_f32 launch");
}

int deadline_arm(unsigned long long *ctl, double timeout_ms, hipStream_t stream)
{
    int dev = 0;
    (void)hipGetDevice(&dev);
    const unsigned long long ticks = (unsigned long long)(timeout_ms * g_ticks_per_ms[dev]) + 1ull;
    hipLaunchKernelGGL(stamp_deadline, dim3(1), dim3(1), 0, stream, ctl, ticks);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? OPEVO_OK : hip_fail(e, "stamp_deadline launch");
}

int deadline_expired(unsigned long long *ctl, hipStream_t stream, bool *expired)
{
    unsigned long long flag = 0;
    hipError_t e = hipMemcpyAsync(&flag, ctl + 2, sizeof flag, hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return hip_fail(e, "reading the deadline flag");
    *expired = flag != 0;
    return OPEVO_OK;
}

}  // namespace opevo

extern "C" int opevo_compare_f32(const float *c, const float *ref, int64_t n, void *stream,
                                 double *max_scaled, double *rel_fro)
{
    if (!c || !ref || n < 1) return opevo::fail(OPEVO_E_ARG, "compare_f32: bad arguments");
    return opevo::compare_f32(c, ref, n, nullptr, 1, static_cast<hipStream_t>(stream), max_scaled, rel_fro);
}

extern "C" int opevo_compare_rows_f32(const float *c, const float *ref_rows, const int32_t *row_index,
                                      int64_t n_rows, int64_t row_len, void *stream,
                                      double *max_scaled, double *rel_fro)
{
    if (!c || !ref_rows || !row_index || n_rows < 1 || row_len < 1)
        return opevo::fail(OPEVO_E_ARG, "compare_rows_f32: bad arguments");
    return opevo::compare_f32(c, ref_rows, n_rows * row_len, row_index, row_len,
                              static_cast<hipStream_t>(stream), max_scaled, rel_fro);
}

extern "C" int opevo_compare_f32_static(const float *c, const float *ref, int64_t n, void *stream, double *result)
{
    if (!c || !ref || !result || n < 1) return opevo::fail(OPEVO_E_ARG, "compare_f32_static: bad arguments");
    if (n > OPEVO_COMPARE_STATIC_MAX_N)
        return opevo::fail(OPEVO_E_ARG, "compare_f32_static: n = %lld exceeds the limit of %lld elements",
                           (long long)n, (long long)OPEVO_COMPARE_STATIC_MAX_N);
    return opevo::compare_f32_static(c, ref, n, static_cast<hipStream_t>(stream), result);
}
