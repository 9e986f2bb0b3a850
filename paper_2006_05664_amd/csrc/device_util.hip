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

// Batched transposition of 16-bit matrices, out[b][c][r] = in[b][r][c], for two problems in one
// launch (workgroups below blocks0 serve the first): the rewrite of an NCHW image and an OIHW kernel
// tensor to channels-last, or of a MatMul's second operand to [N][K].  A workgroup moves one tile of
// tr rows x tc columns through LDS; every thread issues all its loads before it uses the first, and
// no index needs a division by a run-time number.  Two tile shapes, chosen by the host:
//   narrow (tc == cols <= 64, e.g. the 9 columns of a 3 x 3 kernel; tr * tc <= 4096): the tile is one
//     contiguous run of the input and is copied to LDS as it is.
//   wide (tc = 64 columns of a longer row, tr = 64): reads walk c with the lane, writes walk r.
// Where rows and cols are multiples of 4 (vec4) both directions move four elements (8 bytes) per
// lane: a wave instruction costs the same for 2 bytes per lane as for 8.
struct TransposeJob { const unsigned short *in; unsigned short *out; int batches, rows, cols, tr, tc, tiles_r, tiles_c, narrow, vec4; };
typedef unsigned short u16x4_t __attribute__((ext_vector_type(4)));
constexpr int kTilePitch = 68;     // wide tiles: 64 columns + 4, rows stay 8-byte aligned
__global__ __launch_bounds__(256) void transpose_tiles_16(TransposeJob j0, TransposeJob j1, int blocks0)
{
    __shared__ __attribute__((aligned(8))) unsigned short tile[64 * kTilePitch];   // >= 4096 for the narrow tiles
    int blk = blockIdx.x;
    const bool first = blk < blocks0;
    if (!first) blk -= blocks0;
    const unsigned short *jin = first ? j0.in : j1.in;
    unsigned short *jout = first ? j0.out : j1.out;
    const int rows = first ? j0.rows : j1.rows, cols = first ? j0.cols : j1.cols, tr = first ? j0.tr : j1.tr,
              tc = first ? j0.tc : j1.tc, tiles_r = first ? j0.tiles_r : j1.tiles_r, tiles_c = first ? j0.tiles_c : j1.tiles_c,
              narrow = first ? j0.narrow : j1.narrow, vec4 = first ? j0.vec4 : j1.vec4;
    const int tcb = blk % tiles_c, trb = (blk / tiles_c) % tiles_r, b = blk / (tiles_c * tiles_r);
    const int r0 = trb * tr, c0 = tcb * tc;
    const int nr = min(tr, rows - r0), nc = min(tc, cols - c0);
    const unsigned short *in = jin + ((long)b * rows + r0) * cols + c0;
    unsigned short *out = jout + ((long)b * cols + c0) * rows + r0;
    const int tid = threadIdx.x, tx = tid & 63, ty = tid >> 6;
    if (narrow) {
        // contiguous tile of nr * nc <= 4096 elements, kept in LDS with pitch nc
        if (vec4) {
            u16x4_t v[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int i = (tid + k * 256) * 4;
                v[k] = i < nr * nc ? *(const u16x4_t *)(in + i) : (u16x4_t){0, 0, 0, 0};
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int i = (tid + k * 256) * 4;
                if (i < nr * nc) *(u16x4_t *)(tile + i) = v[k];
            }
            __syncthreads();
            for (int c = ty; c < nc; c += 4)
                for (int r = tx * 4; r < nr; r += 256) {
                    u16x4_t o;
                    o.x = tile[r * nc + c]; o.y = tile[(r + 1) * nc + c]; o.z = tile[(r + 2) * nc + c]; o.w = tile[(r + 3) * nc + c];
                    *(u16x4_t *)(out + (long)c * rows + r) = o;
                }
        } else {
            unsigned short v[16];
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                const int i = tid + k * 256;
                v[k] = i < nr * nc ? in[i] : (unsigned short)0;
            }
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                const int i = tid + k * 256;
                if (i < nr * nc) tile[i] = v[k];
            }
            __syncthreads();
            for (int c = ty; c < nc; c += 4)
                for (int r = tx; r < nr; r += 64) out[(long)c * rows + r] = tile[r * nc + c];
        }
    } else if (vec4) {
        // 64 x 64 tile in 4 x 4 blocks: 16 column quads x 16 row groups per pass
        const int cq = tid & 15, rq = tid >> 4;
        u16x4_t v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int rr = rq + 16 * k;
            v[k] = (rr < nr && cq * 4 < nc) ? *(const u16x4_t *)(in + (long)rr * cols + cq * 4) : (u16x4_t){0, 0, 0, 0};
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) *(u16x4_t *)(tile + (rq + 16 * k) * kTilePitch + cq * 4) = v[k];
        __syncthreads();
        // write: 16 row quads x 16 columns per pass; a thread gathers 4 rows of one column
        const int rqw = tid & 15, cg = tid >> 4;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int cc = cg + 16 * k;
            if (cc < nc && rqw * 4 < nr) {
                u16x4_t o;
                o.x = tile[(rqw * 4 + 0) * kTilePitch + cc]; o.y = tile[(rqw * 4 + 1) * kTilePitch + cc];
                o.z = tile[(rqw * 4 + 2) * kTilePitch + cc]; o.w = tile[(rqw * 4 + 3) * kTilePitch + cc];
                *(u16x4_t *)(out + (long)cc * rows + rqw * 4) = o;
            }
        }
    } else {
        // 64 x 64 tile, element by element
        unsigned short v[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const int rr = ty + 4 * k;
            v[k] = (rr < nr && tx < nc) ? in[(long)rr * cols + tx] : (unsigned short)0;
        }
#pragma unroll
        for (int k = 0; k < 16; ++k) tile[(ty + 4 * k) * kTilePitch + tx] = v[k];
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const int cc = ty + 4 * k;
            if (cc < nc && tx < nr) out[(long)cc * rows + tx] = tile[tx * kTilePitch + cc];
        }
    }
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

int transpose_16(const void *in0, void *out0, int64_t batches0, int64_t rows0, int64_t cols0,
                 const void *in1, void *out1, int64_t batches1, int64_t rows1, int64_t cols1, hipStream_t stream)
{
    auto job = [](const void *in, void *out, int64_t batches, int64_t rows, int64_t cols) {
        TransposeJob j;
        j.in = static_cast<const unsigned short *>(in); j.out = static_cast<unsigned short *>(out);
        j.batches = int(batches); j.rows = int(rows); j.cols = int(cols);
        // narrow tile: whole rows where they are short, as many as fit 4096 elements (a multiple of 4
        // of them for the 8-byte form); wide tile: 64 x 64
        const bool aligned = reinterpret_cast<uintptr_t>(in) % 8 == 0 && reinterpret_cast<uintptr_t>(out) % 8 == 0;
        j.narrow = cols <= 64;
        j.vec4 = aligned && rows % 4 == 0 && cols % 4 == 0;
        if (j.narrow) {
            j.tc = int(std::max<int64_t>(cols, 1));
            // rows * cols of a batch is a multiple of 4 whenever rows is: the contiguous copy may then go 8 bytes at a time
            j.vec4 = aligned && rows % 4 == 0;
            int64_t tr = std::max<int64_t>(1, std::min<int64_t>(rows, 4096 / j.tc));
            if (j.vec4 && tr >= 4) tr = tr / 4 * 4;
            j.tr = int(tr);
            if (j.vec4 && (j.tr % 4 != 0)) j.vec4 = 0;
        } else { j.tc = 64; j.tr = 64; }
        j.tiles_r = int((rows + j.tr - 1) / j.tr); j.tiles_c = int((cols + j.tc - 1) / j.tc);
        return j;
    };
    if (!in1) batches1 = 0;
    const TransposeJob j0 = job(in0, out0, batches0, rows0, cols0), j1 = job(in1, out1, batches1, rows1, cols1);
    const int64_t blocks0 = int64_t(j0.batches) * j0.tiles_r * j0.tiles_c, blocks1 = int64_t(j1.batches) * j1.tiles_r * j1.tiles_c;
    if (blocks0 + blocks1 > INT32_MAX || batches0 * rows0 * cols0 >= (int64_t(1) << 40) || rows0 >= (int64_t(1) << 31) ||
        cols0 >= (int64_t(1) << 31) || rows1 >= (int64_t(1) << 31) || cols1 >= (int64_t(1) << 31))
        return fail(OPEVO_E_ARG, "operand re-layout pre-pass: tensors too large");
    if (blocks0 + blocks1 == 0) return OPEVO_OK;
    hipLaunchKernelGGL(transpose_tiles_16, dim3(unsigned(blocks0 + blocks1)), dim3(256), 0, stream, j0, j1, int(blocks0));
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? OPEVO_OK : hip_fail(e, "operand re-layout pre-pass launch");
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
