// Shared prologue of the kernel templates: operator geometry.
//
// Every name in capitals is a compile-time constant supplied per configuration as a -D
// option by the host (see the plan/define renderer): the kernels contain no run-time
// shape arguments, so each configuration is its own specialised program, compiled and run
// on the hardware to be scored (Sec. 1).
//
// All three operators are run as one batched GEMM view  C[b][m][n] = sum_k A[b][m][k] B[b][k][n]:
//   OP 0  MatMul       (App. B.1)  batch = 1
//   OP 1  BatchMatMul  (App. B.2)  grid z = batch / BATCH_INNER, BATCH_INNER batches per workgroup
//   OP 2  Conv2d       (App. B.3, Eq. 5 with stride and padding) as an implicit GEMM:
//         m = output channel, k = (ci, r, s) flattened as the OIHW kernel tensor stores it,
//         n = output pixel (image, y, x); B[k][n] is gathered from the NCHW image on the fly
//         and is zero where the tap falls outside the image.
//
// Workgroup (bx, by, bz) = block_id() (by default blockIdx.x, .y, .z) owns rows [by*BM, +BM) and
// columns "bx-th block of BN columns".  For conv a block of columns is a box of
// NB2 images x BH rows x BW pixels; column c of the block is image c/(BH*BW), row (c/BW)%BH,
// pixel c%BW of that box.

#ifndef A_TRANS
#define A_TRANS 0
#endif
#ifndef KSPLIT
#define KSPLIT 1   // MatMul, Conv2d: workgroups along grid z that share one output tile, each reducing its own K range
#endif
#ifndef SUBM
// A workgroup tile too large for one pass (LDS, accumulators) is computed as SUBM x SUBN sub-tiles of
// BM x BN, one after another: workgroup (n, m) owns rows [m*SUBM*BM, +SUBM*BM) and the columns alike.
#define SUBM 1
#define SUBN 1
#endif
#define OP_MATMUL 0
#define OP_BMM 1
#define OP_CONV 2

typedef unsigned short u16;
typedef unsigned int u32;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

#if IN_DTYPE == 0
typedef float in_t;
__device__ __forceinline__ float to_f32(in_t x) { return x; }
#elif IN_DTYPE == 1
typedef u16 in_t;   // bf16 bits
__device__ __forceinline__ float to_f32(in_t x) { return __builtin_bit_cast(float, (u32)x << 16); }
#else
typedef u16 in_t;   // fp16 bits
__device__ __forceinline__ float to_f32(in_t x) { return (float)__builtin_bit_cast(_Float16, x); }
#endif

// Which tile a workgroup owns: n = block of BN columns, m = block of BM rows, b = batch block.
// Default launch: a three-dimensional grid (n, m, b).  With GRID_LINEAR the launch is
// one-dimensional and the linear workgroup number walks the axes 0 = n, 1 = m, 2 = b in the order
// ORDER0 (fastest), ORDER1, ORDER2; GROUP consecutive tiles of axis ORDER1 are walked together:
// a group goes through the whole of axis ORDER0 (second-axis index fastest inside the group)
// before the next group starts; a ragged last group is narrower.
struct BlockId { int n, m, b; };
__device__ __forceinline__ BlockId block_id()
{
    BlockId id;
#ifdef GRID_LINEAR
    constexpr int ext[3] = {GRID_N1, GRID_M1, GRID_B1};
    constexpr int e0 = ext[ORDER0], e1 = ext[ORDER1];
    const int L = blockIdx.x;
    const int rest = L / (e0 * e1), pid = L % (e0 * e1);
    const int gid = pid / (GROUP * e0), in_group = pid % (GROUP * e0);
    const int first = gid * GROUP;
    const int gsz = (e1 - first < GROUP) ? e1 - first : GROUP;
    int idx[3];
    idx[ORDER0] = in_group / gsz;
    idx[ORDER1] = first + in_group % gsz;
    idx[ORDER2] = rest;
    id.n = idx[0]; id.m = idx[1]; id.b = idx[2];
#else
    id.n = blockIdx.x; id.m = blockIdx.y; id.b = blockIdx.z;
#endif
    return id;
}

// One element of the result.  With the reduction split over KSPLIT workgroups the output has been
// cleared by the host before the launch and every workgroup adds its partial sum (fp32 atomic add
// in device scope, unordered: the rounding of the last bits depends on the arrival order).
__device__ __forceinline__ void c_out(float *p, float v)
{
#if KSPLIT > 1
    __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#else
    *p = v;
#endif
}

#if OP == OP_CONV
// Conv2d with the reduction split over grid z: first position of this workgroup's range of the
// reduction walk (its KSTEPS slabs follow from there)
#if KSPLIT > 1
#define CONV_KBASE(bid) ((bid).b * (KSTEPS * BK))
#else
#define CONV_KBASE(bid) 0
#endif
struct ColBlock { int nb0, y0, x0; };
__device__ __forceinline__ ColBlock col_block(int bx)
{
    ColBlock cb;
    cb.x0 = (bx % W1) * BW;
    cb.y0 = ((bx / W1) % H1) * BH;
    cb.nb0 = (bx / (W1 * H1)) * NB2;
    return cb;
}
// Position k of the reduction as the kernel walks it -> flattened tap (ci*HK + r)*WK + s.
// By default the walk is the flattened order itself.  With TAP_BOX the three reduction axes are
// split separately (App. B.3: C_in, H_k and W_k in two factors each): slab k / BK is the box
// number (cio, ro, so), row-major over CI_O x HK_O x WK_O boxes, and k % BK is the place
// (a, b, c) inside the CI_I x HK_I x WK_I box, row-major as well.
__host__ __device__ constexpr int conv_tap(int k)
{
#ifdef TAP_BOX
    const int kt = k / BK, j = k % BK;
    const int so = kt % WK_O, ro = (kt / WK_O) % HK_O, cio = kt / (WK_O * HK_O);
    const int c = j % WK_I, b = (j / WK_I) % HK_I, a = j / (WK_I * HK_I);
    return ((cio * CI_I + a) * HK + ro * HK_I + b) * WK + so * WK_I + c;
#else
    return k;
#endif
}
// B[k][c] of the implicit GEMM: image value under position k of the reduction for column c of the block.
__device__ __forceinline__ in_t conv_b(const in_t *__restrict__ img, const ColBlock &cb, int kpos, int c)
{
    const int k = conv_tap(kpos);
    const int ci = k / (HK * WK), r = (k / WK) % HK, s = k % WK;
    const int nb = cb.nb0 + c / (BH * BW);
    const int y = (cb.y0 + (c / BW) % BH) * STRIDE + r - PAD_CONV;
    const int x = (cb.x0 + c % BW) * STRIDE + s - PAD_CONV;
    if (y < 0 || y >= HIN || x < 0 || x >= WIN) return (in_t)0;
    return img[(((long)nb * CIN + ci) * HIN + y) * WIN + x];
}
__device__ __forceinline__ long conv_c_index(const ColBlock &cb, int m, int c)
{
    const int nb = cb.nb0 + c / (BH * BW);
    const int y = cb.y0 + (c / BW) % BH;
    const int x = cb.x0 + c % BW;
    return (((long)nb * M + m) * HOUT + y) * WOUT + x;
}
#endif
