// MFMA-only loop: the matrix-pipe ceiling the device sustains under its power limit.
// Every wave keeps a 4x2 arrangement of accumulators busy with ITERS rounds of 32x32x16 MFMAs
// (PEAK_ATOM = 32) or twice as many rounds of 16x16x32 MFMAs (PEAK_ATOM = 16: half the flops per
// instruction, a quarter of the accumulator updates per flop) on register-resident operand fragments (4 of A, 2 of B, whatever the caller put into
// `in`: the clock the device holds depends on how many operand bits toggle, so zeros and
// random data give different ceilings); nothing else runs.
// Flops = blocks * waves * 8 * ITERS * 32768.
#if IN_DTYPE == 1
typedef __attribute__((ext_vector_type(8))) __bf16 frag_t;
#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0)
#define MFMA16(a, b, c) __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0)
#else
typedef __attribute__((ext_vector_type(8))) _Float16 frag_t;
#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0)
#define MFMA16(a, b, c) __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0)
#endif

#ifndef PEAK_ATOM
#define PEAK_ATOM 32
#endif
#if PEAK_ATOM == 16
typedef __attribute__((ext_vector_type(4))) float f32x4_;
extern "C" __global__ __launch_bounds__(256)
void KERNEL_NAME(const u16 *__restrict__ in, const u16 *__restrict__ unused, float *__restrict__ out,
                 unsigned long long *ctl)
{
    frag_t a[4], b[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = __builtin_bit_cast(frag_t, *(const u32x4 *)(in + (i * 256 + threadIdx.x) * 8));
#pragma unroll
    for (int j = 0; j < 2; ++j) b[j] = __builtin_bit_cast(frag_t, *(const u32x4 *)(in + ((4 + j) * 256 + threadIdx.x) * 8));
    f32x4_ acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[i][r] = 0.f;
    for (int it = 0; it < ITERS * 2; ++it) {     // half the flops per instruction: twice the rounds
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = MFMA16(a[i & 3], b[i >> 2], acc[i]);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) s += acc[i][r];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}
#else
extern "C" __global__ __launch_bounds__(256)
void KERNEL_NAME(const u16 *__restrict__ in, const u16 *__restrict__ unused, float *__restrict__ out,
                 unsigned long long *ctl)
{
    frag_t a[4], b[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = __builtin_bit_cast(frag_t, *(const u32x4 *)(in + (i * 256 + threadIdx.x) * 8));
#pragma unroll
    for (int j = 0; j < 2; ++j) b[j] = __builtin_bit_cast(frag_t, *(const u32x4 *)(in + ((4 + j) * 256 + threadIdx.x) * 8));
    f32x16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    for (int it = 0; it < ITERS; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = MFMA(a[i & 3], b[i >> 2], acc[i]);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}
#endif
