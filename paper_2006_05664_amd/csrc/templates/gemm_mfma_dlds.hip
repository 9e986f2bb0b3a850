// MFMA kernel template with operands streamed global memory -> LDS directly (gfx950), for
// MatMul / BatchMatMul members whose tile shapes allow it (the host's decoder decides).
//
// Roles of the tiling factors are those of the register-staged MFMA template: workgroup tile
// BM x BN, WM x WN waves, per-wave tile TM x TN of 32x32x16 atoms, K consumed in KSTEPS slabs of
// BK.  What differs is how a slab travels:
//
//  * Every wave issues wave-wide 16-byte-per-lane loads whose destination is LDS (1 KiB per
//    instruction, no registers, no LDS store instructions).  NSTG stages of BM*BK + BK*BN
//    elements each form a ring; NSTG-1 slabs are in flight while one is being multiplied.
//  * A stage keeps A as [BM][BK] and B as [BK][BN], i.e. both exactly as global memory has
//    them.  The 16-byte chunk c of A row r sits at chunk position c ^ ((r / A_RPW) % ACH), of
//    B row k at c ^ (((k / B_RPW) % ..) << 2): the permutation is applied by choosing which
//    global chunk each lane loads, and it keeps every fragment read free of bank conflicts.
//  * A fragments are 16-byte LDS reads.  B fragments need 8 consecutive k for one n; they
//    are read with the transposing LDS load: in each group of 16 lanes, lane s supplies the
//    address of 4 consecutive n at row k + s/4, and lane i receives the 4 consecutive k of
//    column n0 + i (two such reads per fragment).
//  * The waits are explicit: s_waitcnt vmcnt(n) with n = the loads this wave issued after the
//    slab it needs, then a bare s_barrier (the fence of __syncthreads() would drain every
//    outstanding load).  Each stage is its own LDS object so that the compiler can tell that
//    loads landing in one stage do not alias the fragment reads of another.

#if IN_DTYPE == 1
typedef __attribute__((ext_vector_type(8))) __bf16 frag_t;
#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0)
#else
typedef __attribute__((ext_vector_type(8))) _Float16 frag_t;
#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0)
#endif
typedef __attribute__((ext_vector_type(4))) short v4s;
typedef __attribute__((ext_vector_type(8))) short v8s;
typedef f32x16 acc_t;
#define LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

constexpr int NW = NT / 64;
constexpr int MI = TM / 32, NI = TN / 32;
constexpr int KK = BK / 16;                                   // MFMA K steps per slab
constexpr int A_STAGE = BM * BK, B_STAGE = BK * BN, STAGE = A_STAGE + B_STAGE;   // elements
constexpr int ACH = BK / 8;                                   // 16-byte chunks per A row
constexpr int A_RPW = (16 / ACH) > 0 ? (16 / ACH) : 1;        // A rows per 256-byte bank window
constexpr int BCH = BN / 8;                                   // chunks per B row
constexpr int B_RPW = (16 / BCH) > 0 ? (16 / BCH) : 1;
constexpr int B_SWM = (4 / B_RPW) > 0 ? (4 / B_RPW) : 1;
constexpr int LA = BM * BK * 2 / 1024 / NW, LB = BK * BN * 2 / 1024 / NW;   // loads per wave and slab
constexpr int PER = LA + LB;

__device__ __forceinline__ int a_swz(int row) { return (row / A_RPW) % ACH; }
__device__ __forceinline__ int b_swz(int krow) { return ((krow / B_RPW) % B_SWM) << 2; }

__device__ __forceinline__ void issue_slab(const u16 *__restrict__ Ab, const u16 *__restrict__ Bb, u16 *stage,
                                           int m0, int n0, int k0, int wave, int lane)
{
#pragma unroll
    for (int t = 0; t < LA; ++t) {
        const int instr = wave * LA + t;                 // which 1 KiB piece of the A part
        const int p = instr * 64 + lane;                 // 16-byte position this lane fills
        const int row = p / ACH, kc = (p % ACH) ^ a_swz(row);
        __builtin_amdgcn_global_load_lds(Ab + (long)(m0 + row) * K + k0 + kc * 8, LDS_PTR(stage + instr * 512), 16, 0, 0);
    }
#pragma unroll
    for (int t = 0; t < LB; ++t) {
        const int instr = wave * LB + t;
        const int p = instr * 64 + lane;
        const int krow = p / BCH, c = (p % BCH) ^ b_swz(krow);
        __builtin_amdgcn_global_load_lds(Bb + (long)(k0 + krow) * N + n0 + c * 8, LDS_PTR(stage + A_STAGE + instr * 512), 16, 0, 0);
    }
}

__device__ __forceinline__ void load_frags(frag_t (&af)[MI], frag_t (&bf)[NI], const u16 *stage,
                                           int wm, int wn, int lane, int kk)
{
    const u16 *As = stage, *Bs = stage + A_STAGE;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
        const int row = wm * TM + i * 32 + (lane & 31);
        const int kc = kk * 2 + (lane >> 5);
        af[i] = __builtin_bit_cast(frag_t, *(const u32x4 *)(As + row * BK + ((kc ^ a_swz(row)) << 3)));
    }
    const int s = lane & 15;
#pragma unroll
    for (int j = 0; j < NI; ++j) {
        const int n = wn * TN + j * 32 + 16 * ((lane >> 4) & 1) + 4 * (s & 3);
        v4s h[2];
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int krow = kk * 16 + 8 * (lane >> 5) + 4 * r + (s >> 2);
            const u16 *p = Bs + krow * BN + (((n >> 3) ^ b_swz(krow)) << 3) + (n & 7);
            h[r] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s *)p);
        }
        bf[j] = __builtin_bit_cast(frag_t, __builtin_shufflevector(h[0], h[1], 0, 1, 2, 3, 4, 5, 6, 7));
    }
}

// s_waitcnt vmcnt(n) alone (expcnt and lgkmcnt left at their maxima), gfx9 encoding
#define WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xf) | (((n) >> 4) << 14) | (0x7 << 4) | (0xf << 8))
#define BARRIER() do { asm volatile("" ::: "memory"); __builtin_amdgcn_s_barrier(); asm volatile("" ::: "memory"); } while (0)
#define KCLAMP(k) ((k) < KSTEPS ? (k) : KSTEPS - 1)

extern "C" __global__ __launch_bounds__(NT)
void KERNEL_NAME(const u16 *__restrict__ A, const u16 *__restrict__ B, float *__restrict__ C,
                 unsigned long long *ctl /* deadline control, used by the scalar template only */)
{
    __shared__ __attribute__((aligned(1024))) u16 st0[STAGE];
    __shared__ __attribute__((aligned(1024))) u16 st1[STAGE];
#if NSTG > 2
    __shared__ __attribute__((aligned(1024))) u16 st2[STAGE];
#else
#define st2 st0
#endif
#if NSTG > 3
    __shared__ __attribute__((aligned(1024))) u16 st3[STAGE];
#else
#define st3 st0
#endif
    u16 *const stg[4] = {st0, st1, st2, st3};
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;

    for (int bi = 0; bi < BATCH_INNER; ++bi) {
        const long batch = (long)blockIdx.z * BATCH_INNER + bi;
        const u16 *Ab = A + batch * M * K;
        const u16 *Bb = B + batch * K * N;
        float *Cb = C + batch * M * N;

        acc_t acc[MI][NI];
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

        if (bi > 0) BARRIER();      // every wave is done reading the previous batch's stages
        // prologue: slabs 0 .. NSTG-2 in flight, slab 0 landed, its first fragments read
#pragma unroll
        for (int s = 0; s < NSTG - 1; ++s) issue_slab(Ab, Bb, stg[s], m0, n0, KCLAMP(s) * BK, wave, lane);
        WAIT_VMCNT((NSTG - 2) * PER);
        BARRIER();
        frag_t af[2][MI], bf[2][NI];
        load_frags(af[0], bf[0], stg[0], wm, wn, lane, 0);

        // slab q, resident in stage s
        auto slab_step = [&](int q, int s) {
            if (q > 0) {
                WAIT_VMCNT((NSTG - 2) * PER);   // this wave's part of slab q has landed
                BARRIER();                       // everyone's has, and the stage of slab q-1 is free
                load_frags(af[0], bf[0], stg[s], wm, wn, lane, 0);
            }
            // refill the stage slab q-1 used (past the end: a redundant copy of the last slab)
            issue_slab(Ab, Bb, stg[(s + NSTG - 1) % NSTG], m0, n0, KCLAMP(q + NSTG - 1) * BK, wave, lane);
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                if (kk + 1 < KK) load_frags(af[(kk + 1) & 1], bf[(kk + 1) & 1], stg[s], wm, wn, lane, kk + 1);
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NI; ++j) acc[i][j] = MFMA(af[kk & 1][i], bf[kk & 1][j], acc[i][j]);
            }
        };
        constexpr int KMAIN = KSTEPS / NSTG * NSTG;
        for (int kt = 0; kt < KMAIN; kt += NSTG) {
#pragma unroll
            for (int s = 0; s < NSTG; ++s) slab_step(kt + s, s);
        }
#pragma unroll
        for (int s = 0; s < KSTEPS - KMAIN; ++s) slab_step(KMAIN + s, s);

        // Epilogue: an atom's result sits with column (l % 32) in lane l, register r being
        // row 8*(r/4) + 4*(l/32) + r%4.
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = 8 * (r / 4) + 4 * (lane / 32) + r % 4;
                    Cb[(long)(m0 + wm * TM + i * 32 + row) * N + n0 + wn * TN + j * 32 + (lane & 31)] = acc[i][j][r];
                }
    }
}
