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
//  * Fragment reads run one MFMA step ahead of the MFMAs, across slab boundaries as well, so
//    no LDS latency is exposed after a barrier.
//  * The waits are explicit: s_waitcnt vmcnt(n) with n = the loads this wave issued after the
//    slab it needs, then a bare s_barrier (the fence of __syncthreads() would drain every
//    outstanding load).

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

// One wave-wide 16-byte-per-lane load whose destination is LDS: lane i's 16 bytes land at
// lds_base + 16 * i (lds_base wave-uniform, passed in M0).  It is written as inline assembly so
// that the compiler's own wait-count bookkeeping never sees these loads: whenever it loses track
// of which LDS object such a load fills, it guards later LDS reads with a wait for ALL
// outstanding loads, which would cut the ring down to a single slab in flight.  The kernel
// places every wait these loads need itself (WAIT_VMCNT below).
__device__ __forceinline__ void dma16(const u16 *g, unsigned lds_base)
{
    const unsigned m = __builtin_amdgcn_readfirstlane(lds_base);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(m) : "memory", "m0");
}

// stage: LDS byte address of the stage to fill
__device__ __forceinline__ void issue_slab(const u16 *__restrict__ Ab, const u16 *__restrict__ Bb, unsigned stage,
                                           int m0, int n0, int k0, int wave, int lane)
{
#pragma unroll
    for (int t = 0; t < LA; ++t) {
        const int instr = wave * LA + t;                 // which 1 KiB piece of the A part
        const int p = instr * 64 + lane;                 // 16-byte position this lane fills
        const int row = p / ACH, kc = (p % ACH) ^ a_swz(row);
        dma16(Ab + (long)(m0 + row) * K + k0 + kc * 8, stage + instr * 1024);
    }
#pragma unroll
    for (int t = 0; t < LB; ++t) {
        const int instr = wave * LB + t;
        const int p = instr * 64 + lane;
        const int krow = p / BCH, c = (p % BCH) ^ b_swz(krow);
        dma16(Bb + (long)(k0 + krow) * N + n0 + c * 8, stage + (A_STAGE + instr * 512) * 2);
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
#define VMC(n) ((n) < 63 ? (n) : 63)
#define WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt((VMC(n) & 0xf) | ((VMC(n) >> 4) << 14) | (0x7 << 4) | (0xf << 8))
#define WAIT_LGKM_VMCNT(n) __builtin_amdgcn_s_waitcnt((VMC(n) & 0xf) | ((VMC(n) >> 4) << 14) | (0x7 << 4) | (0x0 << 8))
#define BARRIER() do { asm volatile("" ::: "memory"); __builtin_amdgcn_s_barrier(); asm volatile("" ::: "memory"); } while (0)
#define KCLAMP(k) ((k) < KSTEPS ? (k) : KSTEPS - 1)

extern "C" __global__ __launch_bounds__(NT)
void KERNEL_NAME(const u16 *__restrict__ A, const u16 *__restrict__ B, float *__restrict__ C,
                 unsigned long long *ctl /* deadline control, used by the scalar template only */)
{
    __shared__ __attribute__((aligned(1024))) u16 ring[NSTG * STAGE];
    u16 *const stg[4] = {ring, ring + STAGE, ring + (NSTG > 2 ? 2 : 0) * STAGE, ring + (NSTG > 3 ? 3 : 0) * STAGE};
    const unsigned ring_addr = (unsigned)(unsigned long)(__attribute__((address_space(3))) u16 *)ring;   // LDS byte address
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
        // prologue: slabs 0 .. NSTG-1 in flight (one per stage), slab 0 landed, its first fragments read
#pragma unroll
        for (int s = 0; s < NSTG; ++s) issue_slab(Ab, Bb, ring_addr + s * STAGE * 2, m0, n0, KCLAMP(s) * BK, wave, lane);
        WAIT_VMCNT((NSTG - 1) * PER);
        BARRIER();
        frag_t af[2][MI], bf[2][NI];
        load_frags(af[0], bf[0], stg[0], wm, wn, lane, 0);

        // Slab q, resident in stage s.  The fragment reads run one MFMA step ahead of the MFMAs,
        // across slab boundaries too: before the last step of a slab the wave makes sure slab
        // q + 1 has landed for everyone, reads that slab's first fragments, and only then issues
        // the MFMAs of its own last step, which cover the latency of those reads.  At that barrier
        // every wave holds all of slab q in registers, so stage s is refilled right there.
        auto slab_step = [&](int q, int s) {
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                if (kk + 1 < KK) {
                    load_frags(af[(kk + 1) & 1], bf[(kk + 1) & 1], stg[s], wm, wn, lane, kk + 1);
                } else {
                    WAIT_LGKM_VMCNT((NSTG - 2) * PER);   // own fragments of this step read, own part of slab q+1 landed
                    BARRIER();
                    load_frags(af[0], bf[0], stg[(s + 1) % NSTG], wm, wn, lane, 0);
                    // past the end: a redundant copy of the last slab
                    issue_slab(Ab, Bb, ring_addr + s * STAGE * 2, m0, n0, KCLAMP(q + NSTG) * BK, wave, lane);
                }
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
