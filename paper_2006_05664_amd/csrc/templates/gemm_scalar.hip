// Scalar-FMA kernel template: runs every member of every configuration space (any tile
// shape, any input type), one fp32 FMA per multiply-accumulate.  It is the only template of
// the two-level spaces and the fallback of the four-level spaces where the per-wave tile is
// not made of MFMA atoms.
//
// Workgroup tile BM x BN, K consumed in KSTEPS slabs of BK staged in LDS as fp32.
// The NT threads share the BM*BN outputs round-robin: thread t owns outputs t, t+NT, ...
// (row = index / BN, column = index % BN), E of them, each a register accumulator.
//
// Members of the spaces that land here can be orders of magnitude slower than the MFMA
// kernels, so this template honours a deadline: ctl (may be NULL) points to
// {start tick, allowed ticks, expired flag} in device memory; once per K slab thread 0
// compares the device wall clock with it and, through an LDS word read by all threads
// after the slab's first barrier, the whole workgroup leaves together.  The host then
// scores the trial as invalid (fitness 0).

#ifndef KUNROLL
#define KUNROLL 4   // reduction steps unrolled together where the flag asks for unrolling
#endif
#define PRAGMA_(x) _Pragma(#x)
#define PRAGMA_UNROLL(n) PRAGMA_(unroll n)

extern "C" __global__ __launch_bounds__(NT)
void KERNEL_NAME(const in_t *__restrict__ A, const in_t *__restrict__ B, float *__restrict__ C,
                  unsigned long long *ctl)
{
    extern __shared__ __attribute__((aligned(16))) float smem_f[];
    float *As = smem_f;             // [BM][BK]
    float *Bs = smem_f + BM * BK;   // [BK][BN]
    __shared__ int expired;
    const int tid = threadIdx.x;
    if (tid == 0) expired = 0;
    const BlockId bid = block_id();
    constexpr int E = (BM * BN + NT - 1) / NT;

#if OP == OP_CONV
    const ColBlock cb = col_block(bid.n);
#endif

    for (int bi = 0; bi < BATCH_INNER; ++bi)
    for (int sub = 0; sub < SUBM * SUBN; ++sub) {
        const int m0 = (bid.m * SUBM + sub / SUBN) * BM;
#if OP != OP_CONV
        const int n0 = (bid.n * SUBN + sub % SUBN) * BN;
#endif
#if OP == OP_CONV
        const in_t *Ab = A;   // kernel tensor [M][K]
#else
#if KSPLIT > 1   // MatMul, reduction split over grid z: this workgroup owns K range [bid.b * KSTEPS * BK, + KSTEPS * BK)
        const in_t *Ab = A + (long)bid.b * (KSTEPS * BK);
        const in_t *Bb = B + (long)bid.b * (KSTEPS * BK) * N;
        float *Cb = C;
#else
        const long batch = (long)bid.b * BATCH_INNER + bi;
        const in_t *Ab = A + batch * M * K;
        const in_t *Bb = B + batch * K * N;
        float *Cb = C + batch * M * N;
#endif
#endif
        float acc[E];
#pragma unroll
        for (int e = 0; e < E; ++e) acc[e] = 0.f;

        for (int kt = 0; kt < KSTEPS; ++kt) {
#if OP == OP_CONV
            const int k0 = CONV_KBASE(bid) + kt * BK;
#else
            const int k0 = kt * BK;
#endif
            if (tid == 0 && ctl && ctl[1] != 0 && wall_clock64() - ctl[0] > ctl[1]) {
                expired = 1;
                ctl[2] = 1;
            }
            __syncthreads();
            if (expired) return;
            for (int i = tid; i < BM * BK; i += NT)
#if A_TRANS   // first operand stored [K][M]: walk it along M so that the loads stay coalesced
                As[(i % BM) * BK + i / BM] = to_f32(Ab[(long)(k0 + i / BM) * M + m0 + i % BM]);
#elif OP == OP_CONV
                As[i] = to_f32(Ab[(long)(m0 + i / BK) * K + conv_tap(k0 + i % BK)]);
#else
                As[i] = to_f32(Ab[(long)(m0 + i / BK) * K + k0 + i % BK]);
#endif
            for (int i = tid; i < BK * BN; i += NT) {
#if OP == OP_CONV
                Bs[i] = to_f32(conv_b(B, cb, k0 + i / BN, i % BN));
#else
                Bs[i] = to_f32(Bb[(long)(k0 + i / BN) * N + n0 + i % BN]);
#endif
            }
            __syncthreads();
#if FLAG
            PRAGMA_UNROLL(KUNROLL)
#else
#pragma unroll 1
#endif
            for (int kk = 0; kk < BK; ++kk) {
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const int idx = tid + e * NT;
                    if (idx < BM * BN)
                        acc[e] = __builtin_fmaf(As[(idx / BN) * BK + kk], Bs[kk * BN + idx % BN], acc[e]);
                }
            }
        }
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int idx = tid + e * NT;
            if (idx < BM * BN) {
#if OP == OP_CONV
                c_out(&C[conv_c_index(cb, m0 + idx / BN, idx % BN)], acc[e]);
#else
                c_out(&Cb[(long)(m0 + idx / BN) * N + n0 + idx % BN], acc[e]);
#endif
            }
        }
    }
}
