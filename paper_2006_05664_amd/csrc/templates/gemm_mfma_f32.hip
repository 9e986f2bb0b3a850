// fp32 MFMA kernel template (MatMul / BatchMatMul with fp32 inputs, App. B.1 / B.2 at the paper's
// own precision): 32x32x2 fp32 atoms, fp32 accumulation, for members of the four-level spaces whose
// per-wave tile is made of 32x32 atoms and whose K slab is a multiple of 8.
//
// Roles of the tiling factors as in the 16-bit MFMA template: workgroup tile BM x BN, WM x WN
// waves, per-wave tile TM x TN, K consumed in KSTEPS slabs of BK staged in LDS.
//
// An fp32 atom takes one value per lane and operand: lane l supplies row (column) l % 32 at
// reduction index l / 32, so an instruction reduces two k.  Both operands are staged exactly as
// global memory has them, with 16-byte loads and 16-byte LDS stores and no transposition:
//   As[BM][BK + 4]: a lane reads the four consecutive k of its row with one 16-byte LDS read
//                   (lanes 0..31 the k 8g .. 8g+3, lanes 32..63 the k 8g+4 .. 8g+7) and feeds them
//                   to four MFMAs, which therefore pair k = 8g + j with k = 8g + 4 + j;
//   Bs[BK][BN + 4]: for MFMA j a lane reads the value at row 8g + 4*(l / 32) + j of its column
//                   (32 consecutive floats per half wave: conflict-free).
// Which k are paired inside an instruction does not matter as long as both operands agree.
// A_TRANS (first operand stored [K][M]): A is staged [BK][BM + 4] and read like B.
// Conv2d (implicit GEMM, App. B.3): the kernel tensor is A, the image is gathered into B's layout
// value by value (bounds-checked taps, zero padding).  A K slab of BK taps is staged BKP = BK
// rounded up to 8 wide (rows of zeros), and a wave tile that is no multiple of 32 is rounded up to
// whole atoms: the overhang reads rows / columns of its neighbours (or the slack behind the tile)
// and is never stored.
// FLAG = 1: two LDS stages; the 16-byte pieces of slab kt+1 are loaded into registers before the
//           MFMAs of slab kt and written to the other stage after them (one barrier per slab).
// FLAG = 0: one stage, load -> barrier -> store -> barrier -> compute.

typedef f32x16 acc_t;
#ifndef BKP
#define BKP BK
#endif
#ifndef NWR
#define NWR (WM * WN)   // waves the workgroup really runs
#endif
constexpr int NPASS = (WM * WN) / NWR;
constexpr int MI = (TM + 31) / 32, NI = (TN + 31) / 32;
#if OP == OP_CONV
// rows of A / columns of B that the last atoms of the last waves may read past the tile
constexpr int A_ROWS = (WM - 1) * TM + MI * 32, B_COLS = ((WN - 1) * TN + NI * 32 + 3) / 4 * 4;
constexpr int LDA = BKP + 4;
constexpr int A_STAGE = A_ROWS * LDA;
constexpr int A_CHUNKS = BM * (BKP / 4);                      // (row, 4 taps)
constexpr int LDB = B_COLS + 4;
constexpr int B_STAGE = BKP * LDB;
constexpr int BN4 = (BN + 3) / 4;
constexpr int B_CHUNKS = BKP * BN4;                           // (tap, 4 columns)
#else
#if A_TRANS   // first operand stored [K][M]: staged [BK][BM + 4] and read like B, one value per MFMA
constexpr int LDA = BM + 4;
constexpr int A_STAGE = BK * LDA;
constexpr int A_CHUNKS = BK * (BM / 4);
#else
constexpr int LDA = BK + 4;                                   // floats; rows stay 16-byte aligned
constexpr int A_STAGE = BM * LDA;
constexpr int A_CHUNKS = BM * (BK / 4);                       // 16-byte pieces of a slab
#endif
constexpr int LDB = BN + 4;
constexpr int B_STAGE = BK * LDB;
constexpr int B_CHUNKS = BK * (BN / 4);
#endif
constexpr int NA = (A_CHUNKS + NT - 1) / NT, NB = (B_CHUNKS + NT - 1) / NT;
#ifndef NSTAGE
#define NSTAGE 1
#endif

struct Slab { f32x4 a[NA], b[NB]; };

#if OP == OP_CONV
// k0 = first position of the slab in the reduction walk (slab number * BK)
__device__ __forceinline__ void load_slab(Slab &s, const float *__restrict__ Ab, const float *__restrict__ Bb,
                                          int m0, const ColBlock &cb, int k0, int tid)
{
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int q = tid + i * NT;
        if (A_CHUNKS % NT == 0 || q < A_CHUNKS) {
            const int row = q / (BKP / 4), kc = q % (BKP / 4);
            f32x4 v;
#pragma unroll
            for (int t = 0; t < 4; ++t) v[t] = (kc * 4 + t < BK) ? Ab[(long)(m0 + row) * K + conv_tap(k0 + kc * 4 + t)] : 0.f;
            s.a[i] = v;
        }
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int q = tid + i * NT;
        if (B_CHUNKS % NT == 0 || q < B_CHUNKS) {
            const int krow = q / BN4, c0 = (q % BN4) * 4;
            f32x4 v;
#pragma unroll
            for (int t = 0; t < 4; ++t) v[t] = (krow < BK && c0 + t < BN) ? conv_b(Bb, cb, k0 + krow, c0 + t) : 0.f;
            s.b[i] = v;
        }
    }
}

__device__ __forceinline__ void store_slab(const Slab &s, float *As, float *Bs, int tid)
{
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int q = tid + i * NT;
        if (A_CHUNKS % NT == 0 || q < A_CHUNKS) *(f32x4 *)(As + (q / (BKP / 4)) * LDA + (q % (BKP / 4)) * 4) = s.a[i];
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int q = tid + i * NT;
        if (B_CHUNKS % NT == 0 || q < B_CHUNKS) *(f32x4 *)(Bs + (q / BN4) * LDB + (q % BN4) * 4) = s.b[i];
    }
}
#else
__device__ __forceinline__ void load_slab(Slab &s, const float *__restrict__ Ab, const float *__restrict__ Bb,
                                          int m0, int n0, int k0, int tid)
{
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int q = tid + i * NT;
        if (A_CHUNKS % NT == 0 || q < A_CHUNKS)
#if A_TRANS
            s.a[i] = *(const f32x4 *)(Ab + (long)(k0 + q / (BM / 4)) * M + m0 + (q % (BM / 4)) * 4);
#else
            s.a[i] = *(const f32x4 *)(Ab + (long)(m0 + q / (BK / 4)) * K + k0 + (q % (BK / 4)) * 4);
#endif
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int q = tid + i * NT;
        if (B_CHUNKS % NT == 0 || q < B_CHUNKS)
            s.b[i] = *(const f32x4 *)(Bb + (long)(k0 + q / (BN / 4)) * N + n0 + (q % (BN / 4)) * 4);
    }
}

__device__ __forceinline__ void store_slab(const Slab &s, float *As, float *Bs, int tid)
{
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int q = tid + i * NT;
#if A_TRANS
        if (A_CHUNKS % NT == 0 || q < A_CHUNKS) *(f32x4 *)(As + (q / (BM / 4)) * LDA + (q % (BM / 4)) * 4) = s.a[i];
#else
        if (A_CHUNKS % NT == 0 || q < A_CHUNKS) *(f32x4 *)(As + (q / (BK / 4)) * LDA + (q % (BK / 4)) * 4) = s.a[i];
#endif
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int q = tid + i * NT;
        if (B_CHUNKS % NT == 0 || q < B_CHUNKS) *(f32x4 *)(Bs + (q / (BN / 4)) * LDB + (q % (BN / 4)) * 4) = s.b[i];
    }
}
#endif

__device__ __forceinline__ void compute_slab(acc_t (&acc)[MI][NI], const float *As, const float *Bs, int wm, int wn, int lane)
{
    const int l32 = lane & 31, half = lane >> 5;
#if FLAG
#pragma unroll
#else
#pragma unroll 1
#endif
    for (int g = 0; g < BKP / 8; ++g) {
        f32x4 af[MI];
#if A_TRANS
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j4 = 0; j4 < 4; ++j4) af[i][j4] = As[(g * 8 + 4 * half + j4) * LDA + wm * TM + i * 32 + l32];
#else
#pragma unroll
        for (int i = 0; i < MI; ++i) af[i] = *(const f32x4 *)(As + (wm * TM + i * 32 + l32) * LDA + g * 8 + 4 * half);
#endif
#pragma unroll
        for (int j4 = 0; j4 < 4; ++j4) {
            float bf[NI];
#pragma unroll
            for (int j = 0; j < NI; ++j) bf[j] = Bs[(g * 8 + 4 * half + j4) * LDB + wn * TN + j * 32 + l32];
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i][j4], bf[j], acc[i][j], 0, 0, 0);
        }
    }
}

extern "C" __global__ __launch_bounds__(NT)
void KERNEL_NAME(const float *__restrict__ A, const float *__restrict__ B, float *__restrict__ C,
                 unsigned long long *ctl /* deadline control: folded members only (the scalar template always honours it) */)
{
    extern __shared__ __attribute__((aligned(16))) float smem_f32[];
    float *As = smem_f32, *Bs = smem_f32 + NSTAGE * A_STAGE;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const BlockId bid = block_id();
#if OP == OP_CONV
    const ColBlock cb = col_block(bid.n);
#define LOAD_SLAB(S, kt) load_slab(S, Ab, Bb, m0, cb, CONV_KBASE(bid) + (kt) * BK, tid)
#else
#define LOAD_SLAB(S, kt) load_slab(S, Ab, Bb, m0, n0, (kt) * BK, tid)
#endif

    // more waves asked for than a workgroup holds: NWR real waves take the tiles of WM * WN / NWR waves each,
    // one after another, each with the whole K loop
#if SUBM * SUBN * NPASS > 1
    // Folded members can run for seconds (few workgroups, many passes): like the scalar template they
    // honour the harness's deadline, checked once per pass by thread 0 and passed on through LDS so
    // that the whole workgroup leaves together.
    __shared__ int expired;
    if (tid == 0) expired = 0;
#endif
    for (int bi = 0; bi < BATCH_INNER; ++bi)
    for (int sub = 0; sub < SUBM * SUBN; ++sub)
    for (int pass = 0; pass < NPASS; ++pass) {
#if SUBM * SUBN * NPASS > 1
        if (tid == 0 && ctl && ctl[1] != 0 && wall_clock64() - ctl[0] > ctl[1]) {
            expired = 1;
            ctl[2] = 1;
        }
        __syncthreads();
        if (expired) return;
#endif
        const int vwave = wave + pass * NWR;
        const int wm = vwave / WN, wn = vwave % WN;
        const int m0 = (bid.m * SUBM + sub / SUBN) * BM;
#if OP != OP_CONV
        const int n0 = (bid.n * SUBN + sub % SUBN) * BN;
#endif
#if OP == OP_CONV
        const float *Ab = A, *Bb = B;   // kernel tensor [M][K], image
#elif KSPLIT > 1   // MatMul, reduction split over grid z: this workgroup owns K range [bid.b * KSTEPS * BK, + KSTEPS * BK)
        const float *Ab = A + (long)bid.b * (KSTEPS * BK);
        const float *Bb = B + (long)bid.b * (KSTEPS * BK) * N;
        float *Cb = C;
#else
        const long batch = (long)bid.b * BATCH_INNER + bi;
        const float *Ab = A + batch * M * K;
        const float *Bb = B + batch * K * N;
        float *Cb = C + batch * M * N;
#endif
        acc_t acc[MI][NI];
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

        Slab slab;
#if NSTAGE == 2
        // every wave has left the previous batch's last slab before the stages are written again
        if (bi > 0 || sub > 0 || pass > 0) __syncthreads();
        LOAD_SLAB(slab, 0);
        store_slab(slab, As, Bs, tid);
        __syncthreads();
        for (int kt = 0; kt < KSTEPS; ++kt) {
            const int cur = kt & 1, nxt = cur ^ 1;
            // slab index clamped past the end: one redundant load instead of a branch around the accumulators
            LOAD_SLAB(slab, (kt + 1 < KSTEPS ? kt + 1 : KSTEPS - 1));
            compute_slab(acc, As + cur * A_STAGE, Bs + cur * B_STAGE, wm, wn, lane);
            store_slab(slab, As + nxt * A_STAGE, Bs + nxt * B_STAGE, tid);
            __syncthreads();
        }
#else
        for (int kt = 0; kt < KSTEPS; ++kt) {
            LOAD_SLAB(slab, kt);
            __syncthreads();
            store_slab(slab, As, Bs, tid);
            __syncthreads();
            compute_slab(acc, As, Bs, wm, wn, lane);
        }
        __syncthreads();
#endif
        // an atom's result sits with column (l % 32) in lane l, register r being row 8*(r/4) + 4*(l/32) + r%4
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = i * 32 + 8 * (r / 4) + 4 * (lane >> 5) + r % 4, col = j * 32 + (lane & 31);
#if OP == OP_CONV
                    // the overhang of a rounded-up wave tile is not stored
                    if ((TM % 32 == 0 || row < TM) && (TN % 32 == 0 || col < TN))
                        c_out(&C[conv_c_index(cb, m0 + wm * TM + row, wn * TN + col)], acc[i][j][r]);
#else
                    c_out(&Cb[(long)(m0 + wm * TM + row) * N + n0 + wn * TN + col], acc[i][j][r]);
#endif
                }
    }
}
