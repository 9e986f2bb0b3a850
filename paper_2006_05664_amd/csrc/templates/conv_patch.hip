// Conv2d kernel template with an LDS-resident image patch (bf16 / fp16 inputs, fp32 accumulation) for gfx950.
//
// The convolution of App. B.3 (Eq. 5 with stride and padding) as an implicit GEMM whose operands stay in
// the layouts the caller hands over (image NCHW, kernel tensor OIHW): no pre-pass, one launch.
// A workgroup owns BM output channels x a box of NB2 images x BH rows x BW pixels, as on the other
// templates; WM x WN waves, wave (wm, wn) owning channels [wm*TM, +TM) and columns [wn*TN, +TN) of the
// flattened box, in ATOM x ATOM MFMA atoms (32x32x16 or 16x16x32).
//
// The reduction is walked in KSTEPS slabs of CS input channels, every slab with all HK*WK taps.  Per slab
// the workgroup holds in LDS
//   * the patch: the input pixels under its box for the slab's channels, channels fastest,
//     P[image][py][px][CS (+8)], PH = (BH-1)*STRIDE + HK rows by PW = (BW-1)*STRIDE + WK columns (row pitch PWP >= PW).  An output
//     pixel (y, x) under tap (r, s) reads patch pixel (y*STRIDE + r, x*STRIDE + s): the 8 channels an MFMA lane
//     wants are 16 contiguous bytes, and the tap is a compile-time offset from the lane's own pixel, so one
//     staged pixel serves all the taps that touch it.  Positions outside the image (padding) are zeros: both
//     stages are cleared once, and the fill only ever writes positions inside the image, whose place in the
//     patch is the same for every slab.
//   * the kernel tensor's part, A[tap][BM][CS] (16-byte chunks permuted by row), so that an A fragment is 16 contiguous bytes too.
// Both parts are transposed on the way in, two channels at a time: a thread loads 4-byte pairs of pixels of two
// channels (rows of the NCHW image are contiguous in x; with WIN even, aligned pairs never straddle a row), or the
// 2*HK*WK contiguous values of two input channels of one output channel, swaps halves in registers and stores
// 4-byte words (one pixel or tap, its two channels).  The padding of 8 elements per patch pixel makes 16 consecutive pixels
// start in 16 different groups of 4 banks, which is what conflict-free 16-byte reads need.
//
// KW > 1: KW waves share every wave tile and split the reduction: of the HK*WK*(CS/KA) MFMA steps of a slab, wave k of the
//           KW takes steps k, k + KW, ...; after the last slab the KW partial sums are added through LDS.  With few
//           output atoms per compute unit (the 14 x 14 convolution: six) this is what lets a large wave tile, whose
//           fragments are read from LDS once per step instead of once per wave, still keep all four SIMDs busy.
// FLAG = 1: two stages; the global loads of slab s+1 are in flight (in registers) while slab s is multiplied,
//           and are written to the other stage afterwards: one barrier per slab.
// FLAG = 0: one stage: load, barrier, store, barrier, multiply.

#if IN_DTYPE == 1
typedef __attribute__((ext_vector_type(8))) __bf16 frag_t;
#define MFMA_32(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0)
#define MFMA_16(a, b, c) __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0)
#else
typedef __attribute__((ext_vector_type(8))) _Float16 frag_t;
#define MFMA_32(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0)
#define MFMA_16(a, b, c) __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0)
#endif

#if ATOM == 32
typedef f32x16 acc_t;
#define KA 16
#define NACC 16
#define MFMA(a, b, c) MFMA_32(a, b, c)
#else
typedef f32x4 acc_t;
#define KA 32
#define NACC 4
#define MFMA(a, b, c) MFMA_16(a, b, c)
#endif

constexpr int T = HK * WK;                                    // taps
constexpr int PH = (BH - 1) * STRIDE + HK, PW = (BW - 1) * STRIDE + WK;
// PWP, IPIX (from the host): row pitch and image pitch of the patch in pixels.  The lanes of an MFMA read consecutive
// output pixels of the flattened box, BW to a row; with unit stride and room in the LDS the host makes the row
// pitch congruent to BW modulo 16 (and the image pitch to BH*BW), so that the patch pixel of output pixel n sits at
// n modulo 16 and any 16 lanes served together start in 16 different groups of banks (PITCH / 8 is odd).
static_assert(PWP >= PW && IPIX >= PH * PWP, "patch pitches too small");
constexpr int NPIX = NB2 * IPIX;
constexpr int PITCH = CS + 8;                                 // elements per patch pixel
// The kernel tensor's part has no padding: a row is CS elements = NCH 16-byte chunks, and chunk c of row r is stored at
// chunk c ^ a_swz(r).  16 consecutive rows read the same chunk c together; without the permutation rows 16 / NCH apart
// would start in the same group of banks, with it they take NCH different chunks.  (The patch cannot do the same: which
// rows are read together depends on the tap, while a stored pixel has one place.)
constexpr int NCH = CS / 8;
// (An exclusive-or stays inside the row only for a power of two of chunks: other slab lengths are stored unpermuted.)
__device__ __forceinline__ int a_swz(int row)
{
    return (NCH & (NCH - 1)) != 0 ? 0 : NCH <= 16 ? (row * NCH / 16) % NCH : row % 16;
}
constexpr int DUMP = 64;                                      // elements at the end of a stage that take the stores of pixels outside the patch
constexpr int P_STAGE = NPIX * PITCH, A_STAGE = T * BM * CS, STAGE = P_STAGE + A_STAGE + DUMP;   // elements
constexpr int MI = TM / ATOM, NI = (TN + ATOM - 1) / ATOM;    // atoms per wave tile (the last column of atoms may hang over)
constexpr int KK = CS / KA;                                   // MFMA steps per tap
#ifndef KW
#define KW 1                                                  // waves that share a wave tile and split the reduction steps of every slab
#endif
constexpr int STEPS = T * KK;                                 // MFMA steps of a slab
constexpr int NWAVES = NT / 64;
static_assert(NWAVES == WM * WN * KW && KW <= STEPS, "decoder and template disagree");
static_assert(TM % ATOM == 0 && CS % KA == 0 && BK == CS * T && KSTEPS * CS == CIN, "decoder and template disagree");
static_assert(NSTG * STAGE * 2 <= 160 * 1024, "stages exceed the LDS");
static_assert(NSTG == (FLAG && KSTEPS > 1 ? 2 : 1), "a pipelined member with more than one slab has two stages, every other member one");

// Patch fill: a task is two channels x an aligned pair of pixels: two 4-byte loads (one per channel), a 2 x 2
// transposition in registers, two 4-byte LDS stores (one per pixel: its two channels).  Across the lanes four
// channel pairs are fastest, then the pairs of pixels along the row, the rows and the images, then the remaining
// channel pairs: 64 lanes load from 4 (or 8) channels, 64 contiguous bytes each, and store 16 pixels x 4 words,
// which fall into different banks but for the stride of two pixels.
// An image of odd width has its rows at any 2-byte offset: the same pairs (even x, odd x) are loaded with 4-byte
// loads that are only 2-byte aligned.  The last pixel of a row has no partner there; its load starts one pixel
// to the left, so that no load reaches beyond the row (the last row ends the tensor), and the words are shifted
// down by one pixel before the transposition (bit 0 of the task's byte offset says so).
// An image one pixel wide: a task is two channels x one pixel, two 2-byte loads and one 4-byte store.
constexpr bool ALIGNED = WIN % 2 == 0;
constexpr bool PAIRED = ALIGNED || WIN >= 3;
typedef u32 __attribute__((aligned(2))) u32_a2;
constexpr int CP = CS / 2;                                    // channel pairs of a slab
constexpr int NPAIR = PAIRED ? PW / 2 + 1 : PW;               // aligned pairs that cover PW columns from either parity (odd width: pixels)
constexpr int PAIRS = NPAIR * PH * NB2;
constexpr int P_TASKS = CP * PAIRS;
static_assert(CP % 4 == 0, "channel pairs are dealt to the lanes four at a time");
constexpr int NPT = (P_TASKS + NT - 1) / NT;
// Kernel-tensor fill: a task is one output channel x two input channels: the 2*T values of the two channels are
// contiguous in the OIHW tensor (T 4-byte loads); tap t of both channels makes one 4-byte LDS store.
constexpr int A_TASKS = BM * CP;
constexpr int NAT = (A_TASKS + NT - 1) / NT;

struct Fill {
    u32 pg[NPT];              // byte offset inside the image tensor of the task's pair of pixels, first channel, slab 0
    u32 pd0[NPT], pd1[NPT];   // 4-byte word in the stage of each of the two pixels (this channel pair); a pixel outside
                              // the patch or the image goes to the dump words at the end of the stage: unconditional stores
    u32 ag[NAT];              // byte offset inside the kernel tensor of the task's 2*T values, slab 0
    u32 ad[NAT];              // 4-byte word in the A part of tap 0 (the taps follow BM rows apart)
};
struct Regs {
    u32 p[NPT][2];
    u32 a[NAT][T];
};

__device__ __forceinline__ void plan_fill(Fill &f, const ColBlock &cb, int m0, int tid)
{
    const int yin0 = cb.y0 * STRIDE - PAD_CONV, xin0 = cb.x0 * STRIDE - PAD_CONV;
    const int xs = xin0 & ~1;                                 // first aligned pair at or left of the patch
#pragma unroll
    for (int i = 0; i < NPT; ++i) {
        const int q = tid + i * NT;
        const int pr = (q / 4) % PAIRS, cp = q / (4 * PAIRS) * 4 + q % 4;
        const int jp = pr % NPAIR, py = (pr / NPAIR) % PH, b = pr / (NPAIR * PH);
        const int y = yin0 + py, x = PAIRED ? xs + 2 * jp : xin0 + jp, px = x - xin0;   // px: patch column of the task's first pixel (-1 .. PW)
        const bool in = (P_TASKS % NT == 0 || q < P_TASKS) && y >= 0 && y < HIN && x >= 0 && x < WIN;
        const bool v0 = in && px >= 0 && px < PW, v1 = PAIRED && in && px + 1 >= 0 && px + 1 < PW && (ALIGNED || x + 1 < WIN);
        const int left = (PAIRED && !ALIGNED && x == WIN - 1) ? 1 : 0;
        const int d0 = ((b * IPIX + py * PWP + px) * PITCH) / 2 + cp, dump = (STAGE - DUMP) / 2 + (tid & 31);
        f.pg[i] = (v0 || v1) ? (2u * (u32)((((cb.nb0 + b) * CIN + 2 * cp) * HIN + y) * WIN + x - left) | (u32)left) : 0u;
        f.pd0[i] = (u32)(v0 ? d0 : dump);
        f.pd1[i] = (u32)(v1 ? d0 + PITCH / 2 : dump);
    }
#pragma unroll
    for (int i = 0; i < NAT; ++i) {
        const int q = tid + i * NT;
        const int cp = q % CP, m = q / CP;
        const bool on = A_TASKS % NT == 0 || q < A_TASKS;
        f.ag[i] = on ? 2u * (u32)((m0 + m) * K + 2 * cp * T) : 0u;
        f.ad[i] = on ? (u32)(m * (CS / 2) + (((cp >> 2) ^ a_swz(m)) << 2) + (cp & 3)) : ~0u;   // BM is a multiple of 16: the tap does not change the permutation
    }
}

// global loads of slab s into registers (unconditional: a task with nothing to do reads the slab's first bytes)
__device__ __forceinline__ void load_slab(Regs &r, const Fill &f, const u16 *__restrict__ A, const u16 *__restrict__ B, int s)
{
    const char *Bs = (const char *)(B + (long)s * CS * HIN * WIN);
    const char *As = (const char *)(A + (long)s * CS * T);
#pragma unroll
    for (int i = 0; i < NPT; ++i) {   // the second load is the next channel (offset 0 for an idle task: still inside the tensor)
        if constexpr (ALIGNED) {
            r.p[i][0] = *(const u32 *)(Bs + f.pg[i]);
            r.p[i][1] = *(const u32 *)(Bs + f.pg[i] + 2 * HIN * WIN);
        } else if constexpr (PAIRED) {
            const u32 o = f.pg[i] & ~1u;
            r.p[i][0] = *(const u32_a2 *)(Bs + o);
            r.p[i][1] = *(const u32_a2 *)(Bs + o + 2 * HIN * WIN);
        } else {
            r.p[i][0] = *(const u16 *)(Bs + f.pg[i]);
            r.p[i][1] = *(const u16 *)(Bs + f.pg[i] + 2 * HIN * WIN);
        }
    }
#pragma unroll
    for (int i = 0; i < NAT; ++i)
#pragma unroll
        for (int t = 0; t < T; ++t) r.a[i][t] = *(const u32 *)(As + f.ag[i] + 4 * t);
}

// S = the stage as 4-byte words (the patch part is first, the kernel-tensor part follows)
__device__ __forceinline__ void store_slab(const Regs &r, const Fill &f, u32 *S)
{
#pragma unroll
    for (int i = 0; i < NPT; ++i) {
        u32 p0 = r.p[i][0], p1 = r.p[i][1];
        if constexpr (PAIRED && !ALIGNED) {
            const u32 sh = (f.pg[i] & 1u) << 4;                   // a pair loaded one pixel to the left: the pixel wanted is the upper one
            p0 >>= sh;
            p1 >>= sh;
        }
        S[f.pd0[i]] = (p0 & 0xffffu) | (p1 << 16);                // first pixel: its two channels
        if constexpr (PAIRED) S[f.pd1[i]] = (p0 >> 16) | (p1 & 0xffff0000u);      // second pixel
    }
    u32 *SA = S + P_STAGE / 2;
#pragma unroll
    for (int i = 0; i < NAT; ++i) {
        if (A_TASKS % NT != 0 && f.ad[i] == ~0u) continue;
#pragma unroll
        for (int t = 0; t < T; ++t) {
            // value t of the run is tap t of the first channel, value T + t tap t of the second
            const u32 lo = r.a[i][t / 2], hi = r.a[i][(T + t) / 2];
            const u32 l16 = (t % 2) ? (lo >> 16) : (lo & 0xffffu);
            const u32 h16 = ((T + t) % 2) ? (hi & 0xffff0000u) : (hi << 16);
            SA[f.ad[i] + t * (BM * CS / 2)] = l16 | h16;
        }
    }
}

// a lane's place in the A part: its row of the wave tile's first atom (element offset), which 16-byte chunk of a K step it
// supplies, and its row's chunk permutation
struct ALane { int row, chunk, perm; };

// fragments of step (tap, kk): MI rows of atoms from the A part, NI columns of atoms from the patch
__device__ __forceinline__ void load_frags(frag_t (&af)[MI], frag_t (&bf)[NI], const u16 *As, const u16 *P,
                                           const ALane &al, const int (&b_lane)[NI], int tap, int kk)
{
    const int r = tap / WK, s = tap % WK;
    const int a_row = al.row, a_chunk = al.chunk, a_perm = al.perm;
#pragma unroll
    for (int i = 0; i < MI; ++i)
        af[i] = __builtin_bit_cast(frag_t, *(const u32x4 *)(As + a_row + (((kk * (KA / 8) + a_chunk) ^ a_perm) << 3) + (tap * BM + i * ATOM) * CS));
#pragma unroll
    for (int j = 0; j < NI; ++j)
        bf[j] = __builtin_bit_cast(frag_t, *(const u32x4 *)(P + b_lane[j] + (r * PWP + s) * PITCH + kk * KA));
}

// The MFMA steps WI, WI + KW, ... of a slab, fully unrolled; the fragments of step u + FRAG_AHEAD are read before the
// MFMAs of step u are issued (a ring of FRAG_AHEAD + 1 sets of fragment registers).
// Small wave tiles have too few MFMAs per step to cover the LDS latency of the next step's fragments: they read two steps
// ahead (measured on the 14 x 14 convolution: 5 - 9 % for one-atom tiles, 1.6 % for two atoms, nothing beyond).
#ifndef FRAG_AHEAD
#define FRAG_AHEAD ((TM / ATOM) + (TN + ATOM - 1) / ATOM <= 3 ? 2 : 1)
#endif
template <int WI>
__device__ __forceinline__ void compute_steps(acc_t (&acc)[MI][NI], const u16 *As, const u16 *P, const ALane &al, const int (&b_lane)[NI])
{
    constexpr int NS = (STEPS - WI + KW - 1) / KW;
    constexpr int RING = FRAG_AHEAD + 1;
    frag_t af[RING][MI], bf[RING][NI];
#pragma unroll
    for (int u = 0; u < FRAG_AHEAD && u < NS; ++u) {
        const int t = WI + u * KW;
        load_frags(af[u], bf[u], As, P, al, b_lane, t / KK, t % KK);
    }
#pragma unroll
    for (int u = 0; u < NS; ++u) {
        const int t = WI + (u + FRAG_AHEAD) * KW;
        if (u + FRAG_AHEAD < NS) load_frags(af[(u + FRAG_AHEAD) % RING], bf[(u + FRAG_AHEAD) % RING], As, P, al, b_lane, t / KK, t % KK);
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j) acc[i][j] = MFMA(af[u % RING][i], bf[u % RING][j], acc[i][j]);
        __builtin_amdgcn_sched_barrier(0);             // no more sets of fragments alive than the ring has
    }
}
template <int WI>
__device__ __forceinline__ void compute_for_wave(int wk, acc_t (&acc)[MI][NI], const u16 *As, const u16 *P, const ALane &al, const int (&b_lane)[NI])
{
    if constexpr (WI + 1 < KW) {
        if (wk == WI) compute_steps<WI>(acc, As, P, al, b_lane);
        else compute_for_wave<WI + 1>(wk, acc, As, P, al, b_lane);
    } else {
        compute_steps<WI>(acc, As, P, al, b_lane);
    }
}

// wk: which of the KW waves of its tile this wave is (wave-uniform)
__device__ __forceinline__ void compute_slab(acc_t (&acc)[MI][NI], const u16 *As, const u16 *P, const ALane &al, const int (&b_lane)[NI], int wk)
{
    if constexpr (STEPS * (MI * NI + MI + NI) <= 512) {
        compute_for_wave<0>(wk, acc, As, P, al, b_lane);
    } else {
        // long slabs (many taps): the loop over the steps stays a loop
#pragma unroll 1
        for (int t = wk; t < STEPS; t += KW) {
            const int tap = t / KK, kk = t % KK;
            frag_t af[MI], bf[NI];
            load_frags(af, bf, As, P, al, b_lane, tap, kk);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j) acc[i][j] = MFMA(af[i], bf[j], acc[i][j]);
        }
    }
}

extern "C" __global__ __launch_bounds__(NT)
void KERNEL_NAME(const u16 *__restrict__ A, const u16 *__restrict__ B, float *__restrict__ C,
                  unsigned long long *ctl /* unused: members of this template are never folded */)
{
    extern __shared__ __attribute__((aligned(16))) u16 smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lrow = lane % ATOM, lk = (lane / ATOM) * 8;
    const BlockId bid = block_id();
    const ColBlock cb = col_block(bid.n);
    const int wk = __builtin_amdgcn_readfirstlane(wave / (WM * WN));   // the wave's part of the reduction steps
    const int wmn = wave % (WM * WN), wm = wmn / WN, wn = wmn % WN;
    const int m0 = bid.m * BM;

    Fill fill;
    plan_fill(fill, cb, m0, tid);
    Regs regs;
#if FLAG
    load_slab(regs, fill, A, B, 0);
#endif
    // (pipelined members: while the first slab is on its way) zeros in the patch part of every stage: the patch positions
    // that lie outside the image are never written again
    {
        const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int st = 0; st < NSTG; ++st)
            for (int i = tid; i < P_STAGE / 8; i += NT) ((u32x4 *)(smem + st * STAGE))[i] = zero;
    }

    // this lane's place in the fragments: its row of the A part, and per column of atoms its output pixel's
    // patch pixel under tap (0, 0) (columns past the wave tile read the tile's last pixel and are not stored)
    // (whole atoms of 16 or 32 rows lie between a lane's rows: they all have this row's permutation)
    const ALane al = {(wm * TM + lrow) * CS, lane / ATOM, a_swz(lrow)};
    int b_lane[NI];
#pragma unroll
    for (int j = 0; j < NI; ++j) {
        const int ct = j * ATOM + lrow;
        const int cn = wn * TN + (ct < TN ? ct : TN - 1);
        const int b = cn / (BH * BW), y = (cn / BW) % BH, x = cn % BW;
        b_lane[j] = (b * IPIX + y * STRIDE * PWP + x * STRIDE) * PITCH + lk;
    }

    acc_t acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < NACC; ++r) acc[i][j][r] = 0.f;

#if FLAG
    // Two stages: while slab s is multiplied the loads of slab s+1 are in flight; they are written to the other stage
    // afterwards (one barrier per slab).  Branch-free body (the loads must not sink below the MFMAs): past the last slab
    // the last one is loaded and stored once more, into the stage nobody reads any longer.  (Loading two slabs ahead
    // into a second register set was measured: no faster, and the registers cost members their place on this template.)
    __syncthreads();                                   // the zeros are in place
    store_slab(regs, fill, (u32 *)smem);
    __syncthreads();
#pragma unroll 1
    for (int s = 0; s < KSTEPS; ++s) {
        u16 *cur = smem + (s & 1) * STAGE, *nxt = smem + (NSTG == 2 ? (s + 1) & 1 : 0) * STAGE;
        load_slab(regs, fill, A, B, s + 1 < KSTEPS ? s + 1 : KSTEPS - 1);
        __builtin_amdgcn_sched_barrier(0);             // all loads are issued before the first MFMA ...
        compute_slab(acc, cur + P_STAGE, cur, al, b_lane, wk);
        __builtin_amdgcn_sched_barrier(0);             // ... and the stores follow the last
        if (NSTG == 2) store_slab(regs, fill, (u32 *)nxt);
        __syncthreads();
    }
#else
#pragma unroll 1
    for (int s = 0; s < KSTEPS; ++s) {
        load_slab(regs, fill, A, B, s);
        __syncthreads();                               // slab s-1 has been multiplied (first pass: the zeros are in place)
        store_slab(regs, fill, (u32 *)smem);
        __syncthreads();
        compute_slab(acc, smem + P_STAGE, smem, al, b_lane, wk);
    }
#endif

    // Epilogue.  An atom's result sits with column (l % ATOM) in lane l; 32x32: register r is row
    // 8*(r/4) + 4*(l/32) + r%4; 16x16: register r is row 4*(l/16) + r.
#if KW == 1
#pragma unroll
    for (int i = 0; i < MI; ++i) {
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int ct = j * ATOM + lrow;
            if (TN % ATOM != 0 && ct >= TN) continue;
            const int cn = wn * TN + ct;
#pragma unroll
            for (int r = 0; r < NACC; ++r) {
                const int row = (ATOM == 32) ? 8 * (r / 4) + 4 * (lane / 32) + r % 4 : 4 * (lane / 16) + r;
                const int gm = m0 + wm * TM + i * ATOM + row;
                C[conv_c_index(cb, gm, cn)] = acc[i][j][r];
            }
        }
    }
#else
    // The KW waves of a tile hold partial sums.  In passes of APP atoms (as many as the LDS holds for all waves), every
    // wave writes its accumulators of the pass's atoms to LDS, R[atom][wave][4 registers][lane]; then wave k of a tile adds,
    // in the order of the waves, the KW partial sums of the atoms k, k + KW, ... of the pass and stores them.
    constexpr int ATOMS = MI * NI, Q = NACC / 4;
    constexpr int APP_FIT = LDS_BYTES / (NWAVES * Q * 1024);
    constexpr int APP = APP_FIT < ATOMS ? APP_FIT : ATOMS;
    static_assert(APP >= 1, "the LDS cannot hold one atom of every wave");
    f32x4 *R = (f32x4 *)smem;
#pragma unroll
    for (int a0 = 0; a0 < ATOMS; a0 += APP) {
        __syncthreads();                               // the stages (or the previous pass) are no longer read
#pragma unroll
        for (int a = a0; a < a0 + APP && a < ATOMS; ++a)
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                const acc_t &v = acc[a / NI][a % NI];
                const f32x4 w = {v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]};
                R[(((a - a0) * NWAVES + wave) * Q + q) * 64 + lane] = w;
            }
        __syncthreads();
#pragma unroll 1
        for (int a = a0 + wk; a < a0 + APP && a < ATOMS; a += KW) {
            const int i = a / NI, j = a % NI;
            const int ct = j * ATOM + lrow;
            const int cn = wn * TN + (ct < TN ? ct : TN - 1);
            const long c0 = conv_c_index(cb, m0 + wm * TM + i * ATOM, cn);   // row 0 of the atom; a row is HOUT*WOUT further
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                f32x4 sum = R[(((a - a0) * NWAVES + wmn) * Q + q) * 64 + lane];
#pragma unroll
                for (int k = 1; k < KW; ++k) {
                    const f32x4 v = R[(((a - a0) * NWAVES + k * (WM * WN) + wmn) * Q + q) * 64 + lane];
                    sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
                }
                if (TN % ATOM == 0 || ct < TN) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int r = 4 * q + e;
                        const int row = (ATOM == 32) ? 8 * (r / 4) + 4 * (lane / 32) + r % 4 : 4 * (lane / 16) + r;
                        C[c0 + (long)row * (HOUT * WOUT)] = sum[e];
                    }
                }
            }
        }
    }
#endif
}
