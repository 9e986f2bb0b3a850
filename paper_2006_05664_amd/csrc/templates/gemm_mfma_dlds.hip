// MFMA kernel template with operands streamed global memory -> LDS directly (gfx950), for
// MatMul / BatchMatMul members whose tile shapes allow it (the host's decoder decides).
//
// Roles of the tiling factors are those of the register-staged MFMA template: workgroup tile
// BM x BN, WM x WN waves, per-wave tile TM x TN of 32x32x16 atoms, K consumed in KSTEPS slabs of
// BK.  What differs is how a slab travels and how the instruction stream is laid out:
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
//  * One MFMA step (all atoms of the wave tile for 16 k; for wave tiles of one or two atoms a group
//    of several such steps) uses one of two fragment buffer sets;
//    between its MFMAs the wave issues, one or two at a time, the LDS reads of the next step's
//    fragments (across slab boundaries too) and, in the last step of a slab, the loads that
//    refill the stage.  The order is pinned with scheduling barriers: every LDS read and every
//    load issue sits in the shadow of an MFMA, so a single wave per SIMD can keep its matrix
//    pipe busy, which in turn allows 128 x 128 wave tiles, the shape with the least LDS traffic
//    per flop (LDS bandwidth, not the matrix pipe, limits smaller wave tiles).
//  * The waits are explicit: s_waitcnt vmcnt(n) with n = the loads this wave issued after the
//    slab it needs, then a bare s_barrier (the fence of __syncthreads() would drain every
//    outstanding load).
//  * C is written with non-temporal stores: it is never read again.
//  * B_KMAJOR: the second operand arrives with the reduction index contiguous, [N][K] like the
//    first: either a MatMul whose B a pre-pass transposed, or a Conv2d whose image and kernel
//    tensor a pre-pass rewrote channels-last (CONV_NHWC: the reduction is walked as (r, s, ci), Cin
//    a multiple of 8, so the 8 values of a 16-byte piece are 8 channels of one tap of one pixel).
//    Its stage part is then [BNR][BK], laid out, permuted and read exactly like A's (one 16-byte
//    LDS read per fragment, no transposing reads).  For Conv2d a row is an output pixel of the
//    workgroup's box: every lane computes the byte offset of its piece (pixel, tap, channel group)
//    itself, and pieces that fall outside the image (padding) or past the box's last pixel (the
//    rows that round the part up to whole wave loads) are read from a block of zeros that
//    precedes the image in the workspace.  A wave tile may be ragged along N (TN no multiple of
//    32): the overhang is computed and not stored.

// ATOM: 32 = 32x32x16 MFMAs (16 accumulators per lane and atom), 16 = 16x16x32 MFMAs (4 accumulators: half the
// flops per instruction, but a 32-deep dot product per accumulator update; under the chip's power limit the matrix
// pipes sustain more flops per second on changing operands with these).  Lane l holds, for atom row or column
// l % ATOM, the 8 reduction values from 8 * (l / ATOM) of a KA-wide step.
#if IN_DTYPE == 1
typedef __attribute__((ext_vector_type(8))) __bf16 frag_t;
#if ATOM == 16
#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0)
#else
#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0)
#endif
#else
typedef __attribute__((ext_vector_type(8))) _Float16 frag_t;
#if ATOM == 16
#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0)
#else
#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0)
#endif
#endif
typedef __attribute__((ext_vector_type(4))) short v4s;
typedef __attribute__((ext_vector_type(8))) short v8s;
#if ATOM == 16
typedef __attribute__((ext_vector_type(4))) float acc_t;
#else
typedef f32x16 acc_t;
#endif
constexpr int ACC_N = ATOM == 16 ? 4 : 16;      // accumulators per lane and atom
constexpr int KA = ATOM == 16 ? 32 : 16;        // reduction values one MFMA consumes

#ifndef B_KMAJOR
#define B_KMAJOR 0
#endif
#ifndef CONV_NHWC
#define CONV_NHWC 0
#endif
#if B_KMAJOR && A_TRANS
#error "a K-contiguous second operand is not combined with a transposed first one"
#endif
#if OP == OP_CONV && !(B_KMAJOR && CONV_NHWC)
#error "Conv2d runs on this template with channels-last operands only"
#endif
constexpr int NW = NT / 64;
constexpr int MI = TM / ATOM, NI = (TN + ATOM - 1) / ATOM;
constexpr int KK = BK / KA;                                   // MFMA K steps per slab
#if ATOM == 16 && (A_TRANS || OP == OP_CONV || B_KMAJOR)
#error "16x16x32 atoms: MatMul / BatchMatMul with row-major operands as stored only"
#endif
#if B_KMAJOR
constexpr int B_STAGE = BNR * BK;   // BNR rows of BK: the BN columns of the tile, rounded up to whole wave loads
#else
constexpr int B_STAGE = BK * BN;
#endif
#ifndef ANR
#define ANR BM   // rows of A's stage part: BM, or BM rounded up to whole wave loads (the extra rows repeat row BM-1 and are never read)
#endif
constexpr bool A_PADDED = ANR != BM;
constexpr int A_STAGE = ANR * BK, STAGE = A_STAGE + B_STAGE;   // elements
#if A_TRANS   // first operand stored [K][M]: its stage part is [BK][BM], laid out and read like B's
constexpr int ACH = BM / 8;                                   // 16-byte chunks per A row (a row is one k)
constexpr int A_RPW = (16 / ACH) > 0 ? (16 / ACH) : 1;
constexpr int A_SWM = (4 / A_RPW) > 0 ? (4 / A_RPW) : 1;
#else
constexpr int ACH = BK / 8;                                   // 16-byte chunks per A row
constexpr int A_RPW = (16 / ACH) > 0 ? (16 / ACH) : 1;        // A rows per 256-byte bank window
#endif
constexpr int BCH = B_KMAJOR ? 1 : BN / 8;                    // chunks per B row (B stored [K][N])
constexpr int B_RPW = (16 / BCH) > 0 ? (16 / BCH) : 1;
constexpr int B_SWM = (4 / B_RPW) > 0 ? (4 / B_RPW) : 1;
constexpr int LA = A_STAGE * 2 / 1024 / NW, LB = B_STAGE * 2 / 1024 / NW;   // loads per wave and slab
constexpr int PER = LA + LB;

#if A_TRANS
__device__ __forceinline__ int a_swz(int krow) { return ((krow / A_RPW) % A_SWM) << 2; }
#elif ATOM == 16
// 16-row atoms: lanes 0-15 read 16 rows at one chunk, lanes 16-31 the same rows at the next chunk, and so on.
// A 16-byte LDS read is served in four turns of 16 lanes; the first takes lanes 0-3, 12-15, 20-23 and 24-27, the
// second the other lanes below 32, the last two the same lanes plus 32 (the grouping that explains the bank
// conflict counts measured for the 32-row pattern, none, and for this pattern under the 32-row permutation and
// under a first attempt, two-way each).  The permutations below put the 16 lanes of every turn on 16 different
// 16-byte bank groups for every K step (found by enumerating the linear maps from the row's low four bits).
__device__ __forceinline__ int a_swz(int row)
{
    const int b1 = (row >> 1) & 1, b2 = (row >> 2) & 1, b3 = (row >> 3) & 1;
    return ACH == 4 ? (b3 << 1) : ACH == 8 ? (b1 | (b2 << 1) | (b3 << 2)) : (row & 15);
}
#else
__device__ __forceinline__ int a_swz(int row) { return (row / A_RPW) % ACH; }
#endif
#if ATOM == 16 && !B_KMAJOR
// with 16-column atoms the two 16-lane groups that read B together sit 8 k rows apart on the same columns:
// rows whose bit 3 differs are moved 32 bytes apart as well
__device__ __forceinline__ int b_swz(int krow) { return (((krow / B_RPW) % B_SWM) << 2) ^ (((krow >> 3) & 1) << 1); }
#else
__device__ __forceinline__ int b_swz(int krow) { return ((krow / B_RPW) % B_SWM) << 2; }
#endif

// One wave-wide 16-byte-per-lane load whose destination is LDS: lane i's 16 bytes, read from
// base + off (base wave-uniform, off per lane), land at lds_base + 16 * i (lds_base wave-uniform,
// passed in M0).  It is written as inline assembly so that the compiler's own wait-count
// bookkeeping never sees these loads: whenever it loses track of which LDS object such a load
// fills, it guards later LDS reads with a wait for ALL outstanding loads, which would cut the
// ring down to a single slab in flight.  The kernel places every wait these loads need itself
// (WAIT_VMCNT below).
__device__ __forceinline__ void dma16(const u16 *base, unsigned off, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base), "s"(lds_base) : "memory", "m0");
}

// The 1 KiB piece number `instr` of a stage's A part covers the 16-byte positions
// p = instr * 64 + lane: row p / ACH, chunk position p % ACH, which holds global chunk
// (p % ACH) ^ a_swz(row).  Split into a wave-uniform part (first row of the piece) and a per-lane
// byte offset that repeats every PA pieces, so a wave keeps min(LA, PA) offsets in registers.
constexpr int lane_period(int per_row, int swz_rows)
{
    int p = 1;
    while ((p * 64) % per_row != 0 || (p * 64 / per_row) % swz_rows != 0) ++p;
    return p;
}
#if A_TRANS
constexpr int PA = lane_period(ACH, A_RPW * A_SWM), PB = lane_period(BCH, B_RPW * B_SWM);
#elif B_KMAJOR
constexpr int PA = lane_period(ACH, A_RPW * ACH), PB = PA;
#elif ATOM == 16
constexpr int PA = lane_period(ACH, 16), PB = lane_period(BCH, 16);   // both permutations repeat every 16 rows   // B's permutation repeats every 16 k rows
#else
constexpr int PA = lane_period(ACH, A_RPW * ACH), PB = lane_period(BCH, B_RPW * B_SWM);
#endif
constexpr int NA = (A_PADDED || LA < PA) ? LA : PA, NB = LB < PB ? LB : PB;

__device__ __forceinline__ unsigned a_lane_off(int instr, int lane)
{
    const int p = instr * 64 + lane, row0 = instr * 64 / ACH, row = p / ACH;
#if A_TRANS
    return (unsigned)((row - row0) * M + (((p % ACH) ^ a_swz(row)) << 3)) * 2u;
#else
    // rows past BM (a padded part) repeat row BM-1: in bounds, never read back
    const int rc = (A_PADDED && row > BM - 1) ? BM - 1 : row, r0c = (A_PADDED && row0 > BM - 1) ? BM - 1 : row0;
    return (unsigned)((rc - r0c) * K + (((p % ACH) ^ a_swz(row)) << 3)) * 2u;
#endif
}
#if B_KMAJOR
__device__ __forceinline__ unsigned b_lane_off(int instr, int lane)   // rows of K elements, like A's
{
    const int p = instr * 64 + lane, row0 = instr * 64 / ACH, row = p / ACH;
    return (unsigned)((row - row0) * K + (((p % ACH) ^ a_swz(row)) << 3)) * 2u;
}
#else
__device__ __forceinline__ unsigned b_lane_off(int instr, int lane)
{
    const int p = instr * 64 + lane, krow0 = instr * 64 / BCH, krow = p / BCH;
    return (unsigned)((krow - krow0) * N + (((p % BCH) ^ b_swz(krow)) << 3)) * 2u;
}
#endif
#if OP == OP_CONV
// What a lane needs to know about the pixel whose piece it loads (piece u of its wave's share of the
// B part, the same pixel in every slab), in two registers: base2 = byte offset, from the block of
// zeros that precedes the channels-last image, of channel 0 of the input pixel under tap (0, 0)
// (kept modulo 2^32: that pixel lies outside the image for padded borders), and yx = its
// coordinates as two wrapping 16-bit fields (x low, y high; a negative coordinate wraps to a large
// field).  A row past the box's last pixel gets y = 0x8000, which no tap brings back into the image.
// Which 8 reduction positions of a slab the piece holds (k8) follows from the lane alone; where a
// slab lies inside one tap (CIN % BK == 0) it is folded into base2.
constexpr unsigned ZERO_BLOCK = 256;   // bytes of zeros in front of the image
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
struct PixelPiece { unsigned base2, yx; };
__device__ __forceinline__ int piece_k8(int instr, int lane)
{
    const int p = instr * 64 + lane;
    return ((p % ACH) ^ a_swz(p / ACH)) << 3;
}
__device__ __forceinline__ PixelPiece pixel_piece(const ColBlock &cb, int instr, int lane)
{
    const int p = instr * 64 + lane, c = p / ACH;
    PixelPiece pp;
    const int cc = c < BN ? c : 0;
    const int nb = cb.nb0 + cc / (BH * BW);
    const int y0 = (cb.y0 + (cc / BW) % BH) * STRIDE - PAD_CONV;
    const int x0 = (cb.x0 + cc % BW) * STRIDE - PAD_CONV;
    pp.base2 = ZERO_BLOCK + 2u * (unsigned)(((nb * HIN + y0) * WIN + x0) * CIN);
#if CIN % BK == 0
    pp.base2 += 2u * (unsigned)piece_k8(instr, lane);
#endif
    pp.yx = ((c < BN ? (unsigned)y0 : 0x8000u) << 16) | ((unsigned)x0 & 0xFFFFu);
    return pp;
}
// does tap (r, sx) of the pixel fall inside the image?
__device__ __forceinline__ bool tap_inside(unsigned yx, int r, int sx)
{
    const u16x2 at = __builtin_bit_cast(u16x2, yx) + __builtin_bit_cast(u16x2, ((unsigned)r << 16) | (unsigned)sx);
    const u16x2 lim = {(unsigned short)(WIN - 1), (unsigned short)(HIN - 1)};   // element 0 = low half = x
    return __builtin_bit_cast(unsigned, __builtin_elementwise_min(at, lim)) == __builtin_bit_cast(unsigned, at);
}
#endif

// stage: LDS byte address of the stage to fill; slot: which share of the slab this wave issues
// (wave-uniform, in a scalar register); aoff / boff: a_lane_off / b_lane_off of the wave's pieces.
// piece t (0 .. PER-1) of this wave's share of a slab: the A pieces first, then the B pieces
#if OP == OP_CONV
#define BOFF_T PixelPiece
#define NBOFF LB
#else
#define BOFF_T unsigned
#define NBOFF NB
#endif
__device__ __forceinline__ void issue_piece(int t, const u16 *__restrict__ Ab, const u16 *__restrict__ Bb, unsigned stage,
                                            int m0, int n0, int k0, int slot, const unsigned (&aoff)[NA],
                                            const BOFF_T (&boff)[NBOFF])
{
    if (t < LA) {
        const int instr = slot * LA + t;
#if A_TRANS
        dma16(Ab + (long)(k0 + instr * 64 / ACH) * M + m0, aoff[t % PA], stage + instr * 1024);
#else
        const int row0 = instr * 64 / ACH;
        dma16(Ab + (long)(m0 + ((A_PADDED && row0 > BM - 1) ? BM - 1 : row0)) * K + k0, aoff[A_PADDED ? t : t % PA], stage + instr * 1024);
#endif
    } else {
        const int u = t - LA, instr = slot * LB + u;
#if OP == OP_CONV
        const PixelPiece &pp = boff[u];
#if CIN % BK == 0
        // a slab lies inside one tap: the tap and its offset are the same for every lane (scalar
        // arithmetic on the slab's first position k0); the lane's 8-channel group is already in base2
        const int tap = k0 / CIN, r = tap / WK, sx = tap % WK;
        const unsigned in_off = pp.base2 + 2u * (unsigned)((r * WIN + sx) * CIN + k0 % CIN);
#else
        const int kp = k0 + piece_k8(instr, threadIdx.x & 63);   // position in the (r, s, ci) walk
        const int tap = kp / CIN, ci0 = kp % CIN, r = tap / WK, sx = tap % WK;
        const unsigned in_off = pp.base2 + 2u * (unsigned)((r * WIN + sx) * CIN + ci0);
#endif
        const bool ok = tap_inside(pp.yx, r, sx);
        dma16(Bb, ok ? in_off : 0u, stage + (A_STAGE + instr * 512) * 2);
#elif B_KMAJOR
        dma16(Bb + (long)(n0 + instr * 64 / ACH) * K + k0, boff[u % PB], stage + (A_STAGE + instr * 512) * 2);
#else
        dma16(Bb + (long)(k0 + instr * 64 / BCH) * N + n0, boff[u % PB], stage + (A_STAGE + instr * 512) * 2);
#endif
    }
}
__device__ __forceinline__ frag_t read_a(const u16 *stage, int wm, int lane, int kk, int i)
{
    const int row = wm * TM + i * ATOM + (lane % ATOM);
    const int kc = kk * (KA / 8) + lane / ATOM;
    return __builtin_bit_cast(frag_t, *(const u32x4 *)(stage + row * BK + ((kc ^ a_swz(row)) << 3)));
}
#if A_TRANS
// half an A fragment from the [BK][BM] stage part, with the transposing read (as for B)
__device__ __forceinline__ v4s read_a_half(const u16 *stage, int wm, int lane, int kk, int i, int r)
{
    const int s = lane & 15;
    const int m = wm * TM + i * 32 + 16 * ((lane >> 4) & 1) + 4 * (s & 3);
    const int krow = kk * 16 + 8 * (lane >> 5) + 4 * r + (s >> 2);
    const u16 *p = stage + krow * BM + (((m >> 3) ^ a_swz(krow)) << 3) + (m & 7);
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s *)p);
}
#endif
#if B_KMAJOR
__device__ __forceinline__ frag_t read_bk(const u16 *stage, int wn, int lane, int kk, int j)
{
    const int row = wn * TN + j * ATOM + (lane % ATOM);
    const int kc = kk * (KA / 8) + lane / ATOM;
    return __builtin_bit_cast(frag_t, *(const u32x4 *)(stage + A_STAGE + row * BK + ((kc ^ a_swz(row)) << 3)));
}
#endif
__device__ __forceinline__ v4s read_b_half(const u16 *stage, int wn, int lane, int kk, int j, int r)
{
    const int s = lane & 15;
#if ATOM == 16
    const int n = wn * TN + j * 16 + 4 * (s & 3);
    const int krow = kk * 32 + 8 * (lane >> 4) + 4 * r + (s >> 2);
#else
    const int n = wn * TN + j * 32 + 16 * ((lane >> 4) & 1) + 4 * (s & 3);
    const int krow = kk * 16 + 8 * (lane >> 5) + 4 * r + (s >> 2);
#endif
    const u16 *p = stage + A_STAGE + krow * BN + (((n >> 3) ^ b_swz(krow)) << 3) + (n & 7);
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s *)p);
}

// s_waitcnt vmcnt(n) alone (expcnt and lgkmcnt left at their maxima), gfx9 encoding
#define VMC(n) ((n) < 63 ? (n) : 63)
#define WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt((VMC(n) & 0xf) | ((VMC(n) >> 4) << 14) | (0x7 << 4) | (0xf << 8))
#define WAIT_LGKM_VMCNT(n) __builtin_amdgcn_s_waitcnt((VMC(n) & 0xf) | ((VMC(n) >> 4) << 14) | (0x7 << 4) | (0x0 << 8))
#define WAIT_LGKM() __builtin_amdgcn_s_waitcnt(0xf | (0x3 << 14) | (0x7 << 4) | (0x0 << 8))
#define BARRIER() do { asm volatile("" ::: "memory"); __builtin_amdgcn_s_barrier(); asm volatile("" ::: "memory"); } while (0)
#define KCLAMP(k) ((k) < KSTEPS ? (k) : KSTEPS - 1)

extern "C" __global__ __launch_bounds__(NT)
void KERNEL_NAME(const u16 *__restrict__ A, const u16 *__restrict__ B, float *__restrict__ C,
                 unsigned long long *ctl /* deadline control, used by the scalar template only */)
{
    __shared__ __attribute__((aligned(1024))) u16 ring[NSTG * STAGE];
    const unsigned ring_addr = __builtin_amdgcn_readfirstlane((unsigned)(unsigned long)(__attribute__((address_space(3))) u16 *)ring);   // LDS byte address
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const BlockId bid = block_id();
    const int m0 = bid.m * BM, n0 = bid.n * BN;
    const int uwave = __builtin_amdgcn_readfirstlane(wave);
    const int slot = uwave;
    unsigned aoff[NA];
#pragma unroll
    for (int t = 0; t < NA; ++t) aoff[t] = a_lane_off(slot * LA + t, lane);
#if OP == OP_CONV
    const ColBlock cb = col_block(bid.n);
    PixelPiece boff[LB];
#pragma unroll
    for (int t = 0; t < LB; ++t) boff[t] = pixel_piece(cb, slot * LB + t, lane);
    const int kbase = CONV_KBASE(bid);   // first reduction position of this workgroup's partition
#else
    unsigned boff[NB];
#pragma unroll
    for (int t = 0; t < NB; ++t) boff[t] = b_lane_off(slot * LB + t, lane);
    constexpr int kbase = 0;
#endif

    for (int bi = 0; bi < BATCH_INNER; ++bi) {
#if OP == OP_CONV   // kernel tensor [Cout][Hk][Wk][Cin]; block of zeros followed by the image [B][H][W][Cin]
        const u16 *Ab = A, *Bb = B;
#elif KSPLIT > 1   // MatMul, reduction split over grid z: this workgroup owns K range [bid.b * KSTEPS * BK, + KSTEPS * BK)
        const u16 *Ab = A + (long)bid.b * (KSTEPS * BK);
#if B_KMAJOR
        const u16 *Bb = B + (long)bid.b * (KSTEPS * BK);
#else
        const u16 *Bb = B + (long)bid.b * (KSTEPS * BK) * N;
#endif
        float *Cb = C;
#else
        const long batch = (long)bid.b * BATCH_INNER + bi;
        const u16 *Ab = A + batch * M * K;
        const u16 *Bb = B + batch * K * N;
        float *Cb = C + batch * M * N;
#endif

        acc_t acc[MI][NI];
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int r = 0; r < ACC_N; ++r) acc[i][j][r] = 0.f;

        if (bi > 0) {               // the previous batch: own loads landed, every wave done reading the stages
            WAIT_VMCNT(0);
            BARRIER();
        }
        // prologue: slabs 0 .. NSTG-1 in flight (one per stage), slab 0 landed, its first fragments read
#pragma unroll
        for (int s = 0; s < NSTG; ++s)
#pragma unroll
            for (int t = 0; t < PER; ++t)
                issue_piece(t, Ab, Bb, ring_addr + s * STAGE * 2, m0, n0, kbase + KCLAMP(s) * BK, slot, aoff, boff);
        WAIT_VMCNT((NSTG - 1) * PER);
        BARRIER();
        // Wave tiles of one or two atoms have too few MFMAs per 16-wide K step to cover the latency of the
        // next step's fragment reads (the steps of a slab then form a chain of LDS latencies).  Such
        // members advance in groups of G K steps: the fragments of a whole group are read while the
        // previous group's G * MI * NI MFMAs run.  Two fragment buffer sets of G steps each; the number
        // of groups per slab stays even so that the set a group uses is known at compile time.
        constexpr int G = (MI * NI <= 2 && KK >= 4) ? KK / 2 : 1;
        constexpr int KG = KK / G;
#if B_KMAJOR
        frag_t bf[2 * G][NI];
#define B_FRAG(b, j) bf[b][j]
#else
        v4s bh[2 * G][NI][2];
#define B_FRAG(b, j) __builtin_bit_cast(frag_t, __builtin_shufflevector(bh[b][j][0], bh[b][j][1], 0, 1, 2, 3, 4, 5, 6, 7))
#endif
        constexpr int SLOTS = G * MI * NI;         // MFMAs per group of steps
#if A_TRANS
        v4s ah[2 * G][MI][2];
        constexpr int NR = 2 * MI + 2 * NI;        // fragment reads per MFMA step
        // read number k of the fragments of step (stage, kk) into buffer set b: A fragment 0, the B
        // fragments, the other A fragments (the order the step's MFMAs need them in)
        auto frag_read = [&](int b, const u16 *stage, int kk, int k) {
            if (k < 2) ah[b][0][k] = read_a_half(stage, wm, lane, kk, 0, k);
            else if (k < 2 + 2 * NI) bh[b][(k - 2) / 2][(k - 2) % 2] = read_b_half(stage, wn, lane, kk, (k - 2) / 2, (k - 2) % 2);
            else ah[b][(k - 2 * NI) / 2][(k - 2 * NI) % 2] = read_a_half(stage, wm, lane, kk, (k - 2 * NI) / 2, (k - 2 * NI) % 2);
        };
#define A_FRAG(b, i) __builtin_bit_cast(frag_t, __builtin_shufflevector(ah[b][i][0], ah[b][i][1], 0, 1, 2, 3, 4, 5, 6, 7))
#elif B_KMAJOR
        frag_t af[2 * G][MI];
        constexpr int NR = MI + NI;                // fragment reads per MFMA step: A fragment 0, the B fragments, the other A fragments
        auto frag_read = [&](int b, const u16 *stage, int kk, int k) {
            if (k == 0) af[b][0] = read_a(stage, wm, lane, kk, 0);
            else if (k <= NI) bf[b][k - 1] = read_bk(stage, wn, lane, kk, k - 1);
            else af[b][k - NI] = read_a(stage, wm, lane, kk, k - NI);
        };
#define A_FRAG(b, i) af[b][i]
#else
        frag_t af[2 * G][MI];
        constexpr int NR = MI + 2 * NI;            // fragment reads per MFMA step
        // read number k of the fragments of step (stage, kk) into buffer set b
        auto frag_read = [&](int b, const u16 *stage, int kk, int k) {
            if (k == 0) af[b][0] = read_a(stage, wm, lane, kk, 0);
            else if (k <= 2 * NI) bh[b][(k - 1) / 2][(k - 1) % 2] = read_b_half(stage, wn, lane, kk, (k - 1) / 2, (k - 1) % 2);
            else af[b][k - 2 * NI] = read_a(stage, wm, lane, kk, k - 2 * NI);
        };
#define A_FRAG(b, i) af[b][i]
#endif
        // read number k of the fragments of group kg (steps kg*G .. kg*G+G-1) of a stage into buffer half h
        auto group_read = [&](int h, const u16 *stage, int kg, int k) {
            frag_read(h * G + k / NR, stage, kg * G + k / NR, k % NR);
        };
        constexpr int NRG = G * NR;                // fragment reads per group
#pragma unroll
        for (int k = 0; k < NRG; ++k) group_read(0, ring, 0, k);

        // One group of MFMA steps.  Its MFMAs use one buffer half (the halves alternate from group to group: with
        // an even number of groups per slab that is kg & 1; with a single group per slab, which 16x16x32 atoms on
        // slabs of 32 have, the slab's parity, which is its stage's because the ring has an even number of stages);
        // between them the wave issues, one
        // or two at a time, the reads of the next group's fragments and (in the last group of a slab,
        // after the barrier) the loads that refill the stage.  sched_barrier pins that order.
        auto slab_step = [&](int q, int s) {
#pragma unroll
            for (int kg = 0; kg < KG; ++kg) {
                const bool last = kg + 1 == KG;
                const int nact = NRG + (last ? PER : 0);
                const u16 *nstage = ring + (last ? (s + 1) % NSTG : s) * STAGE;
                static_assert(KG % 2 == 0 || NSTG % 2 == 0, "buffer halves must alternate at compile time");
                const int cur = (((s & 1) * (KG & 1)) + kg) & 1;
                const int nkg = last ? 0 : kg + 1, nh = cur ^ 1;
#pragma unroll
                for (int m = 0; m < SLOTS; ++m) {
                    const int g = m / (MI * NI), i = (m % (MI * NI)) / NI, j = m % NI;
                    acc[i][j] = MFMA(A_FRAG(cur * G + g, i), B_FRAG(cur * G + g, j), acc[i][j]);
                    if (m == 0 && last) {
                        WAIT_LGKM_VMCNT((NSTG - 2) * PER);
                        BARRIER();
                    }
                    constexpr int UMAX = (NRG + PER + SLOTS - 1) / SLOTS + 1;    // most actions behind one MFMA
                    const int lo = (m * nact + SLOTS - 1) / SLOTS, hi = ((m + 1) * nact + SLOTS - 1) / SLOTS;
#pragma unroll
                    for (int u = 0; u < UMAX; ++u) {
                        const int a = lo + u;
                        if (a >= hi) continue;
                        if (!last) group_read(nh, nstage, nkg, a);
                        else {
                            // the last group's actions: the NRG reads with the PER loads spread evenly among them
                            const int nl = a * PER / nact, nl1 = (a + 1) * PER / nact;
                            if (nl1 > nl) issue_piece(nl, Ab, Bb, ring_addr + s * STAGE * 2, m0, n0, kbase + KCLAMP(q + NSTG) * BK, slot, aoff, boff);
                            else group_read(nh, nstage, nkg, a - nl);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        };
        constexpr int KMAIN = KSTEPS / NSTG * NSTG;
        for (int kt = 0; kt < KMAIN; kt += NSTG) {
#pragma unroll
            for (int s = 0; s < NSTG; ++s) slab_step(kt + s, s);
        }
#pragma unroll
        for (int s = 0; s < KSTEPS - KMAIN; ++s) slab_step(KMAIN + s, s);

        // The last NSTG slab steps issued loads past the end of K (redundant copies of the last
        // slab, so that the wait counts stay uniform).  They must have landed before this wave ends:
        // a load that arrives after the workgroup's LDS has been handed to another workgroup would
        // write into memory this kernel no longer owns.
        WAIT_VMCNT(0);
        // Epilogue: an atom's result sits with column (l % ATOM) in lane l; 32x32 atoms: register r is
        // row 8*(r/4) + 4*(l/32) + r%4; 16x16 atoms: row 4*(l/16) + r.
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int r = 0; r < ACC_N; ++r) {
                    const int row = ATOM == 16 ? 4 * (lane / 16) + r : 8 * (r / 4) + 4 * (lane / 32) + r % 4;
#if OP == OP_CONV
                    if (TN % 32 != 0 && j * 32 + (lane & 31) >= TN) continue;   // overhang of a ragged wave tile
                    float *dst = &C[conv_c_index(cb, m0 + wm * TM + i * 32 + row, wn * TN + j * 32 + (lane & 31))];
#else
                    float *dst = &Cb[(long)(m0 + wm * TM + i * ATOM + row) * N + n0 + wn * TN + j * ATOM + (lane % ATOM)];
#endif
#if KSPLIT > 1
                    c_out(dst, acc[i][j][r]);
#else
                    __builtin_nontemporal_store(acc[i][j][r], dst);
#endif
                }
    }
}
