// MFMA kernel template (bf16 / fp16 inputs, fp32 accumulation) for gfx950.
//
// Roles of the tiling factors of one output axis (outermost first):
//   f1 workgroups along the axis (grid), f2 waves of the workgroup along the axis,
//   f3 basic tiles per wave, f4 basic tile.  Workgroup tile BM x BN = (f2 f3 f4 of M) x
//   (f2 f3 f4 of N); WM x WN waves, each owning a TM x TN = (f3 f4) x (f3 f4) tile made of
//   ATOM x ATOM MFMA atoms (32x32x16 or 16x16x32); a basic tile of FMI x FNI atoms is computed
//   as an outer product of FMI A-fragments and FNI B-fragments held in registers.
//   The reduction axis is split in KSTEPS slabs of BK, each staged in LDS.
//
// LDS layout (16-bit elements): As[stage][BM][BK+PAD] and Bs[stage][BN][BK+PAD], both with
// the reduction index contiguous, which is the order an MFMA lane wants its 8 operand values
// in.  A rows arrive that way from global memory; B arrives with n contiguous, so each
// thread loads a KB(k) x 8(n) block (KB = 8, 4 or 2, the largest that still gives every thread
// a block), transposes it in registers and writes 8 LDS rows of 2*KB bytes.  Consecutive lanes
// take consecutive k-blocks of the same 8 columns, so that their transposed stores fall into
// one padded LDS row after another without bank conflicts.
//
// FLAG = 1: two LDS stages and two register slabs: the global loads of slab kt+2 are issued
//           before the MFMAs of slab kt, slab kt+1 (loaded one step earlier) is written to the
//           other stage after them (one barrier per slab); the MFMA loop is fully unrolled and
//           software-pipelined (fragments of the next step are read while this step's MFMAs run).
// FLAG = 0: one stage, load -> barrier -> compute -> barrier; KUNROLL MFMA K steps of a slab are
//           unrolled together (1 unless the configuration space has a parameter for it).
// BMM only, STAGE_LDS = 0: no LDS at all, fragments are read straight from global memory.
// Conv2d only: wave tiles that are no multiple of the atom are rounded up to whole atoms (the
//           overhang is computed and thrown away), and the reduction axis Cin*Hk*Wk rarely has a factor 16, so a slab of BK taps is
//           staged BKP = BK rounded up to the MFMA K step wide, its tail filled with zeros; when
//           BKP != BK the kernel tensor is read element by element (its rows are not 16-byte
//           aligned then) with the same bounds as the image gather, and so it is when the slabs
//           are boxes of separately split C_in, H_k and W_k (TAP_BOX: not contiguous in memory).
//           CONV_NHWC: the operands were rewritten channels-last by a pre-pass (image [B][H][W][Cin],
//           kernel tensor [Cout][Hk][Wk][Cin]) and the reduction is walked as (r, s, ci).  Cin and BK
//           are multiples of 8, so 8 consecutive positions are 8 consecutive channels of one tap:
//           16 contiguous bytes of a pixel (or zeros where the tap falls outside the image), and a
//           row of the kernel tensor is contiguous along the whole walk.  Both operands then travel
//           in 16-byte pieces, consecutive lanes taking consecutive pieces of one row.

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
#define MFMA(a, b, c) MFMA_32(a, b, c)
#else
typedef f32x4 acc_t;
#define KA 32
#define MFMA(a, b, c) MFMA_16(a, b, c)
#endif

#if OP == OP_CONV && defined(TAP_BOX)
#define GATHER_A 1
#define A_TAP(k) conv_tap(k)
#else
#define GATHER_A 0
#define A_TAP(k) (k)
#endif
#ifndef KUNROLL
#define KUNROLL 1   // reduction steps of the non-pipelined (FLAG = 0) loop unrolled together
#endif
#define PRAGMA_(x) _Pragma(#x)
#define PRAGMA_UNROLL(n) PRAGMA_(unroll n)
#ifndef BKP
#define BKP BK
#endif
// Atoms per wave tile.  A Conv2d wave tile need not be a multiple of the atom (pixel tiles come
// from factors of 55, 27, ...): the last atom row / column then hangs over the tile; what it
// computes from its neighbours' rows (or from whatever follows the stage in LDS) is never stored.
#ifndef NWR
#define NWR (WM * WN)   // waves the workgroup really runs
#endif
constexpr int NPASS = (WM * WN) / NWR;
constexpr int MI = (TM + ATOM - 1) / ATOM, NI = (TN + ATOM - 1) / ATOM;
constexpr bool RAGGED_M = TM % ATOM != 0, RAGGED_N = TN % ATOM != 0;
constexpr int FMI = (!RAGGED_M && FM % ATOM == 0) ? FM / ATOM : 1;   // atoms per basic tile
constexpr int FNI = (!RAGGED_N && FN % ATOM == 0) ? FN / ATOM : 1;
constexpr int LDA = BKP + PAD, LDB = BKP + PAD;
__device__ __forceinline__ int lds_off(int row, int k)   // element offset of (row, k) in a stage
{
    return row * (BKP + PAD) + k;
}
constexpr int A_STAGE = BM * LDA, B_STAGE = BN * LDB;
constexpr int A_CHUNKS = BM * (BKP / 8);                      // 16-byte pieces of the A slab
constexpr int NA = (A_CHUNKS + NT - 1) / NT;
#if OP == OP_CONV
constexpr int B_CHUNKS = BN * (BKP / 8);                      // (column, 8 taps) gathers
constexpr int KB = 8;
#else
// B slab in KB(k) x 8(n) blocks; KB shrinks (8 -> 4 -> 2) until every thread owns a block
constexpr int KB = ((BK / 8) * (BN / 8) >= NT) ? 8 : ((BK / 4) * (BN / 8) >= NT) ? 4 : 2;
constexpr int B_CHUNKS = (BK / KB) * (BN / 8);
#endif
constexpr int NB = (B_CHUNKS + NT - 1) / NT;

#ifndef CONV_NHWC
#define CONV_NHWC 0
#endif
#if OP == OP_CONV
#ifndef CONV_TABLE
#define CONV_TABLE 0
#endif
#if CONV_NHWC
// A column of the implicit GEMM (an output pixel) as the channels-last gather needs it: the input
// pixel under tap (0, 0), which lies outside the image for padded borders (y0, x0 may be negative;
// base2, the byte offset of its channel 0 from the kernel's second pointer, is kept modulo 2^32).
// That pointer is a block of 256 zero bytes, which the [B][H][W][Cin] image follows.
struct NhwcCol { u32 base2; int y0, x0; };
__device__ __forceinline__ NhwcCol nhwc_col(const ColBlock &cb, int c)
{
    NhwcCol col;
    const int nb = cb.nb0 + c / (BH * BW);
    col.y0 = (cb.y0 + (c / BW) % BH) * STRIDE - PAD_CONV;
    col.x0 = (cb.x0 + c % BW) * STRIDE - PAD_CONV;
    col.base2 = 256u + 2u * (u32)(((nb * HIN + col.y0) * WIN + col.x0) * CIN);
    return col;
}
constexpr int NB_NHWC = (BN * (BKP / 8) + NT - 1) / NT;
constexpr bool NHWC_COLS_IN_REGS = NB_NHWC <= 8;
struct NhwcCols { NhwcCol c[NHWC_COLS_IN_REGS ? NB_NHWC : 1]; };
#endif
#if CONV_TABLE
// Image gather through a table.  Taken element by element, the gather spends some thirty integer
// instructions per value on splitting the tap into (ci, r, s) and the column into (image, y, x),
// several times what the MFMAs of the slab cost.  Both splits are hoisted.  The tap's part is
// a table built at compile time, two words per position of the reduction walk as the slabs
// stage it (KSTEPS slabs of BKP positions, the positions past BK of each slab unused):
//   off2 = byte offset of the tap inside one image, 2*((ci*HIN + r)*WIN + s);   rs = r << 16 | s.
// The column's part is {base2 = byte offset of the pixel under tap (0, 0, 0), which lies outside the
// tensor for padded borders and is kept modulo 2^32; yx = that pixel's y << 16 | x as two
// wrapping 16-bit fields}, computed once per thread before the K loop when the thread's columns
// repeat with a short period over its pieces, else once per piece.  Per value that leaves one
// packed add (yx + rs, the two fields independent), one packed minimum against (HIN-1, WIN-1) and
// a compare (a coordinate below zero wraps to a large field), one add for the address, the load
// and two selects.  The host only selects this path if the fields are wide enough.
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
constexpr int NTAB = KSPLIT * KSTEPS * BKP;
struct ConvTable { u32 e[2 * NTAB]; };   // 8 positions = {off2[0..8), rs[0..8)}: 64 bytes
constexpr ConvTable make_conv_table()
{
    ConvTable t{};
    for (int kt = 0; kt < KSPLIT * KSTEPS; ++kt)
        for (int j = 0; j < BKP; ++j) {
            u32 off2 = 0, rs = 0;
            if (j < BK) {
                const int k = conv_tap(kt * BK + j);
                const int ci = k / (HK * WK), r = (k / WK) % HK, sx = k % WK;
                off2 = 2u * (u32)((ci * HIN + r) * WIN + sx);
                rs = ((u32)r << 16) | (u32)sx;
            }
            const int p = kt * BKP + j;
            t.e[(p / 8) * 16 + p % 8] = off2;
            t.e[(p / 8) * 16 + 8 + p % 8] = rs;
        }
    return t;
}
__constant__ __attribute__((aligned(64))) ConvTable conv_table = make_conv_table();

struct ConvCol { u32 base2, yx; };
__device__ __forceinline__ ConvCol conv_col(const ColBlock &cb, int c)
{
    ConvCol col;
    const int nb = cb.nb0 + c / (BH * BW);
    const int y0 = (cb.y0 + (c / BW) % BH) * STRIDE - PAD_CONV;
    const int x0 = (cb.x0 + c % BW) * STRIDE - PAD_CONV;
    col.base2 = 2u * (u32)((nb * CIN * HIN + y0) * WIN + x0);
    col.yx = ((u32)y0 << 16) | ((u32)x0 & 0xFFFFu);
    return col;
}
constexpr int gcd_(int a, int b) { return b ? gcd_(b, a % b) : a; }
#endif
#endif

#if A_TRANS && !STAGE_LDS
#error "a transposed first operand needs LDS staging"
#endif
#if A_TRANS
// first operand stored [K][M] (M contiguous): its slab travels like B's, in KBA(k) x 8(m) blocks
constexpr int KBA = ((BK / 8) * (BM / 8) >= NT) ? 8 : ((BK / 4) * (BM / 8) >= NT) ? 4 : 2;
constexpr int AT_CHUNKS = (BK / KBA) * (BM / 8);
constexpr int NAT = (AT_CHUNKS + NT - 1) / NT;
#endif

struct Slab {
#if A_TRANS
    u32x4 at[NAT][KBA];
#else
    u32x4 a[NA];
#endif
#if OP == OP_CONV
    u32x4 b[NB];
#else
    u32x4 b[NB][KB];
#endif
};

// An operand whose rows run along the reduction axis in memory (B[k][n]; A[k][m] when the first
// operand is stored transposed): thread-owned blocks of KBX(k) x 8 elements, loaded as KBX 16-byte
// rows.  Consecutive lanes take consecutive k-blocks of the same 8 columns: their transposed LDS
// rows are then contiguous (no bank conflicts) and each global row still gets whole 128-byte
// segments from the 8 lanes that share a k-block.  base points at element [k0][first column of the tile].
template <int KBX, int CHUNKS, int NX>
__device__ __forceinline__ void load_kmajor(u32x4 (&r)[NX][KBX], const u16 *__restrict__ base, long ld, int tid)
{
#pragma unroll
    for (int i = 0; i < NX; ++i) {
        const int q = tid + i * NT;
        if (CHUNKS % NT == 0 || q < CHUNKS) {
            const int kb = q % (BK / KBX), xb = q / (BK / KBX);
#pragma unroll
            for (int j = 0; j < KBX; ++j) r[i][j] = *(const u32x4 *)(base + (long)(kb * KBX + j) * ld + xb * 8);
        }
    }
}
// ... and stored into a stage part laid out [column][k]: each block is transposed in registers
// (row j of the block is k = kb*KBX + j holding columns xb*8 .. +7) and written as 8 rows of KBX k.
template <int KBX, int CHUNKS, int NX>
__device__ __forceinline__ void store_kmajor(const u32x4 (&r)[NX][KBX], u16 *S, int tid)
{
#pragma unroll
    for (int i = 0; i < NX; ++i) {
        const int q = tid + i * NT;
        if (CHUNKS % NT == 0 || q < CHUNKS) {
            const int kb = q % (BK / KBX), xb = q / (BK / KBX);
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const int d = c / 2;
                u32 o[KBX / 2];
#pragma unroll
                for (int t = 0; t < KBX / 2; ++t)
                    o[t] = (c % 2 == 0) ? ((r[i][2 * t][d] & 0xffffu) | (r[i][2 * t + 1][d] << 16))
                                        : ((r[i][2 * t][d] >> 16) | (r[i][2 * t + 1][d] & 0xffff0000u));
                u16 *dst = S + lds_off(xb * 8 + c, kb * KBX);
                if (KBX == 8) { u32x4 v; v.x = o[0]; v.y = o[1 % (KBX / 2)]; v.z = o[2 % (KBX / 2)]; v.w = o[3 % (KBX / 2)]; *(u32x4 *)dst = v; }
                else if (KBX == 4) { typedef __attribute__((ext_vector_type(2))) unsigned int u32x2; u32x2 v; v.x = o[0]; v.y = o[1 % (KBX / 2)]; *(u32x2 *)dst = v; }
                else { *(u32 *)dst = o[0]; }
            }
        }
    }
}

#if OP == OP_CONV && CONV_TABLE
// piece i of a thread gathers column (tid + i*NT) % BN: the columns repeat every COL_PERIOD pieces
constexpr int COL_PERIOD = BN / gcd_(NT, BN);
constexpr int NCOL = COL_PERIOD < NB ? COL_PERIOD : NB;
constexpr bool COLS_IN_REGS = NCOL <= 8;
struct ConvCols { ConvCol c[COLS_IN_REGS ? NCOL : 1]; };
#endif

__device__ __forceinline__ void load_slab(Slab &s, const u16 *__restrict__ Ab, const u16 *__restrict__ Bb,
                                          int m0, int k0, int tid
#if OP == OP_CONV
                                          , const ColBlock &cb
#if CONV_TABLE
                                          , const ConvCols &cols
#elif CONV_NHWC
                                          , const NhwcCols &ncols
#endif
#else
                                          , int n0
#endif
)
{
#if A_TRANS
    load_kmajor<KBA, AT_CHUNKS, NAT>(s.at, Ab + (long)k0 * M + m0, M, tid);
#else
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int q = tid + i * NT;
        if (A_CHUNKS % NT == 0 || q < A_CHUNKS) {
            const int row = q / (BKP / 8), kc = q % (BKP / 8);
            if (BKP == BK && !GATHER_A) {
                s.a[i] = *(const u32x4 *)(Ab + (long)(m0 + row) * K + k0 + kc * 8);
            } else if (CONV_NHWC) {   // BK is a multiple of 8: a piece is whole or past the slab's end
                const u32x4 zero = {0u, 0u, 0u, 0u};
                const bool in = kc * 8 < BK;
                const u32x4 v = *(const u32x4 *)(Ab + (long)(m0 + row) * K + (in ? k0 + kc * 8 : 0));
                s.a[i] = in ? v : zero;
            } else {   // padded slab: taps past BK are zeros, rows start at any 2-byte offset;
                       // boxed reduction walk: the taps of a slab are not contiguous
                u32 h[8];
#pragma unroll
                for (int t = 0; t < 8; ++t)
                    h[t] = (kc * 8 + t < BK) ? (u32)Ab[(long)(m0 + row) * K + A_TAP(k0 + kc * 8 + t)] : 0u;
                u32x4 v;
                v.x = h[0] | (h[1] << 16); v.y = h[2] | (h[3] << 16);
                v.z = h[4] | (h[5] << 16); v.w = h[6] | (h[7] << 16);
                s.a[i] = v;
            }
        }
    }
#endif
#if OP != OP_CONV
    load_kmajor<KB, B_CHUNKS, NB>(s.b, Bb + (long)k0 * N + n0, N, tid);
#elif CONV_NHWC
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int q = tid + i * NT;
        if (B_CHUNKS % NT == 0 || q < B_CHUNKS) {
            const int c = q / (BKP / 8), kc = q % (BKP / 8);
            const NhwcCol col = NHWC_COLS_IN_REGS ? ncols.c[i] : nhwc_col(cb, c);
            const int kp = k0 + kc * 8;                        // position in the (r, s, ci) walk
            const int tap = kp / CIN, ci0 = kp % CIN, r = tap / WK, sx = tap % WK;
            const bool ok = (BKP == BK || kc * 8 < BK) && (unsigned)(col.y0 + r) < (unsigned)HIN &&
                            (unsigned)(col.x0 + sx) < (unsigned)WIN;
            // unconditional load (from the block of zeros where the tap is outside) and a select
            const u32 o = ok ? col.base2 + 2u * (u32)((r * WIN + sx) * CIN + ci0) : 0u;
            const u32x4 v = *(const u32x4 *)((const char *)Bb + (size_t)o);
            const u32x4 zero = {0u, 0u, 0u, 0u};
            s.b[i] = ok ? v : zero;
        }
    }
#else
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int q = tid + i * NT;
        if (B_CHUNKS % NT == 0 || q < B_CHUNKS) {
            const int c = q % BN, kc = q / BN;
            u32 h[8];
#if CONV_TABLE
            const ConvCol col = COLS_IN_REGS ? cols.c[i % NCOL] : conv_col(cb, c);
            const u32x4 *tp = (const u32x4 *)(conv_table.e + 2 * (k0 / BK * BKP + kc * 8));
            const u32x4 o0 = tp[0], o1 = tp[1], r0 = tp[2], r1 = tp[3];
            const u32 off2[8] = {o0.x, o0.y, o0.z, o0.w, o1.x, o1.y, o1.z, o1.w};
            const u32 rs[8] = {r0.x, r0.y, r0.z, r0.w, r1.x, r1.y, r1.z, r1.w};
            const u16x2 lim = {(unsigned short)(WIN - 1), (unsigned short)(HIN - 1)};   // element 0 = low half = x
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const u16x2 at = __builtin_bit_cast(u16x2, col.yx) + __builtin_bit_cast(u16x2, rs[t]);
                const bool ok = __builtin_bit_cast(u32, __builtin_elementwise_min(at, lim)) == __builtin_bit_cast(u32, at) &&
                                (BKP == BK || kc * 8 + t < BK);
                // unconditional load (of the tensor's first element where the tap is outside the image)
                // and two selects: straight-line code, all eight loads in flight together
                const u32 o = ok ? col.base2 + off2[t] : 0u;
                const u32 v = *(const u16 *)((const char *)Bb + (size_t)o);
                h[t] = ok ? v : 0u;
            }
#else
#pragma unroll
            for (int t = 0; t < 8; ++t) h[t] = (BKP == BK || kc * 8 + t < BK) ? (u32)conv_b(Bb, cb, k0 + kc * 8 + t, c) : 0u;
#endif
            u32x4 v;
            v.x = h[0] | (h[1] << 16); v.y = h[2] | (h[3] << 16);
            v.z = h[4] | (h[5] << 16); v.w = h[6] | (h[7] << 16);
            s.b[i] = v;
        }
    }
#endif
}

__device__ __forceinline__ void store_slab(const Slab &s, u16 *As, u16 *Bs, int tid)
{
#if A_TRANS
    store_kmajor<KBA, AT_CHUNKS, NAT>(s.at, As, tid);
#else
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int q = tid + i * NT;
        if (A_CHUNKS % NT == 0 || q < A_CHUNKS) {
            const int row = q / (BKP / 8), kc = q % (BKP / 8);
            *(u32x4 *)(As + lds_off(row, kc * 8)) = s.a[i];
        }
    }
#endif
#if OP == OP_CONV
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int q = tid + i * NT;
        if (B_CHUNKS % NT == 0 || q < B_CHUNKS) {
#if CONV_NHWC
            const int c = q / (BKP / 8), kc = q % (BKP / 8);
#else
            const int c = q % BN, kc = q / BN;
#endif
            *(u32x4 *)(Bs + lds_off(c, kc * 8)) = s.b[i];
        }
    }
#else
    store_kmajor<KB, B_CHUNKS, NB>(s.b, Bs, tid);
#endif
}

// MFMAs of one LDS-resident slab.  Lane l of a wave supplies, for atom row/column l % ATOM,
// the 8 reduction values starting at 8*(l / ATOM) of each KA-wide step.
// A slab is consumed in steps of one basic tile (FMI x FNI atoms) per KA-wide K step: the
// FMI + FNI fragments of a step are read from LDS, then FMI*FNI MFMAs form their outer product.
__device__ __forceinline__ void load_frags(frag_t (&af)[FMI], frag_t (&bf)[FNI], const u16 *As, const u16 *Bs,
                                           int a_row0, int b_row0, int lk, int step)
{
    constexpr int TJ = NI / FNI, TI = MI / FMI;
    const int kk = step / (TI * TJ), i0 = (step / TJ) % TI * FMI, j0 = step % TJ * FNI;
#pragma unroll
    for (int i = 0; i < FMI; ++i)
        af[i] = __builtin_bit_cast(frag_t, *(const u32x4 *)(As + lds_off(a_row0 + (i0 + i) * ATOM, kk * KA + lk)));
#pragma unroll
    for (int j = 0; j < FNI; ++j)
        bf[j] = __builtin_bit_cast(frag_t, *(const u32x4 *)(Bs + lds_off(b_row0 + (j0 + j) * ATOM, kk * KA + lk)));
}

__device__ __forceinline__ void compute_slab(acc_t (&acc)[MI][NI], const u16 *As, const u16 *Bs,
                                             int a_row0, int b_row0, int lk)
{
    constexpr int TJ = NI / FNI, TI = MI / FMI;
    constexpr int STEPS = (BKP / KA) * TI * TJ;
#if FLAG
    // fully unrolled, fragments of step t+1 are read before the MFMAs of step t are issued
    // (two register sets), so LDS latency hides behind the matrix pipe inside one wave
    frag_t af[2][FMI], bf[2][FNI];
    load_frags(af[0], bf[0], As, Bs, a_row0, b_row0, lk, 0);
#pragma unroll
    for (int t = 0; t < STEPS; ++t) {
        if (t + 1 < STEPS) load_frags(af[(t + 1) & 1], bf[(t + 1) & 1], As, Bs, a_row0, b_row0, lk, t + 1);
        const int i0 = (t / TJ) % TI * FMI, j0 = t % TJ * FNI;
#pragma unroll
        for (int i = 0; i < FMI; ++i)
#pragma unroll
            for (int j = 0; j < FNI; ++j)
                acc[i0 + i][j0 + j] = MFMA(af[t & 1][i], bf[t & 1][j], acc[i0 + i][j0 + j]);
    }
#else
    PRAGMA_UNROLL(KUNROLL)
    for (int kk = 0; kk < BKP / KA; ++kk) {
#pragma unroll
        for (int tt = 0; tt < TI * TJ; ++tt) {
            frag_t af[FMI], bf[FNI];
            load_frags(af, bf, As, Bs, a_row0, b_row0, lk + kk * KA, tt);
            const int i0 = tt / TJ * FMI, j0 = tt % TJ * FNI;
#pragma unroll
            for (int i = 0; i < FMI; ++i)
#pragma unroll
                for (int j = 0; j < FNI; ++j)
                    acc[i0 + i][j0 + j] = MFMA(af[i], bf[j], acc[i0 + i][j0 + j]);
        }
    }
#endif
}

extern "C" __global__ __launch_bounds__(NT)
void KERNEL_NAME(const u16 *__restrict__ A, const u16 *__restrict__ B, float *__restrict__ C,
                  unsigned long long *ctl /* deadline control: folded members only (the scalar template always honours it) */)
{
    extern __shared__ __attribute__((aligned(16))) u16 smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lrow = lane % ATOM, lk = (lane / ATOM) * 8;
    const BlockId bid = block_id();
#if OP == OP_CONV
    const ColBlock cb = col_block(bid.n);
#endif

    // A configuration may ask for more waves than a workgroup can hold (WM * WN > 16).  The workgroup
    // then runs NWR of them (a divisor of WM * WN), and every real wave takes the tiles of
    // WM * WN / NWR waves one after another, each with the whole K loop: slow, and the same result.
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
        const u16 *Ab = A, *Bb = B;
#else
#if KSPLIT > 1   // MatMul, reduction split over grid z: this workgroup owns K range [bid.b * KSTEPS * BK, + KSTEPS * BK)
        const u16 *Ab = A + (long)bid.b * (KSTEPS * BK);
        const u16 *Bb = B + (long)bid.b * (KSTEPS * BK) * N;
        float *Cb = C;
#else
        const long batch = (long)bid.b * BATCH_INNER + bi;
        const u16 *Ab = A + batch * M * K;
        const u16 *Bb = B + batch * K * N;
        float *Cb = C + batch * M * N;
#endif
#endif
        acc_t acc[MI][NI];
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int r = 0; r < (ATOM == 32 ? 16 : 4); ++r) acc[i][j][r] = 0.f;

#if STAGE_LDS
        u16 *As = smem, *Bs = smem + NSTAGE * A_STAGE;
        Slab slab;
#if OP == OP_CONV
#if CONV_TABLE
        ConvCols cols;
        if (COLS_IN_REGS) {
#pragma unroll
            for (int i = 0; i < NCOL; ++i) cols.c[i] = conv_col(cb, (tid + i * NT) % BN);
        }
#define LOAD_INTO(S, kt) load_slab(S, Ab, Bb, m0, CONV_KBASE(bid) + (kt) * BK, tid, cb, cols)
#elif CONV_NHWC
        NhwcCols ncols;
        if (NHWC_COLS_IN_REGS) {
#pragma unroll
            for (int i = 0; i < NB_NHWC; ++i) ncols.c[i] = nhwc_col(cb, ((tid + i * NT) / (BKP / 8)) % BN);
        }
#define LOAD_INTO(S, kt) load_slab(S, Ab, Bb, m0, CONV_KBASE(bid) + (kt) * BK, tid, cb, ncols)
#else
#define LOAD_INTO(S, kt) load_slab(S, Ab, Bb, m0, CONV_KBASE(bid) + (kt) * BK, tid, cb)
#endif
#else
#define LOAD_INTO(S, kt) load_slab(S, Ab, Bb, m0, (kt) * BK, tid, n0)
#endif
#if FLAG
        // Two LDS stages, two register slabs: the loads of slab kt+2 are issued before the MFMAs
        // of slab kt; slab kt+1 (loaded one iteration earlier) is written to the other stage
        // after them.  Global latency therefore has two K steps to hide in.
        Slab slab1;
        constexpr int KPAIRS = KSTEPS / 2 * 2;
        if (bi > 0 || sub > 0 || pass > 0) __syncthreads();
        LOAD_INTO(slab, 0);
        if (KSTEPS > 1) LOAD_INTO(slab1, 1);
        store_slab(slab, As, Bs, tid);
        __syncthreads();
#define KCLAMP(k) ((k) < KSTEPS ? (k) : KSTEPS - 1)
#define COMPUTE(stage) compute_slab(acc, As + (stage) * A_STAGE, Bs + (stage) * B_STAGE, wm * TM + lrow, wn * TN + lrow, lk)
        // branch-free body: slab indices past the end are clamped (a few redundant loads at
        // the tail) so that the accumulators never cross a conditional block
        for (int kt = 0; kt < KPAIRS; kt += 2) {
            LOAD_INTO(slab, KCLAMP(kt + 2));
            COMPUTE(0);
            store_slab(slab1, As + A_STAGE, Bs + B_STAGE, tid);
            __syncthreads();
            LOAD_INTO(slab1, KCLAMP(kt + 3));
            COMPUTE(1);
            store_slab(slab, As, Bs, tid);
            __syncthreads();
        }
        if (KSTEPS % 2) COMPUTE(0);
#else
        for (int kt = 0; kt < KSTEPS; ++kt) {
            LOAD_INTO(slab, kt);
            __syncthreads();
            store_slab(slab, As, Bs, tid);
            __syncthreads();
            compute_slab(acc, As, Bs, wm * TM + lrow, wn * TN + lrow, lk);
        }
        __syncthreads();
#endif
#else  // no LDS staging (BMM, STAGE_LDS = 0): fragments straight from global memory
        for (int k0 = 0; k0 < K; k0 += KA) {
            frag_t af[MI], bf[NI];
#pragma unroll
            for (int i = 0; i < MI; ++i)
                af[i] = __builtin_bit_cast(frag_t, *(const u32x4 *)(Ab + (long)(m0 + wm * TM + i * ATOM + lrow) * K + k0 + lk));
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const u16 *p = Bb + (long)(k0 + lk) * N + n0 + wn * TN + j * ATOM + lrow;
                u32x4 v;
                v.x = (u32)p[0] | ((u32)p[(long)N] << 16);
                v.y = (u32)p[2L * N] | ((u32)p[3L * N] << 16);
                v.z = (u32)p[4L * N] | ((u32)p[5L * N] << 16);
                v.w = (u32)p[6L * N] | ((u32)p[7L * N] << 16);
                bf[j] = __builtin_bit_cast(frag_t, v);
            }
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j) acc[i][j] = MFMA(af[i], bf[j], acc[i][j]);
        }
#endif

        // Epilogue.  An atom's result sits with column (l % ATOM) in lane l; 32x32: register r
        // is row 8*(r/4) + 4*(l/32) + r%4; 16x16: register r is row 4*(l/16) + r.
#pragma unroll
        for (int i = 0; i < MI; ++i) {
#pragma unroll
            for (int j = 0; j < NI; ++j) {
#pragma unroll
                for (int r = 0; r < (ATOM == 32 ? 16 : 4); ++r) {
                    const int row = (ATOM == 32) ? 8 * (r / 4) + 4 * (lane / 32) + r % 4 : 4 * (lane / 16) + r;
                    if ((RAGGED_M && i * ATOM + row >= TM) || (RAGGED_N && j * ATOM + lrow >= TN)) continue;
                    const int gm = m0 + wm * TM + i * ATOM + row;
                    const int cn = wn * TN + j * ATOM + lrow;   // column inside the workgroup tile
#if OP == OP_CONV
                    c_out(&C[conv_c_index(cb, gm, cn)], acc[i][j][r]);
#else
                    c_out(&Cb[(long)gm * N + n0 + cn], acc[i][j][r]);
#endif
                }
            }
        }
    }
}
