/*
 * opevo.h -- C ABI of the MI355X (gfx950) trial-evaluation library for OpEvo.
 *
 * The library solves   x* = argmax_{x in X} f(x),  X = prod_i X_i   (Sec. 3, Eq. 1)
 * where f(x) is the measured TFLOP/s of one tensor operator compiled under
 * configuration x (Sec. 1, Sec. 3), by the evolutionary loop of Alg. 1 (Sec. 4.4).
 * It holds: the configuration-space encoder (Sec. 3), the q-random-walk mutation
 * (Sec. 4.3, Eq. 3; App. A), selection + recombination (Sec. 4.2, Eq. 2), HIP kernel
 * templates for MatMul / BatchMatMul / Conv2d (App. B.1-B.3) instantiated per
 * configuration through hipRTC, and a hipEvent measurement harness.
 *
 * Conventions
 *  - Every call returns an int status: OPEVO_OK (0) or a negative OPEVO_E_* code.
 *    Nothing throws or aborts.  opevo_last_error() returns a thread-local text for
 *    the last failing call on this thread (hipRTC log included).
 *  - Handles (opevo_space, opevo_rng, opevo_tuner, opevo_op, opevo_kernel) are owned by
 *    the library from *_create until *_destroy.  All arrays are caller-owned HOST memory
 *    unless the argument is documented as a DEVICE pointer.  Device pointers and the
 *    stream are borrowed for the duration of the call; the library never frees them.
 *  - Flat configuration encoding (int32): parameters in declaration order; a FACTOR
 *    parameter takes nu slots (its factors, outermost first, product == C); a
 *    PERMUTATION of n items takes n slots (the order, items 0..n-1); DISCRETE and
 *    CATEGORICAL take one slot (index into the value list).
 *  - "Illegal" = not a member of the space: an error of the caller (OPEVO_E_ILLEGAL).
 *    "Invalid" = a member the kernel templates or the hardware cannot run (too many
 *    threads, LDS or registers; compile failure): such a trial is still an evaluation,
 *    with fitness 0 (Sec. 4.2), and the reason is reported as OPEVO_E_INVALID.
 *  - Random numbers: SplitMix64 (state += 0x9E3779B97F4A7C15, then the two
 *    multiply-xorshift rounds), double = (u64 >> 11) * 2^-53, integer below n =
 *    ((u64 >> 32) * n) >> 32.  The order in which each routine draws is stated at
 *    the routine, so a run is reproducible from its seed alone.
 */
#ifndef OPEVO_H
#define OPEVO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define OPEVO_OK            0
#define OPEVO_E_ARG        -1   /* null pointer, bad enum, size or capacity too small            */
#define OPEVO_E_ILLEGAL    -2   /* configuration / vertex is not in the space                     */
#define OPEVO_E_INVALID    -3   /* legal configuration that cannot run (fitness 0, Sec. 4.2)      */
#define OPEVO_E_HIPRTC     -4   /* hipRTC failure (log in opevo_last_error)                       */
#define OPEVO_E_HIP        -5   /* HIP runtime failure, or no usable GPU                          */
#define OPEVO_E_PARITY     -6   /* result disagrees with the supplied reference tensor            */
#define OPEVO_E_TOO_LARGE  -7   /* feasible set too large to enumerate / solve exactly            */
#define OPEVO_E_STATE      -8   /* call sequence error (e.g. best() before any tell())            */

typedef struct opevo_space  opevo_space;
typedef struct opevo_rng    opevo_rng;
typedef struct opevo_tuner  opevo_tuner;
typedef struct opevo_op     opevo_op;
typedef struct opevo_kernel opevo_kernel;

const char *opevo_last_error(void);
const char *opevo_status_name(int status);
/* Library version as a static string. */
const char *opevo_version(void);

/* ------------------------------------------------------------------ random numbers */
int opevo_rng_create(uint64_t seed, opevo_rng **out);
int opevo_rng_destroy(opevo_rng *rng);
int opevo_rng_next_u64(opevo_rng *rng, uint64_t *out);
int opevo_rng_next_double(opevo_rng *rng, double *out);          /* [0,1)            */
int opevo_rng_next_below(opevo_rng *rng, uint32_t n, uint32_t *out); /* [0,n), n > 0 */

/* ------------------------------------------------- configuration space (Sec. 3, Eq. 1) */
typedef enum {
    OPEVO_FACTOR      = 0,  /* nu ordered positive factors with product C; adjacency: move one
                               prime from one factor to another (Sec. 3)                        */
    OPEVO_PERMUTATION = 1,  /* orders of n items; adjacency: one transposition (Sec. 3)         */
    OPEVO_DISCRETE    = 2,  /* strictly ascending reals; adjacency: neighbours in value order   */
    OPEVO_CATEGORICAL = 3   /* J unordered choices; adjacency: complete graph (Sec. 3)          */
} opevo_ptype;

typedef struct {
    int32_t       type;      /* opevo_ptype                                                     */
    int32_t       nu;        /* FACTOR: number of factors (>= 1)                                */
    int64_t       C;         /* FACTOR: the product (>= 1)                                      */
    int32_t       n_values;  /* PERMUTATION: n items; DISCRETE: value count; CATEGORICAL: J     */
    int32_t       reserved;
    const double *values;    /* DISCRETE: n_values strictly ascending numbers (copied); else NULL */
    const char   *name;      /* optional label (copied), may be NULL                            */
} opevo_param_desc;

/* Builds X = prod X_i.  OPEVO_E_ARG for a malformed descriptor, OPEVO_E_TOO_LARGE if a single
 * feasible set has more than 2^24 vertices. */
int opevo_space_create(const opevo_param_desc *params, int n_params, opevo_space **out);
int opevo_space_destroy(opevo_space *space);
int opevo_space_num_params(const opevo_space *space, int *n_params);
int opevo_space_width(const opevo_space *space, int *n_int32);             /* flat length     */
int opevo_space_param_slice(const opevo_space *space, int param, int *offset, int *width);
int opevo_space_param_name(const opevo_space *space, int param, const char **name);
int opevo_space_param_size(const opevo_space *space, int param, int64_t *n_vertices);
int opevo_space_size(const opevo_space *space, double *n_configs);         /* prod |X_i|      */
/* OPEVO_OK if cfg (flat, width ints) is a member of X, else OPEVO_E_ILLEGAL. */
int opevo_space_is_legal(const opevo_space *space, const int32_t *cfg);
/* All vertices of X_param in the canonical order (FACTOR and PERMUTATION: lexicographic;
 * DISCRETE / CATEGORICAL: index order), each `width(param)` ints, into out[cap_vertices*width].
 * *n receives the vertex count; OPEVO_E_ARG if cap_vertices is too small (*n still set). */
int opevo_space_enumerate(const opevo_space *space, int param, int32_t *out,
                          int64_t cap_vertices, int64_t *n);
/* S(v): the vertices adjacent to v in X_param, in the canonical order (FACTOR: source
 * position ascending, then prime ascending, then target position ascending; PERMUTATION:
 * position pairs i<j lexicographic; DISCRETE: lower then upper; CATEGORICAL: index order). */
int opevo_space_neighbors(const opevo_space *space, int param, const int32_t *v,
                          int32_t *out, int cap_vertices, int *n);
/* Mixed-radix index of a configuration: parameter 0 most significant, digit = position of
 * the parameter's vertex in enumerate order.  Only for spaces with fewer than 2^62 members. */
int opevo_space_rank(const opevo_space *space, const int32_t *cfg, int64_t *rank);
int opevo_space_unrank(const opevo_space *space, int64_t rank, int32_t *cfg_out);
/* Uniform member of X: per parameter, in order, vertex index = next_below(|X_i|). */
int opevo_space_random(const opevo_space *space, opevo_rng *rng, int32_t *cfg_out);
/* One q-random walk (Sec. 4.3) on parameter `param`, in place on that parameter's slots of
 * v (a vertex, width(param) ints).  Per step: if S(u) is empty return (no draw); draw
 * next_double(), stop unless it is < q; else u = S(u)[next_below(|S(u)|)].  0 <= q < 1. */
int opevo_space_walk(const opevo_space *space, int param, double q, opevo_rng *rng, int32_t *v);
/* Mutation of a whole configuration: an independent walk on every parameter, in order. */
int opevo_space_mutate(const opevo_space *space, double q, opevo_rng *rng, int32_t *cfg_inout);
/* Exact q-random-walk distribution from `start` (App. A: S = (1-q)(I-Q)^-1 p0) by a dense
 * fp64 solve; probs_out[i] belongs to vertex i of enumerate order.  For feasible sets of at
 * most 2048 vertices (else OPEVO_E_TOO_LARGE).  An isolated start gives the point mass. */
int opevo_qrw_exact(const opevo_space *space, int param, const int32_t *start, double q,
                    double *probs_out, int64_t cap);

/* ------------------------------------- selection, recombination, Alg. 1 (Sec. 4.2, 4.4) */
/* One child by Eq. 2: parents are given best first (n_parents configs, flat) with their
 * fitness (negative / NaN count as 0).  Per parameter, in order: if the fitness total is > 0,
 * t = next_double()*total and the parent is the first j with t < f_1+..+f_j; else
 * j = next_below(n_parents).  The parameter is copied whole from that parent. */
int opevo_recombine(const opevo_space *space, const int32_t *parents, const double *fitness,
                    int n_parents, opevo_rng *rng, int32_t *child_out);

/* Alg. 1 in ask/tell form.  lambda = parents, rho = children per generation, 0 <= q < 1.
 * The tuner keeps the space pointer: destroy the tuner first. */
int opevo_tuner_create(const opevo_space *space, int lambda, int rho, double q, uint64_t seed,
                       opevo_tuner **out);
int opevo_tuner_destroy(opevo_tuner *tuner);
/* Which mutation ask() applies to a recombined child.  0 (default): the q-random walk on every
 * parameter's graph (Sec. 4.3).  1: a control that ignores the graphs, as a plain evolutionary
 * algorithm would mutate: per parameter, in order, draw next_double(); if it is < q the
 * parameter becomes the vertex number next_below(|X_i|) of its feasible set.  Used to measure what
 * the topology-aware walk buys (Sec. 5.5 compares hyperparameters, not this).  The no-duplicate
 * rule applies to both. */
int opevo_tuner_set_mutation(opevo_tuner *tuner, int kind);
/* Next configurations to evaluate, at most max_n (max_n <= 0: no cap): the first call gives
 * lambda random members, later calls give rho children of the top-lambda of everything told
 * so far (ties: earlier trial first).  No configuration is ever returned twice, whether it was
 * told or is still pending: a duplicate child is mutated again from where it stands, up to 100
 * times, then replaced by a uniformly random unsampled member.  *n_out == 0: space exhausted.
 * cfgs_out holds max(lambda, rho) * width ints. */
int opevo_tuner_ask(opevo_tuner *tuner, int32_t *cfgs_out, int max_n, int *n_out);
/* Enqueue n evaluated configurations with their fitness (TFLOP/s; 0 for invalid ones). */
int opevo_tuner_tell(opevo_tuner *tuner, const int32_t *cfgs, const double *fitness, int n);
int opevo_tuner_num_trials(const opevo_tuner *tuner, int *n);
/* Best configuration so far, its fitness and its 0-based trial index. */
int opevo_tuner_best(const opevo_tuner *tuner, int32_t *cfg_out, double *fitness, int *trial);
/* The whole history in trial order. */
int opevo_tuner_history(const opevo_tuner *tuner, int32_t *cfgs_out, double *fitness_out,
                        int cap_trials, int *n);

/* --------------------------------------------------------- operators (App. B.1 - B.3) */
typedef enum { OPEVO_MATMUL = 0, OPEVO_BMM = 1, OPEVO_CONV2D = 2, OPEVO_BMM_TA = 3 } opevo_op_kind;
typedef enum { OPEVO_F32 = 0, OPEVO_BF16 = 1, OPEVO_F16 = 2 } opevo_dtype;

/* Which configuration space / kernel template family an operator is tuned in.
 *  TILE2: every loop axis split in two (outer = workgroups or steps, inner = tile); one
 *         scalar-FMA template that runs every member.  MatMul only.
 *         params: M(2) N(2) K(2).
 *  TILE4: output axes split in four (workgroups, waves per workgroup, basic tiles per wave,
 *         basic tile), reduction axis in two (steps, LDS tile), plus one binary flag:
 *         MatMul  M(4) N(4) K(2) unroll{0,1}        (double-buffered, unrolled main loop)
 *         BMM     B(2) M(4) N(4) K(2) lds{0,1}      (stage operands through LDS or not)
 *         Conv2d  B(2) Cout(4) H(4) W(4) R(2) unroll{0,1},  R = Cin*Hk*Wk
 *         MFMA kernels (bf16/fp16 inputs) where the per-wave tile is made of 32x32 or 16x16
 *         atoms and the LDS tile of whole MFMA K-steps; a scalar-FMA kernel otherwise.
 *         fp32 inputs: 32x32x2 fp32 MFMA atoms; MatMul / BMM where the per-wave tile is made of
 *         32x32 atoms and the LDS tile is a multiple of 8 (and the contiguous axes multiples of 4),
 *         Conv2d with the same widening as above (slabs padded to 8, wave tiles rounded up to 32);
 *         else scalar.
 *         Conv2d widens this: an LDS tile of any length is zero-padded to whole K-steps, and a
 *         per-wave tile that is no multiple of 16 is rounded up to whole 16x16 atoms as long as
 *         that at most doubles the work (the overhang is computed and not stored).
 *         Folding: a member that asks for more than a workgroup has is not scored 0 but run as serial
 *         work, so that the search sees a slow member with its own place in the landscape: a per-wave
 *         tile of more than 256 accumulators per lane is cut (a prime at a time along its longer side)
 *         into sub-tiles that become tiles of waves of their own; a reduction slab too long for the LDS
 *         is halved while it stays a multiple of 32; a workgroup tile too large for the LDS even then
 *         (or for 1024 threads x 256 outputs on the scalar template) is cut into sub-tiles that the
 *         workgroup computes one after another (Conv2d: along the channel side only); more than 16
 *         waves: the workgroup runs the largest divisor of their number that is at most 16 and every
 *         real wave takes the tiles of several waves in turn, each with the whole K loop.  opevo_plan
 *         reports the tile, wave tile and threads the kernel really uses.  What still cannot run
 *         (a pixel box too large for the LDS, staging registers, spills) stays invalid.
 *  TILE4X: TILE4 plus the two remaining parameter types of Sec. 3 as launch tunables.  The
 *         workgroups are launched as a one-dimensional grid and walk the grid axes (0 = N tiles,
 *         1 = M tiles, 2 = batch blocks of a BMM) in the order given by a PERMUTATION parameter
 *         `order` (first = fastest varying); a DISCRETE parameter `group` in {1, 2, 4, 8, 16}
 *         is the number of consecutive tiles of the second axis that are walked together (each
 *         group goes through the whole first axis before the next group starts), which decides
 *         what the workgroups resident at one time share in L2.  Flat encoding: the TILE4 slots,
 *         then the permutation (2 or 3 slots), then the index of the group width.
 *  TILE4P: Conv2d only, the space as App. B.3 lays it out: the reduction axes are split
 *         separately,
 *         Conv2d  B(2) Cout(4) H(4) W(4) Cin(2) Hk(2) Wk(2) unroll{0,1} unroll_steps{1,2,4,8}
 *         so a K slab is a box of Cin_inner x Hk_inner x Wk_inner taps and the kernel walks the
 *         Cin_outer x Hk_outer x Wk_outer boxes in row-major order (a different summation order
 *         from TILE4's flattened walk, the same sum).  unroll_steps (DISCRETE) is the number of
 *         reduction steps unrolled together where the reduction is a loop: the scalar template's
 *         K loop when unroll = 1 (explicit pragma), the MFMA template's loop over the K steps of
 *         a slab when unroll = 0 (with unroll = 1 that template is fully unrolled and pipelined
 *         anyway).  Kernel templates, padding of slabs and rounding of wave tiles as for TILE4.
 *  TILE4K: MatMul only, the reduction axis in three factors as App. B.1 has it:
 *         MatMul  M(4) N(4) K(3) unroll{0,1},   K = (partitions, steps, LDS tile)
 *         The first factor is the number of workgroups (grid z) that share one output tile; each
 *         reduces its own contiguous part of K and adds its partial sums into C with fp32 atomic
 *         adds.  Members with more than one partition need C cleared first: opevo_kernel_launch /
 *         opevo_kernel_time (and opevo_tune) enqueue a small fill kernel over C before every
 *         launch of such a member, and the time of that clear counts as part of the trial.  The sum is the
 *         same up to the rounding of an fp32 addition order that varies from run to run.  For
 *         operators whose output has fewer tiles than the chip has compute units (MM3 of App. B.1:
 *         512 x 1024 from K = 4096) this is what fills the machine.
 *  TILE4C: Conv2d only: TILE4 with the reduction axis in three factors (as TILE4K gives MatMul) and a
 *         second binary choice, the layout the kernel reads its operands in:
 *         Conv2d  B(2) Cout(4) H(4) W(4) R(3) unroll{0,1} layout{0,1},  R = (partitions, steps, LDS tile)
 *         partitions = workgroups along grid z that share an output tile, each reducing its own
 *         contiguous range of R and adding its partial sums into the output with fp32 atomic adds (the
 *         output is cleared by a fill kernel before every launch of such a member, inside the timed
 *         launch): the 256 x 6272 x 2304 GEMM view of the 14 x 14 convolution has too few output
 *         tiles for 256 compute units otherwise.
 *         layout = 0: operands as the caller stores them (NCHW image gathered value by value, OIHW
 *         kernel tensor), R walked as (ci, r, s).  layout = 1: channels last.  Every launch is preceded,
 *         on the same stream and inside the timed launch, by one pre-pass kernel that rewrites the
 *         image as [B][H][W][Cin] and the kernel tensor as [Cout][Hk][Wk][Cin] into a workspace the
 *         kernel object owns (allocated when its module is loaded, freed by opevo_kernel_destroy);
 *         R is then walked as (r, s, ci), 8 consecutive reduction values of a pixel are 16
 *         contiguous bytes, and both operands travel in 16-byte pieces like MatMul's first operand.
 *         Same sum in another order.  Needs Cin and the LDS tile to be multiples of 8 and an MFMA
 *         member; elsewhere layout = 1 runs the layout = 0 kernel.
 *  TILE4T: MatMul only: TILE4 plus a binary choice of the second operand's layout,
 *         MatMul  M(4) N(4) K(2) unroll{0,1} bpack{0,1}
 *         bpack = 1: every launch is preceded, on the same stream and inside the timed launch, by a
 *         pre-pass kernel that transposes B to [N][K] into a workspace the kernel object owns; both
 *         operands are then K-contiguous and read from LDS with plain 16-byte fragment reads.  Only
 *         members of the direct-to-LDS template have such a kernel; elsewhere bpack = 1 runs the
 *         bpack = 0 kernel.
 *  TILE4A: MatMul only: TILE4 plus a binary choice of the MFMA atom,
 *         MatMul  M(4) N(4) K(2) unroll{0,1} atom{0,1}
 *         atom = 1: members of the direct-to-LDS template multiply with 16x16x32 atoms instead of 32x32x16 ones
 *         (same tiles, same LDS traffic, twice the MFMA instructions, a quarter of the accumulator updates per
 *         flop: under the chip's power limit the matrix pipes sustain about a tenth more flops per second on
 *         changing operands that way, while kernels bound by instruction issue lose).  Elsewhere, and where the
 *         unrolled loop body would grow too long, atom = 1 runs the atom = 0 kernel.
 *  TILE4L: Conv2d only: the input channels in two factors and a three-way choice of the operand path,
 *         Conv2d  B(2) Cout(4) H(4) W(4) Cin(2) unroll{0,1} layout{0,1,2} kwaves{1,2,4,8},  Cin = (slabs, channels per slab)
 *         layout = 0: operands as the caller stores them, reduction walked as (ci, r, s): a slab is the slab's
 *         channels with all their Hk*Wk taps (TILE4 with R = (slabs, channels per slab * Hk * Wk)).
 *         layout = 1: channels-last copies written by a pre-pass inside the timed launch, as in TILE4C;
 *         walked as (r, s, ci), a slab being the slab's channels under one tap.
 *         layout = 2: an LDS-resident image patch (App. B.3's loop nest with the taps innermost): per slab the
 *         workgroup stages the input pixels under its box of output pixels once, channels fastest, straight from
 *         the NCHW image, and the slab's part of the OIHW kernel tensor re-ordered tap by tap; every tap then
 *         reads its operands from that patch at a fixed offset from the output pixel.  One launch, no pre-pass,
 *         each staged pixel re-used by all taps that touch it.  16-bit inputs, slabs of whole 16 channels (32 on
 *         16x16x32 atoms), at most 16 waves, and patch + kernel-tensor part within the LDS.  A member that asks
 *         for something else keeps its workgroup tile and is divided among the waves another way: shorter slabs
 *         are merged and slabs too long for the LDS halved, wave tiles of fewer than 16 output channels merged
 *         along Cout, waves beyond 16 merged along the pixels.  Where that does not help (fp32 inputs, fewer than
 *         16 input channels, an image one pixel wide, a patch too large for the LDS) layout = 2 runs the layout = 0 kernel.  Same sum in
 *         another order.
 *         kwaves (DISCRETE, layout = 2 only, inert elsewhere): that many waves share every wave tile and deal the
 *         slab's MFMA steps (taps x groups of channels) round-robin among themselves; their partial sums are added
 *         through LDS after the last slab, in the order of the waves (deterministic).  The workgroup then has
 *         (waves along Cout) x (waves along the pixels) x kwaves waves; where it cannot hold them (16 waves, registers,
 *         LDS for the final sum) the member runs with kwaves = 1. */
typedef enum { OPEVO_TILE2 = 0, OPEVO_TILE4 = 1, OPEVO_TILE4X = 2, OPEVO_TILE4P = 3, OPEVO_TILE4K = 4, OPEVO_TILE4C = 5, OPEVO_TILE4T = 6,
               OPEVO_TILE4A = 7, OPEVO_TILE4L = 8 } opevo_variant;

/* dims:  MATMUL {M, N, K}            C[M,N] = A[M,K] B[K,N]
 *        BMM    {B, M, N, K}         C[b] = A[b] B[b]
 *        BMM_TA {B, M, N, K}         C[b] = A[b]^T B[b] with the first operand stored as [B][K][M]
 *                                    (App. B.2: "transposed first"); same configuration spaces as
 *                                    BMM; runs on every template (members with lds = 0 on the
 *                                    scalar one)
 *        CONV2D {B, Cin, H, W, Cout, Hk, Wk, stride, pad}  NCHW image, OIHW kernel,
 *               out[B,Cout,Hout,Wout], Hout = floor((H+2*pad-Hk)/stride)+1 (App. B.3).
 * All tensors dense row-major.  `in` is the element type of both inputs; accumulation and
 * the output are always fp32. */
int opevo_op_create(int kind, const int64_t *dims, int n_dims, int in_dtype, opevo_op **out);
int opevo_op_destroy(opevo_op *op);
int opevo_op_flops(const opevo_op *op, double *flops);     /* 2*MACs, padding taps counted  */
int opevo_op_bytes(const opevo_op *op, double *bytes);     /* read A, B once + write C once */
int opevo_op_sizes(const opevo_op *op, int64_t *a_elems, int64_t *b_elems, int64_t *c_elems);
/* The operator's configuration space for a variant (caller destroys it). */
int opevo_op_space(const opevo_op *op, int variant, opevo_space **out);

typedef struct {
    int32_t status;        /* OPEVO_OK or OPEVO_E_INVALID                                      */
    int32_t path;          /* 0 scalar FMA, 1 MFMA 32x32x16, 2 MFMA 16x16x32, 3 MFMA 32x32x16 with
                              operands streamed global -> LDS directly, 4 fp32 MFMA 32x32x2,
                              5 Conv2d with an LDS-resident image patch (either atom)          */
    int32_t grid[3];
    int32_t block;         /* threads per workgroup                                            */
    int32_t lds_bytes;
    int32_t acc_per_lane;  /* fp32 accumulators each lane holds                                */
    int32_t tile[3];       /* workgroup tile BM, BN, BK                                        */
    int32_t wave_tile[2];  /* per-wave tile                                                    */
    char    reason[96];    /* why invalid, else empty                                          */
    int32_t sub_tiles[2];  /* folded members: sub-tiles of `tile` along M and N that a workgroup
                              computes one after another (1, 1 otherwise): a workgroup owns
                              sub_tiles[0] * tile[0] rows and sub_tiles[1] * tile[1] columns  */
    int32_t wave_passes;   /* folded members: tiles every wave computes in turn (1 otherwise)  */
} opevo_plan;

/* Decode + validate (host only, no GPU): OPEVO_E_ILLEGAL if cfg is not in the space;
 * otherwise OPEVO_OK with plan->status telling valid / invalid. */
int opevo_kernel_plan(const opevo_op *op, int variant, const int32_t *cfg, opevo_plan *plan);
/* The hipRTC option string ("-DBM=.. ...") and template name the configuration renders to. */
int opevo_kernel_defines(const opevo_op *op, int variant, const int32_t *cfg,
                         char *buf, size_t cap);
/* hipRTC serialises compilations inside one process, so concurrent instantiation (the paper
 * compiles on 8 CPU threads, Sec. 6) runs on worker processes.  Started before the calling
 * process has opened the GPU, a worker is the executable opevo_rtc_worker next to the library
 * (fork + exec; it uses the hipRTC of the ROCm installation under /opt/rocm).  Started later,
 * no exec is done: a worker is then a fork of the caller that only serves compile requests
 * with the hipRTC the caller is bound to.  Workers keep no device file open.  Idempotent;
 * *n_running (may be NULL) = workers alive.  Without a pool every instantiation compiles in
 * the calling process.  opevo_compile_pool_kind: 1 executable workers, 0 forks, -1 no pool.
 * Start the pool before the first GPU call of the process, and never while another thread is
 * compiling: executable workers use the newer compiler of the ROCm installation (their kernels
 * are about a tenth faster), and a fork taken while a thread sits inside hipRTC can leave the
 * child with that thread's locks held.  Fork-only pools are capped at 12 workers. */
int opevo_compile_pool_start(int n_workers, int *n_running);
int opevo_compile_pool_stop(void);
int opevo_compile_pool_kind(int *kind);
/* A limit on the time a caller waits for one instantiation on a worker (seconds; 0, the default, = none).
 * hipRTC cannot be interrupted and no process is started once the GPU may be open, so a compilation that
 * overruns is left to finish in the background (its worker returns to the pool afterwards, the result is
 * dropped) while the call is answered OPEVO_E_INVALID at the deadline: the configuration counts as one that
 * cannot be evaluated (Sec. 4.2: fitness 0).  A few members of the convolution spaces (one wave gathering a
 * long slab value by value, fully unrolled) take a minute or more to compile on a loaded host and would
 * otherwise hold up their whole generation.  No effect without a pool. */
int opevo_compile_pool_deadline(double seconds);

/* Instantiate: render + hipRTC-compile for gfx950 (works without a GPU).  Returns
 * OPEVO_E_INVALID for an invalid configuration (no kernel), OPEVO_E_HIPRTC on a compile
 * failure.  The module is loaded on the first launch.  Two checks on the compiled code of the
 * direct-to-LDS template (path 3), whose hand-placed waits count the loads in flight and so
 * need the fully unrolled, spill-free code: a code object above 128 KiB (the compiler did not
 * unroll the schedule) makes this call return OPEVO_E_INVALID.  On every template, a kernel
 * that the compiler gave private scratch memory (register spills) makes its first launch /
 * timing return OPEVO_E_INVALID: it would be slow, it would break the load counting of path 3,
 * and one spilling member of the register-staged template once gave wrong rows.  opevo_tune
 * scores both as invalid trials. */
int opevo_kernel_build(const opevo_op *op, int variant, const int32_t *cfg,
                       opevo_kernel **out, double *compile_ms);
/* Compiling is by far the longest part of a trial (Sec. 6 gives it 8 CPU threads), and runs of
 * Alg. 1 that differ in seed, q or lambda revisit many configurations.  opevo_kernel_build (and
 * through it opevo_tune) therefore keeps every code object it compiled, keyed by the template
 * text, the member's constants and the compiler options: in memory, up to max_memory_bytes
 * (default 256 MiB, oldest dropped first, 0 switches it off, negative keeps the current limit),
 * and, if dir is not NULL / empty, also as one file per entry in that directory (created if
 * missing; files appear by rename, so processes may share it; a file that does not match its key
 * or is damaged is ignored and compiled again).  Without this call the directory is taken from the
 * environment variable OPEVO_CODE_CACHE_DIR, if set.  A hit makes compile_ms the look-up time.
 * OPEVO_E_ARG if dir cannot be created or written.  _clear drops the in-memory entries (files
 * stay).  _stats: look-ups answered from the cache (disk_hits of them from a file), look-ups that
 * had to compile, entries and bytes held in memory; any pointer may be NULL. */
int opevo_code_cache_configure(const char *dir, int64_t max_memory_bytes);
int opevo_code_cache_clear(void);
int opevo_code_cache_stats(int64_t *hits, int64_t *disk_hits, int64_t *misses, int64_t *entries,
                           int64_t *bytes);
int opevo_kernel_destroy(opevo_kernel *kernel);
int opevo_kernel_code_size(const opevo_kernel *kernel, size_t *bytes);
/* Registers / scratch the compiler used (available after the first launch loaded it). */
int opevo_kernel_resources(opevo_kernel *kernel, int *vgprs, int *sgprs, int *spill_bytes,
                           int *static_lds);
/* One launch on `stream` (a hipStream_t, NULL = default stream).  a, b, c are DEVICE
 * pointers: the two inputs in the operator's input dtype and the fp32 output, sized as
 * opevo_op_sizes says, 16-byte aligned.  MatMul / BMM: a = A, b = B.  Conv2d: a = the kernel
 * tensor [Cout,Cin,Hk,Wk], b = the image [B,Cin,H,W].  Asynchronous. */
int opevo_kernel_launch(opevo_kernel *kernel, const void *a, const void *b, void *c, void *stream);
/* Timing (Sec. 3: f = TFLOP/s): `warmup` untimed launches (the first of them is itself
 * timed, to size a sample, and followed by a synchronisation), then `samples` samples of
 * `launches_per_sample` launches each; warm-ups and samples are enqueued back to back with
 * one hipEvent between consecutive samples on `stream` and a single synchronisation at the
 * end, so the GPU never idles inside the measurement.  ms per launch of each sample into
 * samples_ms (may be NULL), median into *median_ms.  launches_per_sample <= 0: chosen so that
 * one sample spans at least 200 us.  A launch of 20 ms or more is taken as the measurement
 * on its own.  warmup_ms > 0 extends the warm-up until that much GPU time has been spent
 * (at most 4000 launches): after idling the device needs tens of milliseconds to reach its
 * sustained clocks, and a sample taken earlier under-reports the kernel by up to a quarter.
 * timeout_ms > 0 gives scalar-template kernels, and folded members of the register-staged MFMA
 * templates (see TILE4), a deadline of timeout_ms per launch: one that is still running then winds down by itself (every workgroup leaves at its
 * next K slab) and the call returns OPEVO_E_INVALID; 0 = no deadline.  Synchronises `stream`. */
int opevo_kernel_time(opevo_kernel *kernel, const void *a, const void *b, void *c, void *stream,
                      int warmup, double warmup_ms, int launches_per_sample, int samples,
                      double timeout_ms, double *median_ms, double *samples_ms);

/* The matrix-pipe ceiling this device sustains: TFLOP/s of a kernel that only issues
 * 32x32x16 MFMAs of the given input type (OPEVO_BF16 / OPEVO_F16) on register operands, measured
 * like any trial after 40 ms of warm-up.  random_data = 0: all operands zero (no operand bit
 * toggles: the clock stays near its maximum and the result near the nominal peak);
 * random_data != 0: operands uniform in (-1, 1), as a workload's are (the device then lowers its
 * clock to stay inside its power limit, and this is the ceiling a real kernel is up against).
 * Kernel results are best read against both.  Allocates and frees a small device buffer.
 * Synchronises `stream`. */
int opevo_mfma_ceiling(int in_dtype, int random_data, void *stream, double *tflops);
/* The same with the MFMA atom named: 32 = 32x32x16 (what opevo_mfma_ceiling measures), 16 = 16x16x32.  On
 * operands that change, the device sustains more flops per second with the 16x16x32 atom (fewer accumulator
 * updates per flop, so less power per flop); on all-zero operands slightly fewer. */
int opevo_mfma_ceiling_atom(int in_dtype, int random_data, int atom, void *stream, double *tflops);

/* Parity gate: c and ref are DEVICE fp32 arrays of n elements.
 * max_scaled = max |c-ref| / (|ref|+1), rel_fro = ||c-ref||_F / ||ref||_F (0 if both 0).
 * Uses a library-owned device workspace allocated on first use. Synchronises `stream`. */
int opevo_compare_f32(const float *c, const float *ref, int64_t n, void *stream,
                      double *max_scaled, double *rel_fro);

/* The same for a sample of rows: c is viewed as a matrix with row_len columns, ref_rows holds
 * the n_rows reference rows row_index[0..n_rows) (DEVICE int32) back to back.  For outputs
 * whose full reference is too expensive to compute on the host. */
int opevo_compare_rows_f32(const float *c, const float *ref_rows, const int32_t *row_index,
                           int64_t n_rows, int64_t row_len, void *stream,
                           double *max_scaled, double *rel_fro);

/* opevo_compare_f32 for callers that cannot allocate (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the same comparison with the same kernel, but the
 * per-workgroup partial results live in a fixed array of 24 KiB of device memory that is part of the
 * library's code object (one copy per GPU, held until the process ends), the final fold runs on
 * the device in the same order as opevo_compare_f32's host fold, and nothing is copied back:
 * result is a DEVICE pointer to two doubles that receive {max_scaled, rel_fro}, valid once the
 * work enqueued on `stream` has finished.  The call allocates nothing, frees nothing and does
 * not synchronise.  n may be at most OPEVO_COMPARE_STATIC_MAX_N; a larger n is refused with
 * OPEVO_E_ARG.  All calls on one GPU share the one array: calls whose kernels may overlap there
 * (different streams, or graphs replayed concurrently) race and must be serialised by the caller;
 * no clearing is needed between calls (each call overwrites every partial it later reads). */
#define OPEVO_COMPARE_STATIC_MAX_N ((int64_t)1 << 34)
int opevo_compare_f32_static(const float *c, const float *ref, int64_t n, void *stream,
                             double *result);

/* -------------------------------------------------------- whole tuning run (Alg. 1) */
typedef struct {
    const void *a, *b;         /* DEVICE inputs                                                  */
    void       *c;             /* DEVICE fp32 output, overwritten by every trial                 */
    const float *ref;          /* DEVICE fp32 reference for the parity gate, or NULL: the whole
                                  output, or (n_ref_rows > 0) only the sampled rows, back to back */
    const int32_t *ref_row_index;  /* DEVICE row numbers of the sampled reference rows, or NULL   */
    int32_t     n_ref_rows;    /* 0: ref is the whole output                                     */
    int32_t     ref_row_len;   /* columns of the output viewed as a matrix (sampled reference)   */
    void       *stream;        /* hipStream_t                                                    */
    int32_t     trials;        /* evaluation budget, the initial lambda included                 */
    int32_t     lambda, rho;   /* Alg. 1                                                         */
    double      q;
    uint64_t    seed;
    int32_t     compile_threads;   /* concurrent hipRTC instantiations per generation (>= 1)     */
    int32_t     warmup, launches_per_sample, samples;   /* as opevo_kernel_time                  */
    double      warmup_ms;                              /* as opevo_kernel_time, 0 = none        */
    double      trial_timeout_ms;                       /* as opevo_kernel_time, 0 = none        */
    double      tol_max_scaled, tol_rel_fro;            /* parity gate thresholds                */
    /* optional per-trial logs, each `trials` long (cfg_log: trials*width), may be NULL */
    int32_t    *cfg_log;
    double     *fitness_log;   /* TFLOP/s, 0 for invalid / failed                                */
    int32_t    *status_log;    /* OPEVO_OK, OPEVO_E_INVALID, OPEVO_E_HIPRTC, OPEVO_E_PARITY, ... */
    double     *compile_ms_log;
    double     *run_ms_log;    /* median ms per launch                                           */
    double     *wall_s_log;    /* seconds since the start of the run when the trial finished     */
    int32_t     progress_every; /* > 0: after every generation that crosses a multiple of this many
                                   trials, one line on stderr (trials done, best TFLOP/s, seconds);
                                   0: silent.  Independently of this, OPEVO_TUNE_TRACE=1 in the
                                   environment prints one line per trial before its kernel runs
                                   (kernel name = configuration), so that the log of a run that
                                   died names what was on the GPU                                   */
    int32_t     mutation;       /* as opevo_tuner_set_mutation: 0 the paper's q-random walk, 1 control */
    int32_t     speculate_threads; /* > 0: while a generation is compiled and timed, that many further host
                                   threads build the generation Alg. 1 would ask for next if none of the
                                   current children made the top-lambda (a copy of the tuner is asked; the
                                   run's own tuner and its trajectory are untouched).  A guessed kernel is
                                   used when the run really asks for that configuration, else discarded.
                                   Needs as many idle compile workers; 0: off                            */
} opevo_tune_args;

typedef struct {
    int32_t n_trials;          /* evaluated (may be < trials if the space was exhausted)         */
    int32_t best_trial;        /* index of the best trial, -1 if none had fitness > 0            */
    double  best_tflops;
    double  best_ms;
    int32_t n_invalid, n_compile_fail, n_parity_fail;
    double  wall_s, compile_s, run_s;   /* total, hipRTC (wall, overlapped), GPU measurement     */
    int32_t n_built_ahead;     /* trials whose kernel had been built ahead of time (speculate_threads)  */
} opevo_tune_result;

/* Runs Alg. 1 on the GPU: ask -> instantiate the generation's children concurrently ->
 * time each -> parity gate -> tell.  best_cfg_out receives the best configuration
 * (width ints).  A parity failure gives that trial fitness 0 and is counted; it does not
 * stop the run. */
int opevo_tune(const opevo_op *op, int variant, const opevo_tune_args *args,
               int32_t *best_cfg_out, opevo_tune_result *result);

#ifdef __cplusplus
}
#endif
#endif /* OPEVO_H */
