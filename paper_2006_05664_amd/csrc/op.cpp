// Operator descriptors, configuration spaces and the configuration decoder.
#include "op.hpp"

#include <cstdlib>
#include <cstring>
#include <algorithm>
#include <new>
#include <numeric>
#include <sstream>

using namespace opevo;

static const int kMaxThreads = 1024;            // threads per workgroup on gfx950
static const int kMaxLds = 160 * 1024;          // LDS bytes per workgroup on gfx950
static const int64_t kMaxDldsBody = 256;        // unrolled K-loop body of the direct-to-LDS template, instructions
static const int64_t kMaxDldsBody16 = 400;      // the same for members on 16x16x32 atoms
static const int kMaxAcc = 256;                 // fp32 accumulators per lane kept in registers
static const int kPad = 8;                      // LDS row padding of the MFMA template (elements)

int64_t opevo_op::a_elems() const
{
    return kind == OPEVO_CONV2D ? M * K : batch * M * K;   // conv: kernel tensor [Cout][Cin*Hk*Wk]
}

int64_t opevo_op::b_elems() const
{
    return kind == OPEVO_CONV2D ? nimg * cin * hin * win : batch * K * N;
}

namespace opevo {

static opevo_param_desc factor(const char *name, int64_t C, int nu)
{
    opevo_param_desc d;
    std::memset(&d, 0, sizeof d);
    d.type = OPEVO_FACTOR; d.C = C; d.nu = nu; d.name = name;
    return d;
}

static const double kGroupValues[] = {1, 2, 4, 8, 16};
static const int kNumGroupValues = 5;
static const double kUnrollSteps[] = {1, 2, 4, 8};
static const int kNumUnrollSteps = 4;
static const double kReductionWaves[] = {1, 2, 4, 8};
static const int kNumReductionWaves = 4;

static opevo_param_desc permutation(const char *name, int n)
{
    opevo_param_desc d;
    std::memset(&d, 0, sizeof d);
    d.type = OPEVO_PERMUTATION; d.n_values = n; d.name = name;
    return d;
}

static opevo_param_desc discrete(const char *name, const double *values, int n)
{
    opevo_param_desc d;
    std::memset(&d, 0, sizeof d);
    d.type = OPEVO_DISCRETE; d.n_values = n; d.values = values; d.name = name;
    return d;
}

static opevo_param_desc flag(const char *name)
{
    opevo_param_desc d;
    std::memset(&d, 0, sizeof d);
    d.type = OPEVO_CATEGORICAL; d.n_values = 2; d.name = name;
    return d;
}

int op_param_descs(const opevo_op &op, int variant, std::vector<opevo_param_desc> &descs)
{
    descs.clear();
    if (variant == OPEVO_TILE2) {
        if (op.kind != OPEVO_MATMUL) return fail(OPEVO_E_ARG, "the two-level space exists for MatMul only");
        descs = {factor("M", op.M, 2), factor("N", op.N, 2), factor("K", op.K, 2)};
        return OPEVO_OK;
    }
    if (variant == OPEVO_TILE4P) {
        // App. B.3: C_out, H_out, W_out in four factors, C_in, H_k, W_k in two factors each, the binary
        // choice of an explicit unroll and the discrete bound on the unrolled steps; the batch
        // split is kept from the four-level space
        if (op.kind != OPEVO_CONV2D) return fail(OPEVO_E_ARG, "the separately split reduction space exists for Conv2d only");
        descs = {factor("B", op.nimg, 2), factor("Cout", op.M, 4), factor("H", op.hout, 4), factor("W", op.wout, 4),
                 factor("Cin", op.cin, 2), factor("Hk", op.hk, 2), factor("Wk", op.wk, 2), flag("unroll"),
                 discrete("unroll_steps", kUnrollSteps, kNumUnrollSteps)};
        return OPEVO_OK;
    }
    if (variant == OPEVO_TILE4K) {
        // MatMul with the reduction axis in three factors, as App. B.1 splits it; the outermost one is
        // the number of workgroups that share an output tile, each reducing its own part of K
        if (op.kind != OPEVO_MATMUL) return fail(OPEVO_E_ARG, "the split-reduction space exists for MatMul only");
        descs = {factor("M", op.M, 4), factor("N", op.N, 4), factor("K", op.K, 3), flag("unroll")};
        return OPEVO_OK;
    }
    if (variant == OPEVO_TILE4T) {
        // MatMul with the layout of the second operand as a second binary choice: as stored ([K][N]) or
        // transposed to [N][K] by a pre-pass before every launch
        if (op.kind != OPEVO_MATMUL) return fail(OPEVO_E_ARG, "the space with a packed second operand exists for MatMul only");
        descs = {factor("M", op.M, 4), factor("N", op.N, 4), factor("K", op.K, 2), flag("unroll"), flag("bpack")};
        return OPEVO_OK;
    }
    if (variant == OPEVO_TILE4A) {
        // MatMul with the MFMA atom of direct-to-LDS members as a second binary choice: 32x32x16 or 16x16x32
        if (op.kind != OPEVO_MATMUL) return fail(OPEVO_E_ARG, "the space with a choice of MFMA atom exists for MatMul only");
        descs = {factor("M", op.M, 4), factor("N", op.N, 4), factor("K", op.K, 2), flag("unroll"), flag("atom")};
        return OPEVO_OK;
    }
    if (variant == OPEVO_TILE4C) {
        // Conv2d with the fused reduction axis in three factors (partitions along grid z, steps, LDS
        // tile) and the operand layout as a second binary choice
        if (op.kind != OPEVO_CONV2D) return fail(OPEVO_E_ARG, "the split-reduction / channels-last space exists for Conv2d only");
        descs = {factor("B", op.nimg, 2), factor("Cout", op.M, 4), factor("H", op.hout, 4), factor("W", op.wout, 4),
                 factor("R", op.K, 3), flag("unroll"), flag("layout")};
        return OPEVO_OK;
    }
    if (variant == OPEVO_TILE4L) {
        // Conv2d with the input channels in two factors (slabs, channels per slab; every slab holds all the
        // taps) and a three-way choice of how the operands reach the matrix units: gathered from the NCHW
        // image value by value, channels-last copies written by a pre-pass, or an LDS-resident image patch
        // filled straight from the NCHW image; for the last, the number of waves that share a wave tile and split
        // the reduction steps of every slab among themselves
        if (op.kind != OPEVO_CONV2D) return fail(OPEVO_E_ARG, "the space with an LDS-resident image patch exists for Conv2d only");
        descs = {factor("B", op.nimg, 2), factor("Cout", op.M, 4), factor("H", op.hout, 4), factor("W", op.wout, 4),
                 factor("Cin", op.cin, 2), flag("unroll"), flag("layout"), discrete("kwaves", kReductionWaves, kNumReductionWaves)};
        descs[descs.size() - 2].n_values = 3;
        return OPEVO_OK;
    }
    if (variant != OPEVO_TILE4 && variant != OPEVO_TILE4X) return fail(OPEVO_E_ARG, "unknown variant %d", variant);
    switch (op.kind) {
    case OPEVO_MATMUL:
        descs = {factor("M", op.M, 4), factor("N", op.N, 4), factor("K", op.K, 2), flag("unroll")};
        break;
    case OPEVO_BMM:
        descs = {factor("B", op.batch, 2), factor("M", op.M, 4), factor("N", op.N, 4),
                 factor("K", op.K, 2), flag("lds")};
        break;
    case OPEVO_CONV2D:
        descs = {factor("B", op.nimg, 2), factor("Cout", op.M, 4), factor("H", op.hout, 4),
                 factor("W", op.wout, 4), factor("R", op.K, 2), flag("unroll")};
        break;
    default:
        return fail(OPEVO_E_ARG, "unknown operator kind %d", op.kind);
    }
    if (variant == OPEVO_TILE4X) {
        // the order in which a one-dimensional launch walks the grid axes (N tiles, M tiles and,
        // for BMM, batch blocks; first = fastest), and the width of the groups of second-axis
        // tiles it walks together
        descs.push_back(permutation("order", op.kind == OPEVO_BMM ? 3 : 2));
        descs.push_back(discrete("group", kGroupValues, kNumGroupValues));
    }
    return OPEVO_OK;
}

// Row pitch and per-image pitch (in pixels) of the LDS-resident patch for a box of bh x bw output pixels:
// (bh-1)*stride + hk rows of (bw-1)*stride + wk pixels.  padded (unit stride only): the row pitch and the image
// pitch are raised to be congruent to bw and to bh*bw modulo 16, so that consecutive output pixels of the
// flattened box read consecutive groups of LDS banks.
static void patch_pitches(const opevo_op &op, int64_t bh, int64_t bw, bool padded, int64_t &row, int64_t &image)
{
    const int64_t ph = (bh - 1) * op.stride + op.hk, pw = (bw - 1) * op.stride + op.wk;
    row = pw; image = ph * pw;
    if (!padded || op.stride != 1) return;
    row = pw + ((bw - pw) % 16 + 16) % 16;
    image = ph * row + ((bh * bw - ph * row) % 16 + 16) % 16;
}

static void invalid(opevo_plan &p, const char *fmt, long a = 0, long b = 0)
{
    p.status = OPEVO_E_INVALID;
    snprintf(p.reason, sizeof p.reason, fmt, a, b);
}

int decode(const opevo_op &op, int variant, const int32_t *cfg, Decoded &out)
{
    std::vector<opevo_param_desc> descs;
    if (int rc = op_param_descs(op, variant, descs)) return rc;
    // legality: every factor tuple multiplies back to its axis, flags in range
    {
        int off = 0;
        for (const auto &d : descs) {
            if (d.type == OPEVO_FACTOR) {
                int64_t prod = 1;
                for (int j = 0; j < d.nu; ++j) {
                    if (cfg[off + j] < 1) return fail(OPEVO_E_ILLEGAL, "factor %d of %s is < 1", j, d.name);
                    prod *= cfg[off + j];
                    if (prod > d.C) break;
                }
                if (prod != d.C)
                    return fail(OPEVO_E_ILLEGAL, "factors of %s do not multiply to %lld", d.name, (long long)d.C);
                off += d.nu;
            } else if (d.type == OPEVO_PERMUTATION) {
                unsigned seen = 0;
                for (int j = 0; j < d.n_values; ++j) {
                    if (cfg[off + j] < 0 || cfg[off + j] >= d.n_values || (seen >> cfg[off + j] & 1u))
                        return fail(OPEVO_E_ILLEGAL, "%s is not a permutation of 0..%d", d.name, d.n_values - 1);
                    seen |= 1u << cfg[off + j];
                }
                off += d.n_values;
            } else {
                if (cfg[off] < 0 || cfg[off] >= d.n_values)
                    return fail(OPEVO_E_ILLEGAL, "%s out of range", d.name);
                off += 1;
            }
        }
    }

    opevo_plan &p = out.plan;
    std::memset(&p, 0, sizeof p);
    p.status = OPEVO_OK;
    std::ostringstream D;

    // ---- common GEMM-view quantities filled by each variant
    int64_t m1 = 1, n1 = 1, b1 = 1, binner = 1;
    int64_t BM = 1, BN = 1, BK = 1, ksteps = 1, WM = 1, WN = 1, TM = 1, TN = 1, FM = 1, FN = 1;
    int flagv = 0;
    int64_t nb2 = 1, BH = 1, BW = 1, h1 = 1, w1 = 1;
    bool four_level = (variant == OPEVO_TILE4 || variant == OPEVO_TILE4X || variant == OPEVO_TILE4P || variant == OPEVO_TILE4K ||
                       variant == OPEVO_TILE4C || variant == OPEVO_TILE4T || variant == OPEVO_TILE4A || variant == OPEVO_TILE4L);
    int atom16 = 0;                        // MatMul, TILE4A: 1 = 16x16x32 atoms on direct-to-LDS members
    int bpack = 0;                         // MatMul, TILE4T: 1 = second operand transposed to [N][K] by a pre-pass
    int layout = 0;                        // Conv2d, TILE4C: 1 = channels-last operands (pre-pass)
    int64_t subm = 1, subn = 1;            // sub-tiles a workgroup computes one after another (folded members)
    int64_t ksplit = 1;
    int64_t box[6] = {1, 1, 1, 1, 1, 1};   // C_in, H_k, W_k as (boxes, box extent) pairs
    bool tap_box = false;
    int64_t kunroll = 0;                   // 0: the template's default
    int64_t patch_cs = 0;                  // Conv2d, TILE4L, layout 2: channels per slab of the LDS-resident patch (0: not on that template)
    int patch_atom = 0, patch_stages = 1, patch_kw = 1;
    int64_t patch_row = 0, patch_image = 0;   // its row pitch and image pitch in pixels
    int tile4_width = 0;   // slots of the four-level part, after which the launch-order parameters follow

    if (!four_level) {
        m1 = cfg[0]; BM = cfg[1]; n1 = cfg[2]; BN = cfg[3]; ksteps = cfg[4]; BK = cfg[5];
        flagv = 1;
    } else if (op.kind == OPEVO_MATMUL || op.kind == OPEVO_BMM) {
        const int32_t *c = cfg;
        if (op.kind == OPEVO_BMM) { b1 = c[0]; binner = c[1]; c += 2; }
        m1 = c[0]; WM = c[1]; TM = int64_t(c[2]) * c[3]; FM = c[3];
        n1 = c[4]; WN = c[5]; TN = int64_t(c[6]) * c[7]; FN = c[7];
        if (variant == OPEVO_TILE4K) { ksplit = c[8]; b1 = ksplit; ksteps = c[9]; BK = c[10]; flagv = c[11]; }
        else { ksteps = c[8]; BK = c[9]; flagv = c[10]; }
        if (variant == OPEVO_TILE4T) bpack = c[11];
        if (variant == OPEVO_TILE4A) atom16 = c[11];
        BM = WM * TM; BN = WN * TN;
        tile4_width = int(c - cfg) + (variant == OPEVO_TILE4K || variant == OPEVO_TILE4T || variant == OPEVO_TILE4A ? 12 : 11);
    } else {   // conv: B(2) Cout(4) H(4) W(4) R(2) flag
        const int32_t *c = cfg;
        const int64_t nb1 = c[0]; nb2 = c[1];
        m1 = c[2]; WM = c[3]; TM = int64_t(c[4]) * c[5]; FM = c[5];
        const int32_t *h = c + 6, *w = c + 10;
        h1 = h[0]; w1 = w[0];
        BH = int64_t(h[1]) * h[2] * h[3]; BW = int64_t(w[1]) * w[2] * w[3];
        WN = int64_t(h[1]) * w[1];
        TN = nb2 * h[2] * h[3] * w[2] * w[3];
        FN = nb2 * h[3] * w[3];
        n1 = nb1 * h1 * w1;
        if (variant == OPEVO_TILE4P) {
            for (int j = 0; j < 6; ++j) box[j] = c[14 + j];
            ksteps = box[0] * box[2] * box[4];
            BK = box[1] * box[3] * box[5];
            flagv = c[20];
            kunroll = int64_t(kUnrollSteps[c[21]]);
            // a box that spans whole kernel rows (and whole kernel planes if it holds several
            // channels) is a contiguous run of the flattened reduction axis: the plain walk
            const bool contiguous = (box[5] == op.wk || (box[3] == 1 && box[1] == 1)) && (box[3] == op.hk || box[1] == 1);
            tap_box = !contiguous;
            tile4_width = 22;
        } else if (variant == OPEVO_TILE4C) {
            ksplit = c[14]; b1 = ksplit; ksteps = c[15]; BK = c[16]; flagv = c[17]; layout = c[18];
            tile4_width = 19;
        } else if (variant == OPEVO_TILE4L) {
            const int64_t taps = op.hk * op.wk;
            flagv = c[16];
            tile4_width = 19;
            if (c[17] == 1) { layout = 1; ksteps = taps * c[14]; BK = c[15]; }   // channels-last walk (r, s, ci): a slab is c[15] channels of one tap
            else { ksteps = c[14]; BK = c[15] * taps; }                          // walk (ci, r, s): a slab is c[15] channels with all their taps
            // layout 2: the LDS-resident patch, for members it can hold (the others run as with layout 0).
            // 32x32x16 atoms need slabs of whole 16 channels, 16x16x32 atoms of 32; the wave's pixel side is
            // rounded up to whole atoms while that at most doubles the work; the atom that wastes less is taken.
            // kwaves: that many waves share every wave tile and split the MFMA steps of a slab (taps x channel groups).
            // A member that asks for what the template has not is folded rather than sent away (same workgroup tile,
            // another division of it among the waves): slabs of fewer than 16 channels are merged, slabs too long for the
            // LDS halved; wave tiles of fewer than 16 output channels are merged along Cout; with more than 16 waves kwaves
            // is halved, then the waves along the pixels are merged a prime at a time (their tiles grow).
            if (c[17] == 2 && op.dtype != OPEVO_F32 && op.win >= 2 && op.b_elems() < (int64_t(1) << 30) && op.a_elems() < (int64_t(1) << 30)) {
                auto up = [](int64_t v, int64_t a) { return (v + a - 1) / a * a; };
                auto prime = [](int64_t n) { for (int64_t q = 2; q * q <= n; ++q) if (n % q == 0) return q; return n; };
                int64_t cs = c[15], tm = TM, wm = WM;
                while (cs % 16 != 0 && cs < op.cin) cs *= prime(op.cin / cs);
                // ... and slabs too long for the LDS (the kernel tensor's part holds all taps of a slab) are halved while they
                // stay whole 16 channels
                {
                    int64_t prow0 = 0, pimage0 = 0;
                    patch_pitches(op, BH, BW, false, prow0, pimage0);
                    auto stage_bytes = [&](int64_t v) { return (nb2 * pimage0 * (v + 8) + taps * WM * TM * v + 64) * 2; };
                    while (cs % 32 == 0 && stage_bytes(cs) * ((flagv && op.cin / cs > 1) ? 2 : 1) > kMaxLds) cs /= 2;
                }
                const int64_t slabs = op.cin / cs;
                const int64_t ph = (BH - 1) * op.stride + op.hk, pw = (BW - 1) * op.stride + op.wk;
                const int st = (flagv && slabs > 1) ? 2 : 1;
                // the padded pitches if the LDS has room for them, else the plain ones
                int64_t prow = 0, pimage = 0, lds_p = 0;
                for (int padded = 1; padded >= 0; --padded) {
                    patch_pitches(op, BH, BW, padded == 1, prow, pimage);
                    lds_p = st * (nb2 * pimage * (cs + 8) + taps * wm * tm * cs + 64) * 2;   // patch (padded pixels), kernel tensor's part, dump words
                    if (lds_p <= kMaxLds) break;
                }
                // the waves along Cout are merged, a prime at a time, until an atom fits the wave tile
                for (; !patch_cs; ) {
                    for (int64_t kw = int64_t(kReductionWaves[c[18]]); kw >= 1 && !patch_cs && tm % 16 == 0; kw /= 2) {
                        int64_t wn = WN, tn = TN;
                        while (wm * wn * kw > kMaxThreads / 64 && wn > 1) { const int64_t q = prime(wn); wn /= q; tn *= q; }
                        const int64_t nw = wm * wn * kw, nt = 64 * nw;
                        if (nt > kMaxThreads) continue;
                        auto fits = [&](int64_t at) {
                            return tm % at == 0 && cs % (at == 32 ? 16 : 32) == 0 && up(tn, at) <= 2 * tn && tm * up(tn, at) <= 64 * kMaxAcc;
                        };
                        const int at = fits(32) && (!fits(16) || up(tn, 32) == up(tn, 16)) ? 32 : fits(16) ? 16 : 0;
                        if (!at || kw > taps * (cs / (at == 32 ? 16 : 32))) continue;   // no atom fits; more waves than steps
                        // the fill: per thread, tasks of two channels x two pixels (images one pixel wide, which the template would fill pixel by pixel, stay with layout 0) and of two channels x all taps (kernel tensor)
                        const int64_t fill_p = (cs / 2 * (op.win >= 2 ? pw / 2 + 1 : pw) * ph * nb2 + nt - 1) / nt, fill_a = (wm * tm * cs / 2 + nt - 1) / nt;
                        // Registers: a lane has 512 / (waves per SIMD).  Counted: the accumulators, two sets of fragments (4 per
                        // atom row and column; three sets for small wave tiles), the fill (3 + 2 per image task, 2 + taps per
                        // kernel-tensor task: plan + data in flight), 24 for addresses, and where waves share a tile 40 + three
                        // quarters of the accumulators again (the final sum moves them through ordinary registers).  An eighth
                        // over is let through: the compiler fits such members.  Calibrated on compiled members: of 150 random
                        // eligible ones the rule lets no spilling member through and turns away 3 that would have fitted; a
                        // member that spills all the same is refused when its kernel is loaded.
                        const int64_t fill = 5 * fill_p + (2 + taps) * fill_a;
                        const int64_t accs = tm * up(tn, at) / 64;
                        const int64_t frags = tm / at + up(tn, at) / at;
                        const int64_t need = accs + (frags <= 3 ? 12 : 8) * frags + 24 + fill + (kw > 1 ? 40 + accs * 3 / 4 : 0);
                        const int64_t have = 512 / ((nw + 3) / 4);
                        // adding the partial sums of kw waves needs room for one atom of every wave
                        const int64_t lds_r = kw > 1 ? nw * (at == 32 ? 4 : 1) * 1024 : 0;
                        if (lds_p <= kMaxLds && lds_r <= kMaxLds && need <= have + have / 8) {
                            patch_cs = cs; patch_atom = at; patch_stages = st; patch_row = prow; patch_image = pimage; patch_kw = int(kw);
                            // the member as the template runs it
                            WM = wm; TM = tm; WN = wn; TN = tn; FM = std::gcd(FM, TM); FN = std::gcd(FN, TN);
                            ksteps = slabs; BK = cs * taps;
                        }
                    }
                    if (wm == 1) break;
                    const int64_t q = prime(wm); wm /= q; tm *= q;
                }
            }
        } else {
            ksteps = c[14]; BK = c[15]; flagv = c[16];
            tile4_width = 17;
        }
        BM = WM * TM; BN = WN * TN;
    }
    // ---- members that ask for more than a workgroup has are folded into serial work instead of scoring 0
    // (the search then sees a slow member with its own place in the landscape, not a hole; Sec. 4.2 keeps
    // zero fitness for what cannot run at all):
    //  * a per-wave tile that needs more than 256 accumulators per lane (or, for a member with more than
    //    16 waves, more than its occupancy leaves) is cut along its longer side (a prime at a time) into
    //    sub-tiles, each of which becomes the tile of a wave of its own;
    //  * a reduction slab too long for the LDS is halved (twice as many steps) while it stays a
    //    multiple of 32;
    //  * more than 16 waves (below): the workgroup runs the largest divisor of their number that fits,
    //    and every real wave takes the tiles of several waves one after another, each with the whole K loop.
    if (four_level && !patch_cs) {
        auto smallest_prime = [](int64_t n) { for (int64_t q = 2; q * q <= n; ++q) if (n % q == 0) return q; return n; };
        // The registers a lane may use depend on how many waves share a SIMD (512 for one, 256 for two,
        // 128 for four): a member that is folded anyway gets wave tiles that leave room for fragments
        // and staging next to the accumulators at the occupancy it will run at.
        auto real_waves = [&](int64_t v) { for (int64_t dv = kMaxThreads / 64; dv > 1; --dv) if (v % dv == 0) return dv; return int64_t(1); };
        auto acc_cap = [&]() {
            const int64_t per_simd = (real_waves(WM * WN) + 3) / 4;
            return std::min<int64_t>(kMaxAcc, 512 / per_simd / 2 - 8);   // half the registers: the other half holds two slabs in flight and the fragments
        };
        const bool refold = TM * TN > 64 * kMaxAcc || WM * WN > kMaxThreads / 64;
        while (refold && TM * TN > 64 * acc_cap() && TM * TN > 1) {
            const bool cut_m = (TM >= TN && TM > 1) || TN == 1;
            int64_t &T = cut_m ? TM : TN, &W = cut_m ? WM : WN, &F = cut_m ? FM : FN;
            const int64_t q = smallest_prime(T);
            T /= q; W *= q;
            F = std::gcd(F, T);
        }
        //  * a workgroup tile too large for the LDS even with the shortest slab (or, on the scalar template,
        //    for 1024 threads with 256 outputs each) is cut, a prime at a time along its longer side, into
        //    sub-tiles that the workgroup computes one after another (SUBM x SUBN of them).
        const int elem = op.dtype == OPEVO_F32 ? 4 : 2;
        const int stages = (flagv && ksteps > 1) ? 2 : 1;
        auto lds_need = [&]() { return (BM + BN) * std::max<int64_t>((BK + kPad) * elem * stages, BK * 4); };
        const int64_t lds_cap = kMaxLds - 16;   // room for the deadline flag word of folded members
        // (TILE4L's gather members walk (ci, r, s) in slabs of whole channels with all their taps, rarely a multiple of 64:
        // there a slab too long is divided by its smallest prime factor; the gather pads any slab to the MFMA step)
        if (variant == OPEVO_TILE4L && layout != 1)
            while (lds_need() > lds_cap && BK > 32) { const int64_t q = smallest_prime(BK); BK /= q; ksteps *= q; }
        while (lds_need() > lds_cap && BK % 64 == 0 && !tap_box) { BK /= 2; ksteps *= 2; }
        // (the scalar template: 1024 threads have 128 registers per lane each; 16 outputs per thread fit with its unrolled loop)
        const int64_t out_cap = BM * BN > int64_t(kMaxThreads) * kMaxAcc ? int64_t(kMaxThreads) * 16 : INT64_MAX;
        while (lds_need() > lds_cap || BM * BN > out_cap) {
            // a convolution's column block is a box of pixels: only its channel side is cut
            const bool cut_m = op.kind == OPEVO_CONV2D || BM >= BN;
            int64_t &W = cut_m ? WM : WN, &T = cut_m ? TM : TN, &F = cut_m ? FM : FN, &S = cut_m ? subm : subn;
            if (W * T == 1) break;
            if (W > 1) { const int64_t q = smallest_prime(W); W /= q; S *= q; }
            else { const int64_t q = smallest_prime(T); T /= q; S *= q; F = std::gcd(F, T); }
            BM = WM * TM; BN = WN * TN;
        }
    }
    // extended variant: launch order and group width
    const bool linear = (variant == OPEVO_TILE4X);
    int order[3] = {0, 1, 2};
    int64_t group = 1;
    if (linear) {
        const int n_axes = op.kind == OPEVO_BMM ? 3 : 2;
        for (int j = 0; j < n_axes; ++j) order[j] = cfg[tile4_width + j];
        group = int64_t(kGroupValues[cfg[tile4_width + n_axes]]);
    }

    // ---- template choice
    int path = 0;   // scalar
    int64_t BKP = BK;   // width of a K slab as the MFMA template stages and multiplies it
    int64_t TMacc = TM, TNacc = TN;   // wave tile in whole atoms (accumulator registers)
    bool ragged = false;
    // Channels-last operands (TILE4C, layout = 1) need 8-value pieces that never straddle a tap (Cin and
    // the LDS tile multiples of 8) and byte offsets into the image that fit 32 bits; they exist on the
    // MFMA templates only.  Elsewhere the choice is inert and the member runs as with layout = 0.
    const bool nhwc_ok = layout == 1 && op.kind == OPEVO_CONV2D && op.dtype != OPEVO_F32 && op.cin % 8 == 0 &&
                         BK % 8 == 0 && op.b_elems() * 2 + 256 < (int64_t(1) << 32) &&
                         op.hin + 2 * op.pad + op.hk < 32768 && op.win + 2 * op.pad + op.wk < 32768;   // coordinates in 15 bits
    int nstage_dlds = 0;
    bool dlds_atom16 = false;
    int64_t bnr = BN;   // rows of the second operand's stage part on the direct-to-LDS template when it is K-contiguous
    int64_t anr = BM;   // rows of the first operand's stage part there
    // Direct global->LDS streaming (path 3) of a pipelined member whose slabs split into whole 1 KiB wave
    // loads: `rows_b` rows of BK K-contiguous elements for the second operand (0: it is stored [K][N]).
    auto dlds_stages = [&](int64_t rows_a, int64_t rows_b, bool a_km_rows, bool atoms16 = false) -> int {
        const int64_t nw = WM * WN;
        if (subm * subn > 1) return 0;   // folded members stay on the register-staged template
        if (64 * nw > kMaxThreads || !(BK == 32 || BK == 64 || BK == 128)) return 0;
        const int64_t a_bytes = rows_a * BK * 2, b_bytes = (rows_b ? rows_b : BN) * BK * 2;
        if (a_bytes % (1024 * nw) != 0 || b_bytes % (1024 * nw) != 0) return 0;
        if (!rows_b && !(BN % 128 == 0 || BN == 64 || BN == 32)) return 0;
        if (a_km_rows && !(BM % 128 == 0 || BM == 64 || BM == 32)) return 0;   // A rows are M-contiguous then
        const int64_t per = (a_bytes + b_bytes) / (1024 * nw);
        int st_found = 0;
        for (int st = 4; st >= 2; --st)
            if (st * (a_bytes + b_bytes) <= kMaxLds && (st - 2) * per <= 63) { st_found = st; break; }
        if (!st_found) return 0;
        // The template keeps accumulators and fragments in register arrays and relies on its K
        // loop body (one pass over the ring) unrolling completely.  Instructions in that body:
        // per stage and MFMA step the MFMAs and fragment reads, per stage the loads.  Bodies
        // past this size were seen not to unroll (code objects of 0.5-1.5 MB instead of 20 KB);
        // such members use the register-staged template instead.
        const int64_t at = atoms16 ? 16 : 32;
        const int64_t mi = TM / at, ni = (TN + at - 1) / at, kk = BK / (atoms16 ? 32 : 16);
        const int64_t body = st_found * (kk * (mi * ni + (op.trans_a ? 2 : 1) * mi + (rows_b ? 1 : 2) * ni) + per);
        // 16x16x32 atoms: twice the MFMAs for the same tile; such bodies (up to 128 x 128 wave tiles on slabs of 32)
        // were checked to unroll (code objects of about 30 KiB)
        return body > (atoms16 ? kMaxDldsBody16 : kMaxDldsBody) ? 0 : st_found;
    };
    if (four_level && op.dtype != OPEVO_F32) {
        if (op.kind == OPEVO_CONV2D) {
            // The convolution's reduction axis Cin*Hk*Wk rarely has a factor 16 (3*11*11 = 363): a slab
            // of BK taps is staged zero-padded to the next multiple of the MFMA K step, and its
            // operands are gathered element by element, so no alignment is asked of it.
            // Likewise a wave tile that is no multiple of 16 is rounded up to whole 16x16 atoms as long
            // as that at most doubles the work (pixel tiles come from factors of 55, 27, ...).
            const int64_t TMp = (TM + 15) / 16 * 16, TNp = (TN + 15) / 16 * 16;
            if (TM % 32 == 0 && TN % 32 == 0) { path = 1; BKP = (BK + 15) / 16 * 16; }
            else if (TMp * TNp <= 2 * TM * TN) { path = 2; BKP = (BK + 31) / 32 * 32; ragged = (TMp != TM || TNp != TN); TMacc = TMp; TNacc = TNp; }
            // channels-last, pipelined, wave tiles of whole 32-row atoms whose pixel side rounds up to 32
            // without doubling the work: the direct-to-LDS template with a K-contiguous second operand
            const int64_t TN32 = (TN + 31) / 32 * 32;
            if (nhwc_ok && flagv == 1 && TM % 32 == 0 && TN32 <= 2 * TN && TM * TN32 / 64 <= kMaxAcc) {
                const int64_t nw = WM * WN;
                // rows staged: every pixel of the box and every row a wave's last atom reads, rounded up
                // until the part splits into whole 1 KiB loads per wave
                int64_t rows = std::max(BN, (WN - 1) * TN + TN32), rows_a = BM;
                if (BK == 32 || BK == 64 || BK == 128) {
                    const int64_t unit = 1024 * nw / std::gcd(int64_t(1024) * nw, BK * 2);
                    rows = (rows + unit - 1) / unit * unit;
                    rows_a = (rows_a + unit - 1) / unit * unit;
                    if (rows * BK * 2 / (1024 * nw) <= 16 && rows_a * BK * 2 / (1024 * nw) <= 16)
                        nstage_dlds = dlds_stages(rows_a, rows, false);
                }
                if (nstage_dlds) { path = 3; bnr = rows; anr = rows_a; BKP = BK; ragged = false; TMacc = TM; TNacc = TN32; }
            }
        } else {
            const bool align_ok = (op.K % 8 == 0) && (op.N % 8 == 0);
            if (align_ok && TM % 32 == 0 && TN % 32 == 0 && BK % 16 == 0) path = 1;
            else if (align_ok && TM % 16 == 0 && TN % 16 == 0 && BK % 32 == 0) path = 2;
        }
    }
    // fp32 inputs: 32x32x2 fp32 atoms (MatMul / BMM), both operands in 16-byte pieces along their
    // contiguous axis, K slabs in groups of 8
    if (four_level && op.dtype == OPEVO_F32 && op.kind != OPEVO_CONV2D && TM % 32 == 0 && TN % 32 == 0 &&
        BK % 8 == 0 && op.N % 4 == 0 && (op.trans_a ? op.M % 4 == 0 : op.K % 4 == 0))
        path = 4;
    // fp32 Conv2d: operands gathered value by value, so any slab length (staged padded to 8) and any
    // wave tile whose round-up to whole 32x32 atoms at most doubles the work
    if (four_level && op.dtype == OPEVO_F32 && op.kind == OPEVO_CONV2D) {
        const int64_t TMp = (TM + 31) / 32 * 32, TNp = (TN + 31) / 32 * 32;
        if (TMp * TNp <= 2 * TM * TN && op.b_elems() < (int64_t(1) << 31)) {
            path = 4; BKP = (BK + 7) / 8 * 8; TMacc = TMp; TNacc = TNp;
        }
    }
    if (patch_cs) { path = 5; BKP = BK; ragged = false; TMacc = TM; TNacc = (TN + patch_atom - 1) / patch_atom * patch_atom; }
    const bool stage_lds = path == 4 || !(op.kind == OPEVO_BMM && four_level && flagv == 0 && path != 0);
    // Direct global->LDS streaming (path 3) for pipelined MatMul / BMM members of 32x32 atoms whose
    // slabs split into whole 1 KiB wave loads and whose row lengths suit the chunk permutation.  With
    // bpack = 1 (TILE4T) the second operand is read from the [N][K] copy a pre-pass makes.
    const bool b_packed = bpack == 1 && op.kind == OPEVO_MATMUL && !op.trans_a;
    if (path == 1 && flagv == 1 && stage_lds && op.kind != OPEVO_CONV2D) {
        nstage_dlds = dlds_stages(BM, b_packed ? BN : 0, op.trans_a);
        if (nstage_dlds) path = 3;
        // TILE4A, atom = 1: the same member on 16x16x32 atoms (MatMul with row-major operands; a member whose body
        // would grow too long keeps the 32x32x16 atoms)
        if (nstage_dlds && atom16 == 1 && op.kind == OPEVO_MATMUL && !op.trans_a && !b_packed && BK % 32 == 0 &&
            dlds_stages(BM, 0, false, true) == nstage_dlds && (BK % 64 == 0 || nstage_dlds % 2 == 0))   // one K step per slab: an even ring
            dlds_atom16 = true;
    }
    const bool b_kmajor = path == 3 && (b_packed || op.kind == OPEVO_CONV2D);
    const bool nhwc = nhwc_ok && (path == 1 || path == 2 || path == 3);
    // a transposed first operand is staged by the MFMA templates like B (rows of 8 along M), so it
    // needs M % 8 == 0 and LDS staging; other members run on the scalar template
    if (op.trans_a && (path == 1 || path == 2) && (op.M % 8 != 0 || !stage_lds)) path = 0;

    int64_t NT, nwr = WM * WN * patch_kw;   // nwr: waves the workgroup really runs
    if (four_level) {
        if (path == 0) nwr = std::min<int64_t>(nwr, kMaxThreads / 64);   // the scalar template deals outputs round-robin to any number of threads
        else while (path != 5 && nwr > kMaxThreads / 64) {      // largest divisor of WM * WN that fits
            int64_t best = 1;
            for (int64_t dv = kMaxThreads / 64; dv >= 1; --dv) if ((WM * WN) % dv == 0) { best = dv; break; }
            nwr = best;
        }
        NT = 64 * nwr;
    }
    else {
        NT = ((BM * BN + 63) / 64) * 64;
        if (NT > 256) NT = 256;
    }
    int64_t acc = (path == 0) ? (BM * BN + NT - 1) / NT : (TMacc * TNacc) / 64;
    const int nstage = path == 5 ? patch_stages : path == 3 ? nstage_dlds : (path != 0 && flagv && ksteps > 1) ? 2 : 1;
    int64_t lds = 0;
    if (path == 0) lds = (BM * BK + BK * BN) * 4;
    else if (path == 4 && op.kind == OPEVO_CONV2D) {
        const int64_t a_rows = (WM - 1) * TM + TMacc, b_cols = ((WN - 1) * TN + TNacc + 3) / 4 * 4;   // with the overhang
        lds = nstage * (a_rows * (BKP + 4) + BKP * (b_cols + 4)) * 4;
    }
    else if (path == 4) lds = nstage * ((op.trans_a ? BK * (BM + 4) : BM * (BK + 4)) + BK * (BN + 4)) * 4;
    else if (path == 3) lds = nstage * (anr + (b_kmajor ? bnr : BN)) * BK * 2;
    else if (path == 5)   // the stages, or (more than one wave per tile) one atom of every wave if that is more
        lds = std::max<int64_t>(nstage * (nb2 * patch_image * (patch_cs + 8) + op.hk * op.wk * BM * patch_cs + 64) * 2,
                                patch_kw > 1 ? nwr * (patch_atom == 32 ? 4 : 1) * 1024 : 0);
    else if (stage_lds) lds = nstage * (BM + BN) * (BKP + kPad) * 2 + (ragged ? 16 * (BKP + kPad) * 2 : 0);   // overhang rows stay inside the allocation

    p.path = path;
    const int64_t n_blocks = n1 * m1 * b1;
    if (linear) { p.grid[0] = int32_t(n_blocks > INT32_MAX ? INT32_MAX : n_blocks); p.grid[1] = 1; p.grid[2] = 1; }
    else { p.grid[0] = int32_t(n1); p.grid[1] = int32_t(m1); p.grid[2] = int32_t(b1); }
    p.block = int32_t(NT > INT32_MAX ? INT32_MAX : NT);
    p.lds_bytes = int32_t(lds > INT32_MAX ? INT32_MAX : lds);
    p.acc_per_lane = int32_t(acc > INT32_MAX ? INT32_MAX : acc);
    p.tile[0] = int32_t(BM); p.tile[1] = int32_t(BN); p.tile[2] = int32_t(BK);
    p.wave_tile[0] = int32_t(four_level ? TM : BM); p.wave_tile[1] = int32_t(four_level ? TN : BN);
    p.sub_tiles[0] = int32_t(subm); p.sub_tiles[1] = int32_t(subn);
    p.wave_passes = int32_t(four_level && nwr > 0 && path != 5 ? (WM * WN) / nwr : 1);

    // ---- black-box constraints made explicit: such members get fitness 0 (Sec. 4.2)
    if (NT > kMaxThreads) invalid(p, "%ld threads per workgroup > %ld", long(NT), long(kMaxThreads));
    else if (acc > kMaxAcc) invalid(p, "%ld accumulators per lane > %ld", long(acc), long(kMaxAcc));
    else if (lds + ((path == 0 || subm * subn * ((WM * WN) / std::max<int64_t>(nwr, 1)) > 1) ? 16 : 0) > kMaxLds)   // the deadline flag word of the scalar template and of folded members
        invalid(p, "%ld bytes of LDS > %ld", long(lds), long(kMaxLds));
    else if (!linear && (m1 > 65535 || b1 > 65535)) invalid(p, "grid y/z %ld x %ld > 65535", long(m1), long(b1));
    else if (linear && n_blocks > INT32_MAX) invalid(p, "%ld workgroups in a one-dimensional grid", long(n_blocks));
    else if (path == 4) {
        const int64_t chunks = op.kind == OPEVO_CONV2D ? (BM * (BKP / 4) + NT - 1) / NT + (BKP * ((BN + 3) / 4) + NT - 1) / NT
                                                       : (BM * (BK / 4) + NT - 1) / NT + (BK * (BN / 4) + NT - 1) / NT;
        if (chunks * 4 > 256) invalid(p, "%ld staging registers per lane > 256", long(chunks * 4));
    }
    else if (path != 0 && path != 3 && path != 5 && stage_lds) {
        // register budget of the slab in flight: 16-byte pieces per thread
        const int64_t a_chunks = op.trans_a ? 8 * (((BK / 8) * (BM / 8) + NT - 1) / NT) : (BM * (BKP / 8) + NT - 1) / NT;
        const int64_t b_chunks = (op.kind == OPEVO_CONV2D) ? (BN * (BKP / 8) + NT - 1) / NT
                                                           : 8 * (((BK / 8) * (BN / 8) + NT - 1) / NT);
        if ((a_chunks + b_chunks) * 4 > 256)
            invalid(p, "%ld staging registers per lane > 256", long((a_chunks + b_chunks) * 4));
    }

    out.tmpl = path == 0 ? "gemm_scalar" : path == 3 ? "gemm_mfma_dlds" : path == 4 ? "gemm_mfma_f32" : path == 5 ? "conv_patch" : "gemm_mfma";
    // one symbol per configuration, so profiles list each instantiated kernel on its own line
    {
        std::ostringstream nm;
        nm << "opevo_" << (op.kind == OPEVO_MATMUL ? "mm" : op.kind == OPEVO_BMM ? (op.trans_a ? "bmmt" : "bmm") : "conv")
           << (variant == OPEVO_TILE4P ? "p" : variant == OPEVO_TILE4K ? "k" : variant == OPEVO_TILE4C ? "c" : variant == OPEVO_TILE4T ? "t" : variant == OPEVO_TILE4A ? "a" : variant == OPEVO_TILE4L ? "l" : four_level ? "4" : "2");
        int width = 0;
        for (const auto &d : descs) width += d.type == OPEVO_FACTOR ? d.nu : d.type == OPEVO_PERMUTATION ? d.n_values : 1;
        for (int i = 0; i < width; ++i) nm << "_" << cfg[i];
        out.kernel_name = nm.str();
    }
    D << "-DKERNEL_NAME=" << out.kernel_name << " ";
    D << "-DOP=" << op.kind << " -DIN_DTYPE=" << op.dtype << " -DM=" << op.M << " -DN=" << op.N
      << " -DK=" << op.K << " -DBM=" << BM << " -DBN=" << BN << " -DBK=" << BK << " -DKSTEPS=" << ksteps
      << " -DNT=" << NT << " -DBATCH_INNER=" << binner << " -DFLAG=" << flagv << " -DA_TRANS=" << (op.trans_a ? 1 : 0);
    if (path != 0) {
        D << " -DATOM=" << (path == 5 ? patch_atom : (path == 2 || dlds_atom16) ? 16 : 32) << " -DWM=" << WM << " -DWN=" << WN << " -DTM=" << TM
          << " -DTN=" << TN << " -DFM=" << FM << " -DFN=" << FN << " -DPAD=" << kPad
          << " -DNSTAGE=" << nstage << " -DNSTG=" << nstage << " -DSTAGE_LDS=" << (stage_lds ? 1 : 0);
        if (nwr != WM * WN && path != 5) D << " -DNWR=" << nwr;
    }
    if (subm * subn > 1) {
        D << " -DSUBM=" << subm << " -DSUBN=" << subn;
    }
    if (op.kind == OPEVO_CONV2D) {
        D << " -DCIN=" << op.cin << " -DHIN=" << op.hin << " -DWIN=" << op.win << " -DHK=" << op.hk
          << " -DWK=" << op.wk << " -DSTRIDE=" << op.stride << " -DPAD_CONV=" << op.pad
          << " -DHOUT=" << op.hout << " -DWOUT=" << op.wout << " -DNB2=" << nb2 << " -DBH=" << BH
          << " -DBW=" << BW << " -DH1=" << h1 << " -DW1=" << w1 << " -DBKP=" << BKP;
        // the MFMA template gathers the image through a compile-time table of tap offsets where its
        // fields are wide enough (byte offsets into the image tensor in 32 bits, padded image
        // coordinates in 15) and the table stays small (8 bytes per position of the reduction walk)
        const bool table = path != 0 && op.b_elems() < (int64_t(1) << 31) && op.hin + 2 * op.pad < 32768 &&
                           op.win + 2 * op.pad < 32768 && op.hk < 32768 && op.wk < 32768 && ksplit * ksteps * BKP <= 8192 && !nhwc;
        if (path != 0) D << " -DCONV_TABLE=" << (table ? 1 : 0);
        if (nhwc) D << " -DCONV_NHWC=1";
    }
    if (tap_box)
        D << " -DTAP_BOX=1 -DCI_O=" << box[0] << " -DCI_I=" << box[1] << " -DHK_O=" << box[2] << " -DHK_I=" << box[3]
          << " -DWK_O=" << box[4] << " -DWK_I=" << box[5];
    if (path == 5) D << " -DCS=" << patch_cs << " -DPWP=" << patch_row << " -DIPIX=" << patch_image << " -DKW=" << patch_kw << " -DLDS_BYTES=" << lds;
    if (b_kmajor) D << " -DB_KMAJOR=1 -DBNR=" << bnr;
    if (path == 3 && anr != BM) D << " -DANR=" << anr;
    if (kunroll) D << " -DKUNROLL=" << kunroll;
    if (ksplit > 1) D << " -DKSPLIT=" << ksplit;
    out.zero_bytes = ksplit > 1 ? op.c_elems() * 4 : 0;
    out.prepass = nhwc ? 1 : (b_kmajor && op.kind == OPEVO_MATMUL) ? 2 : 0;
    if (linear)
        D << " -DGRID_LINEAR=1 -DGRID_N1=" << n1 << " -DGRID_M1=" << m1 << " -DGRID_B1=" << b1 << " -DORDER0=" << order[0]
          << " -DORDER1=" << order[1] << " -DORDER2=" << order[2] << " -DGROUP=" << group;
    out.defines = D.str();
    return OPEVO_OK;
}

}  // namespace opevo

extern "C" {

int opevo_op_create(int kind, const int64_t *dims, int n_dims, int in_dtype, opevo_op **out)
{
    if (!dims || !out) return fail(OPEVO_E_ARG, "op_create: NULL argument");
    if (in_dtype < OPEVO_F32 || in_dtype > OPEVO_F16) return fail(OPEVO_E_ARG, "op_create: unknown dtype %d", in_dtype);
    opevo_op op;
    if (kind == OPEVO_BMM_TA) { kind = OPEVO_BMM; op.trans_a = true; }
    op.kind = kind; op.dtype = in_dtype;
    const int need = kind == OPEVO_MATMUL ? 3 : kind == OPEVO_BMM ? 4 : kind == OPEVO_CONV2D ? 9 : -1;
    if (need < 0) return fail(OPEVO_E_ARG, "op_create: unknown operator kind %d", kind);
    if (n_dims != need) return fail(OPEVO_E_ARG, "op_create: operator needs %d dims, got %d", need, n_dims);
    for (int i = 0; i < n_dims; ++i) {
        const bool may_be_zero = (kind == OPEVO_CONV2D && i == 8);   // padding
        if (dims[i] < (may_be_zero ? 0 : 1) || dims[i] > (int64_t(1) << 30))
            return fail(OPEVO_E_ARG, "op_create: dims[%d] = %lld out of range", i, (long long)dims[i]);
    }
    if (kind == OPEVO_MATMUL) { op.M = dims[0]; op.N = dims[1]; op.K = dims[2]; }
    else if (kind == OPEVO_BMM) { op.batch = dims[0]; op.M = dims[1]; op.N = dims[2]; op.K = dims[3]; }
    else {
        op.nimg = dims[0]; op.cin = dims[1]; op.hin = dims[2]; op.win = dims[3];
        op.M = dims[4]; op.hk = dims[5]; op.wk = dims[6]; op.stride = dims[7]; op.pad = dims[8];
        const int64_t sh = op.hin + 2 * op.pad - op.hk, sw = op.win + 2 * op.pad - op.wk;
        if (sh < 0 || sw < 0) return fail(OPEVO_E_ARG, "op_create: kernel larger than the padded image");
        op.hout = sh / op.stride + 1;    // App. B.3
        op.wout = sw / op.stride + 1;
        op.K = op.cin * op.hk * op.wk;
        op.N = op.nimg * op.hout * op.wout;
    }
    if (double(op.batch) * double(op.M) * double(op.N) > 4.0e18 || op.a_elems() < 0 || op.b_elems() < 0)
        return fail(OPEVO_E_ARG, "op_create: tensor too large");
    *out = new (std::nothrow) opevo_op(op);
    return *out ? OPEVO_OK : fail(OPEVO_E_ARG, "out of memory");
}

int opevo_op_destroy(opevo_op *op) { delete op; return OPEVO_OK; }

int opevo_op_flops(const opevo_op *op, double *flops)
{
    if (!op || !flops) return fail(OPEVO_E_ARG, "op_flops: NULL argument");
    *flops = op->flops();
    return OPEVO_OK;
}

int opevo_op_bytes(const opevo_op *op, double *bytes)
{
    if (!op || !bytes) return fail(OPEVO_E_ARG, "op_bytes: NULL argument");
    *bytes = double(op->a_elems() + op->b_elems()) * op->elem_size() + double(op->c_elems()) * 4.0;
    return OPEVO_OK;
}

int opevo_op_sizes(const opevo_op *op, int64_t *a_elems, int64_t *b_elems, int64_t *c_elems)
{
    if (!op) return fail(OPEVO_E_ARG, "op_sizes: NULL argument");
    if (a_elems) *a_elems = op->a_elems();
    if (b_elems) *b_elems = op->b_elems();
    if (c_elems) *c_elems = op->c_elems();
    return OPEVO_OK;
}

int opevo_op_space(const opevo_op *op, int variant, opevo_space **out)
{
    if (!op || !out) return fail(OPEVO_E_ARG, "op_space: NULL argument");
    std::vector<opevo_param_desc> descs;
    if (int rc = op_param_descs(*op, variant, descs)) return rc;
    return opevo_space_create(descs.data(), int(descs.size()), out);
}

int opevo_kernel_plan(const opevo_op *op, int variant, const int32_t *cfg, opevo_plan *plan)
{
    if (!op || !cfg || !plan) return fail(OPEVO_E_ARG, "kernel_plan: NULL argument");
    Decoded d;
    if (int rc = decode(*op, variant, cfg, d)) return rc;
    *plan = d.plan;
    return OPEVO_OK;
}

int opevo_kernel_defines(const opevo_op *op, int variant, const int32_t *cfg, char *buf, size_t cap)
{
    if (!op || !cfg || !buf) return fail(OPEVO_E_ARG, "kernel_defines: NULL argument");
    Decoded d;
    if (int rc = decode(*op, variant, cfg, d)) return rc;
    const std::string s = d.tmpl + ": " + d.defines;
    if (s.size() + 1 > cap) return fail(OPEVO_E_ARG, "kernel_defines: buffer too small (%zu needed)", s.size() + 1);
    std::memcpy(buf, s.c_str(), s.size() + 1);
    return OPEVO_OK;
}

}  // extern "C"
