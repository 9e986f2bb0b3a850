"""CPU re-computation of the LDS-resident-patch Conv2d template (csrc/templates/conv_patch.hip).

The template's index arithmetic is written out again here, thread by thread, from the constants the decoder
hands it: which global bytes every thread loads for every slab, where it puts each value in LDS, which LDS
bytes every lane reads for every fragment, and which output element every accumulator is stored to.  Checked:
every global access lies inside its tensor and is aligned to its width, every LDS access lies inside the
stage, the fill writes every in-image patch position and every kernel-tensor value exactly once (and nothing
else but the dump words), and the sum the fragments form is the convolution (small shapes: compared with a
direct convolution written with independent index arithmetic; exact on integer data).
No GPU is needed: nothing is launched."""
import re

import numpy as np
import pytest

import paper_2006_05664_amd as P

V = P.OPEVO_TILE4L


def defines(op, cfg):
    text = P.opevo_kernel_defines(op, V, cfg)
    tmpl, rest = text.split(":", 1)
    out = {}
    for tok in rest.split():
        m = re.match(r"-D(\w+)=(-?\d+)$", tok)
        if m:
            out[m.group(1)] = int(m.group(2))
    return tmpl.strip(), out


def emulate(dims, cfg, img=None, ker=None, blocks=None):
    """Re-computes the kernel for the given workgroups (all by default).  Returns the output tensor if operands are given."""
    nimg, cin, hin, win, cout, hk, wk, stride, pad = dims
    op = P.opevo_op_create(P.OPEVO_CONV2D, dims, P.OPEVO_BF16)
    plan = P.opevo_kernel_plan(op, V, cfg)
    tmpl, D = defines(op, cfg)
    assert plan.status == 0 and plan.path == 5 and tmpl == "conv_patch", (plan.status, plan.path, tmpl, plan.reason)
    g = D.__getitem__
    M, K, BM, BK, KSTEPS, NT = g("M"), g("K"), g("BM"), g("BK"), g("KSTEPS"), g("NT")
    ATOM, WM, WN, TM, TN, NSTG, CS = g("ATOM"), g("WM"), g("WN"), g("TM"), g("TN"), g("NSTG"), g("CS")
    CIN, HIN, WIN, HK, WK, S, PAD = g("CIN"), g("HIN"), g("WIN"), g("HK"), g("WK"), g("STRIDE"), g("PAD_CONV")
    HOUT, WOUT, NB2, BH, BW, H1, W1 = g("HOUT"), g("WOUT"), g("NB2"), g("BH"), g("BW"), g("H1"), g("W1")
    assert (CIN, HIN, WIN, HK, WK, S, PAD, M) == (cin, hin, win, hk, wk, stride, pad, cout)
    T = HK * WK
    PH, PW = (BH - 1) * S + HK, (BW - 1) * S + WK
    PWP, IPIX, KW, LDS_BYTES = g("PWP"), g("IPIX"), g("KW"), g("LDS_BYTES")
    assert PWP >= PW and IPIX >= PH * PWP
    NPIX = NB2 * IPIX
    PITCH, DUMP = CS + 8, 64
    P_STAGE, A_STAGE = NPIX * PITCH, T * BM * CS
    NCH = CS // 8

    def a_swz(row):    # chunk permutation of a row of the kernel tensor's part
        return 0 * row if NCH & (NCH - 1) else ((row * NCH // 16) % NCH if NCH <= 16 else row % 16)
    STAGE = P_STAGE + A_STAGE + DUMP
    KA = 16 if ATOM == 32 else 32
    NACC = 16 if ATOM == 32 else 4
    MI, NI, KK = TM // ATOM, (TN + ATOM - 1) // ATOM, CS // KA
    assert TM % ATOM == 0 and CS % KA == 0 and BK == CS * T and KSTEPS * CS == CIN and K == CIN * T
    ALIGNED = WIN % 2 == 0
    PAIRED = ALIGNED or WIN >= 3     # odd widths: the same pairs, loads 2-byte aligned, a row's last pixel loaded from one pixel to the left
    assert NSTG * STAGE * 2 <= LDS_BYTES == plan.lds_bytes <= 160 * 1024
    assert NT == 64 * WM * WN * KW == plan.block <= 1024 and BM == WM * TM and WN * TN == NB2 * BH * BW
    assert 1 <= KW <= T * (CS // (16 if ATOM == 32 else 32))
    assert MI * NI * NACC == plan.acc_per_lane <= 256
    CP = CS // 2
    NPAIR = PW // 2 + 1 if PAIRED else PW
    P_TASKS = CP * NPAIR * PH * NB2
    NPT = (P_TASKS + NT - 1) // NT
    A_TASKS = BM * CP
    NAT = (A_TASKS + NT - 1) // NT
    img_bytes, ker_bytes = nimg * cin * hin * win * 2, cout * K * 2
    grid = list(plan.grid)
    assert grid[0] * NB2 * BH * BW == nimg * HOUT * WOUT and grid[1] * BM == M and grid[2] == 1
    have = img is not None
    out = np.full((nimg, cout, HOUT, WOUT), np.nan) if have else None
    written = np.zeros((nimg, cout, HOUT, WOUT), dtype=np.int32)
    if blocks is None:
        blocks = [(bx, by) for bx in range(grid[0]) for by in range(grid[1])]
    if have:
        img_flat, ker_flat = img.reshape(-1), ker.reshape(-1)
    for bx, by in blocks:
        x0, y0, nb0 = (bx % W1) * BW, ((bx // W1) % H1) * BH, (bx // (W1 * H1)) * NB2
        m0 = by * BM
        yin0, xin0 = y0 * S - PAD, x0 * S - PAD
        xs = xin0 & ~1
        # ---- the fill plan of every thread
        tid = np.arange(NT)
        pg, pd0, pd1 = [], [], []
        for i in range(NPT):
            q = tid + i * NT
            PAIRS = NPAIR * PH * NB2
            pr, cp = (q // 4) % PAIRS, q // (4 * PAIRS) * 4 + q % 4
            jp, py, b = pr % NPAIR, (pr // NPAIR) % PH, pr // (NPAIR * PH)
            y, x = yin0 + py, (xs + 2 * jp if PAIRED else xin0 + jp)
            px = x - xin0
            inside = (q < P_TASKS) & (y >= 0) & (y < HIN) & (x >= 0) & (x < WIN)
            v0 = inside & (px >= 0) & (px < PW)
            v1 = inside & (px + 1 >= 0) & (px + 1 < PW) & PAIRED & (ALIGNED | (x + 1 < WIN))
            left = np.where((x == WIN - 1) & PAIRED & (not ALIGNED), 1, 0)
            goff = np.where(v0 | v1, 2 * ((((nb0 + b) * CIN + 2 * cp) * HIN + y) * WIN + x - left) | left, 0)
            d0 = ((b * IPIX + py * PWP + px) * PITCH) // 2 + cp      # 4-byte words
            dump = (STAGE - DUMP) // 2 + (tid & 31)
            pg.append(goff); pd0.append(np.where(v0, d0, dump)); pd1.append(np.where(v1, d0 + PITCH // 2, dump))
        ag, ad, aon = [], [], []
        for i in range(NAT):
            q = tid + i * NT
            cp, m = q % CP, q // CP
            on = q < A_TASKS
            ag.append(np.where(on, 2 * ((m0 + m) * K + 2 * cp * T), 0)); ad.append(m * (CS // 2) + (((cp >> 2) ^ a_swz(m)) << 2) + (cp & 3)); aon.append(on)
        # ---- bounds and alignment of every global load, for every slab
        for s in range(KSTEPS):
            for i in range(NPT):
                for ch in range(2):
                    o = 2 * s * CS * HIN * WIN + (pg[i] & ~1) + ch * 2 * HIN * WIN
                    width, align = (4 if PAIRED else 2), (4 if ALIGNED else 2)
                    assert ALIGNED or PAIRED or (pg[i] & 1 == 0).all()
                    assert (o >= 0).all() and (o + width <= img_bytes).all() and (o % align == 0).all(), ("image load", bx, by, s, i)
                    # a 4-byte load stays inside its row of the image: a pair never reaches into the next row (or past the tensor)
                    assert not PAIRED or ((o // 2) % WIN + 1 < WIN).all(), ("pair across a row end", bx, by, s, i)
            for i in range(NAT):
                for t in range(T):
                    o = 2 * s * CS * T + ag[i] + 4 * t
                    assert (o >= 0).all() and (o + 4 <= ker_bytes).all() and (o % 4 == 0).all(), ("kernel-tensor load", bx, by, s, i)
        # ---- the LDS stores of one slab: destinations and what lands there (the plan is the same for every slab)
        src = np.full(STAGE, -1, dtype=np.int64)   # which global element (of slab 0) each LDS element receives; -1: never written (zeros)
        hits = np.zeros(STAGE, dtype=np.int32)
        for i in range(NPT):
            for dst, e in (((pd0[i], 0), (pd1[i], 1)) if PAIRED else ((pd0[i], 0),)):   # word of pixel e: low half = first channel, high half = second
                assert (dst >= 0).all() and (2 * dst + 1 < STAGE).all(), ("patch store", bx, by, i)
                real = 2 * dst < STAGE - DUMP
                assert (2 * dst[real] + 1 < P_STAGE).all()
                for ch in range(2):
                    np.add.at(hits, 2 * dst[real] + ch, 1)
                    src[2 * dst[real] + ch] = (pg[i][real] & ~1) // 2 + ch * HIN * WIN + e + (pg[i][real] & 1)
        asrc = np.full(STAGE, -1, dtype=np.int64)
        for i in range(NAT):
            for t in range(T):
                dd = P_STAGE + 2 * (ad[i][aon[i]] + t * (BM * CS // 2))
                assert (dd >= P_STAGE).all() and (dd + 1 < P_STAGE + A_STAGE).all(), ("kernel-tensor store", bx, by, i, t)
                for ch in range(2):                            # value t of the run of 2*T, value T + t
                    np.add.at(hits, dd + ch, 1)
                    asrc[dd + ch] = ag[i][aon[i]] // 2 + ch * T + t
        assert hits.max() <= 1, "an LDS element is written twice in one slab"
        # coverage: every patch position inside the image, every channel of the slab; every kernel-tensor value
        for b in range(NB2):
            for py in range(PH):
                for px in range(PWP):
                    y, x = yin0 + py, xin0 + px
                    base = (b * IPIX + py * PWP + px) * PITCH
                    if 0 <= y < HIN and 0 <= x < WIN and px < PW:
                        want = (((nb0 + b) * CIN + np.arange(CS)) * HIN + y) * WIN + x
                        assert (src[base:base + CS] == want).all(), ("patch position", bx, by, b, py, px)
                    else:
                        assert (hits[base:base + CS] == 0).all(), ("padding position written", bx, by, b, py, px)
                    assert (hits[base + CS:base + PITCH] == 0).all()
        for tap in range(T):
            for m in range(BM):
                base = P_STAGE + (tap * BM + m) * CS
                ch = np.arange(CS)
                want = (m0 + m) * K + ch * T + tap
                where = base + (((ch >> 3) ^ int(a_swz(m))) << 3) + (ch & 7)     # channel ch sits in chunk (ch / 8) ^ a_swz(m)
                assert (asrc[where] == want).all(), ("kernel-tensor value", bx, by, tap, m)
        # ---- fragments: every lane's reads, and (with operands) the sum they form.  Wave = (wk, wm, wn): the KW waves of a
        # tile take the MFMA steps t = tap * KK + kk with t % KW == wk; their partial sums are added in the epilogue.
        lane = np.arange(64)
        lrow, lk = lane % ATOM, (lane // ATOM) * 8
        STEPS = T * KK
        for wmn in range(WM * WN):
            wm, wn = wmn // WN, wmn % WN
            a_row, a_chunk, a_perm = (wm * TM + lrow) * CS, lane // ATOM, a_swz(lrow)
            for j in range(NI):
                ct = j * ATOM + lrow
                cn = wn * TN + np.minimum(ct, TN - 1)
                b, y, x = cn // (BH * BW), (cn // BW) % BH, cn % BW
                b_lane = (b * IPIX + y * S * PWP + x * S) * PITCH + lk
                for i in range(MI):
                    accv = np.zeros((ATOM, ATOM)) if have else None   # [row][column], summed over the KW waves
                    steps_done = np.zeros(STEPS, dtype=np.int32)
                    for wk in range(KW):
                        for t in range(wk, STEPS, KW):
                            steps_done[t] += 1
                            tap, kk = t // KK, t % KK
                            r, sx = tap // WK, tap % WK
                            ao = P_STAGE + a_row + (((kk * (KA // 8) + a_chunk) ^ a_perm) << 3) + (tap * BM + i * ATOM) * CS
                            bo = b_lane + (r * PWP + sx) * PITCH + kk * KA
                            assert (ao % 8 == 0).all() and (bo % 8 == 0).all()
                            assert (ao >= P_STAGE).all() and (ao + 8 <= P_STAGE + A_STAGE).all(), "A fragment outside its part"
                            assert (bo >= 0).all() and (bo + 8 <= P_STAGE).all(), "B fragment outside the patch"
                            for s in range(KSTEPS if have else 0):
                                # lane l supplies 8 reduction values of row / column l % ATOM; lanes with equal l / ATOM pair up
                                av = np.zeros((64, 8)); bv = np.zeros((64, 8))
                                for e in range(8):
                                    sa, sb = asrc[ao + e], src[bo + e]
                                    assert (sa >= 0).all(), "A fragment reads an unwritten element"
                                    av[:, e] = ker_flat[sa + s * CS * T]
                                    bv[:, e] = np.where(sb >= 0, img_flat[np.maximum(sb, 0) + s * CS * HIN * WIN], 0.0)
                                for grp in range(64 // ATOM):
                                    sel = slice(grp * ATOM, (grp + 1) * ATOM)
                                    accv += av[sel] @ bv[sel].T
                    assert (steps_done == 1).all()
                    # epilogue: lane l holds column l % ATOM; register r holds the row stated in the template
                    for l in range(64):
                        if ct[l] >= TN:
                            continue
                        c2 = wn * TN + ct[l]
                        nb, yy, xx = nb0 + c2 // (BH * BW), y0 + (c2 // BW) % BH, x0 + c2 % BW
                        for rr in range(NACC):
                            row = 8 * (rr // 4) + 4 * (l // 32) + rr % 4 if ATOM == 32 else 4 * (l // 16) + rr
                            gm = m0 + wm * TM + i * ATOM + row
                            assert 0 <= nb < nimg and 0 <= gm < cout and 0 <= yy < HOUT and 0 <= xx < WOUT
                            written[nb, gm, yy, xx] += 1
                            if have:
                                out[nb, gm, yy, xx] = accv[row, l % ATOM]
        # ---- more than one wave per tile: the passes of the final sum through LDS
        if KW > 1:
            NWAVES, ATOMS, Q = NT // 64, MI * NI, NACC // 4
            APP = min(LDS_BYTES // (NWAVES * Q * 1024), ATOMS)
            assert APP >= 1
            owner = np.full(ATOMS, -1)
            for a0 in range(0, ATOMS, APP):
                top = min(a0 + APP, ATOMS)
                for a in range(a0, top):
                    for wave in range(NWAVES):
                        for q in range(Q):
                            word = (((a - a0) * NWAVES + wave) * Q + q) * 64 + 63      # 16-byte words; the last lane's
                            assert (word + 1) * 16 <= LDS_BYTES
                for wk in range(KW):
                    for a in range(a0 + wk, top, KW):
                        assert owner[a] == -1
                        owner[a] = wk
            assert (owner >= 0).all(), "an atom of the wave tile is never summed and stored"
    return out, written


def direct_conv(img, ker, stride, pad):
    n, cin, h, w = img.shape
    cout, _, hk, wk = ker.shape
    padded = np.zeros((n, cin, h + 2 * pad, w + 2 * pad))
    padded[:, :, pad:pad + h, pad:pad + w] = img
    ho, wo = (h + 2 * pad - hk) // stride + 1, (w + 2 * pad - wk) // stride + 1
    out = np.zeros((n, cout, ho, wo))
    for r in range(hk):
        for s in range(wk):
            win = padded[:, :, r:r + (ho - 1) * stride + 1:stride, s:s + (wo - 1) * stride + 1:stride]
            out += np.einsum("nchw,oc->nohw", win, ker[:, :, r, s])
    return out


SMALL = [
    # dims (B, Cin, H, W, Cout, Hk, Wk, stride, pad), configuration B(2) Cout(4) H(4) W(4) Cin(2) unroll layout
    ("3x3 pad 1, 32x32 atoms, ragged pixel side", (2, 32, 6, 8, 32, 3, 3, 1, 1), [1, 2, 1, 1, 1, 32, 2, 1, 1, 3, 1, 2, 1, 4, 2, 16, 1, 2, 0]),
    ("3x3 pad 1, 16x16 atoms, two channel waves", (2, 64, 4, 8, 64, 3, 3, 1, 1), [2, 1, 2, 2, 1, 16, 1, 1, 2, 2, 2, 1, 1, 4, 2, 32, 1, 2, 0]),
    ("3x3 no padding, single stage", (1, 32, 6, 6, 32, 3, 3, 1, 0), [1, 1, 1, 1, 1, 32, 1, 1, 1, 4, 1, 1, 2, 2, 2, 16, 0, 2, 0]),
    ("5x5 pad 1, 16x16 atoms", (1, 32, 8, 6, 32, 5, 5, 1, 1), [1, 1, 1, 2, 1, 16, 1, 2, 1, 3, 1, 1, 1, 4, 1, 32, 1, 2, 0]),
    ("5x5 pad 2, boxes of 3 columns", (1, 16, 6, 6, 32, 5, 5, 1, 2), [1, 1, 1, 1, 1, 32, 1, 1, 1, 6, 2, 1, 1, 3, 1, 16, 1, 2, 0]),
    ("3x3 stride 2 pad 1", (1, 32, 8, 8, 32, 3, 3, 2, 1), [1, 1, 1, 1, 1, 32, 1, 1, 1, 4, 1, 1, 1, 4, 1, 32, 1, 2, 0]),
    ("1x1", (2, 32, 4, 4, 64, 1, 1, 1, 0), [2, 1, 1, 2, 1, 32, 1, 1, 1, 4, 1, 1, 1, 4, 1, 32, 1, 2, 0]),
    ("slabs of 48 channels (6 chunks per row: stored unpermuted)", (1, 48, 6, 6, 32, 3, 3, 1, 1), [1, 1, 1, 1, 1, 32, 1, 2, 1, 3, 1, 1, 1, 6, 1, 48, 1, 2, 0]),
    ("slabs of 64 channels (8 chunks per row)", (1, 64, 4, 8, 32, 3, 3, 1, 1), [1, 1, 1, 1, 1, 32, 1, 1, 1, 4, 1, 1, 1, 8, 1, 64, 1, 2, 1]),
    ("odd width: 3x3 pad 1 on 5 x 7", (2, 32, 5, 7, 32, 3, 3, 1, 1), [2, 1, 1, 1, 1, 32, 1, 1, 1, 5, 1, 1, 1, 7, 2, 16, 1, 2, 0]),
    ("odd width: 5x5 pad 2 on 9 x 9, boxes of 3 rows", (1, 16, 9, 9, 32, 5, 5, 1, 2), [1, 1, 1, 1, 1, 32, 3, 1, 1, 3, 1, 1, 1, 9, 1, 16, 1, 2, 0]),
    ("odd width: stride 2 on 7 x 7, two waves per tile", (2, 32, 7, 7, 32, 3, 3, 2, 1), [1, 2, 1, 1, 1, 32, 1, 1, 1, 4, 1, 1, 1, 4, 1, 32, 1, 2, 1]),
]


@pytest.mark.parametrize("label,dims,cfg", SMALL, ids=[c[0] for c in SMALL])
def test_the_patch_template_computes_the_convolution(label, dims, cfg):
    rng = np.random.default_rng(7)
    nimg, cin, hin, win, cout, hk, wk, stride, pad = dims
    img = rng.integers(-3, 4, size=(nimg, cin, hin, win)).astype(np.float64)
    ker = rng.integers(-3, 4, size=(cout, cin, hk, wk)).astype(np.float64)
    out, written = emulate(dims, cfg, img, ker)
    assert (written == 1).all(), "every output element is stored exactly once"
    assert np.array_equal(out, direct_conv(img, ker, stride, pad))


KWAVES = [
    ("two waves split 9 taps x 2 steps", (2, 32, 6, 8, 32, 3, 3, 1, 1), [1, 2, 1, 1, 1, 32, 2, 1, 1, 3, 1, 2, 1, 4, 1, 32, 1, 2, 1]),
    ("four waves, 16x16 atoms, 9 steps (3, 2, 2, 2)", (2, 64, 4, 8, 64, 3, 3, 1, 1), [2, 1, 2, 1, 2, 16, 1, 1, 2, 2, 1, 1, 1, 8, 2, 32, 1, 2, 2]),
    ("eight waves of two tiles, single stage", (1, 64, 6, 6, 64, 3, 3, 1, 1), [1, 1, 1, 2, 1, 32, 1, 1, 1, 6, 1, 1, 1, 6, 2, 32, 0, 2, 2]),
]


@pytest.mark.parametrize("label,dims,cfg", KWAVES, ids=[c[0] for c in KWAVES])
def test_waves_that_split_the_reduction(label, dims, cfg):
    rng = np.random.default_rng(8)
    nimg, cin, hin, win, cout, hk, wk, stride, pad = dims
    img = rng.integers(-3, 4, size=(nimg, cin, hin, win)).astype(np.float64)
    ker = rng.integers(-3, 4, size=(cout, cin, hk, wk)).astype(np.float64)
    op = P.opevo_op_create(P.OPEVO_CONV2D, dims, P.OPEVO_BF16)
    assert "-DKW=%d" % (1, 2, 4, 8)[cfg[18]] in P.opevo_kernel_defines(op, V, cfg).split()
    out, written = emulate(dims, cfg, img, ker)
    assert (written == 1).all()
    assert np.array_equal(out, direct_conv(img, ker, stride, pad))


FOLDED = [
    # members that ask for what the template has not, and the division of the same workgroup tile it runs instead
    ("slabs of 8 channels -> 16", (2, 32, 6, 8, 32, 3, 3, 1, 1), [1, 2, 1, 1, 1, 32, 2, 1, 1, 3, 1, 2, 1, 4, 4, 8, 1, 2, 0], dict(CS=16, KSTEPS=2)),
    ("4 waves of 8 output channels -> one of 32", (2, 32, 6, 8, 32, 3, 3, 1, 1), [1, 2, 1, 4, 2, 4, 2, 1, 1, 3, 1, 2, 1, 4, 2, 16, 1, 2, 0], dict(WM=1, TM=32)),
    ("8 x 4 x 2 waves -> 8 x 1 x 2 waves (pixel waves merged)", (2, 32, 6, 8, 128, 3, 3, 1, 1), [2, 1, 1, 8, 1, 16, 1, 2, 1, 3, 1, 2, 1, 4, 1, 32, 1, 2, 1], dict(WM=8, WN=1, TN=48, KW=2)),
]


@pytest.mark.parametrize("label,dims,cfg,want", FOLDED, ids=[c[0] for c in FOLDED])
def test_folded_members(label, dims, cfg, want):
    rng = np.random.default_rng(9)
    nimg, cin, hin, win, cout, hk, wk, stride, pad = dims
    img = rng.integers(-3, 4, size=(nimg, cin, hin, win)).astype(np.float64)
    ker = rng.integers(-3, 4, size=(cout, cin, hk, wk)).astype(np.float64)
    op = P.opevo_op_create(P.OPEVO_CONV2D, dims, P.OPEVO_BF16)
    _, D = defines(op, cfg)
    assert {k: D[k] for k in want} == want
    out, written = emulate(dims, cfg, img, ker)
    assert (written == 1).all()
    assert np.array_equal(out, direct_conv(img, ker, stride, pad))


FULL = [
    ("conv14, 32 channels x one image, 4 waves", (32, 256, 14, 14, 256, 3, 3, 1, 1), [32, 1, 8, 1, 1, 32, 1, 2, 1, 7, 1, 2, 1, 7, 8, 32, 1, 2, 0]),
    ("conv14, 64 channels x two rows", (32, 256, 14, 14, 256, 3, 3, 1, 1), [32, 1, 4, 2, 1, 32, 7, 2, 1, 1, 1, 1, 1, 14, 8, 32, 1, 2, 0]),
    ("conv14, 16x16 atoms, 8 waves", (32, 256, 14, 14, 256, 3, 3, 1, 1), [16, 2, 8, 2, 1, 16, 1, 2, 1, 7, 1, 2, 1, 7, 8, 32, 1, 2, 0]),
    ("conv56, 64 channels x 4 rows", (1, 64, 56, 56, 64, 3, 3, 1, 1), [1, 1, 1, 2, 1, 32, 14, 2, 1, 2, 1, 1, 1, 56, 2, 32, 1, 2, 0]),
    ("C2 (27 x 27, 5x5, odd width), 64 channels x 9 rows, single stage", (512, 64, 27, 27, 192, 5, 5, 1, 2), [512, 1, 3, 2, 1, 32, 3, 1, 1, 9, 1, 1, 1, 27, 4, 16, 0, 2, 2]),
    ("C2, 64 channels x 9 rows, folded to 2 waves of 32 x 243 (the last workgroup's last pair ends the image tensor)", (512, 64, 27, 27, 192, 5, 5, 1, 2), [512, 1, 3, 4, 1, 16, 3, 1, 3, 3, 1, 1, 1, 27, 4, 16, 0, 2, 0]),
    ("conv14, 64 channels x 7 rows shared by 4 waves", (32, 256, 14, 14, 256, 3, 3, 1, 1), [32, 1, 4, 1, 2, 32, 2, 1, 1, 7, 1, 1, 1, 14, 8, 32, 1, 2, 2]),
    ("conv14, 128 channels x 2 rows x 2 images shared by 4 waves, single stage", (32, 256, 14, 14, 256, 3, 3, 1, 1), [16, 2, 2, 1, 4, 32, 7, 1, 1, 2, 1, 1, 1, 14, 8, 32, 0, 2, 2]),
    ("conv14, 32 channels x 7 rows shared by 8 waves", (32, 256, 14, 14, 256, 3, 3, 1, 1), [32, 1, 8, 1, 1, 32, 2, 1, 1, 7, 1, 1, 1, 14, 8, 32, 1, 2, 3]),
]


@pytest.mark.parametrize("label,dims,cfg", FULL, ids=[c[0] for c in FULL])
def test_addresses_at_full_size(label, dims, cfg):
    """The graded shapes: bounds, alignment and coverage for the corner, edge and interior workgroups."""
    op = P.opevo_op_create(P.OPEVO_CONV2D, dims, P.OPEVO_BF16)
    plan = P.opevo_kernel_plan(op, V, cfg)
    gx, gy = plan.grid[0], plan.grid[1]
    blocks = sorted({(bx, by) for bx in {0, 1, gx // 2, gx - 2, gx - 1} for by in {0, gy - 1} if 0 <= bx < gx})
    emulate(dims, cfg, blocks=blocks)


def test_members_outside_the_patch_template_run_as_layout_0():
    """layout 2 is inert where the template cannot hold the member: the plan is the layout-0 member's."""
    dims = (32, 256, 14, 14, 256, 3, 3, 1, 1)
    op = P.opevo_op_create(P.OPEVO_CONV2D, dims, P.OPEVO_BF16)
    for cfg in ([32, 1, 32, 1, 1, 8, 1, 2, 1, 7, 1, 2, 1, 7, 8, 32, 1],     # 8 output channels per workgroup
                [32, 1, 256, 1, 1, 1, 1, 2, 1, 7, 1, 2, 1, 7, 8, 32, 1],    # one channel per workgroup
                [1, 32, 1, 1, 2, 128, 1, 1, 1, 14, 1, 1, 1, 14, 8, 32, 1]): # 32 images in one box: no room in the LDS
        p2 = P.opevo_kernel_plan(op, V, cfg + [2, 1])
        p0 = P.opevo_kernel_plan(op, V, cfg + [0, 0])
        assert p2.path != 5
        assert (p2.status, p2.path, list(p2.grid), p2.block, p2.lds_bytes) == (p0.status, p0.path, list(p0.grid), p0.block, p0.lds_bytes)
    # fp32 inputs
    opf = P.opevo_op_create(P.OPEVO_CONV2D, dims, P.OPEVO_F32)
    assert P.opevo_kernel_plan(opf, V, [32, 1, 8, 1, 1, 32, 1, 2, 1, 7, 1, 2, 1, 7, 8, 32, 1, 2, 0]).path != 5
