"""CPU re-computation of every address the direct-to-LDS template forms (no GPU).

The template streams operand slabs global memory -> LDS with wave-wide loads whose global address is
`wave-uniform base + per-lane offset` and whose LDS destination is a wave-uniform byte address, and it
waits for them by counting outstanding loads.  A wrong address there is not a wrong result but a memory
fault, so the arithmetic is repeated here, from the constants the decoder hands the template, for every
workgroup corner, wave, lane, piece and slab of a member: every global access must lie inside its
operand, every LDS destination inside the ring, every piece of every slab must be issued exactly
once into the stage the K loop later reads it from, and the wait counts must imply that a slab has
landed before it is read (loads complete in order).  Checked for the member that once faulted a GPU
in a tuning run (MM2 of App. B.1, 128 x 64 tile, slabs of 128, 2 waves, 3 stages), for hand-picked and
seeded random MatMul / BMM members, and for Conv2d members (channels last, App. B.3 / Eq. 5 with stride
and padding), whose lanes compute pixel offsets themselves."""
import re

import pytest

import paper_2006_05664_amd as P


def _defs(op, variant, cfg):
    text = P.opevo_kernel_defines(op, variant, cfg)
    tmpl, rest = text.split(":", 1)
    d = {}
    for tok in rest.split():
        m = re.match(r"-D(\w+)=(-?\d+)$", tok)
        if m:
            d[m.group(1)] = int(m.group(2))
    return tmpl.strip(), d


def _lane_period(per_row, swz_rows):
    p = 1
    while (p * 64) % per_row or (p * 64 // per_row) % swz_rows:
        p += 1
    return p


def check_member(kind, dims, variant, cfg, corners_only=True, force=None):
    """force: constants to use instead of the decoder's (a member the decoder no longer sends to this
    template is then checked as the template would have run it)."""
    op = P.opevo_op_create(kind, dims, P.OPEVO_BF16)
    plan = P.opevo_kernel_plan(op, variant, cfg)
    tmpl, D = _defs(op, variant, cfg)
    if force:
        D.update(force)
    else:
        assert plan.status == P.OPEVO_OK and plan.path == 3 and tmpl == "gemm_mfma_dlds", (plan.path, tmpl, plan.reason)
    g = D.get
    M, N, K, BM, BN, BK, NT = D["M"], D["N"], D["K"], D["BM"], D["BN"], D["BK"], D["NT"]
    NW, KSTEPS, NSTG, KSPLIT = NT // 64, D["KSTEPS"], D["NSTG"], g("KSPLIT", 1)
    conv = D["OP"] == 2
    kmajor = g("B_KMAJOR", 0) == 1
    a_trans = D["A_TRANS"] == 1
    ANR, BNR = g("ANR", BM), g("BNR", BN)
    assert not (conv and not kmajor) and not (a_trans and kmajor)
    ACH = (BM if a_trans else BK) // 8
    A_RPW = max(16 // ACH, 1)
    A_SWM = max(4 // A_RPW, 1)
    a_swz = (lambda k: ((k // A_RPW) % A_SWM) << 2) if a_trans else (lambda r: (r // A_RPW) % ACH)
    if g("ATOM", 32) == 16:             # 16-row atoms: the permutation found free of bank conflicts for their read pattern
        def a_swz(r):
            b = lambda i: (r >> i) & 1
            return (b(3) << 1) if ACH == 4 else (b(1) | (b(2) << 1) | (b(3) << 2)) if ACH == 8 else (r & 15)
        # a 16-byte read is served in four turns of 16 lanes (lanes 0-3, 12-15, 20-23, 24-27; the other lanes below 32;
        # the same plus 32): in every turn the 16 lanes of a fragment read hit 16 different 16-byte bank groups
        g0 = [0, 1, 2, 3, 12, 13, 14, 15, 20, 21, 22, 23, 24, 25, 26, 27]
        turns = [g0, [l for l in range(32) if l not in g0]]
        turns += [[l + 32 for l in t] for t in turns]
        for kk in range(BK // 32):
            for t in turns:
                groups = {(((l & 15) * BK * 2 + (((4 * kk + (l >> 4)) ^ a_swz(l & 15)) << 4)) % 256) // 16 for l in t}
                assert len(groups) == 16, (BK, kk)
    BCH = 1 if kmajor else BN // 8
    B_RPW = max(16 // BCH, 1)
    B_SWM = max(4 // B_RPW, 1)
    ATOM = g("ATOM", 32)
    assert ATOM in (16, 32) and not (ATOM == 16 and (a_trans or conv))
    if ATOM == 16 and not kmajor:      # rows whose bit 3 differs are moved 32 bytes apart as well
        b_swz = lambda k: (((k // B_RPW) % B_SWM) << 2) ^ (((k >> 3) & 1) << 1)
    else:
        b_swz = lambda k: ((k // B_RPW) % B_SWM) << 2
    A_STAGE = ANR * BK
    B_STAGE = BNR * BK if kmajor else BK * BN
    STAGE = A_STAGE + B_STAGE
    assert NSTG * STAGE * 2 <= 160 * 1024 and (force or NSTG * STAGE * 2 == plan.lds_bytes)
    assert (A_STAGE * 2) % (1024 * NW) == 0 and (B_STAGE * 2) % (1024 * NW) == 0
    LA, LB = A_STAGE * 2 // 1024 // NW, B_STAGE * 2 // 1024 // NW
    PER = LA + LB
    assert (NSTG - 2) * PER <= 63                      # the wait count fits its 6 bits
    TM, TN, WM, WN = D["TM"], D["TN"], D["WM"], D["WN"]
    NI = (TN + ATOM - 1) // ATOM
    KA = 32 if ATOM == 16 else 16
    assert WM * TM == BM and TM % ATOM == 0 and WM * WN == NW and BK % KA == 0
    # fragment reads stay inside the stage parts
    assert (WM - 1) * TM + (TM // ATOM) * ATOM <= (BM if not a_trans else BM)
    assert (WN - 1) * TN + NI * ATOM <= (BNR if kmajor else BN)
    if not conv and not a_trans:
        # What the fragment reads fetch is what the loads put there: A rows as 16-byte pieces of 8 k, B (stored
        # [K][N]) with the transposing read, where a lane supplies the address of 4 consecutive n of one k row.
        where_a, where_b = {}, {}                      # (row, k chunk) / (k row, n chunk) -> element offset in the stage
        for instr in range(A_STAGE * 2 // 1024):
            for lane in range(64):
                pp = instr * 64 + lane
                row = pp // ACH
                where_a[(row, (pp % ACH) ^ a_swz(row))] = pp * 8
        for wm in range(WM):
            for i in range(TM // ATOM):
                for lane in range(64):
                    for kk in range(BK // KA):
                        row, kchunk = wm * TM + i * ATOM + lane % ATOM, kk * (KA // 8) + lane // ATOM
                        assert where_a[(row, kchunk)] == row * BK + ((kchunk ^ a_swz(row)) << 3)
        if not kmajor:
            for instr in range(B_STAGE * 2 // 1024):
                for lane in range(64):
                    pp = instr * 64 + lane
                    krow = pp // BCH
                    where_b[(krow, (pp % BCH) ^ b_swz(krow))] = pp * 8
            for wn in range(WN):
                for j in range(NI):
                    for lane in range(64):
                        for kk in range(BK // KA):
                            for r in range(2):
                                s16 = lane & 15
                                if ATOM == 16:
                                    n, krow = wn * TN + j * 16 + 4 * (s16 & 3), kk * 32 + 8 * (lane >> 4) + 4 * r + (s16 >> 2)
                                else:
                                    n, krow = wn * TN + j * 32 + 16 * ((lane >> 4) & 1) + 4 * (s16 & 3), kk * 16 + 8 * (lane >> 5) + 4 * r + (s16 >> 2)
                                addr = krow * BN + (((n >> 3) ^ b_swz(krow)) << 3) + (n & 7)
                                assert krow < BK and n + 4 <= BN and where_b[(krow, n >> 3)] + (n & 7) == addr
                                # lanes 16g .. 16g+15 together cover k rows 8g' .. +3 (+4 for r = 1) of 16 columns: the
                                # group's result lane i holds column n0 + i, which is the atom's column for that lane
                                g16 = lane >> 4
                                if ATOM == 16:
                                    assert krow - (s16 >> 2) == kk * 32 + 8 * g16 + 4 * r and n - 4 * (s16 & 3) == wn * TN + j * 16
    batch = dims[0] if kind in (P.OPEVO_BMM, P.OPEVO_BMM_TA) else 1
    a_elems = (dims[4] * K) if conv else M * K           # per batch
    b_bytes = (256 + 2 * dims[0] * dims[1] * dims[2] * dims[3]) if conv else 2 * K * N
    grid = list(plan.grid)
    if conv:
        CIN, HIN, WIN, HK, WK, S, PAD = D["CIN"], D["HIN"], D["WIN"], D["HK"], D["WK"], D["STRIDE"], D["PAD_CONV"]
        NB2, BH, BW, H1, W1 = D["NB2"], D["BH"], D["BW"], D["H1"], D["W1"]
        assert grid[2] == KSPLIT and KSPLIT * KSTEPS * BK == K
    ns = range(grid[0]) if not corners_only else sorted({0, grid[0] // 2, grid[0] - 1})
    ms = range(grid[1]) if not corners_only else sorted({0, grid[1] - 1})
    kc = lambda k: min(k, KSTEPS - 1)

    def a_piece(m0, k0, instr, lane):
        """(global byte offset inside A, LDS byte offset inside the stage) of lane's 16 bytes"""
        p = instr * 64 + lane
        row0, row = instr * 64 // ACH, p // ACH
        chunk = ((p % ACH) ^ a_swz(row)) << 3
        if a_trans:      # rows are k, M contiguous
            assert row < BK and chunk + 8 <= BM
            return ((k0 + row) * M + m0 + chunk) * 2, instr * 1024 + lane * 16
        rc, r0c = (min(row, BM - 1), min(row0, BM - 1)) if ANR != BM else (row, row0)
        assert rc < BM and chunk + 8 <= BK
        base = ((m0 + r0c) * K + k0) * 2
        return base + ((rc - r0c) * K + chunk) * 2, instr * 1024 + lane * 16

    for kz in range(KSPLIT if conv else 1):
        for bn in ns:
            for bm in ms:
                m0, n0 = bm * BM, bn * BN
                if conv:
                    x0b, y0b, nb0 = (bn % W1) * BW, ((bn // W1) % H1) * BH, (bn // (W1 * H1)) * NB2
                for wave in range(NW):
                    issued = []          # (stage, slab, piece) in issue order

                    def issue(t, stage, slab):
                        k0 = (kz * KSTEPS + kc(slab)) * BK if conv else kc(slab) * BK
                        if t < LA:
                            instr = wave * LA + t
                            for lane in range(64):
                                goff, loff = a_piece(m0, k0, instr, lane)
                                assert 0 <= goff and goff + 16 <= 2 * a_elems, ("A", cfg, goff)
                                assert 0 <= loff and loff + 16 <= A_STAGE * 2
                        else:
                            u = t - LA
                            instr = wave * LB + u
                            for lane in range(64):
                                p = instr * 64 + lane
                                if conv:
                                    c = p // ACH
                                    k8 = ((p % ACH) ^ a_swz(c)) << 3
                                    cc = c if c < BN else 0
                                    nb = nb0 + cc // (BH * BW)
                                    y0, x0 = (y0b + (cc // BW) % BH) * S - PAD, (x0b + cc % BW) * S - PAD
                                    kp = k0 + k8
                                    tap, ci0 = kp // CIN, kp % CIN
                                    r, sx = tap // WK, tap % WK
                                    assert r < HK and ci0 + 8 <= CIN
                                    ok = c < BN and 0 <= y0 + r < HIN and 0 <= x0 + sx < WIN
                                    goff = 256 + 2 * (((nb * HIN + y0 + r) * WIN + x0 + sx) * CIN + ci0) if ok else 0
                                    assert nb < dims[0]
                                elif kmajor:
                                    row = p // ACH
                                    chunk = ((p % ACH) ^ a_swz(row)) << 3
                                    assert row < BNR == BN and chunk + 8 <= BK
                                    goff = ((n0 + row) * K + k0 + chunk) * 2
                                else:
                                    krow = p // BCH
                                    chunk = ((p % BCH) ^ b_swz(krow)) << 3
                                    assert krow < BK and chunk + 8 <= BN
                                    goff = ((k0 + krow) * N + n0 + chunk) * 2
                                assert 0 <= goff and goff + 16 <= b_bytes, ("B", cfg, goff)
                                loff = (A_STAGE + instr * 512) * 2 + lane * 16
                                assert A_STAGE * 2 <= loff and loff + 16 <= STAGE * 2
                        issued.append((stage, slab, t))

                    def landed(outstanding, slab, stage):
                        done = issued[:len(issued) - min(outstanding, 63)] if outstanding else issued
                        last = {}
                        for st, sl, t in done:
                            if st == stage:
                                last[t] = sl       # what the stage holds is what was issued into it last
                        assert last == {t: slab for t in range(PER)}, ("not landed", cfg, slab, stage)

                    for s in range(NSTG):
                        for t in range(PER):
                            issue(t, s, s)
                    landed((NSTG - 1) * PER, 0, 0)
                    order = [(kt + s, s) for kt in range(0, KSTEPS // NSTG * NSTG, NSTG) for s in range(NSTG)]
                    order += [(KSTEPS // NSTG * NSTG + s, s) for s in range(KSTEPS % NSTG)]
                    for q, s in order:
                        # last group of slab q: wait, barrier, then read slab q+1 from the next stage and refill this one
                        if q + 1 < KSTEPS:
                            landed((NSTG - 2) * PER, q + 1, (s + 1) % NSTG)
                        for t in range(PER):
                            issue(t, s, q + NSTG)
                    assert [x for x in order] == [(q, q % NSTG) for q in range(KSTEPS)]
    P.opevo_op_destroy(op)
    return dict(LA=LA, LB=LB, NSTG=NSTG, PER=PER)


MM2 = (P.OPEVO_MATMUL, (512, 4096, 1024))
MM1 = (P.OPEVO_MATMUL, (512, 1024, 1024))
CONV14 = (P.OPEVO_CONV2D, (32, 256, 14, 14, 256, 3, 3, 1, 1))


def test_the_member_that_faulted_forms_only_in_bounds_addresses():
    """opevo_mm4_4_1_4_32_64_2_4_8_8_128_1 of MM2: 128 x 64 tile, slabs of 128, 2 waves, 3 stages, 8 slabs (two
    of them after the last full turn of the ring).  Every address is in bounds and every wait is sufficient: the
    fault of that run is not explained by the template's arithmetic as written.  (Today the decoder sends this
    member to the register-staged template: its unrolled body is past the size limit.)"""
    cfg = [4, 1, 4, 32, 64, 2, 4, 8, 8, 128, 1]
    op = P.opevo_op_create(*MM2, P.OPEVO_BF16)
    assert P.opevo_kernel_plan(op, P.OPEVO_TILE4, cfg).path == 1            # kept off the direct-to-LDS template
    # as the template ran it then: the most stages that fit 160 KiB, 3 x (128 + 64) x 128 x 2 bytes
    r = check_member(P.OPEVO_MATMUL, MM2[1], P.OPEVO_TILE4, cfg, corners_only=False, force={"NSTG": 3})
    assert r == dict(LA=16, LB=8, NSTG=3, PER=24)


@pytest.mark.parametrize("kd,variant,cfg", [
    (MM1, P.OPEVO_TILE4, [2, 2, 1, 128, 8, 4, 1, 32, 32, 32, 1]),
    (MM1, P.OPEVO_TILE4, [4, 2, 2, 32, 8, 2, 2, 32, 8, 128, 1]),
    (MM1, P.OPEVO_TILE4, [16, 1, 1, 32, 16, 1, 2, 32, 16, 64, 1]),
    ((P.OPEVO_MATMUL, (8192, 8192, 8192)), P.OPEVO_TILE4, [32, 2, 2, 64, 32, 2, 2, 64, 256, 32, 1]),
    ((P.OPEVO_MATMUL, (8192, 8192, 8192)), P.OPEVO_TILE4T, [32, 2, 2, 64, 32, 2, 2, 64, 256, 32, 1, 1]),
    # 16x16x32 atoms: 4 waves of 128 x 128 on slabs of 32, 8 waves of 128 x 64, slabs of 64, narrow N tiles
    ((P.OPEVO_MATMUL, (8192, 8192, 8192)), P.OPEVO_TILE4A, [32, 2, 2, 64, 32, 2, 2, 64, 256, 32, 1, 1]),
    ((P.OPEVO_MATMUL, (8192, 8192, 8192)), P.OPEVO_TILE4A, [32, 2, 8, 16, 32, 4, 2, 32, 256, 32, 1, 1]),
    ((P.OPEVO_MATMUL, (8192, 8192, 8192)), P.OPEVO_TILE4A, [32, 2, 4, 32, 32, 2, 4, 32, 128, 64, 1, 1]),
    (MM1, P.OPEVO_TILE4A, [16, 1, 1, 32, 16, 1, 2, 32, 16, 64, 1, 1]),
    (MM1, P.OPEVO_TILE4A, [8, 2, 1, 32, 32, 1, 1, 32, 8, 128, 1, 1]),
    ((P.OPEVO_MATMUL, (512, 768, 1024)), P.OPEVO_TILE4T, [4, 2, 2, 32, 8, 1, 3, 32, 32, 32, 1, 1]),
    ((P.OPEVO_BMM_TA, (24, 128, 64, 128)), P.OPEVO_TILE4, [12, 2, 1, 2, 2, 32, 1, 1, 2, 32, 2, 64, 1]),
    (CONV14, P.OPEVO_TILE4C, [32, 1, 2, 2, 2, 32, 1, 7, 2, 1, 1, 1, 14, 1, 4, 9, 64, 1, 1]),
    (CONV14, P.OPEVO_TILE4C, [32, 1, 8, 1, 1, 32, 1, 7, 2, 1, 1, 1, 14, 1, 1, 18, 128, 1, 1]),
    ((P.OPEVO_CONV2D, (3, 16, 11, 11, 32, 4, 4, 1, 1)), P.OPEVO_TILE4C, [3, 1, 1, 1, 1, 32, 1, 5, 1, 2, 1, 1, 1, 10, 2, 2, 64, 1, 1]),
    ((P.OPEVO_CONV2D, (4, 32, 10, 10, 64, 3, 3, 2, 1)), P.OPEVO_TILE4C, [1, 4, 1, 2, 1, 32, 1, 1, 1, 5, 1, 1, 1, 5, 3, 3, 32, 1, 1]),
])
def test_handpicked_direct_to_lds_members_form_only_in_bounds_addresses(kd, variant, cfg):
    op = P.opevo_op_create(*kd, P.OPEVO_BF16)
    if P.opevo_kernel_plan(op, variant, cfg).path != 3:
        pytest.skip("not a direct-to-LDS member on this build of the decoder")
    check_member(kd[0], kd[1], variant, cfg, corners_only=len(kd[1]) == 3 and kd[1][0] > 1024)


@pytest.mark.parametrize("kd,variant,seed", [(MM2, P.OPEVO_TILE4, 1), (MM1, P.OPEVO_TILE4T, 2), (MM2, P.OPEVO_TILE4A, 5), (CONV14, P.OPEVO_TILE4C, 3),
                                             ((P.OPEVO_CONV2D, (512, 64, 27, 27, 192, 5, 5, 1, 2)), P.OPEVO_TILE4C, 4)])
def test_sampled_direct_to_lds_members_form_only_in_bounds_addresses(kd, variant, seed):
    op = P.opevo_op_create(*kd, P.OPEVO_BF16)
    sp = P.opevo_op_space(op, variant)
    rng = P.opevo_rng_create(seed)
    seen, n = set(), 0
    for _ in range(60000):
        cfg = P.opevo_space_random(sp, rng)
        plan = P.opevo_kernel_plan(op, variant, cfg)
        if plan.status != P.OPEVO_OK or plan.path != 3:
            continue
        key = (tuple(plan.tile), plan.block, tuple(plan.wave_tile), tuple(plan.grid))
        if key in seen:
            continue
        seen.add(key)
        check_member(kd[0], kd[1], variant, list(cfg))
        n += 1
        if n >= 6:
            break
    assert n >= 3
    P.opevo_rng_destroy(rng); P.opevo_space_destroy(sp)
