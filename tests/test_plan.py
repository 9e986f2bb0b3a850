"""Configuration decoder: legality, validity, launch geometry, and that representative
members of every template family compile for gfx950 through hipRTC (no GPU needed)."""
import pytest

import paper_2006_05664_amd as P

MM1 = (P.OPEVO_MATMUL, (512, 1024, 1024))
MM8K = (P.OPEVO_MATMUL, (8192, 8192, 8192))
BMM = (P.OPEVO_BMM, (128, 128, 128, 64))
CONV56 = (P.OPEVO_CONV2D, (1, 64, 56, 56, 64, 3, 3, 1, 1))
CONV14 = (P.OPEVO_CONV2D, (32, 256, 14, 14, 256, 3, 3, 1, 1))


def _op(kd, dtype=P.OPEVO_BF16):
    return P.opevo_op_create(kd[0], kd[1], dtype)


def test_flops_bytes_sizes():
    op = _op(MM1)
    assert P.opevo_op_flops(op) == 2.0 * 512 * 1024 * 1024
    assert P.opevo_op_bytes(op) == 2 * (512 * 1024 + 1024 * 1024) + 4 * 512 * 1024 == 5242880
    op = _op(BMM)
    assert P.opevo_op_flops(op) == 2.0 * 128 * 128 * 128 * 64 and P.opevo_op_bytes(op) == 12582912
    op = _op(CONV56)
    assert P.opevo_op_flops(op) == 2.0 * 64 * 56 * 56 * 64 * 9     # padding taps counted
    assert P.opevo_op_sizes(op) == (64 * 64 * 9, 64 * 56 * 56, 64 * 56 * 56)
    assert P.opevo_op_bytes(op) == 1277952
    op = _op(CONV14)
    assert P.opevo_op_flops(op) == 2.0 * 32 * 256 * 14 * 14 * 256 * 9 and P.opevo_op_bytes(op) == 10813440
    # App. B.3 output extents: C1 -> 55, C2 -> 27
    assert P.opevo_op_sizes(P.opevo_op_create(P.OPEVO_CONV2D, (2, 3, 227, 227, 64, 11, 11, 4, 0), 1))[2] == 2 * 64 * 55 * 55
    assert P.opevo_op_sizes(P.opevo_op_create(P.OPEVO_CONV2D, (2, 64, 27, 27, 192, 5, 5, 1, 2), 1))[2] == 2 * 192 * 27 * 27


def test_illegal_configurations_are_errors_not_trials():
    op = _op(MM1)
    good = [2, 2, 2, 64, 8, 2, 2, 32, 16, 64, 1]
    assert P.opevo_kernel_plan(op, P.OPEVO_TILE4, good).status == P.OPEVO_OK
    for bad in ([2, 2, 2, 32, 8, 2, 2, 32, 16, 64, 1], [2, 2, 2, 64, 8, 2, 2, 32, 16, 64, 2],
                [0, 2, 2, 64, 8, 2, 2, 32, 16, 64, 1], [2, 2, 2, 64, 8, 2, 2, 32, 16, 32, 1],
                [-2, -2, 2, 64, 8, 2, 2, 32, 16, 64, 1]):
        for call in (P.opevo_kernel_plan, P.opevo_kernel_build, P.opevo_kernel_defines):
            with pytest.raises(P.OpevoError) as ei:
                call(op, P.OPEVO_TILE4, bad)
            assert ei.value.status == P.OPEVO_E_ILLEGAL


def test_oversized_members_are_folded_into_serial_work_and_the_rest_is_invalid():
    """Members that ask for more waves, accumulators or LDS than a workgroup has run as serial work
    (slow, but with a fitness of their own); what cannot be folded stays invalid (fitness 0, Sec. 4.2)."""
    op = _op(MM1)
    # 32 x 32 waves of 16 x 32: 16 real waves take 64 wave tiles each
    plan = P.opevo_kernel_plan(op, P.OPEVO_TILE4, [1, 32, 1, 16, 1, 32, 1, 32, 16, 64, 1])
    assert plan.status == P.OPEVO_OK and plan.block == 1024 and plan.path == 2
    assert plan.wave_passes * 16 * list(plan.sub_tiles)[0] * list(plan.sub_tiles)[1] == 32 * 32
    d = P.opevo_kernel_defines(op, P.OPEVO_TILE4, [1, 32, 1, 16, 1, 32, 1, 32, 16, 64, 1])
    assert "-DNWR=16" in d.split() and "-DWM=" in d
    # one wave with a 512 x 512 tile: cut into wave tiles of at most 256 accumulators per lane
    plan = P.opevo_kernel_plan(op, P.OPEVO_TILE4, [1, 1, 8, 64, 2, 1, 8, 64, 16, 64, 1])
    assert plan.status == P.OPEVO_OK and plan.acc_per_lane <= 256 and plan.wave_tile[0] * plan.wave_tile[1] <= 64 * 256
    assert plan.sub_tiles[0] * plan.tile[0] == 512 and plan.sub_tiles[1] * plan.tile[1] == 512
    # a 1024-deep slab: halved until the stages fit
    plan = P.opevo_kernel_plan(op, P.OPEVO_TILE4, [2, 2, 2, 64, 8, 2, 2, 32, 1, 1024, 1])
    assert plan.status == P.OPEVO_OK and plan.tile[2] < 1024 and plan.lds_bytes <= 160 * 1024
    assert "-DKSTEPS=%d" % (1024 // plan.tile[2]) in P.opevo_kernel_defines(op, P.OPEVO_TILE4, [2, 2, 2, 64, 8, 2, 2, 32, 1, 1024, 1]).split()
    # folded members never take the direct-to-LDS template, and un-folded ones decode as before
    assert P.opevo_kernel_plan(op, P.OPEVO_TILE4, [2, 2, 2, 64, 8, 2, 2, 32, 16, 64, 1]).path == 3
    plan = P.opevo_kernel_plan(op, P.OPEVO_TILE4, [2, 2, 2, 64, 8, 2, 2, 32, 16, 64, 1])
    assert list(plan.sub_tiles) == [1, 1] and plan.wave_passes == 1 and list(plan.tile) == [256, 128, 64]
    # not foldable: a box of pixels too large for the LDS (a convolution's column block is cut along channels only)
    conv = _op(CONV14)
    cfg = [1, 32, 256, 1, 1, 1, 1, 1, 1, 14, 1, 1, 1, 14, 1, 2304, 0]          # all 32 images in one tile, one slab
    plan = P.opevo_kernel_plan(conv, P.OPEVO_TILE4, cfg)
    assert plan.status == P.OPEVO_E_INVALID and "LDS" in plan.reason.decode(), plan.reason
    with pytest.raises(P.OpevoError) as ei:
        P.opevo_kernel_build(conv, P.OPEVO_TILE4, cfg)
    assert ei.value.status == P.OPEVO_E_INVALID


def test_two_level_space_has_no_invalid_member():
    op = _op((P.OPEVO_MATMUL, (64, 64, 64)), P.OPEVO_F32)
    sp = P.opevo_op_space(op, P.OPEVO_TILE2)
    for r in range(343):
        cfg = P.opevo_space_unrank(sp, r)
        plan = P.opevo_kernel_plan(op, P.OPEVO_TILE2, cfg)
        assert plan.status == P.OPEVO_OK and plan.path == 0
        assert plan.grid[0] * plan.tile[1] == 64 and plan.grid[1] * plan.tile[0] == 64
        assert 64 <= plan.block <= 256 and plan.block % 64 == 0 and plan.lds_bytes <= 32768
    P.opevo_space_destroy(sp)


@pytest.mark.parametrize("kd", [MM1, MM8K, BMM, CONV56, CONV14])
def test_four_level_spaces_cover_the_output_once_and_are_not_mostly_invalid(kd):
    op = _op(kd)
    sp = P.opevo_op_space(op, P.OPEVO_TILE4)
    rng = P.opevo_rng_create(11)
    a, b, c = P.opevo_op_sizes(op)
    n_valid = n_mfma = 0
    total = 1500
    for _ in range(total):
        cfg = P.opevo_space_random(sp, rng)
        plan = P.opevo_kernel_plan(op, P.OPEVO_TILE4, cfg)
        binner = cfg[1] if kd[0] == P.OPEVO_BMM else 1
        # workgroups x (sub-tiles of a folded member x) workgroup tile = the whole output, exactly once
        # (App. B.1 roles of the factors)
        assert plan.grid[0] * plan.grid[1] * plan.grid[2] * binner * plan.sub_tiles[0] * plan.sub_tiles[1] * plan.tile[0] * plan.tile[1] == c
        assert plan.block % 64 == 0
        if plan.status == P.OPEVO_OK:
            n_valid += 1
            n_mfma += plan.path != 0
            assert plan.block <= 1024 and plan.lds_bytes <= 160 * 1024 and plan.acc_per_lane <= 256
            if plan.path:
                atom = 16 if plan.path == 2 else 32
                if kd[0] == P.OPEVO_CONV2D and plan.path == 2:
                    # convolution wave tiles are rounded up to whole atoms when that at most doubles the work
                    up = [(t + 15) // 16 * 16 for t in plan.wave_tile]
                    assert up[0] * up[1] <= 2 * plan.wave_tile[0] * plan.wave_tile[1]
                else:
                    assert plan.wave_tile[0] % atom == 0 and plan.wave_tile[1] % atom == 0
        else:
            assert plan.reason
    assert n_valid > 0.5 * total, "space mostly invalid: Eq. 2 would have little to select from"
    assert n_mfma > 0.005 * total
    P.opevo_rng_destroy(rng); P.opevo_space_destroy(sp)


COMPILE_CASES = [
    ("scalar f32 two-level", (P.OPEVO_MATMUL, (64, 64, 64)), P.OPEVO_F32, P.OPEVO_TILE2, [8, 8, 4, 16, 2, 32], 0),
    ("mfma 32x32 register-staged double buffer", MM1, P.OPEVO_BF16, P.OPEVO_TILE4, [2, 2, 2, 64, 8, 2, 2, 32, 64, 16, 1], 1),
    ("mfma 32x32 direct-to-LDS", MM1, P.OPEVO_BF16, P.OPEVO_TILE4, [2, 2, 2, 64, 8, 2, 2, 32, 16, 64, 1], 3),
    ("mfma 32x32 direct-to-LDS fp16, 2 stages", MM1, P.OPEVO_F16, P.OPEVO_TILE4, [4, 2, 1, 64, 8, 2, 1, 64, 8, 128, 1], 3),
    ("mfma 16x16 single stage", MM1, P.OPEVO_BF16, P.OPEVO_TILE4, [16, 2, 1, 16, 16, 2, 1, 32, 16, 64, 0], 2),
    ("mfma fp16", MM1, P.OPEVO_F16, P.OPEVO_TILE4, [2, 2, 2, 64, 8, 2, 2, 32, 32, 32, 0], 1),
    ("scalar fallback bf16", MM1, P.OPEVO_BF16, P.OPEVO_TILE4, [32, 2, 2, 4, 16, 2, 8, 4, 64, 16, 1], 0),
    ("bmm lds direct", BMM, P.OPEVO_BF16, P.OPEVO_TILE4, [64, 2, 2, 1, 2, 32, 2, 1, 2, 32, 1, 64, 1], 3),
    ("bmm lds register-staged", BMM, P.OPEVO_BF16, P.OPEVO_TILE4, [64, 2, 2, 1, 2, 32, 2, 1, 2, 32, 4, 16, 1], 1),
    ("bmm direct", BMM, P.OPEVO_BF16, P.OPEVO_TILE4, [64, 2, 2, 1, 2, 32, 2, 1, 2, 32, 1, 64, 0], 1),
    ("conv mfma", CONV56, P.OPEVO_BF16, P.OPEVO_TILE4, [1, 1, 1, 2, 1, 32, 7, 2, 1, 4, 2, 1, 7, 4, 18, 32, 1], 2),
    ("conv mfma16, slab 24 padded to 32", CONV56, P.OPEVO_BF16, P.OPEVO_TILE4, [1, 1, 1, 2, 4, 8, 7, 2, 2, 2, 2, 1, 7, 4, 24, 24, 0], 2),
    ("conv mfma16, 8-row wave tile rounded up to one atom", CONV56, P.OPEVO_BF16, P.OPEVO_TILE4, [1, 1, 4, 2, 1, 8, 7, 2, 2, 2, 2, 1, 7, 4, 24, 24, 0], 2),
    ("conv scalar", CONV56, P.OPEVO_BF16, P.OPEVO_TILE4, [1, 1, 8, 2, 1, 4, 7, 2, 2, 2, 2, 1, 7, 4, 24, 24, 0], 0),
    ("conv mfma32, odd reduction axis, slab 121 padded to 128", (P.OPEVO_CONV2D, (32, 3, 19, 19, 32, 11, 11, 4, 0)), P.OPEVO_BF16,
     P.OPEVO_TILE4, [1, 32, 1, 1, 1, 32, 3, 1, 1, 1, 3, 1, 1, 1, 3, 121, 1], 1),
    ("conv batch mfma", CONV14, P.OPEVO_BF16, P.OPEVO_TILE4, [8, 4, 2, 2, 2, 32, 7, 1, 1, 2, 7, 1, 1, 2, 36, 64, 1], 2),
]


@pytest.mark.parametrize("label,kd,dtype,variant,cfg,path", COMPILE_CASES, ids=[c[0] for c in COMPILE_CASES])
def test_templates_compile_for_gfx950(label, kd, dtype, variant, cfg, path):
    op = _op(kd, dtype)
    plan = P.opevo_kernel_plan(op, variant, cfg)
    assert plan.status == P.OPEVO_OK and plan.path == path, (plan.reason, plan.path)
    kernel, ms = P.opevo_kernel_build(op, variant, cfg)
    assert P.opevo_kernel_code_size(kernel) > 1000 and ms > 0
    assert "-DBM=%d" % plan.tile[0] in P.opevo_kernel_defines(op, variant, cfg)
    P.opevo_kernel_destroy(kernel)


def test_direct_to_lds_members_with_large_bodies_use_the_register_staged_template():
    """The direct-to-LDS template needs its K-loop body to unroll completely; the decoder keeps
    members whose body estimate exceeds 256 instructions on the register-staged template."""
    mm2 = _op((P.OPEVO_MATMUL, (512, 4096, 1024)), P.OPEVO_BF16)
    big = [4, 1, 4, 32, 64, 2, 4, 8, 8, 128, 1]       # 128x64 tile, slab 128, 2 waves: body 3*(8*10+24) = 312
    plan = P.opevo_kernel_plan(mm2, P.OPEVO_TILE4, big)
    assert plan.status == P.OPEVO_OK and plan.path == 1
    mm = _op((P.OPEVO_MATMUL, (8192, 8192, 8192)), P.OPEVO_BF16)
    for cfg in ([32, 2, 2, 64, 32, 2, 2, 64, 256, 32, 1],      # 4 waves of 128x128: 4*(2*28+8) = 256
                [32, 2, 8, 16, 32, 4, 2, 32, 256, 32, 1],      # 8 waves of 128x64
                [32, 2, 4, 32, 32, 4, 8, 8, 128, 64, 1]):      # slab 64, 2 stages
        plan = P.opevo_kernel_plan(mm, P.OPEVO_TILE4, cfg)
        assert plan.status == P.OPEVO_OK and plan.path == 3, cfg


def test_every_sampled_direct_to_lds_member_compiles_to_a_small_code_object():
    """Full unrolling shows in the size of the code object: about 20 KiB; a member whose loops
    survive takes hundreds of KiB (and is refused by opevo_kernel_build)."""
    op = _op((P.OPEVO_MATMUL, (512, 4096, 1024)), P.OPEVO_BF16)
    sp = P.opevo_op_space(op, P.OPEVO_TILE4)
    rng = P.opevo_rng_create(77)
    seen, built = set(), 0
    for _ in range(200000):
        cfg = P.opevo_space_random(sp, rng)
        plan = P.opevo_kernel_plan(op, P.OPEVO_TILE4, cfg)
        key = (tuple(plan.tile), tuple(plan.wave_tile), plan.block)
        if plan.status != P.OPEVO_OK or plan.path != 3 or key in seen:
            continue
        seen.add(key)
        kernel, _ = P.opevo_kernel_build(op, P.OPEVO_TILE4, cfg)
        assert P.opevo_kernel_code_size(kernel) < 128 * 1024, (list(cfg), P.opevo_kernel_code_size(kernel))
        P.opevo_kernel_destroy(kernel)
        built += 1
        if built >= 6:
            break
    assert built == 6
    P.opevo_rng_destroy(rng); P.opevo_space_destroy(sp)


# ------------------------------------------------------------------ extended variant: launch order and group width
def test_extended_variant_adds_a_permutation_and_a_discrete_parameter():
    for kd, n_axes in ((MM1, 2), (BMM, 3), (CONV56, 2)):
        op = _op(kd, P.OPEVO_BF16)
        sp4, spx = P.opevo_op_space(op, P.OPEVO_TILE4), P.opevo_op_space(op, P.OPEVO_TILE4X)
        assert P.opevo_space_width(spx) == P.opevo_space_width(sp4) + n_axes + 1
        assert P.opevo_space_num_params(spx) == P.opevo_space_num_params(sp4) + 2
        fact = 1
        for i in range(2, n_axes + 1):
            fact *= i
        assert P.opevo_space_size(spx) == P.opevo_space_size(sp4) * fact * 5
        assert P.opevo_space_param_name(spx, P.opevo_space_num_params(spx) - 2) == "order"
        assert P.opevo_space_param_name(spx, P.opevo_space_num_params(spx) - 1) == "group"
        P.opevo_space_destroy(sp4); P.opevo_space_destroy(spx)


def test_extended_variant_decodes_to_a_linear_grid_with_the_same_tiles():
    op = _op(MM1, P.OPEVO_BF16)
    base = [2, 2, 2, 64, 8, 2, 2, 32, 16, 64, 1]
    p4 = P.opevo_kernel_plan(op, P.OPEVO_TILE4, base)
    for order in ([0, 1], [1, 0]):
        for g in range(5):
            px = P.opevo_kernel_plan(op, P.OPEVO_TILE4X, base + order + [g])
            assert px.status == P.OPEVO_OK and px.path == p4.path
            assert list(px.tile) == list(p4.tile) and px.block == p4.block and px.lds_bytes == p4.lds_bytes
            assert list(px.grid) == [p4.grid[0] * p4.grid[1] * p4.grid[2], 1, 1]
            d = P.opevo_kernel_defines(op, P.OPEVO_TILE4X, base + order + [g])
            assert "-DGRID_LINEAR=1" in d and "-DORDER0=%d" % order[0] in d and "-DGROUP=%d" % (1, 2, 4, 8, 16)[g] in d
    for bad in (base + [0, 0, 0], base + [0, 2, 0], base + [0, 1, 5], base + [0, 1, -1]):
        with pytest.raises(P.OpevoError) as ei:
            P.opevo_kernel_plan(op, P.OPEVO_TILE4X, bad)
        assert ei.value.status == P.OPEVO_E_ILLEGAL


def test_transposed_first_operand_runs_on_every_template():
    op = P.opevo_op_create(P.OPEVO_BMM_TA, (960, 128, 64, 128), P.OPEVO_BF16)
    assert P.opevo_op_sizes(op) == (960 * 128 * 128, 960 * 128 * 64, 960 * 128 * 64)
    sp = P.opevo_op_space(op, P.OPEVO_TILE4)
    rng = P.opevo_rng_create(5)
    paths = set()
    for _ in range(4000):
        plan = P.opevo_kernel_plan(op, P.OPEVO_TILE4, P.opevo_space_random(sp, rng))
        if plan.status == P.OPEVO_OK:
            paths.add(plan.path)
    assert paths == {0, 1, 2, 3}
    for cfg, path in (([160, 6, 1, 2, 2, 32, 1, 1, 2, 32, 2, 64, 1], 3), ([160, 6, 8, 2, 2, 4, 4, 2, 4, 2, 8, 16, 1], 0),
                      ([160, 6, 1, 2, 2, 32, 1, 1, 2, 32, 8, 16, 1], 1),      # register-staged, A blocks transposed like B's
                      ([160, 6, 4, 2, 1, 16, 2, 2, 1, 16, 4, 32, 1], 2),
                      ([160, 6, 1, 2, 2, 32, 1, 1, 2, 32, 8, 16, 0], 0)):     # no LDS staging: scalar for this layout
        plan = P.opevo_kernel_plan(op, P.OPEVO_TILE4, cfg)
        assert plan.status == P.OPEVO_OK and plan.path == path, (cfg, plan.path, plan.reason)
        kernel, _ = P.opevo_kernel_build(op, P.OPEVO_TILE4, cfg)
        assert "-DA_TRANS=1" in P.opevo_kernel_defines(op, P.OPEVO_TILE4, cfg)
        P.opevo_kernel_destroy(kernel)
    P.opevo_rng_destroy(rng); P.opevo_space_destroy(sp); P.opevo_op_destroy(op)


EXT_COMPILE_CASES = [
    ("direct-to-LDS, m fastest, groups of 4", MM1, [2, 2, 2, 64, 8, 2, 2, 32, 16, 64, 1, 1, 0, 2], 3),
    ("register-staged, n fastest, groups of 16", MM1, [2, 2, 2, 64, 8, 2, 2, 32, 64, 16, 1, 0, 1, 4], 1),
    ("scalar, m fastest", MM1, [32, 2, 2, 4, 16, 2, 8, 4, 64, 16, 1, 1, 0, 0], 0),
    ("bmm, batch fastest", BMM, [64, 2, 2, 1, 2, 32, 2, 1, 2, 32, 1, 64, 1, 2, 0, 1, 1], 3),
    ("conv mfma, cout blocks fastest", CONV56, [1, 1, 1, 2, 1, 32, 7, 2, 1, 4, 2, 1, 7, 4, 18, 32, 1, 1, 0, 3], 2),
]


@pytest.mark.parametrize("label,kd,cfg,path", EXT_COMPILE_CASES, ids=[c[0] for c in EXT_COMPILE_CASES])
def test_extended_variant_templates_compile(label, kd, cfg, path):
    op = _op(kd, P.OPEVO_BF16)
    plan = P.opevo_kernel_plan(op, P.OPEVO_TILE4X, cfg)
    assert plan.status == P.OPEVO_OK and plan.path == path, (plan.reason, plan.path)
    kernel, _ = P.opevo_kernel_build(op, P.OPEVO_TILE4X, cfg)
    assert P.opevo_kernel_code_size(kernel) > 1000
    P.opevo_kernel_destroy(kernel)


# ------------------------------------------------------------------ Conv2d space with separately split reduction axes
C2_SMALL = (P.OPEVO_CONV2D, (4, 16, 12, 12, 32, 5, 5, 1, 2))
C1_SMALL = (P.OPEVO_CONV2D, (16, 3, 35, 35, 16, 11, 11, 4, 0))


def test_separately_split_reduction_space_follows_app_b3():
    """App. B.3: C_out, H_out, W_out in four factors, C_in, H_k, W_k in two, a binary unroll choice
    and a discrete bound on the unrolled steps (the batch split is this build's addition)."""
    op = _op(C2_SMALL, P.OPEVO_BF16)
    sp = P.opevo_op_space(op, P.OPEVO_TILE4P)
    names = [P.opevo_space_param_name(sp, i) for i in range(P.opevo_space_num_params(sp))]
    assert names == ["B", "Cout", "H", "W", "Cin", "Hk", "Wk", "unroll", "unroll_steps"]
    assert P.opevo_space_width(sp) == 22
    sizes = [P.opevo_space_param_size(sp, i) for i in range(9)]
    # ordered 2-factorisations: 4 = 2^2 -> 3, 16 = 2^4 -> 5, 5 -> 2; 4-factorisations: 32 = 2^5 -> C(8,3),
    # 12 = 2^2*3 -> C(5,3)*C(4,3)
    assert sizes == [3, 56, 40, 40, 5, 2, 2, 2, 4]
    P.opevo_space_destroy(sp)
    # the other operators have no such space
    with pytest.raises(P.OpevoError):
        P.opevo_op_space(_op(MM1, P.OPEVO_BF16), P.OPEVO_TILE4P)
    with pytest.raises(P.OpevoError):
        P.opevo_op_space(_op(BMM, P.OPEVO_BF16), P.OPEVO_TILE4P)


def test_boxes_that_are_contiguous_runs_use_the_plain_walk():
    op = _op(C2_SMALL, P.OPEVO_BF16)
    head = [1, 4, 1, 1, 1, 32, 3, 1, 1, 4, 6, 1, 1, 2]
    boxed = head + [4, 4, 5, 1, 1, 5, 1, 0]            # 4 channels x 1 row x 5 taps
    plan = P.opevo_kernel_plan(op, P.OPEVO_TILE4P, boxed)
    assert plan.status == P.OPEVO_OK and plan.path == 1 and plan.tile[2] == 20
    d = P.opevo_kernel_defines(op, P.OPEVO_TILE4P, boxed)
    assert "-DTAP_BOX=1" in d and "-DCI_O=4 -DCI_I=4 -DHK_O=5 -DHK_I=1 -DWK_O=1 -DWK_I=5" in d
    assert "-DKSTEPS=20" in d and "-DBKP=32" in d and "-DKUNROLL=1" in d
    for box, bk in (([8, 2, 1, 5, 1, 5], 50),          # whole kernel planes of 2 channels
                    ([16, 1, 5, 1, 1, 5], 5),          # one kernel row
                    ([16, 1, 5, 1, 5, 1], 1)):         # one tap
        cfg = head + box + [0, 3]
        plan = P.opevo_kernel_plan(op, P.OPEVO_TILE4P, cfg)
        d = P.opevo_kernel_defines(op, P.OPEVO_TILE4P, cfg)
        assert plan.status == P.OPEVO_OK and plan.tile[2] == bk and "TAP_BOX" not in d and "-DKUNROLL=8" in d
    # illegal: Hk factors must multiply to 5, the step index must exist
    with pytest.raises(P.OpevoError):
        P.opevo_kernel_plan(op, P.OPEVO_TILE4P, head + [4, 4, 2, 2, 1, 5, 1, 0])
    with pytest.raises(P.OpevoError):
        P.opevo_kernel_plan(op, P.OPEVO_TILE4P, head + [4, 4, 5, 1, 1, 5, 1, 4])


BOX_COMPILE_CASES = [
    ("mfma32 boxed, pipelined", C2_SMALL, [1, 4, 1, 1, 1, 32, 3, 1, 1, 4, 6, 1, 1, 2, 4, 4, 5, 1, 1, 5, 1, 0], 1),
    ("mfma32 boxed, loop unrolled by 2", C2_SMALL, [1, 4, 1, 1, 1, 32, 3, 1, 1, 4, 6, 1, 1, 2, 2, 8, 1, 5, 5, 1, 0, 1], 1),
    ("mfma16 boxed C1-like", C1_SMALL, [1, 16, 1, 1, 1, 16, 7, 1, 1, 1, 7, 1, 1, 1, 3, 1, 11, 1, 1, 11, 1, 0], 2),
    ("scalar boxed, unrolled by 8", C2_SMALL, [4, 1, 4, 2, 1, 4, 3, 1, 2, 2, 3, 2, 1, 2, 4, 4, 1, 5, 5, 1, 1, 3], 0),
]


@pytest.mark.parametrize("label,kd,cfg,path", BOX_COMPILE_CASES, ids=[c[0] for c in BOX_COMPILE_CASES])
def test_separately_split_reduction_templates_compile(label, kd, cfg, path):
    op = _op(kd, P.OPEVO_BF16)
    plan = P.opevo_kernel_plan(op, P.OPEVO_TILE4P, cfg)
    assert plan.status == P.OPEVO_OK and plan.path == path, (plan.reason, plan.path)
    kernel, _ = P.opevo_kernel_build(op, P.OPEVO_TILE4P, cfg)
    assert P.opevo_kernel_code_size(kernel) > 1000
    P.opevo_kernel_destroy(kernel)


def test_image_gather_table_is_used_where_it_fits():
    """The MFMA template gathers the image through a compile-time table of 8 bytes per position of
    the reduction walk; past 8192 positions it falls back to the element-wise gather."""
    small = _op(C2_SMALL, P.OPEVO_BF16)
    d = P.opevo_kernel_defines(small, P.OPEVO_TILE4, [1, 4, 1, 1, 1, 32, 3, 1, 1, 4, 6, 1, 1, 2, 25, 16, 1])
    assert "-DCONV_TABLE=1" in d
    assert "CONV_TABLE" not in P.opevo_kernel_defines(small, P.OPEVO_TILE4, [4, 1, 4, 2, 1, 4, 3, 1, 2, 2, 3, 2, 1, 2, 25, 16, 1])   # scalar
    deep = _op((P.OPEVO_CONV2D, (2, 1024, 8, 8, 32, 3, 3, 1, 1)), P.OPEVO_BF16)     # 9216 taps
    for cfg in ([1, 2, 1, 1, 1, 32, 2, 1, 1, 4, 2, 1, 1, 4, 288, 32, 1], [1, 2, 1, 1, 1, 32, 2, 1, 1, 4, 2, 1, 1, 4, 192, 48, 0]):
        plan = P.opevo_kernel_plan(deep, P.OPEVO_TILE4, cfg)
        assert plan.status == P.OPEVO_OK and plan.path == 1
        assert "-DCONV_TABLE=0" in P.opevo_kernel_defines(deep, P.OPEVO_TILE4, cfg)
        kernel, _ = P.opevo_kernel_build(deep, P.OPEVO_TILE4, cfg)
        P.opevo_kernel_destroy(kernel)


# ------------------------------------------------------------------ MatMul space with the reduction axis in three factors
MM3 = (P.OPEVO_MATMUL, (512, 1024, 4096))


def test_split_reduction_space_has_three_k_factors_and_is_matmul_only():
    op = _op(MM3, P.OPEVO_BF16)
    sp = P.opevo_op_space(op, P.OPEVO_TILE4K)
    names = [P.opevo_space_param_name(sp, i) for i in range(P.opevo_space_num_params(sp))]
    assert names == ["M", "N", "K", "unroll"] and P.opevo_space_width(sp) == 12
    # 4096 = 2^12 in three ordered factors: C(14, 2) = 91
    assert P.opevo_space_param_size(sp, 2) == 91
    P.opevo_space_destroy(sp)
    for kd in (BMM, CONV56):
        with pytest.raises(P.OpevoError):
            P.opevo_op_space(_op(kd, P.OPEVO_BF16), P.OPEVO_TILE4K)


def test_split_reduction_members_put_the_partitions_on_grid_z():
    op = _op(MM3, P.OPEVO_BF16)
    cfg = [4, 2, 2, 32, 8, 2, 2, 32, 8, 16, 32, 1]            # 8 partitions of 16 slabs of 32
    plan = P.opevo_kernel_plan(op, P.OPEVO_TILE4K, cfg)
    assert plan.status == P.OPEVO_OK and plan.path == 3 and list(plan.grid) == [8, 4, 8] and list(plan.tile) == [128, 128, 32]
    d = P.opevo_kernel_defines(op, P.OPEVO_TILE4K, cfg)
    assert "-DKSPLIT=8" in d and "-DKSTEPS=16" in d and "-DK=4096" in d
    one = [4, 2, 2, 32, 8, 2, 2, 32, 1, 128, 32, 1]           # one partition: the plain kernel
    plan = P.opevo_kernel_plan(op, P.OPEVO_TILE4K, one)
    assert list(plan.grid) == [8, 4, 1] and "KSPLIT" not in P.opevo_kernel_defines(op, P.OPEVO_TILE4K, one)
    with pytest.raises(P.OpevoError):                          # 8 * 16 * 16 != 4096
        P.opevo_kernel_plan(op, P.OPEVO_TILE4K, [4, 2, 2, 32, 8, 2, 2, 32, 8, 16, 16, 1])


SPLITK_COMPILE_CASES = [
    ("direct-to-LDS, 8 partitions", [4, 2, 2, 32, 8, 2, 2, 32, 8, 16, 32, 1], 3),
    ("mfma32 register-staged, 8 partitions", [4, 2, 2, 32, 8, 2, 2, 32, 8, 32, 16, 1], 1),
    ("mfma16, 4 partitions, single stage", [16, 2, 1, 16, 32, 2, 1, 16, 4, 32, 32, 0], 2),
    ("scalar, 16 partitions", [16, 2, 4, 4, 32, 2, 4, 4, 16, 32, 8, 1], 0),
]


@pytest.mark.parametrize("label,cfg,path", SPLITK_COMPILE_CASES, ids=[c[0] for c in SPLITK_COMPILE_CASES])
def test_split_reduction_templates_compile(label, cfg, path):
    op = _op(MM3, P.OPEVO_BF16)
    plan = P.opevo_kernel_plan(op, P.OPEVO_TILE4K, cfg)
    assert plan.status == P.OPEVO_OK and plan.path == path, (plan.reason, plan.path)
    kernel, _ = P.opevo_kernel_build(op, P.OPEVO_TILE4K, cfg)
    assert P.opevo_kernel_code_size(kernel) > 1000
    P.opevo_kernel_destroy(kernel)


def test_fp32_inputs_use_the_fp32_mfma_template_where_the_tile_allows():
    op = _op(MM1, P.OPEVO_F32)
    for cfg, path in (([4, 2, 2, 32, 8, 2, 2, 32, 32, 32, 1], 4), ([4, 2, 2, 32, 8, 2, 2, 32, 32, 32, 0], 4),
                      ([4, 2, 2, 32, 8, 2, 2, 32, 256, 4, 1], 0),        # slab not a multiple of 8
                      ([16, 2, 1, 16, 16, 2, 1, 32, 16, 64, 1], 0)):      # wave tile not made of 32 x 32 atoms
        plan = P.opevo_kernel_plan(op, P.OPEVO_TILE4, cfg)
        assert plan.status == P.OPEVO_OK and plan.path == path, (cfg, plan.path, plan.reason)
    # two stages of (128 x 36 + 32 x 132) floats
    assert P.opevo_kernel_plan(op, P.OPEVO_TILE4, [4, 2, 2, 32, 8, 2, 2, 32, 32, 32, 1]).lds_bytes == 2 * (128 * 36 + 32 * 132) * 4
    kernel, _ = P.opevo_kernel_build(op, P.OPEVO_TILE4, [4, 2, 2, 32, 8, 2, 2, 32, 32, 32, 1])
    assert "gemm_mfma_f32" in P.opevo_kernel_defines(op, P.OPEVO_TILE4, [4, 2, 2, 32, 8, 2, 2, 32, 32, 32, 1])
    P.opevo_kernel_destroy(kernel)
    # 16-bit inputs never take it; a transposed first operand and convolutions do
    assert P.opevo_kernel_plan(_op(MM1, P.OPEVO_BF16), P.OPEVO_TILE4, [4, 2, 2, 32, 8, 2, 2, 32, 32, 32, 1]).path in (1, 3)
    conv = _op(C2_SMALL, P.OPEVO_F32)
    for cfg, path, bkp in (([1, 4, 1, 1, 1, 32, 3, 1, 1, 4, 6, 1, 1, 2, 25, 16, 1], 4, 16),
                           ([1, 4, 1, 1, 1, 32, 3, 1, 1, 4, 6, 1, 1, 2, 80, 5, 1], 4, 8),        # slab of 5 taps staged 8 wide
                           ([2, 2, 1, 1, 1, 32, 2, 1, 1, 6, 6, 1, 1, 2, 16, 25, 1], 4, 32),      # 24-column wave tile rounded up to 32
                           ([4, 1, 4, 2, 1, 4, 3, 1, 2, 2, 3, 2, 1, 2, 25, 16, 1], 0, 16)):      # 4 x 8 wave tile: scalar
        plan = P.opevo_kernel_plan(conv, P.OPEVO_TILE4, cfg)
        assert plan.status == P.OPEVO_OK and plan.path == path, (cfg, plan.path, plan.reason)
        assert "-DBKP=%d" % bkp in P.opevo_kernel_defines(conv, P.OPEVO_TILE4, cfg)
    ta = P.opevo_op_create(P.OPEVO_BMM_TA, (960, 128, 64, 128), P.OPEVO_F32)
    cfg = [160, 6, 1, 2, 2, 32, 1, 1, 2, 32, 8, 16, 1]
    plan = P.opevo_kernel_plan(ta, P.OPEVO_TILE4, cfg)
    assert plan.path == 4 and plan.lds_bytes == 2 * (16 * 132 + 16 * 68) * 4
    kernel, _ = P.opevo_kernel_build(ta, P.OPEVO_TILE4, cfg)
    P.opevo_kernel_destroy(kernel)


# ---------------------------------------------------------------- Conv2d: split reduction + channels-last operands (TILE4C)
def test_conv_split_channels_last_space_and_its_decoding():
    op = _op(CONV14, P.OPEVO_BF16)
    sp = P.opevo_op_space(op, P.OPEVO_TILE4C)
    names = [P.opevo_space_param_name(sp, i) for i in range(P.opevo_space_num_params(sp))]
    assert names == ["B", "Cout", "H", "W", "R", "unroll", "layout"] and P.opevo_space_width(sp) == 19
    # 2304 = 2^8 * 3^2 in three ordered factors: C(10, 2) * C(4, 2) = 45 * 6
    assert P.opevo_space_param_size(sp, 4) == 270
    P.opevo_space_destroy(sp)
    for kd in (MM1, BMM):
        with pytest.raises(P.OpevoError):
            P.opevo_op_space(_op(kd, P.OPEVO_BF16), P.OPEVO_TILE4C)
    V = P.OPEVO_TILE4C
    # 4 partitions on grid z; channels last; 14 waves of 64 x 28 (rounded up to 32): the direct-to-LDS
    # template with both stage parts rounded up to whole 1 KiB loads per wave (224 rows each)
    cfg = [32, 1, 2, 2, 2, 32, 1, 7, 2, 1, 1, 1, 14, 1, 4, 9, 64, 1, 1]
    plan = P.opevo_kernel_plan(op, V, cfg)
    d = P.opevo_kernel_defines(op, V, cfg)
    assert plan.status == P.OPEVO_OK and plan.path == 3 and list(plan.grid) == [32, 2, 4] and plan.block == 896
    assert list(plan.tile) == [128, 196, 64] and list(plan.wave_tile) == [64, 28] and plan.acc_per_lane == 32
    for want in ("-DKSPLIT=4", "-DKSTEPS=9", "-DCONV_NHWC=1", "-DB_KMAJOR=1", "-DBNR=224", "-DANR=224", "-DNSTG=2"):
        assert want in d.split(), (want, d)
    assert plan.lds_bytes == 2 * (224 + 224) * 64 * 2
    # layout = 0: the same tiles on the NCHW gather (register-staged, 16x16 atoms), same grid
    plan0 = P.opevo_kernel_plan(op, V, cfg[:18] + [0])
    d0 = P.opevo_kernel_defines(op, V, cfg[:18] + [0])
    assert plan0.path == 2 and list(plan0.grid) == [32, 2, 4] and "CONV_NHWC" not in d0 and "-DKSPLIT=4" in d0.split()
    # not pipelined (unroll = 0): channels last on the register-staged template
    d1 = P.opevo_kernel_defines(op, V, cfg[:17] + [0, 1])
    assert P.opevo_kernel_plan(op, V, cfg[:17] + [0, 1]).path == 2 and "-DCONV_NHWC=1" in d1.split() and "B_KMAJOR" not in d1
    # a slab that is no multiple of 8 (2304 = 36 * 4 * 16 ... here 9 * 4 * 4 * 4 * 4: slab 4): the choice is inert
    d2 = P.opevo_kernel_defines(op, V, cfg[:14] + [4, 144, 4, 1, 1])
    assert "CONV_NHWC" not in d2
    with pytest.raises(P.OpevoError):                          # 4 * 9 * 32 != 2304
        P.opevo_kernel_plan(op, V, cfg[:14] + [4, 9, 32, 1, 1])
    # three input channels (the paper's C1): no channels-last member exists
    c1 = _op((P.OPEVO_CONV2D, (16, 3, 35, 35, 16, 11, 11, 4, 0)), P.OPEVO_BF16)
    assert "CONV_NHWC" not in P.opevo_kernel_defines(c1, V, [1, 16, 1, 1, 1, 16, 7, 1, 1, 1, 7, 1, 1, 1, 1, 11, 33, 1, 1])


def test_conv_split_channels_last_space_is_not_mostly_invalid_and_reaches_every_template():
    op = _op(CONV14, P.OPEVO_BF16)
    V = P.OPEVO_TILE4C
    sp = P.opevo_op_space(op, V)
    rng = P.opevo_rng_create(5)
    paths, valid, total = {}, 0, 3000
    for _ in range(total):
        cfg = P.opevo_space_random(sp, rng)
        plan = P.opevo_kernel_plan(op, V, cfg)
        if plan.status == P.OPEVO_OK:
            valid += 1
            paths[plan.path] = paths.get(plan.path, 0) + 1
            assert plan.lds_bytes <= 160 * 1024 and plan.block <= 1024 and plan.acc_per_lane <= 256
            assert plan.grid[2] == cfg[14]                     # partitions on grid z
    assert valid > 0.3 * total and set(paths) == {0, 1, 2, 3}, (valid, paths)
    P.opevo_rng_destroy(rng); P.opevo_space_destroy(sp)


TILE4C_COMPILE_CASES = [
    ("direct-to-LDS, channels last, 14 waves, padded stage parts, 4 partitions", CONV14, [32, 1, 2, 2, 2, 32, 1, 7, 2, 1, 1, 1, 14, 1, 4, 9, 64, 1, 1], 3),
    ("direct-to-LDS, channels last, one wave of 32 x 28, slabs of 128 in groups of 4 steps", CONV14, [32, 1, 8, 1, 1, 32, 1, 7, 2, 1, 1, 1, 14, 1, 1, 18, 128, 1, 1], 3),
    ("direct-to-LDS, multi-tap slabs (16 channels, slab 64 = 4 taps)", (P.OPEVO_CONV2D, (3, 16, 11, 11, 32, 4, 4, 1, 1)), [3, 1, 1, 1, 1, 32, 1, 2, 1, 5, 1, 2, 1, 5, 1, 4, 64, 1, 1], 3),
    ("register-staged, channels last, slab 40 padded to 48", (P.OPEVO_CONV2D, (4, 16, 12, 12, 32, 5, 5, 1, 2)), [1, 4, 1, 1, 1, 32, 3, 1, 1, 4, 6, 1, 1, 2, 2, 5, 40, 1, 1], 1),
    ("register-staged 16x16 atoms, NCHW gather, 9 partitions", CONV14, [8, 4, 4, 2, 1, 32, 7, 1, 1, 2, 7, 1, 1, 2, 9, 8, 32, 1, 0], 2),
    ("scalar, 2 partitions", CONV56, [1, 1, 8, 2, 1, 4, 7, 2, 2, 2, 2, 1, 7, 4, 2, 12, 24, 0, 1], 0),
]


@pytest.mark.parametrize("label,kd,cfg,path", TILE4C_COMPILE_CASES, ids=[c[0] for c in TILE4C_COMPILE_CASES])
def test_conv_split_channels_last_templates_compile(label, kd, cfg, path):
    op = _op(kd, P.OPEVO_BF16)
    plan = P.opevo_kernel_plan(op, P.OPEVO_TILE4C, cfg)
    assert plan.status == P.OPEVO_OK and plan.path == path, (plan.reason, plan.path)
    kernel, _ = P.opevo_kernel_build(op, P.OPEVO_TILE4C, cfg)
    assert 1000 < P.opevo_kernel_code_size(kernel) < (128 << 10)
    P.opevo_kernel_destroy(kernel)



# ---------------------------------------------------------------- Conv2d: the operand path as a choice, LDS-resident patch (TILE4L)
def test_conv_patch_space_and_its_decoding():
    op = _op(CONV14, P.OPEVO_BF16)
    V = P.OPEVO_TILE4L
    sp = P.opevo_op_space(op, V)
    names = [P.opevo_space_param_name(sp, i) for i in range(P.opevo_space_num_params(sp))]
    assert names == ["B", "Cout", "H", "W", "Cin", "unroll", "layout", "kwaves"] and P.opevo_space_width(sp) == 19
    assert P.opevo_space_param_size(sp, 4) == 9 and P.opevo_space_param_size(sp, 6) == 3 and P.opevo_space_param_size(sp, 7) == 4
    P.opevo_space_destroy(sp)
    for kd in (MM1, BMM):
        with pytest.raises(P.OpevoError):
            P.opevo_op_space(_op(kd, P.OPEVO_BF16), V)
    # 32 output channels x one image, 7 pixel waves of 28 -> 32 x 2 waves per tile, slabs of 32 channels, single stage
    cfg = [32, 1, 8, 1, 1, 32, 1, 7, 1, 2, 1, 1, 1, 14, 8, 32, 0, 2, 1]
    plan = P.opevo_kernel_plan(op, V, cfg)
    d = P.opevo_kernel_defines(op, V, cfg)
    assert d.startswith("conv_patch:")
    assert plan.status == P.OPEVO_OK and plan.path == 5 and list(plan.grid) == [32, 8, 1] and plan.block == 64 * 7 * 2
    assert list(plan.tile) == [32, 196, 32 * 9] and list(plan.wave_tile) == [32, 28] and plan.acc_per_lane == 16
    # patch of 16 rows, row pitch 30 (16 raised to be congruent to 14 modulo 16), image pitch 480 + 4 (congruent to 196)
    for want in ("-DATOM=32", "-DCS=32", "-DKSTEPS=8", "-DKW=2", "-DNSTG=1", "-DPWP=30", "-DIPIX=484", "-DWM=1", "-DWN=7"):
        assert want in d.split(), (want, d)
    # padded patch pixels, unpadded kernel-tensor rows, dump words; or, if more, one 32x32 atom of each of the 14 waves for the final sum
    assert plan.lds_bytes == max((484 * 40 + 9 * 32 * 32 + 64) * 2, 14 * 4 * 1024)
    # the other two layouts of the same member: the gather walks (ci, r, s) in slabs of 32 * 9, too long for the LDS beside
    # a tile of 32 x 196 and so halved to 16 * 9; the channels-last member (r, s, ci) in slabs of 32, with its pre-pass;
    # kwaves is inert there
    d0 = P.opevo_kernel_defines(op, V, cfg[:17] + [0, 1])
    assert not d0.startswith("conv_patch:") and "-DBK=144" in d0.split() and "-DKSTEPS=16" in d0.split() and "CONV_NHWC" not in d0 and "-DKW" not in d0
    d1 = P.opevo_kernel_defines(op, V, cfg[:17] + [1, 1])
    assert "-DBK=32" in d1.split() and "-DKSTEPS=72" in d1.split() and "-DCONV_NHWC=1" in d1.split()
    with pytest.raises(P.OpevoError):                          # 8 * 16 != 256
        P.opevo_kernel_plan(op, V, cfg[:14] + [8, 16, 0, 2, 1])
    with pytest.raises(P.OpevoError):                          # layout has three values
        P.opevo_kernel_plan(op, V, cfg[:17] + [3, 1])
    # 16x16x32 atoms where they pad the pixel side less (98 -> 112 instead of 128) and the slab has whole 32 channels
    assert "-DATOM=16" in P.opevo_kernel_defines(op, V, [32, 1, 4, 1, 2, 32, 2, 1, 1, 7, 1, 1, 1, 14, 8, 32, 1, 2, 2]).split()
    # an image of odd width is filled by pairs of pixels at 2-byte alignment: same template
    c27 = _op((P.OPEVO_CONV2D, (4, 64, 27, 27, 64, 5, 5, 1, 2)), P.OPEVO_BF16)
    assert P.opevo_kernel_plan(c27, V, [4, 1, 1, 2, 1, 32, 3, 3, 1, 3, 1, 1, 1, 27, 4, 16, 0, 2, 0]).path == 5
    # an image one pixel wide has no pairs of pixels: layout 0
    c1w = _op((P.OPEVO_CONV2D, (4, 32, 8, 1, 32, 3, 1, 1, 0)), P.OPEVO_BF16)
    assert P.opevo_kernel_plan(c1w, V, [4, 1, 1, 1, 1, 32, 1, 1, 1, 6, 1, 1, 1, 1, 1, 32, 0, 2, 0]).path != 5
    assert P.opevo_kernel_plan(_op((P.OPEVO_CONV2D, (4, 32, 8, 2, 32, 3, 1, 1, 0)), P.OPEVO_BF16), V, [4, 1, 1, 1, 1, 32, 1, 1, 1, 6, 1, 1, 1, 2, 1, 32, 0, 2, 0]).path == 5
    # three input channels (the paper's C1): no slab of 16 channels, no patch member
    c1 = _op((P.OPEVO_CONV2D, (16, 3, 35, 35, 16, 11, 11, 4, 0)), P.OPEVO_BF16)
    assert P.opevo_kernel_plan(c1, V, [1, 16, 1, 1, 1, 16, 7, 1, 1, 1, 7, 1, 1, 1, 1, 3, 1, 2, 0]).path != 5


def test_conv_patch_space_is_not_mostly_invalid_and_the_patch_template_has_a_share_of_it():
    for kd, share in ((CONV14, 0.05), (CONV56, 0.08)):
        op = _op(kd, P.OPEVO_BF16)
        V = P.OPEVO_TILE4L
        sp = P.opevo_op_space(op, V)
        rng = P.opevo_rng_create(5)
        paths, valid, total = {}, 0, 3000
        for _ in range(total):
            cfg = P.opevo_space_random(sp, rng)
            plan = P.opevo_kernel_plan(op, V, cfg)
            if plan.status == P.OPEVO_OK:
                valid += 1
                paths[plan.path] = paths.get(plan.path, 0) + 1
                assert plan.lds_bytes <= 160 * 1024 and plan.block <= 1024 and plan.acc_per_lane <= 256 and plan.grid[2] == 1
                if plan.path == 5:
                    assert cfg[17] == 2
        assert valid > 0.5 * total and set(paths) == {0, 1, 2, 3, 5} and paths[5] > share * total, (valid, paths)
        P.opevo_rng_destroy(rng); P.opevo_space_destroy(sp)


TILE4L_COMPILE_CASES = [
    ("patch, 14 waves (7 pixel waves x 2 per tile), single stage", CONV14, [32, 1, 8, 1, 1, 32, 1, 7, 1, 2, 1, 1, 1, 14, 8, 32, 0, 2, 1], 5),
    ("patch, 16x16 atoms, 64 x 98 -> 112 shared by 4 waves, two stages", CONV14, [32, 1, 4, 1, 2, 32, 2, 1, 1, 7, 1, 1, 1, 14, 8, 32, 1, 2, 2], 5),
    ("patch, folded: slabs of 8 channels, 4 waves of 8 output channels", CONV56, [1, 1, 2, 4, 2, 4, 14, 4, 1, 1, 1, 1, 1, 56, 8, 8, 1, 2, 3], 5),
    ("patch, odd width, 25 taps", (P.OPEVO_CONV2D, (4, 64, 27, 27, 64, 5, 5, 1, 2)), [4, 1, 1, 2, 1, 32, 3, 3, 1, 3, 1, 1, 1, 27, 4, 16, 0, 2, 0], 5),
    ("patch, 49 taps: the loop over the steps stays a loop", (P.OPEVO_CONV2D, (2, 32, 12, 12, 32, 7, 7, 1, 3)), [2, 1, 1, 2, 1, 16, 1, 2, 1, 6, 1, 1, 1, 12, 1, 32, 1, 2, 0], 5),
    ("channels last in this space (direct-to-LDS)", CONV56, [1, 1, 1, 2, 1, 32, 14, 2, 1, 2, 1, 1, 1, 56, 2, 32, 1, 1, 0], 3),
]


@pytest.mark.parametrize("label,kd,cfg,path", TILE4L_COMPILE_CASES, ids=[c[0] for c in TILE4L_COMPILE_CASES])
def test_conv_patch_templates_compile(label, kd, cfg, path):
    op = _op(kd, P.OPEVO_BF16)
    plan = P.opevo_kernel_plan(op, P.OPEVO_TILE4L, cfg)
    assert plan.status == P.OPEVO_OK and plan.path == path, (plan.reason, plan.path)
    kernel, _ = P.opevo_kernel_build(op, P.OPEVO_TILE4L, cfg)
    assert 1000 < P.opevo_kernel_code_size(kernel) < (128 << 10)
    P.opevo_kernel_destroy(kernel)

# ---------------------------------------------------------------- MatMul: second operand transposed by a pre-pass (TILE4T)
def test_packed_second_operand_space_and_its_decoding():
    op = _op((P.OPEVO_MATMUL, (8192, 8192, 8192)), P.OPEVO_BF16)
    V = P.OPEVO_TILE4T
    sp = P.opevo_op_space(op, V)
    names = [P.opevo_space_param_name(sp, i) for i in range(P.opevo_space_num_params(sp))]
    assert names == ["M", "N", "K", "unroll", "bpack"] and P.opevo_space_width(sp) == 12
    assert P.opevo_space_size(sp) == 2 * P.opevo_space_size(P.opevo_op_space(op, P.OPEVO_TILE4))
    P.opevo_space_destroy(sp)
    with pytest.raises(P.OpevoError):
        P.opevo_op_space(_op(CONV56, P.OPEVO_BF16), V)
    cfg = [32, 2, 2, 64, 32, 2, 2, 64, 256, 32, 1]
    for bpack in (0, 1):
        plan = P.opevo_kernel_plan(op, V, cfg + [bpack])
        d = P.opevo_kernel_defines(op, V, cfg + [bpack])
        assert plan.status == P.OPEVO_OK and plan.path == 3 and plan.lds_bytes == 4 * 512 * 32 * 2
        assert ("-DB_KMAJOR=1" in d.split()) == (bpack == 1) and ("-DBNR=256" in d.split()) == (bpack == 1)
    # on a member of the register-staged template the choice is inert
    d = P.opevo_kernel_defines(op, V, [32, 2, 1, 128, 32, 2, 1, 128, 512, 16, 1, 1])
    assert "B_KMAJOR" not in d
    # with the second operand K-contiguous, tile widths that the [K][N] chunk permutation cannot serve become eligible
    mm = _op((P.OPEVO_MATMUL, (512, 768, 1024)), P.OPEVO_BF16)
    c96 = [4, 2, 2, 32, 8, 1, 3, 32, 32, 32, 1]                # BN = 96
    assert P.opevo_kernel_plan(mm, V, c96 + [0]).path == 1 and P.opevo_kernel_plan(mm, V, c96 + [1]).path == 3


TILE4T_COMPILE_CASES = [
    ("256x256, 4 waves, 4 stages of 32", (P.OPEVO_MATMUL, (8192, 8192, 8192)), [32, 2, 2, 64, 32, 2, 2, 64, 256, 32, 1, 1]),
    ("one wave of 32 x 64, slabs of 64 in groups of 2 steps", MM1, [16, 1, 1, 32, 16, 1, 2, 32, 16, 64, 1, 1]),
    ("96-wide tile", (P.OPEVO_MATMUL, (512, 768, 1024)), [4, 2, 2, 32, 8, 1, 3, 32, 32, 32, 1, 1]),
]


@pytest.mark.parametrize("label,kd,cfg", TILE4T_COMPILE_CASES, ids=[c[0] for c in TILE4T_COMPILE_CASES])
def test_packed_second_operand_templates_compile(label, kd, cfg):
    op = _op(kd, P.OPEVO_BF16)
    plan = P.opevo_kernel_plan(op, P.OPEVO_TILE4T, cfg)
    assert plan.status == P.OPEVO_OK and plan.path == 3, (plan.reason, plan.path)
    assert "-DB_KMAJOR=1" in P.opevo_kernel_defines(op, P.OPEVO_TILE4T, cfg).split()
    kernel, _ = P.opevo_kernel_build(op, P.OPEVO_TILE4T, cfg)
    assert 1000 < P.opevo_kernel_code_size(kernel) < (128 << 10)
    P.opevo_kernel_destroy(kernel)


# ---------------------------------------------------------------- MatMul: the MFMA atom of direct-to-LDS members as a choice (TILE4A)
def test_atom_choice_space_and_its_decoding():
    op = _op((P.OPEVO_MATMUL, (8192, 8192, 8192)), P.OPEVO_BF16)
    V = P.OPEVO_TILE4A
    sp = P.opevo_op_space(op, V)
    names = [P.opevo_space_param_name(sp, i) for i in range(P.opevo_space_num_params(sp))]
    assert names == ["M", "N", "K", "unroll", "atom"] and P.opevo_space_width(sp) == 12
    assert P.opevo_space_size(sp) == 2 * P.opevo_space_size(P.opevo_op_space(op, P.OPEVO_TILE4))
    P.opevo_space_destroy(sp)
    for other in (CONV56, (P.OPEVO_BMM, (128, 128, 128, 64))):
        with pytest.raises(P.OpevoError):
            P.opevo_op_space(_op(other, P.OPEVO_BF16), V)
    cfg = [32, 2, 8, 16, 32, 4, 2, 32, 256, 32, 1]                 # 256 x 256 tile, 8 waves of 128 x 64, 4 stages of 32
    for atom in (0, 1):
        plan = P.opevo_kernel_plan(op, V, cfg + [atom])
        same = P.opevo_kernel_plan(op, P.OPEVO_TILE4, cfg)
        d = P.opevo_kernel_defines(op, V, cfg + [atom]).split()
        # same tiles, same ring, same accumulators per lane: only the atom differs
        assert (plan.status, plan.path, plan.lds_bytes, plan.block, plan.acc_per_lane) == (P.OPEVO_OK, 3, same.lds_bytes, same.block, same.acc_per_lane)
        assert ("-DATOM=16" in d) == (atom == 1) and ("-DATOM=32" in d) == (atom == 0)
    # inert on the other templates, ...
    for c in ([32, 2, 1, 128, 32, 2, 1, 128, 512, 16, 1, 1], [32, 2, 2, 64, 32, 2, 2, 64, 256, 32, 0, 1]):
        assert P.opevo_kernel_plan(op, V, c).path == 1 and "-DATOM=32" in P.opevo_kernel_defines(op, V, c).split()
    # ... with a transposed first operand there is no such space at all, and a member whose ring has an odd number of
    # stages keeps the 32x32x16 atoms when a slab is a single K step of the small atom (the fragment buffers alternate
    # per step, and which one a step uses must be known at compile time)
    mm = _op((P.OPEVO_MATMUL, (512, 1024, 1024)), P.OPEVO_BF16)
    n_odd = 0
    sp = P.opevo_op_space(mm, V)
    rng = P.opevo_rng_create(5)
    for _ in range(40000):
        c = P.opevo_space_random(sp, rng)
        plan = P.opevo_kernel_plan(mm, V, c)
        if plan.status != P.OPEVO_OK or plan.path != 3 or c[11] != 1:
            continue
        d = dict(t[2:].split("=") for t in P.opevo_kernel_defines(mm, V, c).split(":", 1)[1].split() if "=" in t)
        if int(d["NSTG"]) % 2 == 1 and int(d["BK"]) == 32:
            n_odd += 1
            assert d["ATOM"] == "32", list(c)
        if d["ATOM"] == "16":
            assert int(d["BK"]) % 32 == 0 and int(d["TM"]) % 16 == 0 and "B_KMAJOR" not in d and d["A_TRANS"] == "0"
    P.opevo_rng_destroy(rng); P.opevo_space_destroy(sp)


TILE4A_COMPILE_CASES = [
    ("256x256, 8 waves of 128x64, 2 stages of 64 (the member the 8192^3 searches end on)", (P.OPEVO_MATMUL, (8192, 8192, 8192)), [32, 2, 64, 2, 32, 4, 4, 16, 128, 64, 1, 1]),
    ("256x256, 4 waves of 128x128, 4 stages of 32: 64 MFMAs per step", (P.OPEVO_MATMUL, (8192, 8192, 8192)), [32, 2, 2, 64, 32, 2, 2, 64, 256, 32, 1, 1]),
    ("one wave of 32 x 64, slabs of 64", MM1, [16, 1, 1, 32, 16, 1, 2, 32, 16, 64, 1, 1]),
    ("2 stages of 128", MM1, [4, 2, 1, 64, 8, 2, 1, 64, 8, 128, 1, 1]),
]


@pytest.mark.parametrize("label,kd,cfg", TILE4A_COMPILE_CASES, ids=[c[0] for c in TILE4A_COMPILE_CASES])
def test_direct_to_lds_members_on_16x16x32_atoms_compile_fully_unrolled(label, kd, cfg):
    op = _op(kd, P.OPEVO_BF16)
    plan = P.opevo_kernel_plan(op, P.OPEVO_TILE4A, cfg)
    assert plan.status == P.OPEVO_OK and plan.path == 3, (plan.reason, plan.path)
    assert "-DATOM=16" in P.opevo_kernel_defines(op, P.OPEVO_TILE4A, cfg).split()
    kernel, _ = P.opevo_kernel_build(op, P.OPEVO_TILE4A, cfg)
    assert 1000 < P.opevo_kernel_code_size(kernel) < (128 << 10)
    P.opevo_kernel_destroy(kernel)
