"""Host logic of the GPU library: launch planning and the exact-cover check of
the kernels' index walk.  Runs without a GPU (no compute call is made)."""
import itertools

import pytest

import paper_2505_13813_amd as grkan
from paper_2505_13813_amd import GRKAN_BF16, GRKAN_F32

# (rows, D, G) of every configuration the bench and parity tests use, cut to a
# size the simulator walks in well under a second, plus awkward shapes
SHAPES = [
    (788, 192, 8),      # tiny config: 96-byte segments -> flat walk
    (1000, 768, 8),     # KAT-T x2 / KAT-B x1
    (300, 384, 8), (300, 1536, 8), (301, 3072, 8),
    (130, 3072, 1), (130, 3072, 64),
    (37, 40, 5), (33, 30, 5), (29, 35, 5), (1, 192, 8), (3, 8, 8), (5, 7, 1), (64, 64, 1),
    (1023, 24, 3), (2, 6 * 1009, 6),
]


@pytest.mark.parametrize("rows,D,G", SHAPES)
@pytest.mark.parametrize("io", [GRKAN_F32, GRKAN_BF16])
def test_walk_covers_every_vector_exactly_once(rows, D, G, io):
    es = 4 if io == GRKAN_F32 else 2
    for align, (num_cu, wg_per_cu), forward in itertools.product((16, 8, es), ((256, 4), (256, 8), (3, 1)),
                                                                (False, True)):
        p = grkan.plan(rows, D, G, io, align_bytes=align, num_cu=num_cu, wg_per_cu=wg_per_cu, forward=forward)
        walk_groups = p.column_split if p.lane_coef else G * p.column_split
        assert p.grid == (walk_groups // p.groups_per_wg) * p.wg_per_bundle
        assert p.column_split == 1 or (not forward and (p.lane_coef or G < 4))
        assert not p.lane_coef or G % p.column_split == 0
        assert p.partials_per_group == p.wg_per_bundle * (1 if p.lane_coef else p.column_split)
        assert not p.lane_coef or p.fixed_col
        assert p.vec * es <= align and (D // G) % p.vec == 0
        assert grkan.plan_cover_errors(rows, D, G, io, p) == 0, p.as_dict()


def test_general_walk_is_used_when_columns_cannot_be_fixed_and_still_covers():
    # d_g = 64 * 1031 (line-aligned segments, so the group walk is chosen): 64 * (waves per group)
    # is never a multiple of d_g / vec within the grid budget
    rows, G, dg = 3, 64, 64 * 1031
    for io in (GRKAN_F32, GRKAN_BF16):
        p = grkan.plan(rows, G * dg, G, io)
        assert (p.fixed_col, p.lane_coef, p.groups_per_wg) == (0, 0, 1)
        assert grkan.plan_cover_errors(rows, G * dg, G, io, p) == 0


def test_group_walk_bundles_groups_when_the_flat_walk_cannot_fix_columns():
    # 96-byte-misaligned segments (d_g = 24 * 10007) whose rows are too long for the flat walk to
    # keep columns fixed: group walk, 4 adjacent groups per workgroup, general columns
    rows, G, dg = 3, 8, 24 * 10007
    p = grkan.plan(rows, G * dg, G, GRKAN_F32)
    assert (p.fixed_col, p.lane_coef, p.groups_per_wg, p.waves_per_group_in_wg) == (0, 0, 4, 1)
    assert grkan.plan_cover_errors(rows, G * dg, G, GRKAN_F32, p) == 0


def test_few_long_groups_are_walked_as_column_blocks():
    # one group of 3072 float32 channels: four blocks of 768 (3072 bytes each); two groups: two blocks each
    p = grkan.plan(50432, 3072, 1, GRKAN_F32)
    assert (p.column_split, p.vecs_per_segment, p.lane_coef, p.fixed_col) == (4, 192, 0, 1)
    assert p.grid == 4 * p.wg_per_bundle and p.partials_per_group == 4 * p.wg_per_bundle
    p = grkan.plan(50432, 3072, 2, GRKAN_F32)
    assert p.column_split == 2
    # the blocks must stay whole cache lines, at least three: 192 float32 channels = 768 bytes split once only
    p = grkan.plan(1000, 192, 1, GRKAN_F32)
    assert (p.column_split, p.vecs_per_segment) == (2, 24)
    # ... and whole vectors: 96 channels of bfloat16 = 192 bytes cannot be split
    assert grkan.plan(1000, 96, 1, GRKAN_BF16).column_split == 1
    # the forward pass and four or more groups are left alone
    assert grkan.plan(50432, 3072, 1, GRKAN_F32, forward=True).column_split == 1
    assert grkan.plan(50432, 3072, 4, GRKAN_F32).column_split == 1
    for rows, D, G in ((130, 3072, 1), (77, 1536, 2), (64, 768, 3), (5, 7, 1)):
        for io in (GRKAN_F32, GRKAN_BF16):
            p = grkan.plan(rows, D, G, io)
            assert grkan.plan_cover_errors(rows, D, G, io, p) == 0, (rows, D, G, io, p.as_dict())


def test_headline_plans():
    # KAT-B x2 fp32: 1536-byte segments are line aligned -> one group per
    # workgroup, all four waves share it, fixed columns, one persistent wave of
    # workgroups
    p = grkan.plan(25216, 3072, 8, GRKAN_F32)
    assert (p.vec, p.groups_per_wg, p.waves_per_group_in_wg, p.fixed_col) == (4, 1, 4, 1)
    assert p.grid <= 256 * 4 and p.grid >= 256 * 4 * 0.95
    assert (64 * p.chunk_stride) % p.vecs_per_segment == 0
    # KAT-B x1 bf16: 192-byte segments -> flat walk, coefficients per lane; the 1536-byte rows are walked
    # as four column blocks of two groups (384 bytes) each
    p = grkan.plan(25216, 768, 8, GRKAN_BF16)
    assert (p.vec, p.lane_coef, p.fixed_col, p.column_split, p.vecs_per_segment) == (8, 1, 1, 4, 24)
    assert p.partials_per_group == p.wg_per_bundle and p.grid == 4 * p.wg_per_bundle
    # stress with 64 groups of 48 channels: flat walk as well, eight blocks of eight groups
    p = grkan.plan(50432, 3072, 64, GRKAN_F32)
    assert (p.lane_coef, p.column_split, p.vecs_per_segment) == (1, 8, 96)
    # stress, one group
    p = grkan.plan(50432, 3072, 1, GRKAN_F32)
    assert p.groups_per_wg == 1 and p.fixed_col == 1
    # the forward pass walks whole rows whatever the segment length
    p = grkan.plan(25216, 3072, 8, GRKAN_F32, forward=True)
    assert (p.lane_coef, p.fixed_col, p.vecs_per_segment) == (1, 1, 768)


def test_plan_is_deterministic():
    a = grkan.plan(25216, 3072, 8, GRKAN_F32).as_dict()
    b = grkan.plan(25216, 3072, 8, GRKAN_F32).as_dict()
    assert a == b


def test_empty_input_plans_no_work():
    p = grkan.plan(0, 192, 8, GRKAN_F32)
    assert p.grid == 0 and p.partials_per_group == 0
    assert grkan.plan_cover_errors(0, 192, 8, GRKAN_F32, p) == 0


@pytest.mark.parametrize("rows,D,G,io,status", [
    (-1, 192, 8, GRKAN_F32, 2), (4, 0, 8, GRKAN_F32, 2), (4, 192, 0, GRKAN_F32, 2),
    (4, 190, 8, GRKAN_F32, 2), (4, 192, 8, 7, 6),
])
def test_plan_rejects_bad_arguments(rows, D, G, io, status):
    with pytest.raises(grkan.GrkanError) as e:
        grkan.plan(rows, D, G, io)
    assert e.value.status == status


def test_a_corrupted_plan_fails_the_cover_check():
    p = grkan.plan(100, 768, 8, GRKAN_F32)
    p.wg_per_bundle -= 3  # fewer waves but the same stride bookkeeping: still a cover
    assert grkan.plan_cover_errors(100, 768, 8, GRKAN_F32, p) == 0
    p.fixed_col = 1
    p.wg_per_bundle += 1  # 64 * waves is no longer a multiple of the segment length
    assert grkan.plan_cover_errors(100, 768, 8, GRKAN_F32, p) != 0


def test_random_shapes_are_always_covered_exactly():
    """Seeded sweep over awkward shapes, alignments, device sizes and both
    passes: whatever walk the planner picks, the kernels' index arithmetic
    must visit every vector once and stay in bounds."""
    import random

    rng = random.Random(20250513)
    modes = set()
    for trial in range(400):
        G = rng.choice([1, 1, 2, 3, 4, 5, 7, 8, 8, 12, 16, 33, 64])
        dg = rng.choice([1, 2, 3, 4, 6, 8, 12, 16, 24, 31, 32, 48, 64, 96, 100, 128, 192, 250, 384])
        rows = rng.choice([0, 1, 2, 3, 17, 64, 65, 127, 200, 301])
        io = rng.choice([GRKAN_F32, GRKAN_BF16])
        es = 4 if io == GRKAN_F32 else 2
        align = rng.choice([a for a in (2, 4, 8, 16) if a >= es])
        num_cu, wg = rng.choice([(256, 2), (256, 4), (256, 8), (304, 3), (8, 1), (1, 1), (64, 7)])
        forward = rng.random() < 0.5
        D = G * dg
        if rows * D > 400_000:
            rows = max(1, 400_000 // D)
        p = grkan.plan(rows, D, G, io, align_bytes=align, num_cu=num_cu, wg_per_cu=wg, forward=forward)
        assert grkan.plan_cover_errors(rows, D, G, io, p) == 0, (trial, rows, D, G, io, align, num_cu, wg, forward,
                                                                   p.as_dict())
        if rows:
            modes.add((p.fixed_col, p.lane_coef, p.groups_per_wg > 1))
    # the sweep reaches the fixed and general group walks, bundled groups and the flat walk
    assert {(1, 0, False), (1, 1, False)} <= modes and any(m[2] for m in modes) and any(m[0] == 0 for m in modes)
