"""Host logic of the contraction launch plan (no GPU): every shape gets a plan that a
kernel instance serves, covers all rows and weight rows, fits the CU's LDS and the
partial-result workspace; the plans of the benchmark shapes are pinned."""
import itertools
import random

import pytest

from paper_2404_19124_amd import binding as B

LDS_PER_CU = 160 * 1024


def check_plan(rows, k, n_head, k_top, n_proj, n_cu):
    p = B.spec_plan_contraction(rows, k, n_head, k_top, n_proj, n_cu)
    what = "rows=%d k=%d n_head=%d k_top=%d n_proj=%d n_cu=%d -> %s" % (rows, k, n_head, k_top, n_proj, n_cu, p)
    assert p["row_blocks"] >= 1 and p["ranges"] >= 1 and p["k_split"] >= 1, what
    # all state rows, no empty block
    assert p["row_blocks"] * p["block_rows"] >= rows > (p["row_blocks"] - 1) * p["block_rows"], what
    # all weight rows: tiles of both matrices, every range owns at least one
    tiles = -(-n_head // p["tile_rows"]) + -(-n_proj // p["tile_rows"])
    if p["kernel"] != 0:
        assert p["tiles"] == tiles, what
        assert p["ranges"] <= p["tiles"], what
        assert p["workgroups"] == p["row_blocks"] * p["ranges"] * p["k_split"], what
    # parts per row: the ranges that hold head tiles
    if n_head == 0:
        assert p["kernel"] == 0 or p["parts"] == 0, what
    else:
        assert 1 <= p["parts"] <= p["ranges"], what
        if n_proj == 0:
            assert p["parts"] == p["ranges"], what
    # the workspace holds max(128 * n_cu, rows * n_cu, 16 * n_cu) (row, part) slots
    assert rows * p["parts"] <= max(128 * n_cu, rows * n_cu), what
    assert 0 < p["lds_bytes"] <= LDS_PER_CU, what
    narrow = p["kernel"] in (1, 2)
    if p["k_split"] > 1:
        assert p["kernel"] != 0 and n_head == 0, what
        assert (k // 64) // p["k_split"] >= 8 and p["workgroups"] <= (2 if narrow else 1) * n_cu, what
    if p["proj_apart"]:
        # two launches instead of one: both halves have plans of their own, on the wide kernel
        assert rows > 64 and n_head > 0 and n_proj > 0 and p["kernel"] >= 1000, what
        head = B.spec_plan_contraction(rows, k, n_head, k_top, 0, n_cu)
        proj = B.spec_plan_contraction(rows, k, 0, 0, n_proj, n_cu)
        assert head["kernel"] >= 1000 and proj["kernel"] >= 1000, what
        # the head alone needs fewer tile rounds than the pair
        per = lambda q: -(-q["tiles"] // q["ranges"])
        assert per(head) < per(p) or head["block_rows"] != p["block_rows"], what
    if p["kernel"] >= 1000:   # wide kernel: one workgroup per CU unless there are more row blocks than CUs
        assert p["workgroups"] <= max(n_cu, p["row_blocks"]), what
        assert p["tile_rows"] <= 256 and p["block_rows"] in (64, 96, 128, 160), what
        mb, rest = divmod(p["kernel"] - 1000, 100)
        assert 32 * mb == p["block_rows"] and rest // 2 >= (k_top if n_head else 0), what
        assert (rest % 2 == 1) == (p["tile_rows"] != 256), what
    if narrow:
        assert p["workgroups"] <= max(2 * n_cu, p["row_blocks"] * p["k_split"]), what
    return p


def test_plan_invariants_over_a_grid_of_shapes():
    rows_l = [1, 2, 15, 16, 17, 31, 32, 33, 48, 64, 65, 96, 97, 128, 160, 161, 192, 320, 384, 465, 768, 960, 1000, 2304, 4096]
    shapes = [(4096, 32000, 4096), (4096, 32000, 0), (4096, 0, 4096), (5120, 0, 4096), (8192, 0, 3072), (3072, 128256, 3072),
              (3072, 128256, 0), (64, 9, 0), (64, 300, 64), (320, 16500, 320), (320, 20300, 0), (6144, 49152, 4096), (128, 777, 128)]
    for rows, (k, n_head, n_proj), n_cu in itertools.product(rows_l, shapes, (256, 304, 64, 1)):
        for k_top in ((1, 2, 3, 5, 8) if n_head else (0,)):
            check_plan(rows, k, n_head, k_top, n_proj, n_cu)


def test_plan_invariants_over_random_shapes():
    rnd = random.Random(20240419)
    for _ in range(4000):
        rows = rnd.choice([rnd.randint(1, 20), rnd.randint(17, 200), rnd.randint(100, 5000)])
        k = 64 * rnd.randint(1, 128)
        n_head = rnd.choice([0, rnd.randint(1, 300), rnd.randint(1, 200000)])
        n_proj = rnd.choice([0, 64 * rnd.randint(1, 128)])
        if n_head + n_proj == 0:
            n_proj = 64
        check_plan(rows, k, n_head, rnd.randint(1, 8) if n_head else 0, n_proj, rnd.choice([256, 256, 304, 128, 40, 7]))


# The plans behind the numbers quoted for the benchmark shapes (7B speculator, 5/3/2 tree): a change here
# is a change of the measured configuration and wants new profiles.
PINNED = [
    # rows, k, n_head, k_top, n_proj -> kernel, block_rows, tile_rows, row_blocks, ranges, parts, k_split
    ((1, 4096, 0, 0, 4096), (0, 16, 16, 1, 256, 256, 1)),
    ((1, 4096, 32000, 5, 4096), (0, 16, 16, 1, 256, 256, 1)),
    ((15, 4096, 32000, 2, 0), (0, 16, 16, 1, 256, 256, 1)),
    ((64, 4096, 0, 0, 4096), (1, 32, 64, 2, 64, 0, 4)),
    ((64, 4096, 32000, 5, 4096), (1213, 64, 144, 1, 252, 223, 1)),
    ((320, 4096, 32000, 3, 4096), (1406, 128, 256, 3, 85, 76, 1)),     # not launched like this: proj_apart
    ((320, 4096, 32000, 3, 0), (1506, 160, 256, 2, 125, 125, 1)),      # the head alone: one tile per range
    ((320, 4096, 0, 0, 4096), (1304, 96, 256, 4, 16, 0, 4)),           # the projection alone, four K parts
    ((960, 4096, 32000, 2, 0), (1504, 160, 256, 6, 42, 42, 1)),
    ((384, 4096, 32000, 3, 0), (1306, 96, 256, 4, 64, 64, 1)),
    ((2304, 3072, 128256, 2, 0), (1504, 160, 256, 15, 17, 17, 1)),
]


@pytest.mark.parametrize("args,want", PINNED, ids=["x".join(map(str, a)) for a, _ in PINNED])
def test_plans_of_the_benchmark_shapes(args, want):
    p = check_plan(*args, 256)
    got = (p["kernel"], p["block_rows"], p["tile_rows"], p["row_blocks"], p["ranges"], p["parts"], p["k_split"])
    assert got == want
    assert p["proj_apart"] == (1 if args == (320, 4096, 32000, 3, 4096) else 0)


@pytest.mark.parametrize("args", [(0, 4096, 32000, 2, 0, 256), (4, 100, 32000, 2, 0, 256), (4, 4096, 0, 0, 0, 256),
                                  (4, 4096, 32000, 9, 0, 256), (4, 4096, 32000, 0, 0, 256), (4, 4096, -1, 2, 64, 256),
                                  (4, 4096, 32000, 2, 0, 0)])
def test_plan_rejects_bad_arguments(args):
    with pytest.raises(B.SpecError) as e:
        B.spec_plan_contraction(*args)
    assert e.value.status == B.SPEC_EINVAL
