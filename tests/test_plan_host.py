"""Host logic of the launch planner, without a GPU: muon_plan_only builds the plan muon_init would build and
muon_plan_tiles hands out its tile tables; the tests check that every product's tiles cover exactly the output they
must, once, whatever the shape mix, the arithmetic and the chunking."""
import numpy as np
import pytest

from paper_2502_16982_amd import binding

SHAPE_SETS = {
    "ragged": [(1, 1), (1, 9), (5, 3), (64, 64), (130, 130), (200, 333), (333, 200), (257, 511), (384, 128), (128, 640)],
    "tiles256": [(1024, 1024), (1024, 1536), (1280, 1024), (384, 640), (640, 1152)],
    "moe_expert": [(2048, 1408), (2048, 1408), (1408, 2048)],
    "block": [(4096, 4096), (4096, 11008), (11008, 4096)],
    # the whole 4096-wide block: its 3088 apply tiles are 12 x 256 + 16, so 16 of them move to the fine launch
    "block_full": [(4096, 4096)] * 4 + [(4096, 11008)] * 2 + [(11008, 4096)],
    "many_small": [(256, 384)] * 40 + [(384, 256)] * 30,
    # 26 x 10 symmetric tiles = 256 + 4 and 26 x 16 apply tiles = 256 + 160: the 4 go to the fine launch, the 160 stay
    "sym_tail": [(1024, 1024)] * 26,
    "extreme": [(4, 1 << 20), (1 << 20, 4), (1, 70000)],
}


def plan(shapes, ns, max_bytes=0):
    n = len(shapes)
    p = binding.param_array(shapes, [1] * n, [1] * n)
    need = binding.muon_workspace_bytes(p, n, ns, max_bytes)
    return binding.muon_plan_only(p, n, ns, need), p


def assert_full_coverage(ctx, shapes, ns, label=""):
    """Every output cell of every product is covered by a tile; a cell is covered twice only where the last
    512 x 128 tile of a column strip was shifted to end at the matrix edge (both tiles then write the same values).
    Works over all chunks of the plan: a matrix's tiles are all in the chunk the plan puts it in."""
    desc = [binding.muon_plan_describe(ctx, i) for i in range(len(shapes))]
    mc = ns != binding.MUON_F32
    chunks = binding.muon_plan_chunks(ctx)
    for product in ("gram", "poly", "apply", "apply_last"):
        sym = product in ("gram", "poly")
        cover, strip_cover = {}, {}
        for i, d in enumerate(desc):
            fine = d["tile_n"]
            tm, tn = d["m_pad"] // fine, d["n_pad"] // fine
            # output grid in fine cells: m x m for the symmetric products; X'^T (n x m) on the matrix cores, X' else
            cover[i] = np.zeros((tm, tm) if sym else ((tn, tm) if mc else (tm, tn)), dtype=np.int32)
            strip_cover[i] = np.zeros_like(cover[i])
        for chunk in range(chunks):
            for level in (0, 1):
                for mat, r0, c0, rows, cols, blocks in binding.muon_plan_tiles(ctx, chunk, product, level):
                    assert desc[mat]["chunk"] == chunk
                    fine = desc[mat]["tile_n"]
                    if not mc:
                        assert level == 0 and (rows, cols) == (64, 64)
                    elif level == 0:
                        assert (rows, cols) == (128, 128)
                    else:
                        assert (rows, cols) in ((256, 256), (512, 128))
                    assert r0 % fine == 0 and c0 % fine == 0 and r0 % 64 == 0 and c0 % 64 == 0
                    # plain bf16: a 256-tile on the diagonal of a symmetric product is computed from its upper triangle
                    halved = ns == binding.MUON_BF16 and sym and (rows, cols) == (256, 256) and r0 == c0
                    assert blocks == (36 if halved else rows * cols // 1024) or not mc
                    grid = cover[mat]
                    assert 0 <= r0 and r0 + rows <= grid.shape[0] * fine and 0 <= c0 and c0 + cols <= grid.shape[1] * fine
                    if sym:
                        assert c0 + cols > r0       # touches the diagonal or lies above it
                    sl = (slice(r0 // fine, (r0 + rows) // fine), slice(c0 // fine, (c0 + cols) // fine))
                    grid[sl] += 1
                    if (rows, cols) == (512, 128):
                        assert c0 + cols == grid.shape[1] * fine    # strips are the last 128 columns
                        strip_cover[mat][sl] += 1
        for i, grid in cover.items():
            twice = grid > 1
            assert (grid[twice] == 2).all() and (strip_cover[i][twice] == 2).all(), (label, product, shapes[i])
            assert twice.sum() <= 3, (label, product, shapes[i])    # at most one shifted tile: < 512 rows of overlap
            if sym:
                upper = np.triu(np.ones_like(grid))
                assert (grid[upper == 1] >= 1).all(), (label, product, shapes[i])
                # below the diagonal only what a diagonal 256-tile computes along with its upper part
                r = 256 // desc[i]["tile_n"] if mc else 1
                blocks_i, blocks_j = np.nonzero(np.tril(grid, -1))
                assert all(bi // r == bj // r for bi, bj in zip(blocks_i, blocks_j)), (label, product, shapes[i])
            else:
                assert (grid >= 1).all(), (label, product, shapes[i])


@pytest.mark.parametrize("ns", [binding.MUON_BF16, binding.MUON_BF16X2, binding.MUON_F32])
@pytest.mark.parametrize("name", sorted(SHAPE_SETS))
def test_every_output_tile_is_computed(name, ns):
    shapes = SHAPE_SETS[name]
    ctx, _ = plan(shapes, ns)
    try:
        assert binding.muon_plan_chunks(ctx) == 1
        assert_full_coverage(ctx, shapes, ns, name)
    finally:
        binding.lib().muon_destroy(ctx)


@pytest.mark.parametrize("seed", range(12))
def test_random_shape_lists_are_covered_in_every_chunking(seed):
    """Seeded random lists (dimensions from 1 to 3000, many of them multiples of 128 or 256 so that strips, moved
    tiles and fine leftovers all occur; sometimes many copies of one shape, which makes the launches persistent),
    planned once with room for everything and once with a workspace that forces several chunks."""
    rng = np.random.RandomState(1000 + seed)
    def dim():
        k = rng.randint(4)
        return int(rng.randint(1, 3000)) if k == 0 else int(128 * rng.randint(1, 24)) if k == 1 else int(256 * rng.randint(1, 12)) if k == 2 else int(64 * rng.randint(1, 40))
    shapes = [(dim(), dim()) for _ in range(int(rng.randint(1, 10)))]
    if seed % 3 == 0:
        shapes += [(int(256 * rng.randint(2, 6)), int(256 * rng.randint(2, 6)))] * int(rng.randint(20, 70))
    ns = [binding.MUON_BF16, binding.MUON_BF16X2, binding.MUON_F32][seed % 3 if seed % 3 != 0 else 0]
    n = len(shapes)
    p = binding.param_array(shapes, [1] * n, [1] * n)
    full = binding.muon_workspace_bytes(p, n, ns, 0)
    least = binding.muon_workspace_bytes(p, n, ns, 1)
    for ws in (full, least + (full - least) // 3):
        ctx = binding.muon_plan_only(p, n, ns, ws)
        try:
            assert_full_coverage(ctx, shapes, ns, "random%d" % seed)
        finally:
            binding.lib().muon_destroy(ctx)


def test_orientation_padding_and_tile_sizes():
    shapes = [(2048, 1408), (1408, 2048), (100, 130), (4096, 4096), (384, 640)]
    ctx, _ = plan(shapes, binding.MUON_BF16)
    try:
        d = [binding.muon_plan_describe(ctx, i) for i in range(5)]
        assert [x["transposed"] for x in d] == [1, 0, 0, 0, 0]
        assert [(x["m"], x["n"]) for x in d] == [(1408, 2048), (1408, 2048), (100, 130), (4096, 4096), (384, 640)]
        assert [(x["m_pad"], x["n_pad"]) for x in d] == [(1408, 2048), (1408, 2048), (128, 256), (4096, 4096), (384, 640)]
        assert [x["tile_m"] for x in d] == [256, 256, 128, 256, 256] and all(x["tile_n"] == 128 for x in d)
        # 1408 = 5 x 256 + 128: fifteen 256-tiles on or above the diagonal and the last 128 columns as three
        # 512 x 128 tiles (rows 0, 512 and, shifted to end at the edge, 896), all in the coarse launch
        gram = [t for t in binding.muon_plan_tiles(ctx, 0, "gram", 1) if t[0] == 0]
        assert sorted(t[1:5] for t in gram if t[3:5] == (512, 128)) == [(0, 1280, 512, 128), (512, 1280, 512, 128), (896, 1280, 512, 128)]
        assert len([t for t in gram if t[3:5] == (256, 256)]) == 15
        assert sorted(t[5] for t in gram if t[3:5] == (256, 256)) == [36] * 5 + [64] * 10
        assert not [t for t in binding.muon_plan_tiles(ctx, 0, "gram", 0) if t[0] == 0]
        app = [t for t in binding.muon_plan_tiles(ctx, 0, "apply", 1) if t[0] == 0]
        assert len([t for t in app if t[3:5] == (256, 256)]) == 8 * 5
        assert sorted(t[1] for t in app if t[3:5] == (512, 128)) == [0, 512, 1024, 1536]
        assert not [t for t in binding.muon_plan_tiles(ctx, 0, "apply", 0) if t[0] == 0]
        # 384 x 640 is too low for a 512-row strip tile: 128 x 128 tiles take what the 256-tiles leave
        gram = [t for t in binding.muon_plan_tiles(ctx, 0, "gram", 1) if t[0] == 4]
        assert [t[3:] for t in gram] == [(256, 256, 36)]
        assert len([t for t in binding.muon_plan_tiles(ctx, 0, "gram", 0) if t[0] == 4]) == 3
        # apply output is X'^T, 640 x 384: two 256-tiles, a 512 x 128 pair over the last 128 columns (rows 0 and 128),
        # and the last 128 rows beside them in two 128 x 128 tiles
        app = [t for t in binding.muon_plan_tiles(ctx, 0, "apply", 1) if t[0] == 4]
        assert sorted(t[1:5] for t in app if t[3:5] == (512, 128)) == [(0, 256, 512, 128), (128, 256, 512, 128)]
        assert sorted(t[1:5] for t in binding.muon_plan_tiles(ctx, 0, "apply", 0) if t[0] == 4) == [(512, 0, 128, 128), (512, 128, 128, 128)]
    finally:
        binding.lib().muon_destroy(ctx)


def test_chunked_plan_keeps_each_matrix_in_one_chunk():
    shapes = [(256, 384)] * 5 + [(384, 256)] * 3
    n = len(shapes)
    p = binding.param_array(shapes, [1] * n, [1] * n)
    small = binding.muon_workspace_bytes(p, n, binding.MUON_BF16, 1)       # room for one matrix at a time
    ctx = binding.muon_plan_only(p, n, binding.MUON_BF16, small)
    try:
        chunks = binding.muon_plan_chunks(ctx)
        assert chunks == n
        seen = set()
        for c in range(chunks):
            mats = {t[0] for level in (0, 1) for t in binding.muon_plan_tiles(ctx, c, "apply", level)}
            assert len(mats) == 1 and not (mats & seen)
            assert {binding.muon_plan_describe(ctx, m)["chunk"] for m in mats} == {c}
            seen |= mats
        assert seen == set(range(n))
    finally:
        binding.lib().muon_destroy(ctx)


def test_plan_only_contexts_are_rejected_by_device_entry_points():
    import ctypes as C
    ctx, p = plan([(128, 256)], binding.MUON_BF16)
    L = binding.lib()
    try:
        hp = binding.default_hparams()
        assert L.muon_step(ctx, p, 1, C.byref(hp), None, None) == -1
        assert L.muon_debug_read_update(ctx, 0, C.c_void_p(256), 0, None) == -1
        assert L.muon_profile_enable(ctx, 1) == -1
        assert L.muon_plan_tiles(ctx, 1, 0, 0, None, 0) == -1      # no such chunk
        assert L.muon_plan_tiles(ctx, 0, 4, 0, None, 0) == -1
        assert L.muon_plan_tiles(ctx, 0, 0, 2, None, 0) == -1
    finally:
        L.muon_destroy(ctx)
    ctx = C.c_void_p(None)
    assert L.muon_plan_only(C.byref(ctx), p, 1, binding.MUON_BF16, 16) == -4
    assert ctx.value is None


def closed_form_executed_flops(m, n):
    """Matrix-core flops one Newton-Schulz iteration issues for an m x n matrix (m <= n, multiples of 128, m >= 512)
    under the planner's tiling: 256-tiles on and above the diagonal for the symmetric products, 256-tiles for the
    apply product, and 512-row tiles over the 128-wide strip an odd multiple of 128 leaves."""
    cm, cn, odd = m // 256, n // 256, (m // 128) % 2
    # diagonal 256-tiles: the 36 upper-triangle blocks of their 64
    sym_area = cm * (cm - 1) // 2 * 256 * 256 + cm * 36 * 1024 + odd * -(-m // 512) * 512 * 128
    app_area = cn * cm * 256 * 256 + odd * -(-n // 512) * 512 * 128 + ((n // 128) % 2) * 2 * cm * 128 * 128
    return 2 * (sym_area * n + sym_area * m + app_area * m)


def test_last_round_of_a_persistent_launch_goes_to_the_fine_launch():
    """Launches whose tiles all run the same K are persistent, one block per compute unit (256 when no device is
    asked): when the table is a few tiles longer than a multiple of that, those tiles are issued as four 128 x 128
    tiles each in the fine launch, and every block of the coarse launch gets the same number of tiles."""
    shapes = SHAPE_SETS["block_full"]
    ctx, _ = plan(shapes, binding.MUON_BF16)
    try:
        coarse = binding.muon_plan_tiles(ctx, 0, "apply", 1)
        fine = binding.muon_plan_tiles(ctx, 0, "apply", 0)
        assert len(coarse) == 3072 and len(fine) == 64
        assert all(t[3:5] == (128, 128) for t in fine)
        # whole 256 x 256 tiles: the four quarters of each moved tile are all there
        corners = {(t[0], t[1] // 256, t[2] // 256) for t in fine}
        assert len(corners) == 16
        for m, i, j in corners:
            assert {(m, 256 * i + a, 256 * j + b) for a in (0, 128) for b in (0, 128)} <= {t[:3] for t in fine}
        # the symmetric launches mix K = 4096 and K = 11008 in the Gram product: not persistent, nothing moved
        assert len(binding.muon_plan_tiles(ctx, 0, "gram", 1)) == 7 * 136
        assert len(binding.muon_plan_tiles(ctx, 0, "gram", 0)) == 0
    finally:
        binding.lib().muon_destroy(ctx)
    # 96 tiles over a multiple of 256 are too many to be worth a second launch: left alone
    ctx, _ = plan(SHAPE_SETS["block"], binding.MUON_BF16)
    try:
        assert len(binding.muon_plan_tiles(ctx, 0, "apply", 1)) == 1632
        assert len(binding.muon_plan_tiles(ctx, 0, "apply", 0)) == 0
    finally:
        binding.lib().muon_destroy(ctx)


@pytest.mark.parametrize("name", ["dense12_w1024", "block_w4096", "moe_bank_66x2048x1408"])
def test_bench_counts_the_flops_the_plan_issues(name):
    """bench.py's executed-flop figure is summed over the planner's tile tables; it must equal the closed form of the
    tiling for the benchmark shapes."""
    import bench
    from paper_2502_16982_amd import workloads
    wl = workloads.workload(name)
    want = sum(closed_form_executed_flops(min(a, b), max(a, b)) for a, b in wl.shapes)
    assert bench.executed_ns_flops(wl, 1) == want
    assert bench.executed_ns_flops(wl, 5) == 5 * want
    # symmetry saves between a quarter and a third of the nominal count on these shapes
    assert 0.62 < want / wl.ns_flops(1) < 0.78


@pytest.mark.parametrize("shape,product", [((4096, 4096), "gram"), ((4096, 11008), "apply"), ((11008, 4096), "apply")])
def test_tiles_that_run_together_on_a_die_share_operand_panels(shape, product):
    """Entry b of a tile table runs on accelerator die b % 8 (workgroups are handed out round-robin), one tile per
    compute unit, 32 at a time.  A die's sequence is a contiguous run of a blocked order of the tile grid (4 x 8 or
    8 x 4 blocks), so any 32 consecutive tiles of it lie in at most two blocks and touch at most 2 x 12 operand panels
    in that die's L2, against 33 for a row-major run; the first die's first 32 tiles are one whole block."""
    ctx, _ = plan([shape], binding.MUON_BF16)
    try:
        tiles = [t for t in binding.muon_plan_tiles(ctx, 0, product, 1) if t[3:5] == (256, 256)]
        worst = 0
        for die in range(8):
            seq = tiles[die::8]
            width = min(32, len(seq))
            for start in range(0, len(seq) - width + 1, width):
                block = seq[start:start + width]
                worst = max(worst, len({t[1] for t in block}) + len({t[2] for t in block}))
        assert worst <= 24, worst
        if product == "apply":
            first = tiles[0::8][:32]
            assert len({t[1] for t in first}) + len({t[2] for t in first}) == 12
    finally:
        binding.lib().muon_destroy(ctx)
