"""CPU-side checks of the library: it loads, exports the declared symbols, and its
host logic (argument errors, greedy search, register rule) behaves as the paper states."""
import ctypes
import json
import os
import re

import numpy as np
import pytest

import paper_2305_08872_amd as am

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(am.library_path()):
        from paper_2305_08872_amd import build
        build.build()
    return am.load_library()


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "amulet.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(amulet_[a-z0-9_]+)\s*\(", header))
    names.discard("amulet_score_fn")
    assert {"amulet_mmlike_f32", "amulet_count_i8", "amulet_tune", "amulet_strerror"} <= names
    for n in sorted(names):
        assert hasattr(lib, n), "libamulet.so does not export " + n


def test_argument_errors_are_reported_before_any_launch(lib):
    f = lib.amulet_mmlike_f32
    one = ctypes.c_void_p(16)  # never dereferenced: every call below fails validation first
    assert f(9, 1, 1, 1, one, 1, one, 1, one, one, 1, None) == -1
    assert f(1, -1, 1, 1, one, 1, one, 1, one, one, 1, None) == -2
    assert f(1, 1, 1, 1, None, 1, one, 1, one, one, 1, None) == -3
    assert f(1, 1, 1, 1, one, 1, one, 1, None, one, 1, None) == -3   # discount needs params
    assert f(1, 2, 3, 4, one, 3, one, 3, one, one, 3, None) == -4    # lda < K
    assert f(1, 2, 3, 4, one, 4, one, 2, one, one, 3, None) == -4    # ldb < N
    assert f(1, 2, 3, 4, one, 4, one, 3, one, one, 2, None) == -4    # ldr < N
    assert f(1, 2 ** 31, 3, 4, one, 4, one, 3, one, one, 3, None) == -7
    assert f(1, 0, 3, 4, None, 4, None, 3, None, None, 3, None) == 0  # empty: no-op
    assert lib.amulet_mmlike_f32_shape(1, 99, 2, 3, 4, one, 4, one, 3, one, one, 3, None) == -6
    g = lib.amulet_count_i8
    assert g(2, 3, 4, one, 3, one, 3, one, 3, None) == -4
    assert g(2, 3, 4, None, 4, one, 3, one, 3, None) == -3
    assert g(2, 3, 0, None, 4, None, 3, None, 3, None) == 0
    assert am.amulet_strerror(-4).startswith("leading dimension")
    assert lib.amulet_tune(55, 8, 8, 8, None) == -1


def test_packed_pitch_never_collides_and_argument_errors(lib):
    """The packed pitch holds the row, keeps rows on whole 128-byte lines and is never a pitch
    the library itself calls colliding; a call that wants to pack checks its workspace before
    anything is launched."""
    for eb in (1, 4, 8):
        for cols in [1, 3, 31, 32, 1000, 1024, 4096, 8191, 8192, 16384, 32768, 65536, 100000, 2 ** 20]:
            ld = am.amulet_packed_ld(cols, eb)
            assert ld >= cols and (ld * eb) % 128 == 0 and ld * eb < cols * eb + 256
            assert not am.amulet_pitch_collides(ld, eb)
            assert (ld * eb) % 4096 != 0
    assert am.amulet_packed_ld(0, 4) == 0 and am.amulet_packed_ld(5, 3) == 0
    # the measured rule: multiples of 32 KiB from 64 KiB on
    assert [am.amulet_pitch_collides(n, 4) for n in (4096, 8192, 12288, 16384, 16400, 20480, 24576, 32768, 65536)] == \
        [False, False, False, True, False, False, True, True, True]
    assert am.amulet_pitch_collides(8192, 8) and not am.amulet_pitch_collides(8192, 4)
    assert am.amulet_autopack_workspace_bytes(4, 10, 16384) == 10 * 16416 * 4
    one = ctypes.c_void_p(16)   # never dereferenced: every call below fails validation first
    assert lib.amulet_pack(3, 1, 1, one, 1, one, 1, None) == -2
    assert lib.amulet_pack(4, -1, 1, one, 1, one, 1, None) == -2
    assert lib.amulet_pack(4, 2, 2, None, 2, one, 2, None) == -3
    assert lib.amulet_pack(4, 2, 2, one, 1, one, 2, None) == -4
    assert lib.amulet_pack(4, 0, 2, None, 2, None, 2, None) == 0
    f = lib.amulet_mmlike_f32_autopack
    # discount, 8 x 128 x 16384 with a colliding lda: wants 8 * 16416 * 4 bytes
    assert f(1, 0, 0, 0, 8, 128, 16384, one, 16384, one, 128, one, 0, one, one, 128, one, 100, None) == -8
    assert f(9, 0, 0, 0, 8, 128, 16384, one, 16384, one, 128, one, 0, one, one, 128, one, 100, None) == -1
    assert f(1, 0, 0, 0, 8, 128, 16384, one, 16383, one, 128, one, 0, one, one, 128, one, 100, None) == -4
    assert lib.amulet_mmlike_f64_autopack(1, 0, 0, 0, 8, 128, 8192, one, 8192, one, 128, one, 0, one, one, 128,
                                          one, 100, None) == -8
    assert am.amulet_strerror(-8).startswith("workspace")
    # join count with transposed operands: the workspace holds the transposed copies
    assert am.amulet_count_i8_workspace_bytes(False, False, 100, 200, 300) == 0
    assert am.amulet_count_i8_repack_workspace_bytes(100, 200, 300) == \
        256 * am.amulet_packed_ld(320, 1) + 320 * am.amulet_packed_ld(256, 1)   # K in 64s, M and N in 256s
    assert am.amulet_count_i8_repack_workspace_bytes(0, 200, 300) == 0
    assert am.amulet_count_i8_workspace_bytes(True, False, 100, 200, 300) == 100 * am.amulet_packed_ld(300, 1)
    assert am.amulet_count_i8_workspace_bytes(True, True, 100, 200, 300) == \
        100 * am.amulet_packed_ld(300, 1) + 300 * am.amulet_packed_ld(200, 1)
    h = lib.amulet_count_i8_general
    assert h(1, 0, 100, 200, 300, one, 100, one, 200, one, 200, None, 0, None) == -3      # needs a workspace
    assert h(1, 0, 100, 200, 300, one, 100, one, 200, one, 200, one, 10, None) == -8      # too small
    assert h(1, 0, 100, 200, 300, one, 99, one, 200, one, 200, one, 1 << 20, None) == -4  # lda < M
    assert h(0, 1, 100, 200, 300, one, 300, one, 299, one, 200, one, 1 << 20, None) == -4  # ldb < K
    assert h(0, 0, 0, 200, 300, None, 300, None, 200, None, 200, None, 0, None) == 0


@pytest.fixture(scope="module")
def table1(golden_dir):
    with open(os.path.join(golden_dir, "table1_kc_nc_seconds.json")) as f:
        return json.load(f)


@pytest.mark.parametrize("machine", ["machine1", "machine2"])
def test_greedy_search_reproduces_table1_choice(lib, table1, machine):
    """Feeding the paper's measured k_c x n_c grid as the timer, the two-stage
    search must land on the parameters the paper says it finds."""
    grid = table1[machine]["seconds"]
    axis = table1["axis"]
    calls = []

    def score(i0, i1):
        calls.append((i0, i1))
        return grid[i0][i1]

    b0, b1, n = am.amulet_greedy_search(len(axis), len(axis), score)
    assert (axis[b0], axis[b1]) == tuple(table1[machine]["paper_choice"])
    assert n == len(calls)
    # stage 1 visits the whole first column, stage 2 stops at the first increase
    assert calls[:len(axis)] == [(i, 0) for i in range(len(axis))]
    assert len(calls) == len(axis) + b1 + (1 if b1 + 1 < len(axis) else 0)


def test_greedy_search_edge_cases(lib):
    assert am.amulet_greedy_search(1, 1, lambda a, b: 1.0)[:2] == (0, 0)
    # monotone improvement along axis 1 walks to the end
    assert am.amulet_greedy_search(3, 4, lambda a, b: 10 - a - b)[:2] == (2, 3)
    with pytest.raises(am.AmuletError):
        am.amulet_greedy_search(0, 3, lambda a, b: 0.0)


def test_register_rule_matches_paper_worked_example(lib, golden_dir):
    with open(os.path.join(golden_dir, "register_count_example.json")) as f:
        ex = json.load(f)
    a = ex["args"]
    need = am.amulet_register_demand(ex["I_h"], ex["I_w"], ex["S_w"], a["n_const"], a["n_i"], a["n_j"],
                                     a["n_ij"], a["n_temp"])
    assert need == ex["demand_12x16"]
    assert am.amulet_register_demand(11, ex["I_w"], ex["S_w"], a["n_const"], a["n_i"], a["n_j"],
                                     a["n_ij"], a["n_temp"]) == ex["demand_11x16"]
    assert am.amulet_choose_kernel_height(12, ex["I_w"], ex["S_w"], a["n_const"], a["n_i"], a["n_j"],
                                          a["n_ij"], a["n_temp"], ex["budget"]) == ex["chosen_I_h"]
    # plain matmul: 12*2 + 1 + 2 = 27 <= 32, the full 12x16 kernel fits (Sec. 3 inequality)
    assert am.amulet_register_demand(12, 16, 8, 0, 0, 0, 0, 0) == 27
    assert am.amulet_choose_kernel_height(12, 16, 8, 0, 0, 0, 0, 0, 32) == 12


def test_shape_table_is_the_two_axis_grid(lib):
    n = am.amulet_shape_count(am.AMULET_DISCOUNT)
    assert n == 20 and am.amulet_shape_count(77) == 0      # k axis of 5 points x 4 tiles
    assert am.amulet_shape_count(am.AMULET_IDENTITY) == 13  # two staging depths x 4 tiles, plus the five matrix-core shapes
    assert am.amulet_shape_name(1, 9) == "valu_32x256_w8_k16_s2" and am.amulet_shape_name(0, 9).startswith("mfma_")
    names = [am.amulet_shape_name(1, i) for i in range(n)]
    assert len(set(names)) == n and all(x.startswith("valu_") for x in names)
    assert 0 <= am.amulet_selected_shape(1, 8192, 8192, 8192) < n
    assert am.amulet_shape_count(am.AMULET_TASK_COUNT_I8) >= 1


def test_identity_tile_follows_how_the_tile_counts_suit_the_chip(lib):
    """The built-in choice for the identity task (256 compute units assumed where no GPU is present):
    64 x 64 tiles with fewer 128 x 128 tiles than units, and up to four large tiles per unit where
    the small tiles' count leaves clearly less of a unit's last tile unused; the 128 x 128 streamed
    shapes otherwise.  fp64 reads the shape id's tile index (0 = 64 x 64, 1 = 128 x 128) and also
    takes the small tile at exactly one large tile per unit."""
    small = am.amulet_shape_count(am.AMULET_IDENTITY) - 1
    assert am.amulet_shape_name(am.AMULET_IDENTITY, small) == "mfma_f32_64x64_dma4"
    sel = lambda M, N: am.amulet_selected_shape(am.AMULET_IDENTITY, M, N, 4096)
    for M, N in [(512, 512), (1024, 1024), (1792, 1792), (3072, 3072), (3584, 3584), (2560, 2560), (2047, 2049)]:
        assert sel(M, N) == small, (M, N)
    for M, N in [(2048, 2048), (4096, 4096), (2816, 2816), (8192, 512), (8192, 8192), (16384, 2300)]:
        assert sel(M, N) in (small - 2, small - 1), (M, N)      # the ring of 3 or of 4
    sel64 = lambda M, N: am.amulet_selected_shape_f64(am.AMULET_IDENTITY, M, N, 4096) % 2
    assert [sel64(1024, 1024), sel64(2048, 2048), sel64(3072, 3072), sel64(2816, 2816), sel64(4096, 4096)] == [0, 0, 0, 1, 1]


def test_tile_order_covers_every_tile_exactly_once(lib):
    """The XCD-aware workgroup -> tile map: every tile of the grid has exactly one owner, padding
    workgroups own none, and every XCD gets the same number of tiles to within one (workgroup b
    runs on XCD b % 8), whether or not the tile counts divide by the 8 parts."""
    rng = np.random.Generator(np.random.PCG64(5))
    drawn = [(int(rng.integers(1, 90)), int(rng.integers(1, 90))) for _ in range(24)]
    for tiles_m, tiles_n in [(1, 1), (16, 1), (128, 8), (512, 32), (7, 3), (5, 9), (64, 4), (33, 2), (3, 100),
                             (1, 8), (9, 17), (512, 9), (64, 17), (1000, 1), (22, 22), (33, 33), (129, 17), (2, 2), (1, 3)] + drawn:
        grid = am.amulet_tile_grid(tiles_m, tiles_n)
        assert grid % 8 == 0 and grid >= tiles_m * tiles_n
        owners = {}
        xcds_used = set()
        for b in range(grid):
            t = am.amulet_tile_of_workgroup(b, tiles_m, tiles_n)
            if t is None:
                continue
            assert 0 <= t[0] < tiles_m and 0 <= t[1] < tiles_n
            assert t not in owners, (tiles_m, tiles_n, b, owners.get(t))
            owners[t] = b
            xcds_used.add(b % 8)
        assert len(owners) == tiles_m * tiles_n
        # load balance: the XCDs' tile counts differ by at most one
        per_xcd = [sum(1 for b in owners.values() if b % 8 == x) for x in range(8)]
        assert max(per_xcd) * 8 == grid
        assert max(per_xcd) - min(per_xcd) <= 1, (tiles_m, tiles_n, per_xcd)
        if tiles_m * tiles_n >= 8:
            assert len(xcds_used) == 8
        exact = all(c == per_xcd[0] for c in per_xcd) and any(
            tiles_n % px == 0 and tiles_m % (8 // px) == 0 for px in (8, 4, 2, 1))
        for x in xcds_used:
            ts = sorted(t for t, b in owners.items() if b % 8 == x)
            rows, cols = {t[0] for t in ts}, {t[1] for t in ts}
            if exact:
                # grids that divide: an XCD's tiles form one rectangle
                assert len(ts) == len(rows) * len(cols)
                assert max(rows) - min(rows) + 1 == len(rows) and max(cols) - min(cols) + 1 == len(cols)
            else:
                # otherwise a run of the panel order: inside column panels no wider than a part
                # would be, plus at most the end of one panel and the start of the next
                pw = (tiles_n + 7) // 8
                assert len({t[1] // pw for t in ts}) <= 2 or per_xcd[x] > pw * tiles_m, (tiles_m, tiles_n, x, ts)
    # wide grids: 8 column bands, one per XCD
    assert am.amulet_tile_grid(512, 32) == 8 * 4 * 512
    assert am.amulet_tile_of_workgroup(8 * 4 * 512 - 1, 512, 32) == (511, 31)
    with pytest.raises(am.AmuletError):
        am.amulet_tile_of_workgroup(10 ** 9, 4, 4)


def test_refused_launch_is_reported_by_the_vector_alu_path(lib):
    """A launch the runtime refuses must come back as AMULET_ERR_LAUNCH from every vector-ALU task
    and threshold form (the launcher once dropped the error and returned success).  The seam
    refuses the launch on the host, so this runs without a GPU: the pointers are never read."""
    one = ctypes.c_void_p(256)
    try:
        for task in (am.AMULET_DISCOUNT, am.AMULET_BOOST, am.AMULET_COUNT_GT):
            for shape in range(am.amulet_shape_count(task)):
                am.amulet_debug_fail_launches(1)
                rc = lib.amulet_mmlike_f32_shape(task, shape, 300, 700, 200, one, 200, one, 700, one, one, 700, None)
                assert rc == -5, (task, shape, rc)
            for form in range(4):
                for ta, tb in [(0, 0), (1, 0), (0, 1), (1, 1)]:
                    am.amulet_debug_fail_launches(1)
                    rc = lib.amulet_mmlike_f32_general(task, form, ta, tb, -1, 300, 700, 200, one, 300 if ta else 200,
                                                       one, 200 if tb else 700, one, 700, one, one, 700, None)
                    assert rc == -5, (task, form, ta, tb, rc)
        # a launch that goes out in several parts stops at the part that was refused
        am.amulet_debug_fail_launches(1)
        assert lib.amulet_mmlike_f32(1, 64, 2 ** 31 - 2 ** 16 - 1, 4, one, 4, one, 2 ** 31, one, one, 2 ** 31, None) == -5
        assert "fail" in am.amulet_last_launch_error().lower() or "launch" in am.amulet_last_launch_error().lower()
        am.amulet_debug_fail_launches(1)
        assert lib.amulet_mmlike_f64(1, 0, 300, 700, 200, one, 200, one, 700, one, 0, one, one, 700, None) == -5
    finally:
        am.amulet_debug_fail_launches(0)


def test_selection_cache_is_keyed_by_size_bucket(lib):
    """Without a tuned entry every size gets the built-in default; the default of a bucket's
    sizes is the same function of the sizes as before (the cache key alone changed)."""
    am.amulet_clear_selections()
    assert am.amulet_selected_shape(1, 8192, 8192, 8192) == am.amulet_selected_shape(1, 8191, 8000, 8100)
    with pytest.raises(am.AmuletError):
        am.amulet_selected_shape(77, 8, 8, 8)


def test_deterministic_mode_switch(lib):
    was = am.amulet_get_deterministic()
    try:
        am.amulet_set_deterministic(True)
        assert am.amulet_get_deterministic() is True
        am.amulet_set_deterministic(False)
        assert am.amulet_get_deterministic() is False
    finally:
        am.amulet_set_deterministic(was)
