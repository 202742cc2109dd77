"""Host replay of the device launch plans (CPU only): every lane of every
launch is walked with the index functions the kernels use; all addresses must
be in bounds and the routing dst <- src must equal the map's pieces."""
import numpy as np
import pytest

from paper_2002_12798_amd import binding as B
from paper_2002_12798_amd import synth
from tests import chains

FAMILIES = [-1, B.AMAP_K_ELEMENT, B.AMAP_K_ROWS, B.AMAP_K_TILE, B.AMAP_K_WAVE]


def _replay_all(m):
    ran = 0
    for k in FAMILIES:
        try:
            assert B.amap_plan_selfcheck(m, k) == 0, k
            ran += 1
        except B.AmapError as e:
            assert e.status == B.AMAP_E_UNSUPPORTED and k != -1
    return ran


@pytest.mark.parametrize("name", synth.WORKLOAD_NAMES)
def test_workload_plans(name):
    w = synth.workload(name)
    m = B.amap_compose(w.src_shapes, w.elem_size, w.ops)
    assert _replay_all(m) >= 3


def test_planned_families():
    fam = {n: B.amap_describe(B.amap_compose(w.src_shapes, w.elem_size, w.ops)).kernel_id
           for n, w in ((n, synth.workload(n)) for n in synth.WORKLOAD_NAMES)}
    assert fam["cfg0"] == B.AMAP_K_TILE  # copy piece + channel padding planned as one group
    assert fam["cfg1"] == B.AMAP_K_TILE and fam["cfg3"] == B.AMAP_K_TILE
    assert fam["cfg2_fwd"] == fam["cfg2_rev"] == fam["cfg4"] == B.AMAP_K_ROWS


@pytest.mark.parametrize("seed", range(200))
def test_random_chain_plans(seed):
    src_shapes, ops = chains.random_chain(seed)
    m = B.amap_compose(src_shapes, 2 if seed % 2 else 4, ops)
    if B.amap_describe(m).strided:
        _replay_all(m)


@pytest.mark.parametrize("seed", range(200))
def test_random_chain_plans_with_repeat_tile_and_downward_slices(seed):
    src_shapes, ops = chains.random_chain(seed, extended=True)
    m = B.amap_compose(src_shapes, 2 if seed % 2 else 4, ops)
    if B.amap_describe(m).strided:
        _replay_all(m)


# shapes with aligned inner extents so that the vector / tile paths are planned
ALIGNED = [
    ((3, 40, 24), 2, [("transpose", (0, 2, 1))]),
    ((3, 40, 24), 4, [("transpose", (2, 1, 0))]),
    ((2, 5, 16, 72), 2, [("transpose", (0, 2, 3, 1)), ("pad", (0, 1, 1, 0), (0, 2, 1, 3), 9)]),
    ((4, 36, 8, 8), 4, [("reshape", (4, 36, 64)), ("transpose", (0, 2, 1)), ("slice", 1, 8, 56, 1)]),
    ((6, 200), 2, [("transpose", (1, 0))]),
    ((130, 66), 2, [("transpose", (1, 0))]),
    ((2, 3, 64, 8), 2, [("transpose", (0, 2, 1, 3)), ("reshape", (2, 64, 24))]),
    ((7, 33, 65), 4, [("transpose", (2, 0, 1))]),
    ((5, 264, 40), 2, [("slice", 1, 8, 264, 2), ("transpose", (0, 2, 1))]),
    # repeat / tile / downward slices: loops with source stride 0 and negative source strides
    ((4, 24, 64), 2, [("repeat", 1, 3), ("transpose", (0, 2, 1))]),              # stride-0 loop inside P
    ((4, 24, 64), 2, [("tile", 0, 3), ("transpose", (0, 2, 1))]),                # stride-0 batch loop
    ((6, 1, 128), 4, [("tile", 1, 40)]),                                         # broadcast, row copy
    ((3, 48, 40), 2, [("slice", 1, 47, -1, -1), ("transpose", (0, 2, 1))]),      # P walks the source backwards
    ((3, 48, 40), 2, [("slice", 2, 39, -1, -1)]),                                # reversed contiguous axis
    ((3, 48, 40), 4, [("slice", 0, 2, -1, -2), ("repeat", 2, 2), ("tile", 1, 2)]),
    ((5, 16, 72), 2, [("transpose", (0, 2, 1)), ("repeat", 2, 4), ("pad", (0, 0, 8), (0, 0, 8), 3)]),
    # repeat along the contiguous dimension by a power of two: the expanding row kernel
    ((3, 20, 28), 2, [("repeat", 1, 2), ("repeat", 2, 2)]),
    ((3, 20, 32), 2, [("repeat", 2, 4)]),
    ((7, 9, 40), 2, [("repeat", 2, 8), ("slice", 1, 8, -1, -1)]),
    ((3, 20, 28), 4, [("repeat", 2, 2), ("tile", 0, 2)]),
    ((3, 20, 28), 4, [("repeat", 2, 4)]),
    ((3, 20, 30), 2, [("repeat", 2, 2)]),          # 30 source elements per row: not a whole number of half vectors
    ((3, 20, 28), 2, [("repeat", 2, 3)]),          # not a power of two
    # reversed contiguous axis: mirrored vector loads
    ((5, 12, 64), 2, [("slice", 2, 63, -1, -1)]),
    ((5, 12, 64), 4, [("slice", 2, 63, -1, -1), ("slice", 1, 11, -1, -1)]),
    ((5, 12, 72), 2, [("slice", 2, 67, 3, -1)]),   # 64 of 72 elements, ending inside the row
    ((5, 12, 64), 2, [("slice", 2, 63, -1, -1), ("pad", (0, 0, 8), (0, 0, 8), 1)]),
]


@pytest.mark.parametrize("case", range(len(ALIGNED)))
def test_aligned_plans(case):
    shape, es, ops = ALIGNED[case]
    m = B.amap_compose([shape], es, ops)
    assert B.amap_describe(m).strided
    assert _replay_all(m) >= 2


# short dst rows (16 to 128 bytes): the cross-lane form, one vector per lane
XLANE = [
    ((5, 8, 96), 2, [("transpose", (0, 2, 1))]),                                  # rows of one vector
    ((5, 16, 96), 2, [("transpose", (0, 2, 1))]),                                 # two vectors
    ((3, 4, 52), 4, [("transpose", (0, 2, 1))]),                                  # 4-byte elements, one vector
    ((3, 8, 52), 4, [("transpose", (0, 2, 1))]),
    ((3, 12, 40), 4, [("transpose", (0, 2, 1))]),                                 # three vectors: 20 rows of 3 per wavefront
    ((2, 40, 72), 2, [("transpose", (0, 2, 1))]),                                 # five vectors
    ((2, 64, 24), 2, [("transpose", (0, 2, 1))]),                                 # eight vectors, 128-byte rows
    ((3, 16, 6, 8), 4, [("transpose", (0, 2, 3, 1)), ("reshape", (3, 48, 16)),
                        ("slice", 1, 8, 40, 1), ("pad", (0, 0, 0), (0, 0, 4), 7)]),  # copy piece + fill beside it (a group)
    ((2, 8, 88), 2, [("transpose", (0, 2, 1)), ("pad", (0, 0, 8), (0, 0, 16), 3)]),  # fill on both sides of the row
    ((2, 8, 40), 2, [("slice", 1, 7, -1, -1), ("transpose", (0, 2, 1))]),         # P walks the source backwards
    ((2, 24, 40), 2, [("slice", 1, 0, 24, 3), ("transpose", (0, 2, 1))]),         # strided P
    ((4, 8, 8), 2, [("transpose", (0, 2, 1))]),                                   # a single unit per batch point
    ((2, 3, 8, 24), 2, [("transpose", (0, 1, 3, 2))]),                            # two batch loops
]


@pytest.mark.parametrize("case", range(len(XLANE)))
def test_cross_lane_plans(case, monkeypatch, capfd):
    shape, es, ops = XLANE[case]
    monkeypatch.setenv("AMAP_XLANE", "2")      # planned wherever the form applies
    monkeypatch.setenv("AMAP_PLAN_TRACE", "1")
    capfd.readouterr()
    m = B.amap_compose([shape], es, ops)
    assert B.amap_plan_selfcheck(m, -1) == 0
    assert "amap plan: xlane" in capfd.readouterr().err
    monkeypatch.delenv("AMAP_PLAN_TRACE")
    assert _replay_all(m) >= 2
    monkeypatch.setenv("AMAP_WAVES_LOG", "0")  # one wavefront per workgroup
    assert B.amap_plan_selfcheck(B.amap_compose([shape], es, ops), -1) == 0


def test_cross_lane_default_is_the_measured_winner(monkeypatch, capfd):
    """By default only 2-byte elements in dst rows of one or two vectors take the cross-lane form."""
    monkeypatch.setenv("AMAP_PLAN_TRACE", "1")
    took = []
    for shape, es, ops in XLANE:
        capfd.readouterr()
        m = B.amap_compose([shape], es, ops)
        assert B.amap_plan_selfcheck(m, -1) == 0
        took.append("amap plan: xlane" in capfd.readouterr().err)
    for (shape, es, ops), t in zip(XLANE, took):
        if any(op[0] == "pad" for op in ops):
            continue                               # the row is several pieces, grouped or not
        inner = B.dst_shape(B.amap_compose([shape], es, ops))[-1]
        assert t == (es == 2 and inner <= 16), (shape, es, ops, t)
    monkeypatch.setenv("AMAP_XLANE", "0")
    for shape, es, ops in XLANE:
        capfd.readouterr()
        m = B.amap_compose([shape], es, ops)
        assert B.amap_plan_selfcheck(m, -1) == 0
        assert "amap plan: xlane" not in capfd.readouterr().err


# rows shorter than 1 KiB whose next loop differs between dst and source: planned in a blocked order
# from 2^21 vectors up; the floor is lowered here so that small tensors take that order
BLOCKED_ROWS = [
    ((4, 24, 3, 6, 64), 2, [("transpose", (2, 0, 3, 1, 4))]),                     # head split: [b,s,3,h,64] -> [3,b,h,s,64]
    ((4, 6, 24, 64), 2, [("transpose", (0, 2, 1, 3)), ("reshape", (4, 24, 384))]),  # head merge
    ((3, 10, 7, 32), 4, [("transpose", (0, 2, 1, 3))]),                           # 128-byte rows of 4-byte elements, odd extents
    ((2, 9, 5, 3, 16), 2, [("transpose", (0, 3, 2, 1, 4))]),                      # 32-byte rows, three outer loops permuted
    ((5, 12, 20, 8), 2, [("transpose", (0, 2, 1, 3)), ("pad", (0, 1, 0, 0), (0, 2, 0, 0), 4)]),
    ((2, 16, 64, 64), 2, [("transpose", (0, 2, 1, 3)), ("slice", 1, 8, 40, 1)]),
]


@pytest.mark.parametrize("case", range(len(BLOCKED_ROWS)))
def test_blocked_row_order_plans(case, monkeypatch):
    shape, es, ops = BLOCKED_ROWS[case]
    for run in ("256", "1024", "4096"):
        monkeypatch.setenv("AMAP_ROWS_BLOCK_MIN_LOG2", "0")
        monkeypatch.setenv("AMAP_ROWS_RUN", run)
        m = B.amap_compose([shape], es, ops)
        assert B.amap_describe(m).kernel_id == B.AMAP_K_ROWS
        assert _replay_all(m) >= 2
        for nw in ("0", "2"):
            monkeypatch.setenv("AMAP_WAVES_LOG", nw)
            assert B.amap_plan_selfcheck(B.amap_compose([shape], es, ops), -1) == 0
        monkeypatch.delenv("AMAP_WAVES_LOG")


def test_blocked_row_order_of_random_chains(monkeypatch):
    monkeypatch.setenv("AMAP_ROWS_BLOCK_MIN_LOG2", "0")
    for seed in range(0, 200, 2):
        src_shapes, ops = chains.random_chain(seed, extended=seed % 4 == 0)
        m = B.amap_compose(src_shapes, 2 if seed % 3 else 4, ops)
        if B.amap_describe(m).strided:
            assert B.amap_plan_selfcheck(m, -1) == 0
    for shape, es, ops in ALIGNED:
        assert B.amap_plan_selfcheck(B.amap_compose([shape], es, ops), -1) == 0


# ---- tensors beyond 32-bit offsets: every piece gets a 64-bit window origin and pieces that span
# too much are cut.  The span limit is lowered so that small tensors take that path.

@pytest.fixture
def tiny_windows(monkeypatch):
    monkeypatch.setenv("AMAP_MAX_SPAN_LOG2", "10")   # at most 1024 elements per piece and side
    yield
    monkeypatch.delenv("AMAP_MAX_SPAN_LOG2")


def test_windowed_plans_of_aligned_cases(tiny_windows):
    for shape, es, ops in ALIGNED:
        m = B.amap_compose([shape], es, ops)
        assert B.amap_describe(m).strided
        assert _replay_all(m) >= 2, (shape, ops)


@pytest.mark.parametrize("block", range(4))
def test_windowed_plans_of_random_chains(tiny_windows, block):
    for seed in range(block * 50, block * 50 + 50):
        src_shapes, ops = chains.random_chain(seed, extended=seed % 2 == 0, max_volume=60000)
        m = B.amap_compose(src_shapes, 2 if seed % 3 else 4, ops)
        if B.amap_describe(m).strided:
            _replay_all(m)


def test_windowed_plans_of_scaled_workloads(monkeypatch):
    monkeypatch.setenv("AMAP_MAX_SPAN_LOG2", "14")   # cfg1's channel loop moves 3136 source elements per step
    for name, kw in [("cfg0", {}), ("cfg1", {"n": 1}), ("cfg2_fwd", {"b": 1}), ("cfg2_rev", {"b": 1}), ("cfg3", {"n": 1})]:
        w = synth.workload(name, **kw)
        m = B.amap_compose(w.src_shapes, w.elem_size, w.ops)
        assert B.amap_plan_selfcheck(m, -1) == 0, name


# maps whose dst is contiguous over several loops while the source offers no vectors: planned as
# gathered rows (16-byte dst vectors, one load per element)
GATHERED = [
    ((4, 3, 16, 24), 2, [("transpose", (0, 2, 3, 1))]),                       # planar image -> interleaved, 3 channels
    ((4, 16, 24, 3), 2, [("transpose", (0, 3, 1, 2))]),                       # and back
    ((4, 3, 16, 24), 4, [("transpose", (0, 2, 3, 1))]),
    ((2, 5, 12, 8), 2, [("repeat", 3, 3)]),                                   # repeat by 3 along the contiguous dim
    ((2, 4, 12, 8), 2, [("repeat", 2, 3), ("repeat", 3, 3)]),                 # up-sampling by 3: four loops in the run
    ((64, 40, 5), 2, [("transpose", (0, 2, 1))]),                             # source stride 5
    ((6, 8, 5), 4, [("transpose", (2, 0, 1)), ("slice", 1, 5, -1, -1)]),      # a loop of the run walks backwards
    ((3, 7, 16), 2, [("transpose", (0, 2, 1)), ("pad", (0, 8, 0), (0, 0, 1), 7), ("slice", 2, 0, 8, 1)]),
]


@pytest.mark.parametrize("case", range(len(GATHERED)))
def test_gathered_rows_plans(case, monkeypatch):
    shape, es, ops = GATHERED[case]
    m = B.amap_compose([shape], es, ops)
    info = B.amap_describe(m)
    if case != len(GATHERED) - 1:
        assert info.kernel_id == B.AMAP_K_ROWS and info.vec_bytes == 16, case
    assert _replay_all(m) >= 2
    # the same map with the gather form switched off falls back to narrower accesses and still replays
    monkeypatch.setenv("AMAP_GATHER", "0")
    m0 = B.amap_compose([shape], es, ops)
    assert B.amap_describe(m0).vec_bytes < 16 or case == len(GATHERED) - 1
    assert _replay_all(m0) >= 2
    # windows (tensors cut for 32-bit offsets) on top of the gather form
    monkeypatch.setenv("AMAP_GATHER", "1")
    monkeypatch.setenv("AMAP_MAX_SPAN_LOG2", "9")
    assert _replay_all(B.amap_compose([shape], es, ops)) >= 1


# a small odd number of planes innermost on one side, outer on the other: whole vectors both ways
INTERLEAVED = [
    ((4, 3, 16, 24), 2, [("transpose", (0, 2, 3, 1))]),                        # planar -> interleaved
    ((4, 16, 24, 3), 2, [("transpose", (0, 3, 1, 2))]),                        # interleaved -> planar
    ((4, 16, 24, 3), 4, [("transpose", (0, 3, 1, 2))]),
    ((2, 5, 64), 2, [("transpose", (0, 2, 1))]),
    ((2, 64, 5), 2, [("transpose", (0, 2, 1))]),
    ((3, 6, 40), 2, [("transpose", (0, 2, 1))]),
    ((3, 40, 7), 4, [("transpose", (0, 2, 1))]),
    ((2, 7, 48), 2, [("transpose", (0, 2, 1)), ("slice", 1, 8, 40, 1)]),       # planes read at an offset
    ((2, 3, 8, 16), 2, [("slice", 2, 7, -1, -1), ("transpose", (0, 2, 3, 1))]),  # rows of the image upside down
    ((2, 8, 6, 8), 2, [("reshape", (2, 2, 2, 2, 6, 8)), ("transpose", (0, 1, 4, 2, 5, 3)), ("reshape", (2, 2, 12, 16))]),   # pixel shuffle, r = 2
    ((2, 2, 12, 16), 2, [("reshape", (2, 2, 6, 2, 8, 2)), ("transpose", (0, 1, 3, 5, 2, 4)), ("reshape", (2, 8, 6, 8))]),   # and back
    ((3, 4, 32), 4, [("transpose", (0, 2, 1))]),                               # 4 planes of 4-byte elements
    ((5, 3, 20), 2, [("transpose", (0, 2, 1))]),                               # 20 positions: no whole vectors -> other forms
]


@pytest.mark.parametrize("case", range(len(INTERLEAVED)))
def test_interleaved_rows_plans(case, monkeypatch):
    shape, es, ops = INTERLEAVED[case]
    m = B.amap_compose([shape], es, ops)
    info = B.amap_describe(m)
    if case != len(INTERLEAVED) - 1:
        assert info.vec_bytes == 16          # rows, or (4 planes of 4-byte elements) a tile form with whole vectors
    assert _replay_all(m) >= 2
    monkeypatch.setenv("AMAP_INTER", "0")           # the gathered form instead
    assert _replay_all(B.amap_compose([shape], es, ops)) >= 2
    monkeypatch.setenv("AMAP_INTER", "1")
    monkeypatch.setenv("AMAP_MAX_SPAN_LOG2", "9")   # cut into windows
    assert _replay_all(B.amap_compose([shape], es, ops)) >= 1


# a slice with a small step along the contiguous dimension: with step 2 on 2-byte elements one plane of an
# interleaved source is kept in registers; other steps and 4-byte elements use gathered rows
KEEP_PLANE = [
    ((4, 6, 64), 2, [("slice", 2, 0, 64, 2)]),      # window starts at the first kept element
    ((4, 6, 64), 2, [("slice", 2, 1, 64, 2)]),      # last kept element is the tensor's last: window ends there
    ((128,), 2, [("slice", 0, 1, 128, 2)]),
    ((128,), 2, [("slice", 0, 0, 128, 2)]),
    ((6, 48), 4, [("slice", 1, 0, 48, 3)]),
    ((6, 48), 4, [("slice", 1, 1, 48, 3)]),
    ((6, 48), 4, [("slice", 1, 2, 48, 3)]),
    ((5, 3, 64), 2, [("slice", 2, 3, 64, 4)]),
    ((5, 3, 66), 2, [("slice", 2, 2, 66, 2)]),      # rows of odd pitch in vectors
    ((5, 64), 2, [("slice", 0, 4, -1, -1), ("slice", 1, 1, 64, 2)]),  # rows backwards
    ((11,), 4, [("slice", 0, 0, 11, 3)]),           # neither window fits the source: gathered instead
    ((4, 80), 2, [("slice", 1, 0, 80, 5)]),         # step 5: gathered
    ((3, 2, 64), 2, [("slice", 2, 0, 64, 2), ("transpose", (1, 0, 2))]),
]


@pytest.mark.parametrize("case", range(len(KEEP_PLANE)))
def test_keep_plane_rows_plans(case, monkeypatch):
    shape, es, ops = KEEP_PLANE[case]
    m = B.amap_compose([shape], es, ops)
    assert B.amap_describe(m).vec_bytes == 16
    assert _replay_all(m) >= 1
    monkeypatch.setenv("AMAP_INTER", "0")           # the gathered form instead
    assert _replay_all(B.amap_compose([shape], es, ops)) >= 1
    monkeypatch.setenv("AMAP_INTER", "1")
    monkeypatch.setenv("AMAP_MAX_SPAN_LOG2", "9")   # cut into windows
    assert _replay_all(B.amap_compose([shape], es, ops)) >= 1


# a transposing piece that is contiguous on one side while that side's row length offers no vectors
# (7 x 7 = 49 positions under 128 channels): blocks of 64 rows pass through LDS as one flat run
FLAT = [
    ((4, 128, 7, 7), 2, [("transpose", (0, 2, 3, 1))]),                          # the source is the flat side
    ((4, 7, 7, 128), 2, [("transpose", (0, 3, 1, 2))]),                          # dst is
    ((3, 72, 5, 5), 4, [("transpose", (0, 2, 3, 1))]),                           # last block of 8 rows
    ((3, 5, 5, 72), 4, [("transpose", (0, 3, 1, 2))]),
    ((2, 200, 9), 2, [("transpose", (0, 2, 1))]),
    ((2, 9, 200), 2, [("transpose", (0, 2, 1))]),
    ((4, 130, 7, 7), 2, [("slice", 1, 2, 130, 1), ("transpose", (0, 2, 3, 1))]),  # flat run starts at an odd 4 bytes
    ((4, 7, 7, 136), 2, [("slice", 3, 0, 128, 1), ("transpose", (0, 3, 1, 2))]),  # source rows with a pitch
    ((2, 64, 6, 3), 2, [("transpose", (0, 2, 3, 1))]),                           # 18 positions: pairs only
    ((2, 3, 64, 5, 5), 2, [("transpose", (1, 0, 3, 4, 2))]),                     # batch loops in another order
    ((2, 320, 3, 3), 2, [("transpose", (0, 2, 3, 1)), ("pad", (0, 1, 1, 0), (0, 1, 1, 0), 0)]),  # into a padded image: the row is two loops
    ((4, 128, 7, 7), 2, [("transpose", (0, 2, 3, 1)), ("pad", (0, 1, 1, 0), (0, 1, 1, 0), 0)]),
    ((4, 9, 9, 128), 2, [("slice", 1, 1, 8, 1), ("slice", 2, 1, 8, 1), ("transpose", (0, 3, 1, 2))]),  # a crop made channel-major
    ((2, 64, 3, 3, 3), 4, [("transpose", (0, 2, 3, 4, 1)), ("pad", (0, 1, 0, 1, 0), (0, 0, 1, 1, 0), 0)]),  # three loops
    ((2, 56, 7, 7), 2, [("transpose", (0, 2, 3, 1))]),                           # fewer than 64 rows: one block of 56
    ((5, 7, 7, 48), 2, [("transpose", (0, 3, 1, 2))]),
    ((5, 16, 5, 5), 4, [("transpose", (0, 2, 3, 1))]),
    ((2, 72, 511), 2, [("transpose", (0, 2, 1))]),                               # rows of 511: 65,408 bytes of LDS, the most a tile takes
    ((2, 255, 136), 4, [("transpose", (0, 2, 1))]),                              # fp32, dst contiguous: 65,280 bytes
    ((3, 9, 9, 64), 2, [("slice", 1, 7, 0, -1), ("slice", 2, 1, 8, 1), ("slice", 0, 2, -1, -1), ("transpose", (0, 3, 1, 2))]),  # image rows and the batch backwards
    ((3, 64, 7, 7), 2, [("slice", 0, 2, -1, -1), ("slice", 1, 63, -1, -1), ("transpose", (0, 2, 3, 1))]),                     # batch and channels backwards
    ((1, 64, 25), 4, [("transpose", (0, 2, 1)), ("repeat", 0, 3)]),              # one image written three times
    ((2, 72, 17, 17), 2, [("transpose", (0, 2, 3, 1))]),                         # rows of 289: 37 KiB of LDS
    ((2, 17, 17, 72), 2, [("transpose", (0, 3, 1, 2))]),
    ((2, 48, 35, 35), 2, [("transpose", (0, 2, 3, 1))]),                         # rows of 1225: 16 rows per block
    ((2, 35, 35, 48), 2, [("transpose", (0, 3, 1, 2))]),
    ((2, 40, 23, 23), 4, [("transpose", (0, 2, 3, 1))]),                         # rows of 529 x 4 bytes: 16 rows per block
    ((2, 26, 26, 96), 2, [("transpose", (0, 3, 1, 2))]),                         # rows of 676: 32 rows per block
    ((2, 64, 75, 75), 4, [("transpose", (0, 2, 3, 1))]),                         # rows of 5625: too long for LDS (cut into two tile pieces)
    ((2, 75, 75, 64), 4, [("transpose", (0, 3, 1, 2))]),                         # blocks of 64 rows x 128 columns
    ((2, 72, 47, 47), 2, [("transpose", (0, 2, 3, 1)), ("pad", (0, 1, 1, 0), (0, 1, 1, 0), 0)]),   # 2209 positions into a padded image
    ((2, 49, 49, 72), 2, [("slice", 1, 1, 48, 1), ("slice", 2, 1, 48, 1), ("transpose", (0, 3, 1, 2))]),
    ((3, 7, 7, 64), 2, [("transpose", (0, 3, 1, 2)), ("pad", (0, 1, 0, 0), (0, 0, 0, 0), 0)]),     # dst run starts at element 49 of every image
    ((67, 131), 2, [("transpose", (1, 0))]),                                     # both extents odd
    ((2, 70, 9, 9), 4, [("transpose", (0, 2, 3, 1))]),                           # 70 rows of fp32: no whole vectors along the rows
    ((2, 9, 9, 70), 4, [("transpose", (0, 3, 1, 2))]),
]


# neighbours of the flat forms that must take other forms
FLAT_OTHER = [
    ((3, 64, 7, 7), 2, [("transpose", (0, 2, 3, 1)), ("pad", (0, 0, 0, 1), (0, 0, 0, 0), 0)]),     # dst rows start at element 1: no flat form
    ((3, 72, 5, 6), 2, [("slice", 3, 5, -1, -1), ("transpose", (0, 2, 3, 1))]),   # x backwards: rows are no longer one run -> other forms
    ((2, 8, 7, 7), 2, [("transpose", (0, 2, 3, 1))]),                            # 8 rows only: other forms
]


@pytest.mark.parametrize("case", range(len(FLAT) + len(FLAT_OTHER)))
def test_flat_tiles_plan(case, monkeypatch):
    shape, es, ops = (FLAT + FLAT_OTHER)[case]
    m = B.amap_compose([shape], es, ops)
    info = B.amap_describe(m)
    # (fp32 rows that are no whole vectors on the dst side take other forms; the 49-element fill runs of the third start at odd elements)
    if case < len(FLAT) and (shape, es) not in (((2, 70, 9, 9), 4), ((3, 7, 7, 64), 2)):
        # (the family reported is that of the largest piece: the border fill where the image is padded)
        assert info.vec_bytes == 16 and (B.KERNEL_NAMES[info.kernel_id] == "tile" or "pad" in [o[0] for o in ops])
    assert _replay_all(m) >= 2
    monkeypatch.setenv("AMAP_FLAT", "0")            # gathered rows / split tiles instead
    assert _replay_all(B.amap_compose([shape], es, ops)) >= 2
    monkeypatch.setenv("AMAP_FLAT", "1")
    monkeypatch.setenv("AMAP_WAVES_LOG", "2")       # 4 wavefronts per workgroup
    assert _replay_all(B.amap_compose([shape], es, ops)) >= 2
    monkeypatch.delenv("AMAP_WAVES_LOG")
    monkeypatch.setenv("AMAP_MAX_SPAN_LOG2", "11")  # cut into windows
    assert _replay_all(B.amap_compose([shape], es, ops)) >= 1


# tile vectors along a source run made of two loops (x then y of an image that lands in a padded one,
# or with rows taken from a larger image): the run is a whole number of vectors, its rows are not
STRADDLE = [
    ((2, 64, 12, 12), 2, [("transpose", (0, 2, 3, 1)), ("pad", (0, 1, 1, 0), (0, 1, 1, 0), 0)]),
    ((2, 64, 6, 6), 4, [("transpose", (0, 2, 3, 1)), ("pad", (0, 1, 1, 0), (0, 1, 1, 0), 0)]),
    ((2, 32, 28, 28), 2, [("transpose", (0, 2, 3, 1)), ("pad", (0, 1, 1, 0), (0, 1, 1, 0), 0)]),
    ((3, 40, 4, 6, 4), 2, [("transpose", (0, 2, 3, 4, 1)), ("pad", (0, 0, 1, 1, 0), (0, 1, 0, 1, 0), 0)]),   # three loops: 96 positions
]


@pytest.mark.parametrize("case", range(len(STRADDLE)))
def test_tile_vectors_straddle_the_loops_of_a_source_run(case, monkeypatch):
    shape, es, ops = STRADDLE[case]
    m = B.amap_compose([shape], es, ops)
    assert B.amap_describe(m).vec_bytes == 16
    assert _replay_all(m) >= 3
    monkeypatch.setenv("AMAP_FLAT", "0")             # (short runs would pass through LDS as flat tiles otherwise)
    assert B.amap_describe(m).vec_bytes == 16 and _replay_all(B.amap_compose([shape], es, ops)) >= 3
    monkeypatch.setenv("AMAP_TILE_CHAIN_VEC", "0")   # vectors inside the innermost loop only
    m0 = B.amap_compose([shape], es, ops)
    assert B.amap_describe(m0).vec_bytes < 16
    assert _replay_all(m0) >= 3
    monkeypatch.setenv("AMAP_TILE_CHAIN_VEC", "1")
    monkeypatch.setenv("AMAP_FLAT", "1")
    monkeypatch.setenv("AMAP_MAX_SPAN_LOG2", "11")
    assert _replay_all(B.amap_compose([shape], es, ops)) >= 1


CONCAT_ODD_IMAGES = [
    ([(3, c, 17, 17) for c in (64, 96, 64, 32)], 2, [("concat", 1), ("transpose", (0, 2, 3, 1))]),
    ([(3, c, 7, 7) for c in (64, 80, 128)], 2, [("concat", 1), ("transpose", (0, 2, 3, 1)), ("pad", (0, 1, 1, 0), (0, 1, 1, 0), 0)]),
    ([(2, c, 5, 5) for c in (32, 64)], 4, [("concat", 1), ("transpose", (0, 2, 3, 1))]),
    ([(2, 9, 9, c) for c in (64, 72)], 2, [("concat", 3), ("transpose", (0, 3, 1, 2))]),
]


@pytest.mark.parametrize("case", range(len(CONCAT_ODD_IMAGES)))
def test_concat_of_images_with_rows_of_no_whole_vectors(case, monkeypatch):
    """Pieces that are neighbours along the dst-contiguous dimension are first tried as one group of
    tile pieces; where the image rows offer no vectors the group is not possible and every piece is
    planned on its own (as a flat tile).  (Planning the group's head as a flat tile crashed the host.)"""
    shapes, es, ops = CONCAT_ODD_IMAGES[case]
    m = B.amap_compose(shapes, es, ops)
    assert _replay_all(m) >= 2
    monkeypatch.setenv("AMAP_WAVES_LOG", "2")
    assert _replay_all(B.amap_compose(shapes, es, ops)) >= 2


def _forms(capfd, monkeypatch, shape, es, ops):
    """The forms the planner picks, from its trace on stderr."""
    monkeypatch.setenv("AMAP_PLAN_TRACE", "1")
    capfd.readouterr()
    m = B.amap_compose([shape], es, ops)
    B.amap_describe(m)
    err = capfd.readouterr().err
    monkeypatch.delenv("AMAP_PLAN_TRACE")
    lines = [line for line in err.splitlines() if line.startswith("amap plan:")]
    last = max(i for i, line in enumerate(lines) if line.split()[2] == "begin")   # the plan of the whole chain
    return {line.split()[2] for line in lines[last + 1:]}


def test_planned_forms_of_the_special_cases(capfd, monkeypatch):
    t = lambda *perm: [("transpose", perm)]
    assert "flat-src" in _forms(capfd, monkeypatch, (4, 128, 7, 7), 2, t(0, 2, 3, 1))
    assert "flat-dst" in _forms(capfd, monkeypatch, (4, 7, 7, 128), 2, t(0, 3, 1, 2))
    # rows of 1225: few channels keep the cut into whole-vector part + tail, many take the blocked form; the way back 16-row blocks
    assert "tile" in _forms(capfd, monkeypatch, (2, 48, 35, 35), 2, t(0, 2, 3, 1))
    assert "flat-blocked-src" in _forms(capfd, monkeypatch, (2, 136, 35, 35), 2, t(0, 2, 3, 1))
    assert "flat-dst" in _forms(capfd, monkeypatch, (2, 35, 35, 48), 2, t(0, 3, 1, 2))
    # long rows of one loop with the source as the contiguous side: whole-vector part + one-element tail
    assert "tile" in _forms(capfd, monkeypatch, (2, 64, 75, 75), 4, t(0, 2, 3, 1))
    assert "flat-blocked-src" in _forms(capfd, monkeypatch, (2, 72, 47, 47), 2, t(0, 2, 3, 1) + [("pad", (0, 1, 1, 0), (0, 1, 1, 0), 0)])
    assert "flat-blocked-dst" in _forms(capfd, monkeypatch, (2, 75, 75, 64), 4, t(0, 3, 1, 2))
    assert "flat-src" in _forms(capfd, monkeypatch, (4, 128, 7, 7), 2, t(0, 2, 3, 1) + [("pad", (0, 1, 1, 0), (0, 1, 1, 0), 0)])
    # dst not aligned to vectors, or a row count that is no whole number of vectors: blocked form towards the contiguous dst
    assert "flat-blocked-dst" in _forms(capfd, monkeypatch, (3, 7, 7, 64), 2, t(0, 3, 1, 2) + [("pad", (0, 1, 0, 0), (0, 0, 0, 0), 0)])
    assert "flat-blocked-dst" in _forms(capfd, monkeypatch, (67, 131), 2, t(1, 0))
    assert not any(f.startswith("flat") for f in _forms(capfd, monkeypatch, (3, 64, 7, 7), 2, t(0, 2, 3, 1) + [("pad", (0, 0, 0, 1), (0, 0, 0, 0), 0)]))
    assert "rows-keep-plane" in _forms(capfd, monkeypatch, (4, 6, 64), 2, [("slice", 2, 1, 64, 2)])
    assert "rows-gather" in _forms(capfd, monkeypatch, (6, 48), 4, [("slice", 1, 1, 48, 3)])
    assert "rows-interleave" in _forms(capfd, monkeypatch, (4, 3, 16, 24), 2, t(0, 2, 3, 1))
    assert "rows-deinterleave" in _forms(capfd, monkeypatch, (4, 16, 24, 3), 2, t(0, 3, 1, 2))
    assert "rows-expand" in _forms(capfd, monkeypatch, (4, 6, 16), 2, [("repeat", 2, 2)])
    assert "rows-reverse" in _forms(capfd, monkeypatch, (4, 6, 16), 2, [("slice", 2, 15, -1, -1)])
    assert "tile" in _forms(capfd, monkeypatch, (2, 64, 16, 16), 2, t(0, 2, 3, 1))
    # 28 x 28 into a padded image: tile vectors of 16 bytes across image rows
    assert _forms(capfd, monkeypatch, (2, 64, 28, 28), 2, t(0, 2, 3, 1) + [("pad", (0, 1, 1, 0), (0, 1, 1, 0), 0)]) >= {"tile", "rows-fill"}


def _random_transposing_map(rng):
    """A transposition of the two innermost axes with row lengths, row counts, batch loops, slices,
    pads and crops drawn so that the flat tile forms, their neighbours and their fallbacks all occur."""
    es = int(rng.choice([2, 4]))
    v = 16 // es
    c = int(rng.choice([9, 10, 11, 13, 18, 25, 27, 49, 50, 81, 121, 289, 625, 1225, 2209])) if rng.random() < 0.8 else int(rng.integers(8, 600))
    er = v * int(rng.integers(16 // v, 40)) if rng.random() < 0.7 else int(rng.integers(16, 300))
    nb = int(rng.integers(1, 4)) if c < 1000 else 1
    if c > 1000:
        er = min(er, 160)
    ops = []
    mode = rng.random()
    if mode < 0.25:      # channel-major images into a padded channels-last tensor
        h, w = int(rng.integers(2, 8)), int(rng.integers(2, 10))
        shape = (nb, er, h, w)
        ops = [("transpose", (0, 2, 3, 1)),
               ("pad", (0, int(rng.integers(0, 3)), int(rng.integers(0, 3)), 0), (0, int(rng.integers(0, 3)), int(rng.integers(1, 3)), 0), 0)]
    elif mode < 0.5:     # the crop of a padded channels-last tensor made channel-major
        h, w, a, b = int(rng.integers(2, 8)), int(rng.integers(2, 10)), int(rng.integers(0, 3)), int(rng.integers(1, 3))
        shape = (nb, h + a + 1, w + b + 1, er)
        ops = [("slice", 1, a, a + h, 1), ("slice", 2, b, b + w, 1), ("transpose", (0, 3, 1, 2))]
    else:
        extra = int(rng.integers(0, 3 * v))
        shape = (nb, er + extra, c) if mode < 0.75 else (nb, c, er + extra)
        ax = 1 if mode < 0.75 else 2
        if extra:
            st = int(rng.integers(0, extra + 1))
            ops.append(("slice", ax, st, st + er, 1))
        ops.append(("transpose", (0, 2, 1)))
    return shape, es, ops


def test_random_transposing_maps_replay(monkeypatch):
    rng = np.random.default_rng(2024)
    for it in range(160):
        shape, es, ops = _random_transposing_map(rng)
        monkeypatch.delenv("AMAP_WAVES_LOG", raising=False)
        if it % 3 == 0:
            monkeypatch.setenv("AMAP_WAVES_LOG", str(it % 2 * 2))
        m = B.amap_compose([shape], es, ops)
        assert _replay_all(m) >= 1, (shape, es, ops)


FIXED_WIDTH_FORMS = [
    ((4, 6, 16), 2, [("repeat", 2, 2)]),                      # expanded in registers
    ((4, 6, 16), 4, [("repeat", 2, 4)]),
    ((4, 6, 16), 2, [("slice", 2, 15, -1, -1)]),              # reversed in registers
    ((3, 5, 8), 4, [("slice", 2, 7, -1, -1)]),
]


@pytest.mark.parametrize("cap", ["8", "4", "2"])
def test_vector_cap_never_reaches_the_16_byte_row_forms(cap, monkeypatch):
    """The expanding, reversing, gathered and interleaving row forms are written for 16-byte
    vectors.  Under a narrower cap (a switch for A/B timing) the planner must pick other forms;
    the replay walks those forms with the width the kernel uses, so a wrong plan shows as
    out-of-bounds or doubly written elements (as it did: 772 errors for a repeat by 2 under an
    8-byte cap before the planner checked the cap)."""
    monkeypatch.setenv("AMAP_VEC_BYTES", cap)
    for shape, es, ops in FIXED_WIDTH_FORMS + GATHERED + INTERLEAVED + KEEP_PLANE + FLAT + FLAT_OTHER:
        m = B.amap_compose([shape], es, ops)
        assert B.amap_describe(m).vec_bytes <= max(int(cap), es), (shape, ops)
        assert _replay_all(m) >= 1
