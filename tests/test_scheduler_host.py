"""The tile scheduler on the host (no GPU): vfm_schedule_units runs the launchers' unit map and
the kernels' own block -> (head, tile) -> rows mapping on the CPU.  Checked here: every (head,
token) is handed out exactly once, no tile straddles a clip (cross-clip blocks are never
enumerated), clips go longest first, each XCD gets one contiguous run of units, and the grid
is padded by fewer than 8 idle workgroups."""
import numpy as np
import pytest

from paper_2503_12964_amd import binding, workloads as W

XCDS = 8


def _units_in_order(units):
    """Workgroup b belongs to XCD b % 8 and is that XCD's (b // 8)-th: list the live units in
    the order XCD 0's run, XCD 1's run, ... (the head-major unit numbering)."""
    chunk = len(units) // XCDS
    order = [units[x + XCDS * i] for x in range(XCDS) for i in range(chunk)]
    return [tuple(int(v) for v in u) for u in order]


def _check(cu, heads, rows, units=None):
    """cu: boundaries of one launch's clips (absolute packed positions; cu[0] may be > 0 when the
    launch is one run of a longer call); units: that launch's grid."""
    cu = np.asarray(cu, dtype=np.int64)
    if units is None:
        units = binding.vfm_schedule_units(cu, heads, rows)
    base = int(cu[0])
    cu = cu - base
    units = np.array(units, dtype=np.int64)
    units[units[:, 0] >= 0, 1] -= base
    total = int(cu[-1])
    lens = np.diff(cu)
    n_tiles = int(sum((n + rows - 1) // rows for n in lens))
    assert len(units) % XCDS == 0
    assert len(units) == XCDS * ((n_tiles * heads + XCDS - 1) // XCDS)
    ordered = _units_in_order(units)
    live = [u for u in ordered if u[0] >= 0]
    assert len(live) == n_tiles * heads and len(units) - len(live) < XCDS
    # idle workgroups only at the end of the numbering (the last XCD's run is the short one)
    assert ordered[:len(live)] == live
    cover = np.zeros((heads, total), dtype=np.int32)
    clip_of = np.repeat(np.arange(len(lens)), lens)
    for head, first, n in live:
        assert 0 <= head < heads and 1 <= n <= rows and 0 <= first and first + n <= total
        assert clip_of[first] == clip_of[first + n - 1], "a tile straddles two clips"
        assert (first - cu[clip_of[first]]) % rows == 0, "tiles start on the clip's own tile grid"
        cover[head, first:first + n] += 1
    assert np.all(cover == 1), "every (head, token) exactly once"
    # head-major, and within a head the clips come longest first (ties in packed order)
    heads_seen = [u[0] for u in live]
    assert heads_seen == sorted(heads_seen)
    for h in range(heads):
        clips = [int(clip_of[first]) for head, first, _ in live if head == h]
        runs = [c for i, c in enumerate(clips) if i == 0 or c != clips[i - 1]]
        assert len(runs) == len(set(runs)), "a clip's tiles are consecutive"
        want = sorted((c for c in range(len(lens)) if lens[c] > 0), key=lambda c: (-lens[c], c))
        assert runs == want
    return units


@pytest.mark.parametrize("rows", [128, 256])
def test_paper_workloads(rows):
    for name in ("C2", "C3", "C4"):
        wl = W.WORKLOADS[name]
        units = _check(wl.cu_seqlens, wl.n_heads, rows)
        live = int(np.sum(units[:, 0] >= 0))
        if name == "C4":       # 56,320 tokens: 220 tiles of 256 rows, 440 of 128, times 32 heads
            assert live == (56320 // rows) * 32
        if name == "C3":       # the block-diagonal schedule: tiles follow the clips, not total^2
            assert live == sum((n + rows - 1) // rows for n in wl.seqlens) * 24


@pytest.mark.parametrize("seed", range(12))
def test_random_clip_mixes(seed):
    rng = np.random.default_rng(seed)
    lens = [int(rng.integers(0, 3)) if rng.integers(0, 4) == 0 else int(rng.integers(1, 2000))
            for _ in range(int(rng.integers(1, 30)))]
    cu = np.concatenate([[0], np.cumsum(lens)])
    if cu[-1] == 0:
        lens[0] = 5
        cu = np.concatenate([[0], np.cumsum(lens)])
    _check(cu, int(rng.integers(1, 7)), int(rng.choice([32, 64, 128, 256])))


def test_equal_lengths_keep_packed_order_and_empty_input_has_no_workgroups():
    units = _check([0, 100, 200, 300], 1, 64)
    firsts = [int(u[1]) for u in _units_in_order(units) if u[0] >= 0]
    assert firsts == [0, 64, 100, 164, 200, 264]
    assert len(binding.vfm_schedule_units([0, 0, 0], 4, 256)) == 0


def test_more_clips_than_a_table_holds_are_scheduled_run_by_run():
    # 600 clips of 0..700 tokens: three launches (256 + 256 + 88 clips), whose grids follow one
    # another; each is a complete schedule of its own run of clips
    rng = np.random.default_rng(3)
    lens = rng.integers(0, 700, size=600)
    cu = np.concatenate([[0], np.cumsum(lens)])
    heads, rows = 3, 128
    units = binding.vfm_schedule_units(cu, heads, rows)
    at = 0
    for s0 in range(0, 600, 256):
        run = cu[s0:min(600, s0 + 256) + 1]
        n_tiles = int(sum((n + rows - 1) // rows for n in np.diff(run)))
        grid = XCDS * ((n_tiles * heads + XCDS - 1) // XCDS)
        _check(run, heads, rows, units[at:at + grid])
        at += grid
    assert at == len(units)


def test_forward_schedule_with_its_own_tile_height():
    # the forward cuts 128-row tiles when no clip of the launch has more than 1,024 tokens
    # (and always at head_dim 64), 256-row tiles otherwise
    for name, want in (("C2", 256), ("C4", 256)):
        wl = W.WORKLOADS[name]
        rows = binding.vfm_attn_fwd_tile_rows(wl.cu_seqlens, wl.head_dim)
        assert rows == want
        _check(wl.cu_seqlens, wl.n_heads, rows)
    images = np.arange(0, 289) * 256                        # 288 images of 256 tokens: two runs
    for run in (0, 1):
        assert binding.vfm_attn_fwd_tile_rows(images, 128, run) == 128
    spatial = W.WORKLOADS["C3"].spatial_cu_seqlens          # 36 frames of 256..1,024 tokens
    assert binding.vfm_attn_fwd_tile_rows(spatial, 128) == 128
    _check(spatial, 24, 128)
    assert binding.vfm_attn_fwd_tile_rows(W.WORKLOADS["C4"].cu_seqlens, 64) == 128


def test_argument_errors():
    lib = binding.load_library()
    import ctypes
    n = ctypes.c_int(0)
    cu = np.array([0, 10], dtype=np.int32)
    p = cu.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    buf = np.zeros((8, 3), dtype=np.int32)
    pb = buf.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    assert lib.vfm_schedule_units(None, 1, 10, 1, 256, pb, 8, ctypes.byref(n)) == 1      # NULL
    assert lib.vfm_schedule_units(p, 1, 10, 0, 256, pb, 8, ctypes.byref(n)) == 2         # no heads
    assert lib.vfm_schedule_units(p, 1, 10, 1, 0, pb, 8, ctypes.byref(n)) == 2           # no rows
    assert lib.vfm_schedule_units(p, 1, 11, 1, 256, pb, 8, ctypes.byref(n)) == 3         # cu vs total
    assert lib.vfm_schedule_units(p, 1, 10, 1, 256, pb, 4, ctypes.byref(n)) == 2 and n.value == 8   # too small
    assert lib.vfm_schedule_units(p, 1, 10, 1, 256, pb, 8, ctypes.byref(n)) == 0 and n.value == 8
    assert buf[0].tolist() == [0, 0, 10] and all(buf[i, 0] == -1 for i in range(1, 8))
