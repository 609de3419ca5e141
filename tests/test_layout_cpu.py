"""Tile layout of the fused kernels (csrc/spdnn_layout.h), checked on the host build.

What the kernels rely on: the lane sets are a partition of the wave; the fixed and the
balanced column -> slot rules are permutations of the tile; the four columns of a
staging lane sit 512 bytes apart; and the 16 lanes that a 16-byte LDS store serves
together hit 16 different bank quads.
"""
import ctypes
import os

import numpy as np
import pytest

from paper_2007_14152_amd import build as _build

KCAP = 4096


@pytest.fixture(scope="module")
def lay():
    if not os.path.exists(_build.ORDER_HOST_LIB):
        _build.build()
    L = ctypes.CDLL(_build.ORDER_HOST_LIB)
    u32 = ctypes.c_uint32
    for name in ("tile_offset", "tile_pair_bytes", "set_of_lane", "rank_in_set", "col_slot", "store_group"):
        f = getattr(L, "spdnn_%s_host" % name)
        f.argtypes = [u32]
        f.restype = u32
    L.spdnn_lane_of_group_host.argtypes = [ctypes.c_int, ctypes.c_int]
    L.spdnn_lane_of_group_host.restype = ctypes.c_int
    return L


def test_lane_sets_partition_the_wave(lay):
    lanes = [lay.spdnn_lane_of_group_host(s, i) for s in range(4) for i in range(16)]
    assert sorted(lanes) == list(range(64))
    for s in range(4):
        for i in range(16):
            l = lay.spdnn_lane_of_group_host(s, i)
            assert lay.spdnn_set_of_lane_host(l) == s and lay.spdnn_rank_in_set_host(l) == i
    # the sets are whole quartets: {0,3,5,6}, {1,2,4,7} and both shifted by 8
    quartets = [sorted({lay.spdnn_lane_of_group_host(s, i) >> 2 for i in range(16)}) for s in range(4)]
    assert quartets == [[0, 3, 5, 6], [1, 2, 4, 7], [8, 11, 13, 14], [9, 10, 12, 15]]


def test_tile_offset_interleaves_buffers_in_256_byte_rows(lay):
    off = np.array([lay.spdnn_tile_offset_host(c) for c in range(KCAP)])
    assert np.all(off % 16 == 0)
    assert len(set(off.tolist())) == KCAP
    assert np.all((off >> 4) % 16 == np.arange(KCAP) % 16)        # bank quad = slot mod 16
    assert np.all((off // 256) % 2 == 0)                             # buffer 1 = +256
    assert off.max() + 256 + 16 <= lay.spdnn_tile_pair_bytes_host(KCAP) == 2 * KCAP * 16
    assert lay.spdnn_tile_pair_bytes_host(1) == 512 and lay.spdnn_tile_pair_bytes_host(1024) == 32768


def test_fixed_layout_is_a_conflict_free_permutation(lay):
    slot = np.array([lay.spdnn_col_slot_host(c) for c in range(KCAP)])
    assert sorted(slot.tolist()) == list(range(KCAP))
    # columns 4t .. 4t+3 of a staging lane: 512 bytes apart
    off = np.array([lay.spdnn_tile_offset_host(int(s)) for s in slot])
    for a in range(1, 4):
        assert np.all(off[a::4] == off[0::4] + 512 * a)
    # every store (fixed a) of every lane set hits 16 different quads
    for wave in range(KCAP // 256):
        for s in range(4):
            lanes = [lay.spdnn_lane_of_group_host(s, i) for i in range(16)]
            for a in range(4):
                quads = {int(slot[4 * (wave * 64 + l) + a]) & 15 for l in lanes}
                assert len(quads) == 16


def test_store_groups_of_the_balanced_layout(lay):
    grp = np.array([lay.spdnn_store_group_host(c) for c in range(KCAP)])
    assert grp.min() == 0 and grp.max() == KCAP // 16 - 1
    assert np.all(np.bincount(grp) == 16)
    # a group = the columns 4t+a of the 16 lanes of one set of one wave
    for g in range(KCAP // 16):
        cols = np.nonzero(grp == g)[0]
        assert len({int(c) & 3 for c in cols}) == 1
        lanes = sorted(int(c) >> 2 for c in cols)
        wave = lanes[0] >> 6
        s = lay.spdnn_set_of_lane_host(lanes[0] & 63)
        assert lanes == sorted(wave * 64 + lay.spdnn_lane_of_group_host(s, i) for i in range(16))
    # a lane's four columns own consecutive 256-byte rows of the tile
    off0 = np.array([lay.spdnn_tile_offset_host(int(g) << 4) for g in grp])
    for a in range(1, 4):
        assert np.all(off0[a::4] == off0[0::4] + 512 * a)


def test_two_row_tile_layout(lay):
    """Tile of the two-rows-per-entry kernel: row2_pos is a permutation of every 128-column span,
    the four columns of a staging lane sit 32 entries (256 bytes) apart, and the 32 lanes that an
    8-byte LDS access serves together (half a wave) hit 32 different bank pairs."""
    lay.spdnn_row2_pos_host.argtypes = [ctypes.c_uint32]
    lay.spdnn_row2_pos_host.restype = ctypes.c_uint32
    pos = np.array([lay.spdnn_row2_pos_host(c) for c in range(16384)])
    assert sorted(pos.tolist()) == list(range(16384))
    for span in range(0, 16384, 128):
        assert sorted(pos[span:span + 128].tolist()) == list(range(span, span + 128))
    t = np.arange(4096)
    for a in range(4):
        assert np.all(pos[4 * t + a] == pos[4 * t] + 32 * a)
        for half in range(0, 4096, 32):           # lanes half .. half+31 store their column a together
            assert sorted((pos[4 * t[half:half + 32] + a] % 32).tolist()) == list(range(32))
    assert np.all(pos % 32 == (np.arange(16384) >> 2) % 32)


def test_units_of_interleaved_segments(lay):
    """unit_neuron: for every segment length the units partition the N neurons, a unit's local index
    counts its neurons in ascending order, four neighbouring local indices are four neighbouring
    neurons (one 16-byte store), and in a strided pattern of the matching period a unit's neurons
    read as many columns as it has neurons."""
    f = lay.spdnn_unit_neuron_host
    f.argtypes = [ctypes.c_int] * 4
    f.restype = ctypes.c_int
    for N in (4096, 12288, 65536):
        nunit = N // 4096
        for a in range(6, 13):
            stride = nunit << a
            nr = np.array([[f(u, p, a, stride) for p in range(0, 4096, 1 if N == 4096 else 4)] for u in range(nunit)])
            if N == 4096:
                assert np.array_equal(nr[0], np.arange(4096))   # one unit: the identity, whatever the segments
            step = 1 if N == 4096 else 4
            full = (nr[:, :, None] + np.arange(step)[None, None, :]).reshape(nunit, -1)  # neighbours of every 4th index
            assert sorted(full.ravel().tolist()) == list(range(N))
            assert np.all(np.diff(full, axis=1) > 0)
            if step == 4:
                for u in range(nunit):
                    assert all(f(u, p + 1, a, stride) == f(u, p, a, stride) + 1 for p in range(0, 4096, 4))
    # N = 65536, neuron j reads j + k * 1024 (mod N): segments of 64 neurons every 1024
    N, S, a = 65536, 1024, 6
    p = np.arange(4096)
    for u in (0, 5, 15):
        nrn = (p >> a) * S + (u << a) + (p & 63)
        assert np.array_equal(nrn[::97], [f(u, int(q), a, S) for q in p[::97]])
        cols = (nrn[:, None] + np.arange(32)[None, :] * 1024) % N
        assert len(np.unique(cols)) == 4096


def test_cyclic_windows(lay):
    """Windows are arcs of the circle of N columns: win_rel / win_col are inverse to each other, and
    win_union returns the shortest arc that holds both arguments (brute force on a small circle)."""
    N = 48
    for c_lo in range(0, N, 4):
        for c in range(N):
            r = lay.spdnn_win_rel_host(c, c_lo, N)
            assert 0 <= r < N and lay.spdnn_win_col_host(c_lo, r, N) == c
    rng = np.random.default_rng(3)
    out = (ctypes.c_int * 2)()

    def members(x, y):
        return {(x + i) % N for i in range(y)}

    for _ in range(400):
        ax, cx = (int(v) for v in rng.integers(0, N, 2))
        ay, cy = (int(v) for v in rng.integers(0, N // 2, 2))
        lay.spdnn_win_union_host(ax, ay, cx, cy, N, out)
        ux, uy = out[0], out[1]
        need = members(ax, ay) | members(cx, cy)
        assert need <= members(ux, uy) and uy <= N
        # no shorter arc holds both: try every start
        best = min((y for x in range(N) for y in range(N + 1) if need <= members(x, y)), default=0)
        if ay and cy:
            # both arcs must be covered whole, in one piece each: the shortest such arc starts at one of the two starts
            cand = []
            for x, first, second in ((ax, (ax, ay), (cx, cy)), (cx, (cx, cy), (ax, ay))):
                d = (second[0] - first[0]) % N
                cand.append(max(first[1], d + second[1]))
            assert uy == min(min(cand), N)
        assert uy >= best
