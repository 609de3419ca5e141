"""How the set-up cuts a general layer (neurons of any number of connections, Section II-A-1) into workgroups
(csrc/spdnn_cut.h), run through its host build: every neuron in exactly one workgroup, workgroups within their
limits, and the two cuts chosen and shaped as documented."""
import ctypes

import numpy as np
import pytest

from paper_2007_14152_amd import build as hip_build

WG, PART, STAGE = 1024, 32, 4096


@pytest.fixture(scope="module")
def lib():
    L = ctypes.CDLL(hip_build.ORDER_HOST_LIB)
    L.spdnn_cut_workgroups_host.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                            ctypes.c_int, ctypes.c_void_p, ctypes.c_int]
    return L


def passes_of(deg):
    parts = max(1, -(-int(deg.max()) // PART))
    p = 1
    while p < parts:
        p *= 2
    return p


def cut(lib, deg, windows, G=4):
    """deg: connections per neuron; windows: [N/4, 2] lowest and highest column of every four neurons."""
    N = len(deg)
    ptr = np.zeros(N + 1, dtype=np.int32)
    np.cumsum(deg, out=ptr[1:])
    qw = np.ascontiguousarray(windows, dtype=np.int32)
    P = passes_of(deg)
    nblk = -(-N // WG)
    cap = 4 * P * nblk + 64
    out = np.zeros((cap, 2), dtype=np.int32)
    n = lib.spdnn_cut_workgroups_host(ptr.ctypes.data, qw.ctypes.data, N, P, nblk, G, out.ctypes.data, cap)
    assert n >= 0
    return out[:n], P, nblk


def lanes_of(deg):
    return -(-np.asarray(deg) // PART)


def check_partition(ranges, deg):
    N = len(deg)
    lanes = lanes_of(deg)
    nxt = 0
    for first, count in ranges:
        if count == 0:
            assert first == N          # an empty workgroup says so
            continue
        assert first == nxt and count % 4 == 0 and 0 < count <= WG
        assert lanes[first:first + count].sum() <= WG
        nxt = first + count
    assert nxt == N


def whole_row_windows(N):
    return np.tile(np.array([[0, N - 1]], dtype=np.int32), (N // 4, 1))


def aligned_windows(N, width):
    j = np.arange(0, N, 4)
    lo = (j // width) * width
    return np.stack([lo, lo + width - 1], axis=1).astype(np.int32)


def test_neurons_of_16_to_64_connections_get_the_plain_cut_with_equal_lanes_per_run(lib):
    rng = np.random.default_rng(1)
    N = 65536
    deg = rng.integers(16, 65, size=N)
    ranges, P, nblk = cut(lib, deg, aligned_windows(N, 4096))
    assert P == 2
    check_partition(ranges, deg)
    assert len(ranges) == N // (WG // P)                       # as many workgroups as the cut by neurons has
    lanes = lanes_of(deg)
    per_wg = np.array([lanes[f:f + c].sum() for f, c in ranges])
    runs = per_wg.reshape(-1, 8)                               # 8 workgroups share a window and an XCD
    # inside a run the workgroups differ by at most the lanes of four neurons; the cut by neurons would differ more
    assert (runs.max(axis=1) - runs.min(axis=1)).max() <= 2 * 4 * P
    by_neurons = lanes.reshape(-1, WG // P).sum(axis=1).reshape(-1, 8)
    assert (by_neurons.max(axis=1) - by_neurons.min(axis=1)).mean() > 3 * (runs.max(axis=1) - runs.min(axis=1)).mean()
    # every run covers its own 4096 neurons: run r starts at workgroup 8 r
    starts = np.array([f for f, c in ranges]).reshape(-1, 8)[:, 0]
    assert (starts == np.arange(N // 4096) * 4096).all()


def test_few_long_neurons_get_the_packed_cut(lib):
    rng = np.random.default_rng(2)
    N = 16384
    deg = rng.integers(0, 33, size=N)
    deg[rng.integers(0, N, size=20)] = 2000                    # 63 lanes each
    ranges, P, nblk = cut(lib, deg, whole_row_windows(N))
    assert P == 64
    check_partition(ranges, deg)
    plain = N // (WG // P)
    assert 4 * len(ranges) <= 3 * plain and len(ranges) <= P * nblk
    assert all(c > 0 for f, c in ranges)                       # the packed cut has no empty workgroups
    lanes = lanes_of(deg)
    # packed: the next four neurons would not have fitted (or the workgroup has 1024 neurons)
    for (f, c), (f2, c2) in zip(ranges[:-1], ranges[1:]):
        assert c == WG or lanes[f:f + c].sum() + lanes[f2:f2 + 4].sum() > WG


def test_a_packed_workgroup_is_not_widened_beyond_one_stage(lib):
    N = 16384
    deg = np.full(N, 8)
    deg[::64] = 40                                             # P = 2, few lanes: the packed cut wins
    ranges, P, nblk = cut(lib, deg, aligned_windows(N, 2048))
    check_partition(ranges, deg)
    assert 4 * len(ranges) <= 3 * (N // (WG // P))
    for f, c in ranges:                                        # windows of 2048 columns: no workgroup spans three of them
        lo = (f // 2048) * 2048
        hi = ((f + c - 1) // 2048) * 2048 + 2047
        assert hi - lo < STAGE


@pytest.mark.parametrize("N,kmin,kmax", [(2052, 5, 300), (96, 0, 100), (1024, 33, 64), (4100, 16, 64), (8192, 0, 2100)])
def test_ragged_sizes_and_outliers_are_partitions_within_the_room_there_is(lib, N, kmin, kmax):
    rng = np.random.default_rng(N + kmax)
    deg = rng.integers(kmin, kmax + 1, size=N)
    deg[rng.uniform(size=N) < 0.05] = 0
    ranges, P, nblk = cut(lib, deg, whole_row_windows(N))
    check_partition(ranges, deg)
    assert len(ranges) <= P * nblk                             # the arena's room


def test_all_neurons_of_the_longest_kind_fall_back_to_the_cut_by_neurons(lib):
    N = 8192
    deg = np.full(N, 64)                                       # every workgroup of 512 neurons is exactly full
    ranges, P, nblk = cut(lib, deg, whole_row_windows(N))
    check_partition(ranges, deg)
    assert [tuple(r) for r in ranges] == [(j, 512) for j in range(0, N, 512)]
