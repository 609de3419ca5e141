"""The seeded generator: structure of the draws, agreement of the numpy and
torch backends, and stability of the bits (golden digests)."""
import importlib.util
import os

import numpy as np
import pytest

import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


@pytest.mark.parametrize("N,window", [(64, None), (1024, None), (8192, 1024)])
def test_columns_distinct_sorted_in_window(N, window):
    a = synth.gen_layer(N, 2, 77, window)
    assert a.shape == (N, 32) and a.dtype == np.int32
    assert np.all(np.diff(a, axis=1) > 0)
    assert a.min() >= 0 and a.max() < N
    if window:
        w = a // window
        assert np.all(w.min(1) == w.max(1))
        blocks = w[:, 0].reshape(N // window, window)
        assert np.all(blocks == blocks[:, :1])
        assert sorted(blocks[:, 0].tolist()) == list(range(N // window)), "windows are a permutation"
    b = synth.gen_layer(N, 3, 77, window)
    assert not np.array_equal(a, b), "every layer has its own pattern"


def test_backends_agree():
    for N, window in [(256, None), (8192, 2048)]:
        a = synth.gen_layer(N, 5, 3, window)
        b = synth.gen_layer(N, 5, 3, window, device="cpu").numpy()
        assert np.array_equal(a, b)
    for dens in (0.15, "mixed"):
        y = synth.gen_y0(300, 512, 9, density=dens)
        t = synth.gen_y0(300, 512, 9, density=dens, device="cpu", chunk_rows=7).numpy()
        assert np.array_equal(y, t)
        sub = synth.gen_y0(300, 512, 9, density=dens, rows=[4, 250])
        assert np.array_equal(sub, y[[4, 250]])


def test_y0_is_binary_with_the_stated_density():
    y = synth.gen_y0(400, 4096, 1)
    assert set(np.unique(y).tolist()) == {0.0, 1.0}
    assert abs(y.mean() - 0.15) < 0.002
    m = synth.gen_y0(4000, 1024, 1, density="mixed").mean(1)
    assert ((m > 0.02) & (m < 0.25)).sum() + ((m > 0.35) & (m < 0.65)).sum() == 4000
    assert 0.4 < (m > 0.3).mean() < 0.6


def test_golden_digests():
    spec = importlib.util.spec_from_file_location("mk", os.path.join(GOLD, "make_synth_golden.py"))
    mk = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mk)
    want = open(os.path.join(GOLD, "synth_golden.txt")).read().strip().splitlines()
    assert list(mk.lines()) == want


def test_scattered_window_variant():
    """scatter_columns renames the columns by one permutation per layer: each block's set of
    columns keeps its size but spreads over the row; rows stay sorted and distinct; both
    backends agree."""
    import torch
    N, w = 8192, 1024
    a = synth.gen_layer(N, 3, 11, w)
    b = synth.scatter_columns(a, N, 3, 11)
    assert b.dtype == np.int32 and b.shape == a.shape and (np.diff(b, axis=1) > 0).all()
    for blk in range(N // w):
        ua, ub = np.unique(a[blk * w:(blk + 1) * w]), np.unique(b[blk * w:(blk + 1) * w])
        assert len(ua) == len(ub) <= w and ua.max() - ua.min() < w and ub.max() - ub.min() > N // 2
    # a permutation: two columns are equal after renaming iff they were equal before
    assert len(np.unique(b)) == len(np.unique(a))
    assert not np.array_equal(b, synth.scatter_columns(a, N, 4, 11))
    assert np.array_equal(b, synth.scatter_columns(torch.from_numpy(a), N, 3, 11, device="cpu").numpy())


def test_strided_layers():
    a = synth.gen_layer_strided(4096, 128)
    assert a.shape == (4096, 32) and a.dtype == np.int32
    assert np.all(np.diff(a, axis=1) > 0) and a.min() == 0 and a.max() == 4095
    j = 777
    assert sorted(((j + np.arange(32) * 128) % 4096).tolist()) == a[j].tolist()
    # every column is read by exactly 32 neurons
    assert np.all(np.bincount(a.ravel(), minlength=4096) == 32)
