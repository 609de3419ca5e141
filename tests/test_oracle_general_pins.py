"""Pins for the oracle's general-layer (CSR) form: neurons with any number of
connections (Section II-A-1: W_l may be any sparse matrix).  Each test checks
oracle/ against something other than itself: a dense matrix product in numpy,
closed forms, and invariants of Eq. 1.  No GPU needed.
"""
import numpy as np
import pytest

import oracle
import synth

EPS32 = float(np.finfo(np.float32).eps)


def rand_general(rng, N, L, kmax, values="mixed", empty_frac=0.1):
    ptr, idx, val = [], [], []
    for _ in range(L):
        deg = rng.integers(0, kmax + 1, size=N)
        deg[rng.uniform(size=N) < empty_frac] = 0
        p = np.zeros(N + 1, dtype=np.int32)
        np.cumsum(deg, out=p[1:])
        a = rng.integers(0, N, size=int(p[N])).astype(np.int32)      # repeats allowed
        if values == "mixed":
            v = rng.uniform(-0.25, 0.5, size=int(p[N])).astype(np.float32)
        else:
            v = np.full(int(p[N]), values, dtype=np.float32)
        ptr.append(p)
        idx.append(a)
        val.append(v)
    b = -rng.uniform(0.0, 0.3, size=N).astype(np.float32)
    return ptr, idx, val, b


def dense_matrices(ptr, idx, val, N):
    """W[j, c] = sum of the values of output j's connections to input c."""
    Ws = []
    for p, a, v in zip(ptr, idx, val):
        W = np.zeros((N, N))
        rows = np.repeat(np.arange(N), np.diff(p))
        np.add.at(W, (rows, a), v.astype(np.float64))
        Ws.append(W)
    return Ws


def dense_forward(ptr, idx, val, bias, Y0):
    Y = np.asarray(Y0, dtype=np.float64)
    mags = []
    for W in dense_matrices(ptr, idx, val, Y.shape[1]):
        Z = Y @ W.T + bias.astype(np.float64)[None, :]
        mags.append(np.abs(Y) @ np.abs(W).T + np.abs(bias.astype(np.float64))[None, :])
        Y = np.minimum(np.maximum(Z, 0.0), 32.0)
    return Y, mags


def scatter_full(res, batch, N):
    out = np.zeros((batch, N), dtype=res.Y.dtype)
    out[res.active_rows] = res.Y
    return out


@pytest.mark.parametrize("N,L,batch,kmax", [(32, 1, 5, 7), (64, 3, 8, 40), (96, 2, 6, 100), (128, 4, 5, 33)])
def test_brute_force_dense_general(N, L, batch, kmax):
    rng = np.random.default_rng(4000 + N + kmax)
    ptr, idx, val, b = rand_general(rng, N, L, kmax)
    Y0 = rng.uniform(0, 1, size=(batch, N)).astype(np.float32)
    ref, mags = dense_forward(ptr, idx, val, b, Y0)
    r64 = oracle.infer(idx, val, b, Y0.astype(np.float64), no_skip=True, f64=True, ptr=ptr)
    assert np.allclose(scatter_full(r64, batch, N), ref, rtol=0, atol=1e-11)
    r32 = oracle.infer(idx, val, b, Y0, ptr=ptr)
    got32 = scatter_full(r32, batch, N).astype(np.float64)
    if L == 1:
        # one rounding per connection and one for the bias: (kmax + 2) * eps * sum|y*w|
        assert np.all(np.abs(got32 - ref) <= (kmax + 2) * EPS32 * mags[0] + 1e-30)
    else:
        assert np.allclose(got32, ref, rtol=2e-5, atol=2e-5)
    sure = np.nonzero((ref > 1e-3).any(1))[0]
    assert set(sure) <= set(r32.active_rows.tolist())
    assert set(r32.active_rows.tolist()) <= set(np.nonzero((ref > -1e-6).any(1))[0].tolist())


def test_transposed_or_shifted_rows_would_fail():
    """The dense reference tells W from its transpose and ptr[j] from ptr[j+1]: reading
    the pattern the other way round, or neuron j's entries as neuron j+1's, gives
    different numbers."""
    rng = np.random.default_rng(11)
    N = 64
    ptr, idx, val, b = rand_general(rng, N, 1, 20, empty_frac=0.0)
    Y0 = rng.uniform(0, 1, size=(4, N)).astype(np.float32)
    ref, _ = dense_forward(ptr, idx, val, b, Y0)
    W = dense_matrices(ptr, idx, val, N)[0]
    clip = lambda z: np.minimum(np.maximum(z, 0), 32)
    assert not np.allclose(ref, clip(Y0.astype(np.float64) @ W + b[None, :]), atol=1e-3)
    assert not np.allclose(ref, clip(Y0.astype(np.float64) @ np.roll(W, 1, axis=0).T + b[None, :]), atol=1e-3)
    got = scatter_full(oracle.infer(idx, val, b, Y0, ptr=ptr), 4, N)
    assert np.allclose(got, ref, atol=1e-5)


def test_constant_row_closed_form_with_neuron_sums():
    """A row of constant c gives neuron j the value clip(c * s_j + b_j), s_j the sum of
    its weights, whatever the pattern; neurons without connections give clip(b_j) = 0."""
    rng = np.random.default_rng(12)
    N = 96
    ptr, idx, val, b = rand_general(rng, N, 1, 50, values=0.125, empty_frac=0.2)
    deg = np.diff(ptr[0])
    assert (deg == 0).any() and (deg > 32).any()
    cs = np.array([0.0, 0.25, 1.0, 7.0, 32.0], dtype=np.float32)
    Y0 = np.repeat(cs[:, None], N, axis=1)
    res = oracle.infer(idx, val, b, Y0, ptr=ptr)
    got = scatter_full(res, len(cs), N)
    # c * (deg / 8) is exact in float for these c; one rounding in the bias addition
    expect = np.minimum(np.maximum((cs[:, None] * (deg[None, :] * np.float32(0.125))).astype(np.float32) + b[None, :], 0), 32)
    assert np.array_equal(got, expect.astype(np.float32))
    assert np.all(got[:, deg == 0] == 0)
    assert (got == 32).any()          # the upper clip is reached
    assert 0 not in res.active_rows   # the all-zero row is dropped


def test_fixed_32_is_the_special_case():
    """With 32 connections for every neuron the general form is the fixed form, bit for bit."""
    c = synth.config(0)
    N = c["N"]
    idx = [synth.gen_layer(N, l, c["seed"]) for l in range(3)]
    val = [synth.gen_values(N) for _ in range(3)]
    b = synth.gen_bias(N, c["bias"])
    Y0 = synth.gen_y0(40, N, c["seed"], density="mixed")
    ptr = [np.arange(0, 32 * N + 1, 32, dtype=np.int32)] * 3
    a = oracle.infer(idx, val, b, Y0)
    g = oracle.infer([i.reshape(-1) for i in idx], [v.reshape(-1) for v in val], b, Y0, ptr=ptr)
    assert np.array_equal(a.active_rows, g.active_rows) and np.array_equal(a.Y, g.Y)
    assert np.array_equal(a.active_per_layer, g.active_per_layer)


def test_zero_weight_connections_change_nothing():
    """Appending connections of weight zero to every neuron (the padding of the sliced
    storage of Section III-A-3) leaves every output bit unchanged."""
    rng = np.random.default_rng(13)
    N, L, batch = 64, 3, 9
    ptr, idx, val, b = rand_general(rng, N, L, 20)
    ptr2, idx2, val2 = [], [], []
    for p, a, v in zip(ptr, idx, val):
        deg = np.diff(p)
        extra = rng.integers(0, 6, size=N)
        q = np.zeros(N + 1, dtype=np.int32)
        np.cumsum(deg + extra, out=q[1:])
        a2 = np.zeros(int(q[N]), dtype=np.int32)
        v2 = np.zeros(int(q[N]), dtype=np.float32)
        for j in range(N):
            a2[q[j]:q[j] + deg[j]] = a[p[j]:p[j + 1]]
            v2[q[j]:q[j] + deg[j]] = v[p[j]:p[j + 1]]
            a2[q[j] + deg[j]:q[j + 1]] = rng.integers(0, N, size=extra[j])
        ptr2.append(q)
        idx2.append(a2)
        val2.append(v2)
    Y0 = rng.uniform(0, 1, size=(batch, N)).astype(np.float32)
    r1 = oracle.infer(idx, val, b, Y0, ptr=ptr)
    r2 = oracle.infer(idx2, val2, b, Y0, ptr=ptr2)
    assert np.array_equal(r1.active_rows, r2.active_rows) and np.array_equal(r1.Y, r2.Y)


def test_skip_equals_no_skip_general():
    rng = np.random.default_rng(14)
    N, L, batch = 64, 5, 30
    ptr, idx, val, b = rand_general(rng, N, L, 45, values=0.05)
    Y0 = (rng.uniform(size=(batch, N)) < rng.uniform(0.0, 0.6, size=(batch, 1))).astype(np.float32)
    a = oracle.infer(idx, val, b, Y0, ptr=ptr)
    n = oracle.infer(idx, val, b, Y0, ptr=ptr, no_skip=True)
    assert 0 < a.n_active < batch
    assert np.array_equal(a.active_rows, n.active_rows) and np.array_equal(a.Y, n.Y)


def test_generator_general_layers():
    """Lengths inside [kmin, kmax], columns in range, weight sums near 2, same bytes on a second call."""
    N = 2048
    p, a, v = synth.gen_layer_general(N, 3, 99, 0, 80)
    d = np.diff(p)
    assert d.min() == 0 and d.max() == 80 and p[0] == 0 and p[N] == len(a) == len(v)
    assert a.min() >= 0 and a.max() < N and a.dtype == np.int32 and v.dtype == np.float32
    s = np.add.reduceat(v.astype(np.float64), p[:-1][d > 0])
    # m/2**23 is uniform in [1, 3): mean 2, the sum over d of them / d has sd <= 0.58/sqrt(d)
    assert abs(s[d[d > 0] >= 16].mean() - 2.0) < 0.02
    p2, a2, v2 = synth.gen_layer_general(N, 3, 99, 0, 80)
    assert np.array_equal(p, p2) and np.array_equal(a, a2) and np.array_equal(v, v2)
    pw, aw, vw = synth.gen_layer_general(N, 3, 99, 8, 24, window=256, uniform_weight=True)
    assert (vw == np.float32(0.0625)).all()
    blk = np.repeat(np.arange(N), np.diff(pw)) // 256
    base = synth.window_bases(N, 3, 99, 256)[0][::256]
    assert ((aw >= base[blk]) & (aw < base[blk] + 256)).all()
