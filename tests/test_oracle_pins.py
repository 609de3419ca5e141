"""Pins for the CPU oracle: everything here checks oracle/ against something
other than itself -- a dense matrix product written out in numpy, integer
closed forms, fixed points the mathematics gives, and invariants of Eq. 1
(Section II-A-1).  No GPU needed.
"""
import numpy as np
import pytest
from scipy.stats import binom

import oracle
import synth

EPS32 = float(np.finfo(np.float32).eps)


def rand_model(rng, N, L, distinct=True, values="mixed", bias="neg"):
    idx, val = [], []
    for _ in range(L):
        if distinct:
            a = np.stack([np.sort(rng.choice(N, 32, replace=False)) for _ in range(N)]).astype(np.int32)
        else:
            a = rng.integers(0, N, size=(N, 32)).astype(np.int32)
        if values == "mixed":
            v = rng.uniform(-0.25, 0.5, size=(N, 32)).astype(np.float32)
        elif values == "pos":
            v = rng.uniform(0.0, 0.2, size=(N, 32)).astype(np.float32)
        else:
            v = np.full((N, 32), values, dtype=np.float32)
        idx.append(a)
        val.append(v)
    if bias == "neg":
        b = -rng.uniform(0.0, 0.3, size=N).astype(np.float32)
    else:
        b = np.full(N, bias, dtype=np.float32)
    return idx, val, b


def dense_forward(idx, val, bias, Y0):
    """Eq. 1 written out with dense N x N matrices in float64, no pruning.
    W[j, c] = sum of the values of output j's connections to input c."""
    Y = np.asarray(Y0, dtype=np.float64)
    N = Y.shape[1]
    mags = []
    for a, v in zip(idx, val):
        W = np.zeros((N, N))
        for j in range(N):
            for k in range(32):
                W[j, a[j, k]] += float(v[j, k])
        Z = Y @ W.T + bias.astype(np.float64)[None, :]
        mags.append(np.abs(Y) @ np.abs(W).T + np.abs(bias.astype(np.float64))[None, :])
        Y = np.minimum(np.maximum(Z, 0.0), 32.0)
    return Y, mags


def scatter_full(res, batch, N):
    """Oracle result -> dense [batch, N] with dropped rows as zero."""
    out = np.zeros((batch, N), dtype=res.Y.dtype)
    out[res.active_rows] = res.Y
    return out


@pytest.mark.parametrize("N,L,batch,distinct", [(32, 1, 5, True), (64, 3, 8, True), (128, 4, 6, True),
                                                (48, 2, 7, False)])
def test_brute_force_dense(N, L, batch, distinct):
    rng = np.random.default_rng(1000 + N + L)
    idx, val, b = rand_model(rng, N, L, distinct=distinct)
    Y0 = rng.uniform(0, 1, size=(batch, N)).astype(np.float32)
    ref, mags = dense_forward(idx, val, b, Y0)
    # double-precision oracle, no skipping: equal up to summation order in double
    r64 = oracle.infer(idx, val, b, Y0.astype(np.float64), no_skip=True, f64=True)
    got64 = scatter_full(r64, batch, N)
    assert np.allclose(got64, ref, rtol=0, atol=1e-11)
    # float oracle: within the standard bound 32*eps*sum|y*w| for one layer
    r32 = oracle.infer(idx, val, b, Y0)
    got32 = scatter_full(r32, batch, N).astype(np.float64)
    if L == 1:
        bound = 34 * EPS32 * mags[0] + 1e-30
        assert np.all(np.abs(got32 - ref) <= bound)
    else:
        assert np.allclose(got32, ref, rtol=2e-5, atol=2e-5)
    # the active list is exactly the rows with a positive element
    expect_rows = np.nonzero((ref > 1e-6).any(1))[0]
    sure = np.nonzero((ref > 1e-3).any(1))[0]
    assert set(sure) <= set(r32.active_rows.tolist())
    assert set(r64.active_rows.tolist()) >= set(expect_rows.tolist())


def test_transposed_operand_would_fail():
    """The dense reference distinguishes W from its transpose: a pattern that is
    far from symmetric gives different results when read the other way round."""
    rng = np.random.default_rng(5)
    N = 64
    idx, val, b = rand_model(rng, N, 1)
    Y0 = rng.uniform(0, 1, size=(4, N)).astype(np.float32)
    ref, _ = dense_forward(idx, val, b, Y0)
    W = np.zeros((N, N))
    for j in range(N):
        for k in range(32):
            W[j, idx[0][j, k]] += float(val[0][j, k])
    wrong = np.minimum(np.maximum(Y0.astype(np.float64) @ W + b[None, :], 0), 32)
    assert not np.allclose(ref, wrong, atol=1e-3)
    got = scatter_full(oracle.infer(idx, val, b, Y0), 4, N)
    assert np.allclose(got, ref, atol=1e-5)


@pytest.mark.parametrize("cfg,rows", [(0, 1000), (2, 48), (3, 12), (4, 4)])
def test_layer0_integer_closed_form(cfg, rows):
    """With binary inputs and weights 1/16 the first layer is integer counting:
    Y_1[r][j] = max(k/16 + b, 0), k = number of ones among the 32 gathered
    inputs; k/16 is exact in float and the one addition rounds once."""
    c = synth.config(cfg)
    N = c["N"]
    idx = synth.gen_layer(N, 0, c["seed"], c["window"])
    val = synth.gen_values(N)
    b = synth.gen_bias(N, c["bias"])
    Y0 = synth.gen_y0(c["batch"], N, c["seed"], rows=np.arange(rows))
    k = Y0.astype(np.int64)[:, idx.reshape(-1)].reshape(rows, N, 32).sum(-1)
    z = (k.astype(np.float32) * np.float32(0.0625)) + np.float32(c["bias"])
    expect = np.maximum(z, np.float32(0)).astype(np.float32)
    res = oracle.infer([idx], [val], b, Y0)
    got = scatter_full(res, rows, N)
    assert got.dtype == np.float32
    assert np.array_equal(got, expect)
    assert np.array_equal(res.active_rows, np.nonzero((expect > 0).any(1))[0])
    # statistics of the draw: P(positive) = P(Bin(32, 0.15) >= kmin)
    kmin = int(np.floor(-c["bias"] * 16)) + 1
    p = binom.sf(kmin - 1, 32, synth.DENSITY)
    frac = (expect > 0).mean()
    # elements of one row share that row's realised density, so the spread is
    # governed by the number of rows, not of elements
    assert abs(frac - p) < 0.15 / np.sqrt(rows), (frac, p)
    assert float(expect[expect > 0].min()) == float(np.float32(kmin * 0.0625) + np.float32(c["bias"]))


def test_positive_fraction_values():
    """The layer-0 survival probabilities quoted for the four bias values."""
    want = {-0.30: 0.535642, -0.35: 0.345632, -0.40: 0.194742, -0.45: 0.095840}
    for b, p in want.items():
        kmin = int(np.floor(-b * 16)) + 1
        assert abs(binom.sf(kmin - 1, 32, 0.15) - p) < 5e-6


@pytest.mark.parametrize("bias,seq", [(-0.3, [1.7, 3.1, 5.9, 11.5, 22.7, 32.0, 32.0, 32.0]),
                                      (-0.45, [1.55, 2.65, 4.85, 9.25, 18.05, 32.0, 32.0])])
def test_uniform_row_fixed_points(bias, seq):
    """Every neuron's weights sum to 32/16 = 2, so a constant row c maps to the
    constant clip(2c + b) whatever the pattern: pins iteration and the clip."""
    N = 256
    L = len(seq)
    idx = [synth.gen_layer(N, l, 99) for l in range(L)]
    val = [synth.gen_values(N) for _ in range(L)]
    b = synth.gen_bias(N, bias)
    Y0 = np.ones((3, N), dtype=np.float32)
    Y0[1] = 0.0                      # a dead row between two live ones
    for depth in range(1, L + 1):
        res = oracle.infer(idx[:depth], val[:depth], b, Y0)
        assert res.active_rows.tolist() == [0, 2]
        assert np.allclose(res.Y, seq[depth - 1], rtol=1e-5, atol=0)
        if seq[depth - 1] == 32.0:
            assert np.all(res.Y == np.float32(32.0))


def identity_model(N, L, rng):
    idx, val = [], []
    for _ in range(L):
        a = rng.integers(0, N, size=(N, 32)).astype(np.int32)
        v = np.zeros((N, 32), dtype=np.float32)
        slot = rng.integers(0, 32, size=N)
        a[np.arange(N), slot] = np.arange(N)
        v[np.arange(N), slot] = 1.0
        idx.append(a)
        val.append(v)
    return idx, val, np.zeros(N, dtype=np.float32)


def test_identity_pattern_passes_through_clipped():
    rng = np.random.default_rng(11)
    N = 96
    idx, val, b = identity_model(N, 3, rng)
    Y0 = rng.uniform(-5, 40, size=(9, N)).astype(np.float32)
    Y0[4] = -1.0
    res = oracle.infer(idx, val, b, Y0)
    expect = np.clip(Y0, 0, 32)
    rows = np.nonzero((expect > 0).any(1))[0]
    assert np.array_equal(res.active_rows, rows)
    assert np.array_equal(res.Y, expect[rows])
    assert 4 not in res.active_rows


def test_zero_input_stays_zero():
    rng = np.random.default_rng(12)
    idx, val, b = rand_model(rng, 64, 3)
    res = oracle.infer(idx, val, b, np.zeros((5, 64), dtype=np.float32))
    assert res.n_active == 0 and res.Y.shape == (0, 64)
    assert res.active_per_layer.tolist() == [5, 0, 0, 0]
    assert res.layers_evaluated == 1
    full = oracle.infer(idx, val, b, np.zeros((5, 64), dtype=np.float32), no_skip=True)
    assert full.n_active == 0 and full.layers_evaluated == 3


def test_outputs_in_range_and_lists_consistent():
    rng = np.random.default_rng(13)
    idx, val, b = rand_model(rng, 128, 4, values="pos")
    Y0 = rng.uniform(0, 30, size=(20, 128)).astype(np.float32)
    Y0[::3] = 0
    res = oracle.infer(idx, val, b, Y0)
    assert res.Y.min() >= 0 and res.Y.max() <= 32
    assert (res.Y.max(1) > 0).all()
    assert np.all(np.diff(res.active_rows) > 0)
    assert np.all(np.diff(res.active_per_layer) <= 0)
    assert res.active_per_layer[-1] == res.n_active
    assert res.Y.max() == 32.0, "this model saturates: the clip must have acted"


def test_row_independence_and_permutation():
    rng = np.random.default_rng(14)
    idx, val, b = rand_model(rng, 64, 3)
    Y0 = rng.uniform(0, 2, size=(12, 64)).astype(np.float32)
    Y0[[2, 7]] = 0
    full = oracle.infer(idx, val, b, Y0)
    sub_rows = np.array([1, 2, 5, 7, 11])
    sub = oracle.infer(idx, val, b, Y0[sub_rows])
    dense_full = scatter_full(full, 12, 64)
    assert np.array_equal(scatter_full(sub, 5, 64), dense_full[sub_rows])
    perm = rng.permutation(12)
    pr = oracle.infer(idx, val, b, Y0[perm])
    assert np.array_equal(scatter_full(pr, 12, 64), dense_full[perm])
    assert sorted(perm[pr.active_rows].tolist()) == full.active_rows.tolist()


def test_monotone_in_input_for_nonnegative_weights():
    rng = np.random.default_rng(15)
    idx, val, b = rand_model(rng, 64, 3, values="pos")
    Y0 = rng.uniform(0, 1, size=(6, 64)).astype(np.float32)
    Y1 = Y0 + rng.uniform(0, 0.5, size=Y0.shape).astype(np.float32)
    a = scatter_full(oracle.infer(idx, val, b, Y0), 6, 64)
    c = scatter_full(oracle.infer(idx, val, b, Y1), 6, 64)
    assert np.all(c >= a)


def test_skip_equals_no_skip():
    c = synth.config(0)
    N, L = c["N"], 4
    idx = [synth.gen_layer(N, l, c["seed"]) for l in range(L)]
    val = [synth.gen_values(N) for _ in range(L)]
    b = synth.gen_bias(N, c["bias"])
    Y0 = synth.gen_y0(200, N, c["seed"], density="mixed")
    for depth in (1, 2, 4):
        a = oracle.infer(idx[:depth], val[:depth], b, Y0)
        n = oracle.infer(idx[:depth], val[:depth], b, Y0, no_skip=True)
        assert np.array_equal(a.active_rows, n.active_rows)
        assert np.array_equal(a.Y, n.Y)
        assert np.array_equal(a.active_per_layer, n.active_per_layer)
    assert 0 < a.n_active < 200, "mixed densities: some rows die, some survive"


def test_float_vs_double_within_bound():
    rng = np.random.default_rng(16)
    idx, val, b = rand_model(rng, 128, 1)
    Y0 = rng.uniform(0, 4, size=(10, 128)).astype(np.float32)
    f = scatter_full(oracle.infer(idx, val, b, Y0), 10, 128).astype(np.float64)
    d = scatter_full(oracle.infer(idx, val, b, Y0.astype(np.float64), f64=True), 10, 128)
    _, mags = dense_forward(idx, val, b, Y0)
    assert np.all(np.abs(f - d) <= 34 * EPS32 * mags[0])


def test_missing_layer_is_an_error_only_if_reached():
    rng = np.random.default_rng(17)
    idx, val, b = rand_model(rng, 64, 3)
    z = np.zeros((2, 64), dtype=np.float32)
    r = oracle.infer([idx[0], None, None], [val[0], None, None], b, z)
    assert r.n_active == 0
    Y0 = np.full((2, 64), 30, dtype=np.float32)
    with pytest.raises(RuntimeError):
        oracle.infer([idx[0], None], [np.abs(val[0]), None], np.zeros(64, np.float32), Y0)


def test_fragile_rows_are_reported():
    """A row whose largest pre-activation is within 1e-4 of zero is flagged at
    that layer; rows far from zero are not."""
    N = 64
    idx, val, _ = identity_model(N, 1, np.random.default_rng(18))
    b = np.full(N, -1.0, dtype=np.float32)
    Y0 = np.zeros((3, N), dtype=np.float32)
    Y0[0, 5] = 1.00005      # z = +5e-5  -> active but fragile
    Y0[1, 5] = 0.99995      # z = -5e-5  -> dead but fragile
    Y0[2, 5] = 1.5          # z = 0.5    -> solidly active
    r = oracle.infer(idx, val, b, Y0)
    assert r.fragile_layer.tolist() == [0, 0, -1]
    assert r.active_rows.tolist() == [0, 2]


def test_config0_dynamics():
    """With density 0.15 and bias -0.3 the mean pre-activation is 0: every row
    still has positives after layer 0, almost none after layer 1, none soon
    after -- the benchmark's active set is empty long before layer L."""
    c = synth.config(0)
    N = c["N"]
    idx = [synth.gen_layer(N, l, c["seed"]) for l in range(6)]
    val = [synth.gen_values(N)] * 6
    b = synth.gen_bias(N, c["bias"])
    Y0 = synth.gen_y0(c["batch"], N, c["seed"])
    r = oracle.infer(idx, val, b, Y0)
    apl = r.active_per_layer.tolist()
    assert apl[0] == 1000 and apl[1] == 1000
    assert apl[2] < 100 and apl[-1] == 0


def test_table1_metric_arithmetic():
    """Throughput = inputs * neurons * 32 * layers / time (Section IV-A): the
    printed times and TeraEdges/s of Table I agree under that reading."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "table1_v100.txt")
    n = 0
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        N, L, te, sec = line.split()
        got = synth.nominal_edges(int(N), int(L), 60000) / float(sec) / 1e12
        assert abs(got - float(te)) / float(te) < 0.01, line
        n += 1
    assert n >= 10
