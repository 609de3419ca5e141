"""GPU parity: the HIP path, called through the C-ABI binding, against the CPU
oracle on the same seeded inputs (see parity_util for the bar)."""
import numpy as np
import pytest

import oracle
import synth
from parity_util import MAX_FRAGILE_FRAC, check_against_oracle, close, config_model, gpu_infer

pytestmark = pytest.mark.gpu


def rand_model(rng, N, L, distinct=True, sort=True, lo=-0.25, hi=0.5):
    idx, val = [], []
    for _ in range(L):
        if distinct:
            a = np.stack([rng.choice(N, 32, replace=False) for _ in range(N)])
        else:
            a = rng.integers(0, N, size=(N, 32))
        if sort:
            a = np.sort(a, axis=1)
        idx.append(a.astype(np.int32))
        val.append(rng.uniform(lo, hi, size=(N, 32)).astype(np.float32))
    bias = -rng.uniform(0.0, 0.3, size=N).astype(np.float32)
    return idx, val, bias


@pytest.mark.parametrize("N,L,batch,distinct,sort", [
    (32, 3, 5, True, True),        # smallest N, ragged row group
    (96, 4, 37, True, True),
    (64, 2, 8, False, False),      # duplicated and unsorted columns
    (1028, 2, 70, True, True),     # second output block has 4 neurons
    (2052, 3, 33, True, False),    # three output blocks, unsorted
    (5000, 2, 9, True, True),      # window wider than one LDS stage
])
def test_random_models(N, L, batch, distinct, sort):
    """Arbitrary patterns and non-negative weights of any size: the stated bar."""
    rng = np.random.default_rng(N * 131 + L)
    idx, val, bias = rand_model(rng, N, L, distinct, sort, lo=0.0, hi=0.12)
    Y0 = rng.uniform(0, 1, size=(batch, N)).astype(np.float32)
    Y0[batch // 2] = 0
    ref = oracle.infer(idx, val, bias, Y0)
    n, rows, Y = gpu_infer(idx, val, bias, Y0)
    common, _ = check_against_oracle(ref, n, rows, Y, what="random N=%d" % N)
    assert common > 0


@pytest.mark.parametrize("N,L,batch,kind", [
    (12288, 2, 37, "uniform"),     # 3 stages of 4096 columns: many neurons exceed 16 connections in a stage (spill list)
    (40000, 2, 13, "uniform"),     # 10 stages: 8 steps per stage
    (12288, 1, 9, "clustered"),    # every neuron's 32 columns in one stage: does not fit -> staged kernel
    (16384, 2, 21, "small_arena"), # arena sized for narrow windows -> staged kernel
])
def test_wide_windows(N, L, batch, kind):
    """Layers whose blocks read more than two LDS stages of columns."""
    import paper_2007_14152_amd as sp
    rng = np.random.default_rng(N + L)
    if kind == "clustered":
        idx = []
        for _ in range(L):
            base = rng.integers(0, N // 4096, size=N) * 4096
            a = np.stack([np.sort(b + rng.choice(4096, 32, replace=False)) for b in base])
            idx.append(a.astype(np.int32))
        val = [rng.uniform(0.0, 0.12, size=(N, 32)).astype(np.float32) for _ in range(L)]
        bias = -rng.uniform(0.0, 0.3, size=N).astype(np.float32)
    else:
        idx, val, bias = rand_model(rng, N, L, True, True, lo=0.0, hi=0.12)
    Y0 = rng.uniform(0, 1, size=(batch, N)).astype(np.float32)
    Y0[1] = 0
    ref = oracle.infer(idx, val, bias, Y0)
    m = sp.Model(idx, val, bias, window_hint=4096 if kind == "small_arena" else None)
    assert m.widest_window > 8192
    n, rows, Y = gpu_infer(idx, val, bias, Y0, model=m)
    m.close()
    common, _ = check_against_oracle(ref, n, rows, Y, what="wide %s N=%d" % (kind, N))
    assert common > 0


@pytest.mark.parametrize("N,batch", [(64, 9), (1028, 21), (5000, 6), (16384, 5)])
def test_mixed_sign_weights_one_layer(N, batch):
    """Weights of both signs cancel, so the result can be far smaller than the terms
    that were added; the library adds a neuron's 32 products in its own order, and
    the float bound for any order is |error| <= 32*eps*sum|y*w| (+ one rounding of
    the bias add), which is what this case is held to."""
    rng = np.random.default_rng(N + 7)
    idx, val, bias = rand_model(rng, N, 1, True, True, lo=-0.25, hi=0.5)
    Y0 = rng.uniform(0, 4, size=(batch, N)).astype(np.float32)
    ref = oracle.infer(idx, val, bias, Y0.astype(np.float64), f64=True, no_skip=True)
    exact = np.zeros((batch, N))
    exact[ref.active_rows] = ref.Y
    mag = np.zeros((batch, N))
    for j in range(N):
        mag[:, j] = np.abs(Y0[:, idx[0][j]].astype(np.float64) * val[0][j].astype(np.float64)).sum(1)
    mag += np.abs(bias.astype(np.float64))[None, :]
    n, rows, Y = gpu_infer(idx, val, bias, Y0)
    got = np.zeros((batch, N))
    got[rows] = Y
    eps = float(np.finfo(np.float32).eps)
    assert np.all(np.abs(got - exact) <= 34 * eps * mag + 1e-30)
    sure = np.nonzero((exact > 1e-3).any(1))[0]
    assert set(sure.tolist()) <= set(rows.tolist())


@pytest.mark.parametrize("N,batch,L", [(64, 9, 3), (1028, 21, 4), (4096, 7, 3)])
def test_mixed_sign_weights_several_layers(N, batch, L):
    """Mixed-sign weights through several layers, against the double-precision oracle with the float
    bound carried from layer to layer: ReLU and clip do not expand errors, so
        err_{l+1}[r][j] <= sum_k |w_jk| * err_l[r][idx_jk] + 34*eps*(sum_k |y_k * w_jk| + |b_j|),
    whatever order the 32 products are added in.  The active set is asserted on the rows whose exact
    largest output clears its bound (and on the rows with no output near zero)."""
    rng = np.random.default_rng(N + 11)
    idx, val, bias = rand_model(rng, N, L, True, True, lo=-0.2, hi=0.3)
    Y0 = rng.uniform(0, 4, size=(batch, N)).astype(np.float32)
    eps = float(np.finfo(np.float32).eps)
    y = Y0.astype(np.float64)                  # exact activations of every row, no skipping
    err = np.zeros_like(y)
    for l in range(L):
        w = val[l].astype(np.float64)
        z = np.einsum("rjk,jk->rj", y[:, idx[l]], w) + bias.astype(np.float64)[None, :]
        mag = np.einsum("rjk,jk->rj", np.abs(y[:, idx[l]]), np.abs(w)) + np.abs(bias.astype(np.float64))[None, :]
        err = np.einsum("rjk,jk->rj", err[:, idx[l]], np.abs(w)) + 34 * eps * mag
        y = np.clip(z, 0.0, 32.0)
    ref = oracle.infer(idx, val, bias, Y0.astype(np.float64), f64=True, no_skip=True)
    exact = np.zeros((batch, N))
    exact[ref.active_rows] = ref.Y
    assert np.allclose(exact, y, rtol=0, atol=1e-12), "the test's own recurrence restates Eq. 1"
    n, rows, Y = gpu_infer(idx, val, bias, Y0)
    got = np.zeros((batch, N))
    got[rows] = Y
    assert np.all(np.abs(got - exact) <= 1.01 * err + 1e-30)
    sure_alive = np.nonzero((exact > 1.01 * err + 1e-30).any(1))[0]
    assert set(sure_alive.tolist()) <= set(rows.tolist())
    assert len(sure_alive) > 0


@pytest.mark.parametrize("layers", [1, 2, 3, 120])
def test_config0(layers):
    c, idx, val, bias = config_model(0, layers)
    Y0 = synth.gen_y0(c["batch"], c["N"], c["seed"])
    ref = oracle.infer(idx, val, bias, Y0)
    n, rows, Y = gpu_infer(idx, val, bias, Y0)
    check_against_oracle(ref, n, rows, Y, what="cfg0 L=%d" % layers, max_fragile_frac=MAX_FRAGILE_FRAC)
    if layers == 1:
        assert n == 1000
    if layers == 120:
        assert n == 0 and ref.n_active == 0


@pytest.mark.parametrize("cfg,batch,layers", [(0, 3001, 12), (2, 403, 9), (3, 70, 9), (4, 41, 9)])
def test_sustained_activity(cfg, batch, layers):
    """Mixed row densities: part of the rows die in the first layers, the rest
    saturate at the clip and survive, so compaction sees partial survival."""
    c, idx, val, bias = config_model(cfg, layers)
    Y0 = synth.gen_y0(batch, c["N"], c["seed"], density="mixed")
    ref = oracle.infer(idx, val, bias, Y0)
    assert 0 < ref.n_active < batch
    n, rows, Y = gpu_infer(idx, val, bias, Y0)
    check_against_oracle(ref, n, rows, Y, what="sustained cfg%d" % cfg, max_fragile_frac=MAX_FRAGILE_FRAC)
    assert Y.max() == 32.0


@pytest.mark.parametrize("cfg,batch", [(2, 300), (3, 64), (4, 48)])
@pytest.mark.parametrize("layers", [1, 2])
def test_config_shapes_first_layers(cfg, batch, layers):
    c, idx, val, bias = config_model(cfg, layers)
    Y0 = synth.gen_y0(c["batch"], c["N"], c["seed"], rows=np.arange(batch))
    ref = oracle.infer(idx, val, bias, Y0)
    n, rows, Y = gpu_infer(idx, val, bias, Y0)
    check_against_oracle(ref, n, rows, Y, what="cfg%d L=%d" % (cfg, layers))
    if layers == 1:
        assert n == batch


def test_identity_and_clip():
    rng = np.random.default_rng(3)
    N = 128
    idx = [rng.integers(0, N, size=(N, 32)).astype(np.int32) for _ in range(2)]
    val = [np.zeros((N, 32), dtype=np.float32) for _ in range(2)]
    for a, v in zip(idx, val):
        slot = rng.integers(0, 32, size=N)
        a[np.arange(N), slot] = np.arange(N)
        v[np.arange(N), slot] = 1.0
    bias = np.zeros(N, dtype=np.float32)
    Y0 = rng.uniform(-5, 40, size=(11, N)).astype(np.float32)
    Y0[3] = -2.0
    n, rows, Y = gpu_infer(idx, val, bias, Y0)
    expect = np.clip(Y0, 0, 32)
    keep = np.nonzero((expect > 0).any(1))[0]
    assert np.array_equal(rows, keep) and np.array_equal(Y, expect[keep])


def test_edge_cases():
    import torch
    import paper_2007_14152_amd as sp
    rng = np.random.default_rng(4)
    N = 64
    idx, val, bias = rand_model(rng, N, 2, lo=0.0, hi=0.3)
    m = sp.Model(idx, val, bias)
    # empty batch
    n, rows, Y = m.infer(torch.zeros((0, N), device="cuda"))
    assert n == 0 and rows.numel() == 0
    # all-zero input: nothing survives
    n, rows, Y = m.infer(torch.zeros((9, N), device="cuda"))
    assert n == 0
    # single row; only the last row alive; same handle reused with shrinking batches
    Y0 = np.zeros((13, N), dtype=np.float32)
    Y0[12] = 1.0
    ref = oracle.infer(idx, val, bias, Y0)
    for _ in range(2):
        n, rows, Y = gpu_infer(idx, val, bias, Y0, model=m)
        check_against_oracle(ref, n, rows, Y, what="last row")
        assert rows.tolist() == [12]
    one = np.ones((1, N), dtype=np.float32)
    ref1 = oracle.infer(idx, val, bias, one)
    n, rows, Y = gpu_infer(idx, val, bias, one, model=m)
    check_against_oracle(ref1, n, rows, Y, what="one row")
    # work arena too small / column out of range
    need = sp.spdnn_work_bytes(N, 13)
    w = torch.empty(need, dtype=torch.uint8, device="cuda")
    y = torch.zeros((13, N), device="cuda")
    r = torch.zeros(13, dtype=torch.int32, device="cuda")
    with pytest.raises(sp.SpdnnError) as e:
        sp.spdnn_infer(m.h, y.data_ptr(), 13, w.data_ptr(), need - 1, r.data_ptr(), 0)
    assert e.value.code == sp.SPDNN_ESIZE
    m.close()
    bad = [a.copy() for a in idx]
    bad[1][5, 7] = N
    with pytest.raises(sp.SpdnnError) as e:
        sp.Model(bad, val, bias)
    assert e.value.code == sp.SPDNN_EINVAL


def test_deterministic_and_device_weights():
    import torch
    import paper_2007_14152_amd as sp
    c, idx, val, bias = config_model(0, 4)
    Y0 = synth.gen_y0(777, c["N"], c["seed"], density="mixed")
    a = gpu_infer(idx, val, bias, Y0)
    b = gpu_infer(idx, val, bias, Y0)
    assert a[0] == b[0] and np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2])
    # weights handed over as device arrays, generated by the torch backend on the GPU
    _, didx, dval, dbias = config_model(0, 4, device="cuda:0")
    for h, d in zip(idx, didx):
        assert np.array_equal(h, d.cpu().numpy())
    m = sp.Model(didx, dval, dbias)
    y0 = synth.gen_y0(777, c["N"], c["seed"], density="mixed", device="cuda:0")
    assert np.array_equal(y0.cpu().numpy(), Y0)
    n, rows, Y = m.infer(y0)
    assert n == a[0] and np.array_equal(rows.cpu().numpy(), a[1]) and np.array_equal(Y.cpu().numpy(), a[2])
    m.set_profiling(True)
    m.infer(y0)
    run, rows_in, ms = m.profile()
    assert run == 4 and rows_in[0] == 777 and np.all(np.diff(rows_in) <= 0) and np.all(ms > 0)
    m.close()


def test_two_models_and_a_stream_of_the_callers():
    """Two handles alive at once, one of them on a stream the caller made (default priority),
    called in turns and with changing batch sizes: each gives what it gives alone."""
    import torch
    import paper_2007_14152_amd as sp
    c, idx, val, bias = config_model(0, 5)
    c2, idx2, val2, bias2 = config_model(2, 3)
    Ya = synth.gen_y0(500, c["N"], c["seed"], density="mixed")
    Yb = synth.gen_y0(90, c2["N"], c2["seed"], density="mixed")
    alone_a = gpu_infer(idx, val, bias, Ya)
    alone_a_small = gpu_infer(idx, val, bias, Ya[:33])
    alone_b = gpu_infer(idx2, val2, bias2, Yb)
    side = torch.cuda.Stream()
    ma = sp.Model(idx, val, bias, stream=side)
    mb = sp.Model(idx2, val2, bias2)
    ya = torch.from_numpy(Ya).to("cuda:0")
    yb = torch.from_numpy(Yb).to("cuda:0")
    torch.cuda.synchronize()   # the inputs were produced on torch's stream, ma runs on its own
    for _ in range(2):
        for y, m, ref in ((ya, ma, alone_a), (yb, mb, alone_b), (ya[:33].contiguous(), ma, alone_a_small)):
            torch.cuda.synchronize()
            n, rows, Y = m.infer(y)
            assert n == ref[0] and np.array_equal(rows.cpu().numpy(), ref[1]) and np.array_equal(Y.cpu().numpy(), ref[2])
    ma.close()
    mb.close()


def _uniform_model(rng, N, L, window, w=0.0625):
    """Every neuron: 32 distinct columns inside the 'window'-wide span its 'window'-aligned group of
    neurons shares; one weight for all connections."""
    idx = []
    for _ in range(L):
        base = (np.arange(N) // window) * window
        a = np.stack([b + rng.choice(min(window, N - b), 32, replace=False) for b in base])
        idx.append(np.sort(a, axis=1).astype(np.int32))
    val = [np.full((N, 32), w, dtype=np.float32) for _ in range(L)]
    bias = np.full(N, -0.05, dtype=np.float32)
    return idx, val, bias


@pytest.mark.parametrize("N,L,batch,window,w", [
    (2048, 3, 21, 2048, 0.0625),    # one unit of two output blocks
    (6144, 2, 13, 2048, 0.0625),    # three units
    (8192, 3, 50, 4096, 0.0625),    # two units share a window
    (4096, 2, 9, 4096, 0.07),       # a weight that is not a power of two
    (4096, 2, 1, 1024, -0.03),      # one negative weight for all: rows die after the first layer
])
def test_two_neurons_per_lane(N, L, batch, window, w):
    """Layers with a single weight value run on the kernel with two output neurons per
    lane; one different weight sends the same model to the one-neuron kernel.  Both
    must agree with the oracle."""
    import paper_2007_14152_amd as sp
    rng = np.random.default_rng(N * 7 + L)
    idx, val, bias = _uniform_model(rng, N, L, window, w)
    Y0 = (rng.uniform(0, 1, size=(batch, N)) < 0.3).astype(np.float32)
    ref = oracle.infer(idx, val, bias, Y0)
    m = sp.Model(idx, val, bias)
    assert [m.layer_kernel(l) for l in range(L)] == [sp.SPDNN_KERNEL_PAIR] * L
    n, rows, Y = gpu_infer(idx, val, bias, Y0, model=m)
    m.close()
    check_against_oracle(ref, n, rows, Y, what="pair N=%d" % N)
    # the same model with one weight changed by one ulp-ish amount in every layer: no longer uniform
    val2 = [v.copy() for v in val]
    for v in val2:
        v[N // 2, 5] = np.float32(w) * np.float32(1.0 + 2.0 ** -20)
    ref2 = oracle.infer(idx, val2, bias, Y0)
    m2 = sp.Model(idx, val2, bias)
    assert [m2.layer_kernel(l) for l in range(L)] == [sp.SPDNN_KERNEL_SINGLE] * L
    n2, rows2, Y2 = gpu_infer(idx, val2, bias, Y0, model=m2)
    m2.close()
    check_against_oracle(ref2, n2, rows2, Y2, what="single N=%d" % N)


def test_kernel_choice():
    """Which fused kernel a layer gets (spdnn_layer_kernel)."""
    import paper_2007_14152_amd as sp
    rng = np.random.default_rng(5)
    cases = [
        (1024, 1024, sp.SPDNN_KERNEL_SINGLE),    # uniform weight, but N is not a multiple of 2048
        (4096, 4096, sp.SPDNN_KERNEL_PAIR),
        (8192, 8192, sp.SPDNN_KERNEL_ROW2),        # one weight, N a multiple of 4096, window within 16384 columns
        (16384, 16384, sp.SPDNN_KERNEL_ROW2),
        (6144, 6144, sp.SPDNN_KERNEL_WIDE_PAIR4),  # two LDS stages, one weight, N not a multiple of 4096
        (32768, 32768, sp.SPDNN_KERNEL_WIDE_PAIR),   # window wider than 16384 columns
        (17408, 17408, sp.SPDNN_KERNEL_WIDE),       # five stages, N not a multiple of 2048
    ]
    for N, window, kind in cases:
        idx, val, bias = _uniform_model(rng, N, 1, window)
        m = sp.Model(idx, val, bias)
        assert m.layer_kernel(0) == kind, (N, window, m.layer_kernel(0))
        with pytest.raises(sp.SpdnnError):
            m.layer_kernel(1)
        m.close()


@pytest.mark.parametrize("N,L,batch", [
    (8192, 3, 23),     # tiles of two rows, four neurons per lane: two segments of 4096 columns
    (6144, 2, 7),      # two stages of 32 steps, the second narrower
    (16384, 2, 19),    # tiles of two rows, four segments
    (16384, 3, 1),     # ... a single row (ragged group of two)
    (18432, 2, 6),     # five stages, the last one narrower than the others
    (32768, 1, 5),     # eight stages
])
def test_wide_two_neurons_per_lane(N, L, batch):
    """Wide layers with a single weight value: four neurons per lane on two-row tiles where N
    allows it, else two output neurons per lane (compact slots, zero entry for unused steps,
    spill list).  One different weight sends the model to the one-neuron wide kernel."""
    import paper_2007_14152_amd as sp
    rng = np.random.default_rng(N + 3 * L)
    idx, val, bias = _uniform_model(rng, N, L, N)
    Y0 = (rng.uniform(0, 1, size=(batch, N)) < 0.3).astype(np.float32)
    ref = oracle.infer(idx, val, bias, Y0)
    m = sp.Model(idx, val, bias)
    want = (sp.SPDNN_KERNEL_ROW2 if N % 4096 == 0 and N <= 16384 else
            sp.SPDNN_KERNEL_WIDE_PAIR4 if N <= 16384 else sp.SPDNN_KERNEL_WIDE_PAIR)
    assert [m.layer_kernel(l) for l in range(L)] == [want] * L
    n, rows, Y = gpu_infer(idx, val, bias, Y0, model=m)
    m.close()
    common, _ = check_against_oracle(ref, n, rows, Y, what="wide pair N=%d" % N)
    assert common > 0
    val2 = [v.copy() for v in val]
    for v in val2:
        v[7, 0] = np.float32(0.0625 * (1.0 + 2.0 ** -20))
    ref2 = oracle.infer(idx, val2, bias, Y0)
    m2 = sp.Model(idx, val2, bias)
    assert [m2.layer_kernel(l) for l in range(L)] == [sp.SPDNN_KERNEL_WIDE if N > 8192 else sp.SPDNN_KERNEL_STAGED] * L
    n2, rows2, Y2 = gpu_infer(idx, val2, bias, Y0, model=m2)
    m2.close()
    check_against_oracle(ref2, n2, rows2, Y2, what="wide N=%d" % N)


@pytest.mark.parametrize("N", [10240, 12288])
def test_wide_two_neurons_per_lane_three_stages(N):
    """Three LDS stages (N = 10240: two neurons per lane, the fourth step of every row group is
    idle; N = 12288: three segments of a two-row tile): every neuron has 11, 11 and 10 connections
    in the three 4096-column stages, a few neurons 17 + 15 + 0 (one spilled in the staged format)."""
    import paper_2007_14152_amd as sp
    L, batch = 2, 11
    rng = np.random.default_rng(77)
    idx = []
    for _ in range(L):
        a = np.empty((N, 32), dtype=np.int64)
        for j in range(N):
            counts = (17, 15, 0) if j % 997 == 0 else (11, 11, 10)
            a[j] = np.concatenate([s0 * 4096 + rng.choice(min(4096, N - s0 * 4096), c, replace=False)
                                   for s0, c in enumerate(counts)])
        idx.append(np.sort(a, axis=1).astype(np.int32))
    val = [np.full((N, 32), 0.0625, dtype=np.float32) for _ in range(L)]
    bias = np.full(N, -0.05, dtype=np.float32)
    Y0 = (rng.uniform(0, 1, size=(batch, N)) < 0.3).astype(np.float32)
    ref = oracle.infer(idx, val, bias, Y0)
    m = sp.Model(idx, val, bias)
    want = sp.SPDNN_KERNEL_ROW2 if N % 4096 == 0 else sp.SPDNN_KERNEL_WIDE_PAIR4
    assert [m.layer_kernel(l) for l in range(L)] == [want] * L
    n, rows, Y = gpu_infer(idx, val, bias, Y0, model=m)
    m.close()
    common, _ = check_against_oracle(ref, n, rows, Y, what="wide pair, 3 stages")
    assert common > 0


def test_layers_with_fewer_stages_than_the_widest():
    """A model whose widest layer needs 10 stages (8 steps per stage in the wide format) and
    whose other layer needs 8 (16 steps per stage, more steps per neuron in total): the weight
    arena, sized for the widest window, must hold both."""
    import paper_2007_14152_amd as sp
    N, batch = 40960, 5
    rng = np.random.default_rng(11)
    i0, v0, bias = _uniform_model(rng, N, 1, N)
    i1 = [np.sort(np.stack([rng.choice(32768, 32, replace=False) for _ in range(N)]), axis=1).astype(np.int32)]
    v1 = [np.full((N, 32), 0.0625, dtype=np.float32)]
    idx, val = i0 + i1, v0 + v1
    for v in val:
        v[3, 3] = np.float32(0.0625 * (1.0 + 2.0 ** -20))   # two weight values: one neuron per lane
    Y0 = (rng.uniform(0, 1, size=(batch, N)) < 0.3).astype(np.float32)
    ref = oracle.infer(idx, val, bias, Y0)
    m = sp.Model(idx, val, bias)
    # (with 8 steps per stage a uniform pattern of this size may not fit the wide format: staged kernel then)
    assert m.layer_kernel(0) in (sp.SPDNN_KERNEL_WIDE, sp.SPDNN_KERNEL_STAGED)
    assert m.layer_kernel(1) == sp.SPDNN_KERNEL_WIDE
    n, rows, Y = gpu_infer(idx, val, bias, Y0, model=m)
    m.close()
    common, _ = check_against_oracle(ref, n, rows, Y, what="10 + 8 stages")
    assert common > 0


@pytest.mark.parametrize("cfg,layers,batch,density", [
    (0, 1, 200, "mixed"),      # a single layer: one buffer in use
    (0, 2, 200, "mixed"),
    (0, 12, 900, "mixed"),     # every layer runs; buffers are refilled five times each
    (0, 12, 300, None),        # the rows die after a few layers: copies still in flight when the loop stops
    (2, 5, 120, "mixed"),      # two neurons per lane
    (3, 3, 40, "mixed"),       # wide format (more arrays per layer block)
])
def test_out_of_core_weights_match_resident_weights(cfg, layers, batch, density):
    """Weights streamed from pinned host memory through two device buffers (Section III-B-1):
    same bits as with all weights resident, on repeated calls and against the oracle."""
    import torch
    import paper_2007_14152_amd as sp
    c, idx, val, bias = config_model(cfg, layers)
    Y0 = synth.gen_y0(batch, c["N"], c["seed"], density=density or synth.DENSITY)
    res = sp.Model(idx, val, bias)
    ooc = sp.Model(idx, val, bias, out_of_core=True)
    assert ooc.arena.numel() < res.arena.numel() or layers <= 2
    assert [ooc.layer_kernel(l) for l in range(layers)] == [res.layer_kernel(l) for l in range(layers)]
    y0 = torch.from_numpy(Y0).to("cuda:0")
    want = res.infer(y0)
    for rep in range(3):
        y = y0 if rep != 1 else y0[:batch // 2].contiguous()
        w = want if rep != 1 else res.infer(y)
        n, rows, Y = ooc.infer(y)
        assert n == w[0] and torch.equal(rows, w[1]) and torch.equal(Y, w[2]), "call %d" % rep
    ref = oracle.infer(idx, val, bias, Y0)
    check_against_oracle(ref, want[0], want[1].cpu().numpy(), want[2].cpu().numpy(), what="out of core cfg%d" % cfg)
    res.close()
    ooc.close()


def test_out_of_core_sizes_and_errors():
    import torch
    import paper_2007_14152_amd as sp
    c, idx, val, bias = config_model(0, 4)
    N = c["N"]
    dbytes, hbytes = sp.spdnn_ooc_bytes(N, 4, N)
    assert hbytes == 4 * (hbytes // 4) and dbytes < sp.spdnn_weights_bytes_for_window(N, 400, N)
    d400, h400 = sp.spdnn_ooc_bytes(N, 400, N)
    assert h400 == 100 * hbytes and d400 - dbytes < 400 * 64   # the device side grows by a few counters per layer only
    dev = torch.empty(dbytes, dtype=torch.uint8, device="cuda:0")
    host = torch.empty(hbytes, dtype=torch.uint8, pin_memory=True)
    ip = [a.ctypes.data for a in idx]
    vp = [a.ctypes.data for a in val]
    for db, hb in ((dbytes - 1, hbytes), (dbytes, hbytes - 1)):
        with pytest.raises(sp.SpdnnError) as e:
            sp.spdnn_create_ooc(N, 4, ip, vp, bias.ctypes.data, sp.SPDNN_HOST, dev.data_ptr(), db, host.data_ptr(), hb)
        assert e.value.code == sp.SPDNN_ESIZE
    with pytest.raises(sp.SpdnnError) as e:
        sp.spdnn_create_ooc(N, 4, ip, vp, bias.ctypes.data, sp.SPDNN_HOST, dev.data_ptr(), dbytes, 0, hbytes)
    assert e.value.code == sp.SPDNN_EINVAL


def test_batch_larger_than_one_compaction_chunk():
    """The compaction handles 65536 rows per chunk: batches beyond one and two chunks, with
    survivors and dropped rows in every chunk."""
    rng = np.random.default_rng(77)
    N, L, batch = 64, 4, 140001
    idx, val, bias = rand_model(rng, N, L, True, True, lo=0.0, hi=0.12)
    Y0 = (rng.uniform(size=(batch, N)) < rng.uniform(0.0, 0.5, size=(batch, 1))).astype(np.float32)
    ref = oracle.infer(idx, val, bias, Y0)
    assert 1000 < ref.n_active < batch - 1000
    assert (ref.active_rows < 65536).any() and (ref.active_rows >= 131072).any()
    n, rows, Y = gpu_infer(idx, val, bias, Y0)
    common, _ = check_against_oracle(ref, n, rows, Y, what="three compaction chunks")
    assert common > 1000


@pytest.mark.parametrize("N,batch,kernel", [
    (1024, 50001, "fused_layer_kernel<false>"),   # one neuron per lane, one column block, 250 row chunks
    (4096, 30001, "fused_pair_kernel"),           # two neurons per lane
    (8192, 12002, "fused_row2_kernel"),           # two-row tiles: slices of the list in pairs of rows
    (4100, 9999, None),                           # ragged last output block, window wider than one stage
])
def test_rows_die_in_every_layer_closed_form(N, batch, kernel):
    """The list of active rows is derived by every layer's own kernel from the flags of the layer before
    (Listing 1's pruning between two layers).  Row r holds the integer v_r in every column, every neuron
    averages 32 inputs and the bias is -1, so a layer turns v into v - 1, exactly: v_r > l rows are alive
    on entry to layer l, scattered over the whole batch, and the survivors hold v_r - L.  Checked against
    that closed form on all rows and layers, and against the oracle on a sample."""
    import torch
    import paper_2007_14152_amd as sp
    dev = "cuda:0"
    L, vmax = 8, 12
    rng = np.random.default_rng(N + batch)
    v = rng.integers(1, vmax + 1, size=batch)
    idx = [torch.from_numpy(np.sort(rng.integers(0, N, size=(N, 32)), axis=1).astype(np.int32)).to(dev) for _ in range(L)]
    val = torch.full((N, 32), 1.0 / 32, dtype=torch.float32, device=dev)
    bias = torch.full((N,), -1.0, dtype=torch.float32, device=dev)
    y0 = torch.from_numpy(v.astype(np.float32)).to(dev)[:, None].expand(batch, N).contiguous()
    m = sp.Model(idx, [val] * L, bias, device=dev)
    assert kernel is None or sp.KERNEL_NAMES[m.layer_kernel(0)] == kernel
    m.set_profiling(True)
    n, rows, Y = m.infer(y0)
    run, rows_in, _ = m.profile()
    assert run == L
    assert [int(x) for x in rows_in[:L]] == [int((v > l).sum()) for l in range(L)]
    alive = np.nonzero(v > L)[0]
    assert n == len(alive) and np.array_equal(rows.cpu().numpy(), alive)
    want = torch.from_numpy((v[alive] - L).astype(np.float32)).to(dev)
    assert bool((Y == want[:, None]).all())
    # the oracle on a sample, first and last rows included
    ids = np.unique(np.concatenate([[0, batch - 1], rng.choice(batch, 24, replace=False)]))
    ref = oracle.infer([i.cpu().numpy() for i in idx], [val.cpu().numpy()] * L, bias.cpu().numpy(),
                       np.repeat(v[ids].astype(np.float32)[:, None], N, axis=1))
    assert np.array_equal(ids[ref.active_rows], np.intersect1d(ids, alive))
    m.close()


@pytest.mark.parametrize("N,L", [(1024, 7), (96, 5)])
def test_all_layers_in_one_launch_equals_one_launch_per_layer(N, L):
    """Networks of at most 1024 neurons run all layers in one launch when a workgroup's share of the rows is
    small (Listing 1's loop over the layers inside the workgroup), one launch per layer otherwise.  The
    arithmetic per row is the same: the rows of a small batch must come out bit for bit as the same rows do
    inside a large batch, with the same rows alive on entry to every layer; and both agree with the oracle."""
    import torch
    import paper_2007_14152_amd as sp
    dev = "cuda:0"
    rng = np.random.default_rng(N + L)
    idx = [np.sort(rng.integers(0, N, size=(N, 32)), axis=1).astype(np.int32) for _ in range(L)]
    val = [rng.uniform(0.02, 0.11, size=(N, 32)).astype(np.float32) for _ in range(L)]
    bias = -rng.uniform(0.0, 0.4, size=N).astype(np.float32)
    big, small = 40000, 3001
    Y0 = synth.gen_y0(big, N, 17, density="mixed")
    m = sp.Model(idx, val, bias, device=dev)
    assert m.one_launch(small) and not m.one_launch(big) and m.one_launch(128 * 256) and not m.one_launch(128 * 256 + 4)
    m.set_profiling(True)
    y_big = torch.from_numpy(Y0).to(dev)
    nb, rb, Yb = m.infer(y_big)
    run_b, rows_b, _ = m.profile()
    ns, rs, Ys = m.infer(y_big[:small].contiguous())
    run_s, rows_s, ms_s = m.profile()
    rb_h, rs_h = rb.cpu().numpy(), rs.cpu().numpy()
    assert 0 < ns < small
    keep = rb_h < small
    assert np.array_equal(rb_h[keep], rs_h)
    assert torch.equal(Yb[torch.from_numpy(keep).to(dev)], Ys)
    ref = oracle.infer(idx, val, bias, Y0[:small])
    check_against_oracle(ref, ns, rs_h, Ys.cpu().numpy(), what="one launch N=%d" % N)
    # rows on entry to every layer, from the launch's own counters
    assert run_s == L and [int(x) for x in rows_s[:L]] == [int(x) for x in ref.active_per_layer[:L]]
    assert float(ms_s.sum()) > 0 and all(float(x) > 0 for x in ms_s[:L])
    # every row dies: "launched" ends one layer after the first without rows, as with one launch per layer
    zero = torch.zeros((500, N), dtype=torch.float32, device=dev)
    n0, _, _ = m.infer(zero)
    run0, rows0, _ = m.profile()
    assert n0 == 0 and run0 == 2 and [int(x) for x in rows0[:2]] == [500, 0]
    m.close()


@pytest.mark.parametrize("uniform", [True, False])
def test_largest_n_with_columns_anywhere(uniform):
    """N = 65536 (the largest the 16-bit column offsets allow) with columns drawn from the whole
    row: 16 LDS stages per output block."""
    import paper_2007_14152_amd as sp
    N, L, batch = 65536, 2, 9
    rng = np.random.default_rng(65536 + uniform)
    idx = [synth.gen_layer(N, l, 4242) for l in range(L)]
    val = [np.full((N, 32), 0.0625, np.float32) if uniform else rng.uniform(0.0, 0.12, size=(N, 32)).astype(np.float32)
           for _ in range(L)]
    bias = np.full(N, -0.3, dtype=np.float32)
    Y0 = (rng.uniform(size=(batch, N)) < np.linspace(0.1, 0.6, batch)[:, None]).astype(np.float32)
    ref = oracle.infer(idx, val, bias, Y0)
    assert 0 < ref.n_active
    m = sp.Model(idx, val, bias)
    assert m.widest_window == N
    n, rows, Y = gpu_infer(idx, val, bias, Y0, model=m)
    kinds = [m.layer_kernel(l) for l in range(L)]
    m.close()
    assert kinds == [sp.SPDNN_KERNEL_WIDE] * L
    common, _ = check_against_oracle(ref, n, rows, Y, what="N=65536 anywhere uniform=%s" % uniform)
    assert common > 0


def test_scattered_windows():
    """cfg-4-like windows whose members are scattered over the row by a permutation per layer:
    each block still reads 1024 different columns, but from everywhere, so the layers run as wide
    layers; results against the oracle."""
    import paper_2007_14152_amd as sp
    N, L, batch, w = 16384, 3, 40, 1024
    idx = [synth.scatter_columns(synth.gen_layer(N, l, 31, w), N, l, 31) for l in range(L)]
    val = [synth.gen_values(N) for _ in range(L)]
    bias = synth.gen_bias(N, -0.3)
    Y0 = synth.gen_y0(batch, N, 31, density="mixed")
    ref = oracle.infer(idx, val, bias, Y0)
    assert 0 < ref.n_active < batch
    m = sp.Model(idx, val, bias)
    assert m.widest_window > N - 512
    n, rows, Y = gpu_infer(idx, val, bias, Y0, model=m)
    m.close()
    common, _ = check_against_oracle(ref, n, rows, Y, what="scattered windows")
    assert common > 0


@pytest.mark.parametrize("N,w,batch", [(65536, 4096, 21), (32768, 2048, 9)])
def test_scattered_windows_gathered_footprint(N, w, batch):
    """The other reading of "permuted window": the members of every window are scattered over the whole
    row.  A unit of 4096 output neurons then touches at most 4096 groups of four columns, which the
    two-row-tile kernel stages as a gathered list (the preload list of Section III-A-2) instead of a
    contiguous window; results against the oracle."""
    import paper_2007_14152_amd as sp
    L = 2
    idx = [synth.scatter_columns(synth.gen_layer(N, l, 77, w), N, l, 77) for l in range(L)]
    val = [synth.gen_values(N) for _ in range(L)]
    bias = synth.gen_bias(N, -0.3)
    Y0 = synth.gen_y0(batch, N, 77, density="mixed")
    ref = oracle.infer(idx, val, bias, Y0)
    assert 0 < ref.n_active < batch
    m = sp.Model(idx, val, bias)
    assert m.widest_window > N - 256
    assert [m.layer_kernel(l) for l in range(L)] == [sp.SPDNN_KERNEL_ROW2] * L
    n, rows, Y = gpu_infer(idx, val, bias, Y0, model=m)
    m.close()
    common, _ = check_against_oracle(ref, n, rows, Y, what="scattered windows, gathered footprint")
    assert common > 0


@pytest.mark.parametrize("N,strides,uniform,kinds", [
    (1024, (1, 32), True, "SINGLE"),            # one block: the whole row is its window
    (8192, (1, 32), True, "PAIR"),              # the last unit's window runs over the row end
    (8192, (32, 1), False, "SINGLE"),           # the same with two weight values: one neuron per lane
    (8192, (160,), False, "STAGED"),            # two stages, cyclic
    (16384, (256, 1, 32), True, "PAIR PAIR PAIR"),  # stride 256: two neurons per lane under new names for neurons and columns
    (16384, (256,), False, "WIDE"),             # three stages, one neuron per lane
    (10240, (256,), True, "WIDE_PAIR4"),        # three stages, two neurons per lane, step lists in registers
    (32768, (700,), True, "WIDE_PAIR"),         # six stages, two neurons per lane
    (65536, (1500,), False, "WIDE"),            # twelve stages of eight steps
    (65536, (1024, 2048, 32), True, "PAIR PAIR PAIR"),  # units of 64 segments of 32 and 32 segments of 64 neurons, renamed
    (16384, (512,), True, "PAIR"),              # 8 units of 32 segments of 64 neurons
    (12288, (384,), True, "PAIR"),              # six units, segments every 384 neurons
    (65536, (-1024,), True, "ROW2"),            # (see below) neighbouring units share columns: no renaming; units of
                                                # interleaved segments on two-row tiles
])
def test_strided_layers_wrap_around_the_row_end(N, strides, uniform, kinds):
    """Strided, modular patterns (neuron j reads (j + k*S) mod N): the footprint of the last blocks runs
    over the row end, so their windows are narrow only as arcs of the circle of columns.  Every kernel
    family with such cyclic windows, against the oracle."""
    import paper_2007_14152_amd as sp
    rng = np.random.default_rng(N + len(strides))
    L, batch = len(strides), 11
    def layer(s_):
        if s_ > 0:
            return synth.gen_layer_strided(N, s_)
        # stride -s_, every other connection 32 columns further on: the columns of neighbouring 32-residue classes overlap
        j = np.arange(N, dtype=np.int64)[:, None]
        k = np.arange(32, dtype=np.int64)[None, :]
        return np.sort((j + k * (-s_) + (k & 1) * 32) % N, axis=1).astype(np.int32)
    idx = [layer(s_) for s_ in strides]
    if uniform:
        val = [synth.gen_values(N) for _ in range(L)]
    else:
        val = [rng.uniform(0.03, 0.1, size=(N, 32)).astype(np.float32) for _ in range(L)]
    bias = synth.gen_bias(N, -0.3)
    Y0 = synth.gen_y0(batch, N, 5, density="mixed")
    ref = oracle.infer(idx, val, bias, Y0)
    assert 0 < ref.n_active <= batch
    m = sp.Model(idx, val, bias)
    want = [getattr(sp, "SPDNN_KERNEL_" + k) for k in kinds.split()]
    assert [m.layer_kernel(l) for l in range(L)] == (want if len(want) == L else want * L)
    n, rows, Y = gpu_infer(idx, val, bias, Y0, model=m)
    m.close()
    common, _ = check_against_oracle(ref, n, rows, Y, what="strided N=%d %s" % (N, strides))
    assert common > 0


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_seeded_sweep_over_layer_shapes(seed):
    """Drawn combinations of N, depth, batch, one weight or many, and strides: whatever kernel and launch mode
    the library picks for them (one launch for all layers, one to four neurons per lane, units of interleaved
    segments, wide windows), the result is the oracle's."""
    import paper_2007_14152_amd as sp
    seen = set()
    for case in range(16):
        rng = np.random.default_rng(seed * 100003 + case)
        if case % 2 == 0:
            N = int(rng.choice([32, 64, 100, 512, 1024, 1028, 2048, 4096]))
            L = int(rng.integers(1, 5))
            batch = int(rng.choice([1, 3, 7, 129, 1000, 5000, 40000 if N <= 1024 else 300]))
            idx = [np.sort(rng.integers(0, N, size=(N, 32)), axis=1).astype(np.int32) for _ in range(L)]
            uni = rng.uniform() < 0.4
            val = [np.full((N, 32), 0.0625, np.float32) if uni else rng.uniform(0.02, 0.11, size=(N, 32)).astype(np.float32)
                   for _ in range(L)]
            bias = -rng.uniform(0.0, 0.4, size=N).astype(np.float32)
        else:
            N = int(rng.choice([4096, 8192, 12288, 16384, 32768]))
            L = int(rng.integers(1, 4))
            batch = int(rng.choice([2, 9, 31]))
            idx = [synth.gen_layer_strided(N, int(rng.choice([1, 4, 32, N // 64, N // 32, N // 16, 1000]))) for _ in range(L)]
            val = [synth.gen_values(N) for _ in range(L)]
            bias = synth.gen_bias(N, -0.3)
        Y0 = synth.gen_y0(batch, N, case, density="mixed")
        ref = oracle.infer(idx, val, bias, Y0)
        m = sp.Model(idx, val, bias)
        what = "sweep %d/%d N=%d L=%d batch=%d one launch=%s kernels=%s" % (
            seed, case, N, L, batch, m.one_launch(batch), [sp.KERNEL_NAMES[m.layer_kernel(l)] for l in range(L)])
        seen.add("one launch" if m.one_launch(batch) else sp.KERNEL_NAMES[m.layer_kernel(0)])
        n, rows, Y = gpu_infer(idx, val, bias, Y0, model=m)
        m.close()
        check_against_oracle(ref, n, rows, Y, what=what)
    assert len(seen) >= 3, seen


@pytest.mark.parametrize("rows_per_batch", [1000, 257, 64, 5000])
def test_inputs_in_host_memory_in_serial_batches(rows_per_batch):
    """Section III-B-2: the inputs stay on the host and go through the GPU batch by batch
    (spdnn_infer_host), the copy of the next batch under the kernels of the current one.  Checked
    against the oracle's result for the whole input; also identical to one spdnn_infer call."""
    import torch
    import paper_2007_14152_amd as sp
    c, idx, val, bias = config_model(0, 6)
    batch = 1000
    Y0 = synth.gen_y0(batch, c["N"], c["seed"], density="mixed")
    ref = oracle.infer(idx, val, bias, Y0)
    assert 0 < ref.n_active < batch
    m = sp.Model(idx, val, bias)
    host = torch.from_numpy(Y0).pin_memory()
    for rep in range(2):
        n, rows, Y = m.infer_batched(host, rows_per_batch)
        common, _ = check_against_oracle(ref, n, rows.cpu().numpy(), Y.cpu().numpy(),
                                         what="host batches of %d" % rows_per_batch, max_fragile_frac=MAX_FRAGILE_FRAC)
        assert common > 0
    want = m.infer(torch.from_numpy(Y0).to("cuda:0"))
    assert n == want[0] and torch.equal(rows, want[1]) and torch.equal(Y, want[2])
    # pageable host memory works too (the copies then do not overlap the kernels)
    n2, rows2, Y2 = m.infer_batched(torch.from_numpy(Y0), rows_per_batch)
    assert n2 == n and torch.equal(rows2, rows) and torch.equal(Y2, Y)
    n, rows, Y = m.infer_batched(host[:0].contiguous(), rows_per_batch)
    assert n == 0 and rows.numel() == 0
    with pytest.raises(sp.SpdnnError) as e:   # work arena one byte short
        need = sp.spdnn_host_work_bytes(c["N"], 64)
        work = torch.empty(need, dtype=torch.uint8, device="cuda:0")
        out = torch.empty(batch, dtype=torch.int32, device="cuda:0")
        sp.spdnn_infer_host(m.h, host.data_ptr(), batch, 64, work.data_ptr(), need - 1, out.data_ptr(), 0)
    assert e.value.code == sp.SPDNN_ESIZE
    m.close()
