"""GPU parity for general sparse layers (any number of connections per neuron,
spdnn_create_csr): the HIP path, called through the C-ABI binding, against the CPU
oracle's general form on the same seeded inputs.  Same bar as the fixed-32 tests
(parity_util): active rows bit-exact except fragile ones, Y within 1e-5 relative or
1e-6 absolute."""
import numpy as np
import pytest

import oracle
import synth
from parity_util import check_against_oracle

pytestmark = pytest.mark.gpu


def lanes_per_neuron(ptr):
    """Parts of 32 connections of the layer's longest neuron, rounded up to a power of two."""
    parts = max(1, -(-int(np.diff(ptr).max()) // 32))
    return 1 << (parts - 1).bit_length()


def rand_general(rng, N, L, kmin, kmax, lo=0.0, hi=0.12, empty_frac=0.05, width=None):
    """Random general layers; width = columns of neuron j lie in a window of that many
    columns around j (None: anywhere)."""
    ptr, idx, val = [], [], []
    for _ in range(L):
        deg = rng.integers(kmin, kmax + 1, size=N)
        deg[rng.uniform(size=N) < empty_frac] = 0
        p = np.zeros(N + 1, dtype=np.int32)
        np.cumsum(deg, out=p[1:])
        nnz = int(p[N])
        if width is None:
            a = rng.integers(0, N, size=nnz)
        else:
            owner = np.repeat(np.arange(N), deg)
            a = np.clip(owner + rng.integers(-width // 2, width // 2, size=nnz), 0, N - 1)
        ptr.append(p)
        idx.append(a.astype(np.int32))
        val.append(rng.uniform(lo, hi, size=nnz).astype(np.float32))
    bias = -rng.uniform(0.0, 0.3, size=N).astype(np.float32)
    return ptr, idx, val, bias


def gpu_infer_general(ptr, idx, val, bias, Y0, model=None):
    import torch
    import paper_2007_14152_amd as sp
    own = model is None
    if own:
        model = sp.Model.from_csr(ptr, idx, val, bias)
    y0 = torch.from_numpy(np.ascontiguousarray(Y0, dtype=np.float32)).to("cuda:0")
    n, rows, Y = model.infer(y0)
    out = (n, rows.cpu().numpy().copy(), Y.cpu().numpy().copy())
    if own:
        model.close()
    return out


@pytest.mark.parametrize("N,L,batch,kmax", [
    (32, 3, 5, 32),       # smallest N, ragged row group
    (64, 2, 9, 7),        # short neurons only
    (1028, 3, 70, 32),    # second output block has 4 neurons
    (5000, 2, 11, 20),    # window wider than one LDS stage
])
def test_short_neurons_one_pass(N, L, batch, kmax):
    """At most 32 connections per neuron: one pass per layer, padded with zero weights."""
    import paper_2007_14152_amd as sp
    rng = np.random.default_rng(N * 7 + kmax)
    ptr, idx, val, bias = rand_general(rng, N, L, 0, kmax, hi=0.25)
    Y0 = rng.uniform(0, 1, size=(batch, N)).astype(np.float32)
    Y0[batch // 2] = 0
    ref = oracle.infer(idx, val, bias, Y0, ptr=ptr)
    m = sp.Model.from_csr(ptr, idx, val, bias)
    assert [m.layer_passes(l) for l in range(L)] == [1] * L
    n, rows, Y = gpu_infer_general(ptr, idx, val, bias, Y0, model=m)
    m.close()
    common, _ = check_against_oracle(ref, n, rows, Y, what="general short N=%d" % N)
    assert common > 0


@pytest.mark.parametrize("N,L,batch,kmax,width", [
    (96, 3, 37, 70, None),      # up to 3 parts of 32: 4 lanes per neuron
    (2052, 3, 33, 100, None),   # 4 lanes per neuron, 256 neurons per workgroup: 9 of them, the last launch all empty
    (5000, 2, 9, 64, None),     # two LDS stages, exactly 2 lanes per neuron
    (9000, 2, 10, 45, 1500),    # narrow windows, one stage
    (20000, 2, 6, 40, None),    # 5 stages: the staged kernel walks them
    (1024, 2, 19, 300, None),   # 16 lanes per neuron, 64 neurons per workgroup
    (64, 2, 11, 2100, None),    # 128 lanes per neuron: 8 neurons per workgroup, finishing lanes fill an eighth of a wave
])
def test_long_neurons_several_passes(N, L, batch, kmax, width):
    """More than 32 connections: a neuron is spread over P = 2^ceil(log2(ceil(K/32))) lanes, whose sums meet in LDS;
    the layer runs as P launches, each computing a slice of the neurons (reported as passes)."""
    import paper_2007_14152_amd as sp
    rng = np.random.default_rng(N * 3 + kmax)
    ptr, idx, val, bias = rand_general(rng, N, L, 0, kmax, hi=4.0 / kmax, width=width)
    Y0 = rng.uniform(0, 1, size=(batch, N)).astype(np.float32)
    Y0[1] = 0
    ref = oracle.infer(idx, val, bias, Y0, ptr=ptr)
    m = sp.Model.from_csr(ptr, idx, val, bias)
    want = [lanes_per_neuron(p) for p in ptr]
    assert [m.layer_passes(l) for l in range(L)] == want and max(want) > 1
    assert m.layer_kernel(0) in (sp.SPDNN_KERNEL_SINGLE, sp.SPDNN_KERNEL_STAGED)
    if width:   # the arena was sized for the patterns' window, not for the worst case
        assert m.widest_window <= 1024 + width + 8
        assert m.arena.numel() < sp.spdnn_weights_bytes(N, sum(want))
    else:
        assert m.widest_window >= N - 64
    n, rows, Y = gpu_infer_general(ptr, idx, val, bias, Y0, model=m)
    m.close()
    common, _ = check_against_oracle(ref, n, rows, Y, what="general long N=%d" % N)
    assert common > 0


def test_layers_of_different_kinds_in_one_model():
    """Short, long and exactly-32 uniform layers in one model: the exactly-32 layer with one
    weight value still gets the two-neurons-per-lane kernel."""
    import paper_2007_14152_amd as sp
    N, batch = 2048, 50
    rng = np.random.default_rng(5)
    p0, i0, v0, bias = rand_general(rng, N, 1, 0, 20, hi=0.3)
    p1, i1, v1, _ = rand_general(rng, N, 1, 10, 70, hi=0.08)
    fixed = synth.gen_layer(N, 2, 77)
    p2 = [np.arange(0, 32 * N + 1, 32, dtype=np.int32)]
    i2 = [fixed.reshape(-1)]
    v2 = [np.full(32 * N, 0.0625, dtype=np.float32)]
    ptr, idx, val = p0 + p1 + p2, i0 + i1 + i2, v0 + v1 + v2
    Y0 = rng.uniform(0, 1, size=(batch, N)).astype(np.float32)
    ref = oracle.infer(idx, val, bias, Y0, ptr=ptr)
    m = sp.Model.from_csr(ptr, idx, val, bias)
    assert [m.layer_passes(l) for l in range(3)] == [1, 4, 1]
    assert m.layer_kernel(2) == sp.SPDNN_KERNEL_PAIR
    n, rows, Y = gpu_infer_general(ptr, idx, val, bias, Y0, model=m)
    m.close()
    common, _ = check_against_oracle(ref, n, rows, Y, what="mixed kinds")
    assert common > 0


def test_exactly_32_equals_the_fixed_entry_point():
    """The same model through spdnn_create and spdnn_create_csr: identical bits."""
    import torch
    import paper_2007_14152_amd as sp
    c = synth.config(0)
    N, L = c["N"], 5
    idx = [synth.gen_layer(N, l, c["seed"]) for l in range(L)]
    val = [synth.gen_values(N) for _ in range(L)]
    bias = synth.gen_bias(N, c["bias"])
    Y0 = synth.gen_y0(600, N, c["seed"], density="mixed")
    y0 = torch.from_numpy(Y0).to("cuda:0")
    a = sp.Model(idx, val, bias)
    na, ra, Ya = a.infer(y0)
    ptr = [np.arange(0, 32 * N + 1, 32, dtype=np.int32)] * L
    g = sp.Model.from_csr(ptr, [i.reshape(-1) for i in idx], [v.reshape(-1) for v in val], bias)
    ng, rg, Yg = g.infer(y0)
    assert na == ng and 0 < na < 600
    assert torch.equal(ra, rg) and torch.equal(Ya, Yg)
    a.close()
    g.close()


@pytest.mark.parametrize("N,batch,layers,kmin,kmax", [(4096, 300, 10, 8, 72), (1024, 1000, 8, 0, 40)])
def test_generated_general_layers_sustained(N, batch, layers, kmin, kmax):
    """Seeded general layers (neuron lengths kmin..kmax, weight sums about 2) with binary
    inputs of mixed row density: part of the rows die, the rest saturate at the clip."""
    import paper_2007_14152_amd as sp
    seed = 20200799
    gen = [synth.gen_layer_general(N, l, seed, kmin, kmax) for l in range(layers)]
    ptr, idx, val = [g[0] for g in gen], [g[1] for g in gen], [g[2] for g in gen]
    bias = synth.gen_bias(N, -0.3)
    Y0 = synth.gen_y0(batch, N, seed, density="mixed")
    ref = oracle.infer(idx, val, bias, Y0, ptr=ptr)
    assert 0 < ref.n_active < batch
    n, rows, Y = gpu_infer_general(ptr, idx, val, bias, Y0)
    check_against_oracle(ref, n, rows, Y, what="generated general N=%d" % N)
    assert Y.max() == 32.0


@pytest.mark.parametrize("kmin,kmax,packed", [(0, 100, True), (33, 64, False)])
def test_long_neurons_with_windows_stay_in_one_stage(kmin, kmax, packed):
    """Neurons of blocks of 2048 draw their columns from windows of 2048 columns that lie anywhere in the row
    (the locality of cfg 4).  The workgroups of a layer with several lanes per neuron are runs of neighbouring
    neurons; whether they are packed by what their neurons need (0..100 connections) or all alike (33..64), none
    may reach over a window boundary, or its tile would no longer fit one LDS stage."""
    import paper_2007_14152_amd as sp
    N, batch, window, seed = 16384, 9, 2048, 31
    gen = [synth.gen_layer_general(N, l, seed, kmin, kmax, window) for l in range(2)]
    ptr, idx, val = [g[0] for g in gen], [g[1] for g in gen], [g[2] for g in gen]
    bias = synth.gen_bias(N, -0.3)
    Y0 = synth.gen_y0(batch, N, seed, density="mixed")
    ref = oracle.infer(idx, val, bias, Y0, ptr=ptr)
    m = sp.Model.from_csr(ptr, idx, val, bias)
    assert [m.layer_passes(l) for l in range(2)] == [lanes_per_neuron(p) for p in ptr]
    assert [m.layer_kernel(l) for l in range(2)] == [sp.SPDNN_KERNEL_SINGLE] * 2
    assert m.widest_window <= window
    # what the set-up decides by: workgroups packed by parts against 1024 / P neurons each
    parts = [-(-np.diff(p) // 32) for p in ptr]
    assert all((pp.sum() / 1024 * 4 <= 3 * (N // (1024 // lanes_per_neuron(p)))) == packed for pp, p in zip(parts, ptr))
    n, rows, Y = gpu_infer_general(ptr, idx, val, bias, Y0, model=m)
    m.close()
    common, _ = check_against_oracle(ref, n, rows, Y, what="windows, %d..%d connections" % (kmin, kmax))
    assert common > 0


def test_mixed_sign_weights_long_neurons():
    """Weights of both signs over up to 90 connections: held to the float bound for any
    summation order, (K + 2) * eps * sum|y*w|, against the oracle in double."""
    rng = np.random.default_rng(21)
    N, batch, kmax = 1028, 17, 90
    ptr, idx, val, bias = rand_general(rng, N, 1, 0, kmax, lo=-0.1, hi=0.2)
    Y0 = rng.uniform(0, 4, size=(batch, N)).astype(np.float32)
    ref = oracle.infer(idx, val, bias, Y0.astype(np.float64), f64=True, no_skip=True, ptr=ptr)
    exact = np.zeros((batch, N))
    exact[ref.active_rows] = ref.Y
    owner = np.repeat(np.arange(N), np.diff(ptr[0]))
    mag = np.zeros((batch, N))
    np.add.at(mag.T, owner, np.abs(Y0[:, idx[0]].astype(np.float64) * val[0].astype(np.float64)).T)
    mag += np.abs(bias.astype(np.float64))[None, :]
    n, rows, Y = gpu_infer_general(ptr, idx, val, bias, Y0)
    got = np.zeros((batch, N))
    got[rows] = Y
    eps = float(np.finfo(np.float32).eps)
    assert np.all(np.abs(got - exact) <= (kmax + 2) * eps * mag + 1e-30)
    sure = np.nonzero((exact > 1e-3).any(1))[0]
    assert set(sure.tolist()) <= set(rows.tolist())


def test_general_errors_and_edges():
    import torch
    import paper_2007_14152_amd as sp
    rng = np.random.default_rng(3)
    N = 256
    ptr, idx, val, bias = rand_general(rng, N, 2, 0, 50)
    # ptr that decreases
    bad = [p.copy() for p in ptr]
    bad[1][10] = bad[1][9] - 1
    with pytest.raises(sp.SpdnnError) as e:
        sp.Model.from_csr(bad, idx, val, bias)
    assert e.value.code == sp.SPDNN_EINVAL
    # column outside [0, N)
    badi = [a.copy() for a in idx]
    badi[0][3] = N
    with pytest.raises(sp.SpdnnError) as e:
        sp.Model.from_csr(ptr, badi, val, bias)
    assert e.value.code == sp.SPDNN_EINVAL
    # positive bias
    with pytest.raises(sp.SpdnnError) as e:
        sp.Model.from_csr(ptr, idx, val, np.full(N, 0.1, dtype=np.float32))
    assert e.value.code == sp.SPDNN_EBIAS
    # arena one byte short of what the passes need
    dev = "cuda:0"
    tp = [torch.from_numpy(p).to(dev) for p in ptr]
    ti = [torch.from_numpy(a).to(dev) for a in idx]
    tv = [torch.from_numpy(v).to(dev) for v in val]
    tb = torch.from_numpy(bias).to(dev)
    scratch = torch.empty(4096, dtype=torch.uint8, device=dev)
    passes, total, widest = sp.spdnn_csr_passes(N, 2, [p.data_ptr() for p in tp], scratch.data_ptr(), scratch.numel(),
                                                torch.cuda.current_stream().cuda_stream,
                                                idx_ptrs=[a.data_ptr() for a in ti])
    assert widest == N   # columns anywhere: every block spans the whole row
    assert passes.tolist() == [lanes_per_neuron(p) for p in ptr] and total == int(passes.sum())
    need = sp.spdnn_weights_bytes_for_window(N, total, 4)
    arena = torch.empty(need, dtype=torch.uint8, device=dev)
    with pytest.raises(sp.SpdnnError) as e:
        sp.spdnn_create_csr(N, 2, [p.data_ptr() for p in tp], [a.data_ptr() for a in ti], [v.data_ptr() for v in tv],
                            tb.data_ptr(), arena.data_ptr(), need - 1, torch.cuda.current_stream().cuda_stream)
    assert e.value.code == sp.SPDNN_ESIZE
    # a layer with no connections at all: every output is the clipped bias, all rows die
    empty = [np.zeros(N + 1, dtype=np.int32)]
    n, rows, Y = gpu_infer_general(empty, [np.zeros(0, dtype=np.int32)], [np.zeros(0, dtype=np.float32)], bias,
                                   np.ones((5, N), dtype=np.float32))
    assert n == 0
    # batch of one row
    one = np.ones((1, N), dtype=np.float32)
    ref = oracle.infer(idx, val, bias, one, ptr=ptr)
    n, rows, Y = gpu_infer_general(ptr, idx, val, bias, one)
    check_against_oracle(ref, n, rows, Y, what="general one row")


def _sweep_case(seed):
    """One seeded case of the sweep below: shapes, pattern kind, weights and neuron lengths all drawn."""
    rng = np.random.default_rng(9000 + seed)
    N = int(rng.choice([32, 36, 100, 512, 1024, 1028, 2048, 3000, 4096, 6148, 8192]))
    L = int(rng.integers(1, 4))
    batch = int(rng.integers(1, 98))
    kind = ["fixed", "short", "long"][seed % 3]
    width = [None, 64, 1024][int(rng.integers(0, 3))]
    uniform = bool(rng.integers(0, 2))
    kmax = {"fixed": 32, "short": int(rng.integers(1, 33)), "long": int(rng.integers(33, 90))}[kind]
    ptr, idx, val = [], [], []
    for _ in range(L):
        deg = np.full(N, 32) if kind == "fixed" else rng.integers(0, kmax + 1, size=N)
        p = np.zeros(N + 1, dtype=np.int32)
        np.cumsum(deg, out=p[1:])
        nnz = int(p[N])
        owner = np.repeat(np.arange(N), deg)
        if width is None or width >= N:
            a = rng.integers(0, N, size=nnz)
        else:
            a = np.clip((owner // width) * width + rng.integers(0, width, size=nnz), 0, N - 1)
        v = np.full(nnz, 0.0625, np.float32) if uniform else rng.uniform(0.0, 4.0 / max(kmax, 1), size=nnz).astype(np.float32)
        ptr.append(p)
        idx.append(a.astype(np.int32))
        val.append(v)
    bias = -rng.uniform(0.0, 0.3, size=N).astype(np.float32)
    Y0 = (rng.uniform(size=(batch, N)) < rng.uniform(0.05, 0.7, size=(batch, 1))).astype(np.float32)
    return dict(N=N, L=L, batch=batch, kind=kind, width=width, uniform=uniform, kmax=kmax), ptr, idx, val, bias, Y0


@pytest.mark.parametrize("seed", range(30))
def test_seeded_sweep_of_shapes_patterns_and_lengths(seed):
    """Thirty drawn combinations of N (ragged blocks, one to eight blocks), depth, batch, window width,
    one weight or many, and neuron lengths (exactly 32 through spdnn_create, 0..32 and 33..89 through
    spdnn_create_csr): each against the oracle."""
    import paper_2007_14152_amd as sp
    from parity_util import gpu_infer
    what, ptr, idx, val, bias, Y0 = _sweep_case(seed)
    ref = oracle.infer(idx, val, bias, Y0, ptr=ptr)
    if what["kind"] == "fixed":
        N = what["N"]
        n, rows, Y = gpu_infer([a.reshape(N, 32) for a in idx], [v.reshape(N, 32) for v in val], bias, Y0)
    else:
        n, rows, Y = gpu_infer_general(ptr, idx, val, bias, Y0)
    check_against_oracle(ref, n, rows, Y, what=str(what))
