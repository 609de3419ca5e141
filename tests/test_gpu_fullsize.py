"""Parity at the benchmark's full sizes (60 000 rows, the launch configuration the
benchmark times): the library runs the whole batch on the GPU; the oracle
evaluates a seeded sample of rows (rows are independent, Eq. 1), and the sample
is compared one by one.  Whole-output properties are checked on the GPU result
with torch reductions."""
import numpy as np
import pytest

import oracle
import synth
from parity_util import MAX_FRAGILE_FRAC, check_against_oracle, config_model, launch_row_chunk_bounds

pytestmark = pytest.mark.gpu


def sample_rows(model, batch, sample, seed):
    """Seeded sample of rows, always with the first and the last row and the four rows on each side of
    every row-chunk boundary of the launch."""
    rng = np.random.default_rng(seed)
    ids = set(rng.choice(batch, min(sample, batch), replace=False).tolist()) | {0, batch - 1}
    for b in launch_row_chunk_bounds(model, batch):
        ids |= set(range(max(0, b - 4), min(batch, b + 4)))
    return np.array(sorted(ids))


def compare_sample(ref, ids, n, rows_h, Y, N, dev, what):
    """The library's output restricted to the sampled rows against the oracle's result for them."""
    import torch
    pos = np.searchsorted(rows_h, ids)
    pos_c = np.minimum(pos, max(n - 1, 0))
    present = (rows_h[pos_c] == ids) if n else np.zeros(len(ids), bool)
    sub_rows = ids[present]
    sub_Y = Y[torch.from_numpy(pos_c[present]).to(dev)].cpu().numpy() if present.any() else np.zeros((0, N), np.float32)
    return check_against_oracle(ref, len(sub_rows), sub_rows, sub_Y, row_ids=ids, what=what, max_fragile_frac=MAX_FRAGILE_FRAC)


# cfg 1: every one of the 60 000 rows goes through the oracle
@pytest.mark.parametrize("cfg,layers,sample", [(1, 1, 60000), (1, 2, 60000), (1, 3, 60000), (2, 1, 2048), (2, 2, 2048),
                                              (3, 1, 512), (3, 2, 512), (4, 1, 512), (4, 2, 512)])
def test_full_batch_sampled_rows(cfg, layers, sample):
    import torch
    import paper_2007_14152_amd as sp
    dev = "cuda:0"
    c, didx, dval, dbias = config_model(cfg, layers, device=dev)
    N, batch = c["N"], c["batch"]
    print("cfg", cfg, "layers", layers, "N", N, "batch", batch, flush=True)
    m = sp.Model(didx, dval, dbias, device=dev)
    y0 = synth.gen_y0(batch, N, c["seed"], device=dev)
    n, rows, Y = m.infer(y0)
    del y0
    rows_h = rows.cpu().numpy()
    # whole-output properties
    assert n == rows_h.shape[0] and np.all(np.diff(rows_h) > 0)
    assert rows_h.size == 0 or (rows_h[0] >= 0 and rows_h[-1] < batch)
    if n:
        mx = torch.stack([Y[s:s + 4096].max(dim=1).values.min() for s in range(0, n, 4096)]).min()
        assert float(mx) > 0.0, "every listed row has a positive element"
        assert float(Y.min()) >= 0.0 and float(Y.max()) <= 32.0
    # sampled rows against the oracle, one by one
    ids = sample_rows(m, batch, sample, 100 + cfg)
    assert len(ids) >= sample
    idx = [a.cpu().numpy() for a in didx]
    val = [a.cpu().numpy() for a in dval]
    ref = oracle.infer(idx, val, dbias.cpu().numpy(), synth.gen_y0(batch, N, c["seed"], rows=ids))
    common, _ = compare_sample(ref, ids, n, rows_h, Y, N, dev, "cfg%d L=%d sampled" % (cfg, layers))
    if layers == 1:
        assert n == batch and common == len(ids)
    if ref.n_active == 0 and len(ids) == batch:
        assert n == 0
    if cfg >= 2 and layers == 2:   # these configurations are dead after two layers: oracle sample and whole GPU batch
        assert ref.n_active == 0 and n == 0
    m.close()


def test_full_depth_model_of_the_benchmark():
    """The model the benchmark times: cfg 4 with all 1920 layers, the whole batch, the launch sequence
    of spdnn_infer with its early stop.  Per-layer row counts come from the library's profile; the
    oracle follows a row sample through as many layers as any sampled row reaches."""
    import torch
    import paper_2007_14152_amd as sp
    dev = "cuda:0"
    c = synth.config(4)
    N, L, batch = c["N"], c["L"], c["batch"]
    print("full-depth cfg 4: generating", L, "layers", flush=True)
    didx = torch.empty((L, N, 32), dtype=torch.int32, device=dev)
    for l in range(L):
        didx[l] = synth.gen_layer(N, l, c["seed"], c["window"], device=dev)
    dval1 = synth.gen_values(N, device=dev)       # every layer has the same weights: one array serves all
    dbias = synth.gen_bias(N, c["bias"], device=dev)
    print("full-depth cfg 4: set-up", flush=True)
    m = sp.Model([didx[l] for l in range(L)], [dval1] * L, dbias, device=dev)
    assert m.L == L and all(m.layer_kernel(l) == sp.SPDNN_KERNEL_PAIR for l in (0, 1, L // 2, L - 1))
    y0 = synth.gen_y0(batch, N, c["seed"], device=dev)
    m.set_profiling(True)
    print("full-depth cfg 4: inference", flush=True)
    n, rows, Y = m.infer(y0)
    run, rows_in, ms = m.profile()
    del y0
    ids = sample_rows(m, batch, 256, 104)
    reach = 4                                    # layers the oracle is given; it fails loudly if a row gets further
    idx = [didx[l].cpu().numpy() if l < reach else None for l in range(L)]
    val = [dval1.cpu().numpy() if l < reach else None for l in range(L)]
    ref = oracle.infer(idx, val, dbias.cpu().numpy(), synth.gen_y0(batch, N, c["seed"], rows=ids))
    assert ref.n_active == 0 and n == 0 and rows.numel() == 0
    # rows on entry to every launched layer: all of them twice (every row has a positive output after
    # layer 0), then none; the library stops a bounded number of layers after the first empty count
    assert rows_in[0] == batch and rows_in[1] == batch
    assert np.all(np.diff(rows_in) <= 0) and rows_in[-1] == 0
    first_empty = int(np.argmax(rows_in == 0))
    assert ref.active_per_layer[first_empty] == 0, "the sample dies no later than the whole batch"
    assert ref.active_per_layer[1] == len(ids)
    assert run < 16 and run - first_empty <= 8
    m.close()


@pytest.mark.parametrize("cfg,batch,follow", [(4, 2048, 8), (2, 6000, 40)])
def test_sustained_activity_at_full_depth(cfg, batch, follow):
    """The regime of Table I: rows that stay active through all L layers (Section IV-B).  Mixed row
    densities, every layer of the configuration's shape; the oracle follows `follow` rows through all
    layers: those that die must be dropped, the survivors must be listed with Y_L at the clip."""
    import torch
    import paper_2007_14152_amd as sp
    dev = "cuda:0"
    c = synth.config(cfg)
    N, L = c["N"], c["L"]
    print("sustained full depth cfg", cfg, "L", L, "batch", batch, flush=True)
    didx = torch.empty((L, N, 32), dtype=torch.int32, device=dev)
    for l in range(L):
        didx[l] = synth.gen_layer(N, l, c["seed"], c["window"], device=dev)
    dval1 = synth.gen_values(N, device=dev)
    dbias = synth.gen_bias(N, c["bias"], device=dev)
    m = sp.Model([didx[l] for l in range(L)], [dval1] * L, dbias, device=dev)
    y0 = synth.gen_y0(batch, N, c["seed"], density="mixed", device=dev)
    m.set_profiling(True)
    n, rows, Y = m.infer(y0)
    run, rows_in, ms = m.profile()
    rows_h = rows.cpu().numpy()
    assert run == L and 0 < n < batch
    assert rows_in[0] == batch and np.all(np.diff(rows_in) <= 0) and rows_in[-1] >= n
    assert float(Y.min()) >= 0.0 and float(Y.max()) == 32.0
    # rows to follow: half of them survivors of the GPU run, half not, plus the first and the last row
    rng = np.random.default_rng(500 + cfg)
    alive = rng.choice(rows_h, follow // 2, replace=False)
    dead = rng.choice(np.setdiff1d(np.arange(batch), rows_h), follow - follow // 2, replace=False)
    ids = np.array(sorted(set(alive.tolist()) | set(dead.tolist()) | {0, batch - 1}))
    print("oracle follows", len(ids), "rows through", L, "layers", flush=True)
    idx_h = didx.cpu().numpy()
    val_h = dval1.cpu().numpy()
    ref = oracle.infer([idx_h[l] for l in range(L)], [val_h] * L, dbias.cpu().numpy(),
                       synth.gen_y0(batch, N, c["seed"], density="mixed", rows=ids))
    assert ref.layers_evaluated == L and 0 < ref.n_active < len(ids)
    common, _ = compare_sample(ref, ids, n, rows_h, Y, N, dev, "sustained cfg%d full depth" % cfg)
    assert common == ref.n_active
    assert ref.Y.max() == 32.0
    m.close()


@pytest.mark.parametrize("cfg,layers,kmin,kmax,density,sample", [(4, 1, 16, 64, None, 10), (2, 4, 8, 72, "mixed", 40)])
def test_full_batch_general_layers_sampled_rows(cfg, layers, kmin, kmax, density, sample):
    """The general-layer variant the benchmark can time (bench.py --general): 60 000 rows, neurons of
    kmin..kmax connections, several passes per layer; sampled rows against the oracle's general form."""
    import torch
    import paper_2007_14152_amd as sp
    dev = "cuda:0"
    c = synth.config(cfg)
    N, batch = c["N"], c["batch"]
    dens = density or synth.DENSITY
    print("general cfg", cfg, "layers", layers, "N", N, "batch", batch, flush=True)
    gen = [synth.gen_layer_general(N, l, c["seed"], kmin, kmax, c["window"]) for l in range(layers)]
    ptr, idx, val = [g[0] for g in gen], [g[1] for g in gen], [g[2] for g in gen]
    bias = synth.gen_bias(N, c["bias"])
    m = sp.Model.from_csr(ptr, idx, val, bias, device=dev)
    assert max(m.layer_passes(l) for l in range(layers)) > 1
    y0 = synth.gen_y0(batch, N, c["seed"], density=dens, device=dev)
    n, rows, Y = m.infer(y0)
    del y0
    rows_h = rows.cpu().numpy()
    assert n == rows_h.shape[0] and np.all(np.diff(rows_h) > 0)
    if n:
        assert float(Y.min()) >= 0.0 and float(Y.max()) <= 32.0
    rng = np.random.default_rng(300 + cfg)
    ids = np.sort(rng.choice(batch, sample, replace=False))
    ids[0], ids[-1] = 0, batch - 1
    ref = oracle.infer(idx, val, bias, synth.gen_y0(batch, N, c["seed"], density=dens, rows=ids), ptr=ptr)
    pos = np.searchsorted(rows_h, ids)
    pos_c = np.minimum(pos, max(n - 1, 0))
    present = (rows_h[pos_c] == ids) if n else np.zeros(len(ids), bool)
    sub_rows = ids[present]
    sub_Y = Y[torch.from_numpy(pos_c[present]).to(dev)].cpu().numpy() if present.any() else np.zeros((0, N), np.float32)
    common, _ = check_against_oracle(ref, len(sub_rows), sub_rows, sub_Y, row_ids=ids,
                                     what="general cfg%d L=%d sampled" % (cfg, layers))
    if density == "mixed":
        assert 0 < common < sample
    m.close()
