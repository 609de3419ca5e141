"""Parity at the benchmark's full sizes (60 000 rows, the launch configuration the
benchmark times): the library runs the whole batch on the GPU; the oracle
evaluates a seeded sample of rows (rows are independent, Eq. 1), and the sample
is compared one by one.  Whole-output properties are checked on the GPU result
with torch reductions."""
import numpy as np
import pytest

import oracle
import synth
from parity_util import check_against_oracle, config_model

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cfg,layers,sample", [(1, 1, 96), (1, 2, 96), (1, 3, 96), (2, 1, 48), (2, 2, 48),
                                              (3, 1, 24), (3, 2, 24), (4, 1, 12), (4, 2, 12)])
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
    rng = np.random.default_rng(100 + cfg)
    ids = np.sort(rng.choice(batch, sample, replace=False))
    ids[0], ids[-1] = 0, batch - 1          # first and last row (ragged tail of the last group)
    idx = [a.cpu().numpy() for a in didx]
    val = [a.cpu().numpy() for a in dval]
    ref = oracle.infer(idx, val, dbias.cpu().numpy(), synth.gen_y0(batch, N, c["seed"], rows=ids))
    pos = np.searchsorted(rows_h, ids)
    pos_c = np.minimum(pos, max(n - 1, 0))
    present = (rows_h[pos_c] == ids) if n else np.zeros(len(ids), bool)
    sub_rows = ids[present]
    sub_Y = Y[torch.from_numpy(pos_c[present]).to(dev)].cpu().numpy() if present.any() else np.zeros((0, N), np.float32)
    common, _ = check_against_oracle(ref, len(sub_rows), sub_rows, sub_Y, row_ids=ids,
                                     what="cfg%d L=%d sampled" % (cfg, layers))
    if layers == 1:
        assert n == batch and common == sample
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
