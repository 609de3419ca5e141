"""spdnn_infer_static, the entry point for callers that cannot allocate device memory: its work
memory is the library's fixed scratch array.  Checked against spdnn_infer (same kernels, so the
outputs must be identical) on two calls in a row, the second with a smaller input, and against the
oracle; sizes beyond the array are refused before any GPU work."""
import numpy as np
import pytest

import oracle
import synth
from parity_util import MAX_FRAGILE_FRAC, check_against_oracle, config_model

pytestmark = pytest.mark.gpu


def test_static_scratch_entry_point_matches_the_arena_one():
    import torch
    import paper_2007_14152_amd as sp
    dev = "cuda:0"
    c, idx, val, bias = config_model(0, 7)
    N = c["N"]
    m = sp.Model(idx, val, bias, device=dev)
    for batch in (1500, 333):            # the second call is smaller: the array still holds the first call's lists
        Y0 = synth.gen_y0(batch, N, c["seed"] + batch, density="mixed")
        y0 = torch.from_numpy(Y0).to(dev)
        print("static scratch: batch", batch, flush=True)
        n_s, rows_s, Y_s = m.infer_static(y0)
        n_a, rows_a, Y_a = m.infer(y0)
        assert n_s == n_a and 0 < n_s < batch
        assert torch.equal(rows_s, rows_a) and torch.equal(Y_s, Y_a)
        ref = oracle.infer(idx, val, bias, Y0)
        check_against_oracle(ref, n_s, rows_s.cpu().numpy(), Y_s.cpu().numpy(), what="static batch %d" % batch, max_fragile_frac=MAX_FRAGILE_FRAC)
    # once more after the arena entry point has run, without the final feature map
    n_s, rows_s, _ = m.infer_static(y0, want_Y=False)
    assert n_s == n_a and torch.equal(rows_s, rows_a)
    # empty batch
    n0, rows0, _ = m.infer_static(y0[:0].contiguous())
    assert n0 == 0 and rows0.numel() == 0
    # a batch whose work memory exceeds the array is refused with a clear error, nothing runs
    too_many = sp.SPDNN_STATIC_SCRATCH_BYTES // (2 * N * 4) + 1
    assert sp.spdnn_work_bytes(N, too_many) > sp.SPDNN_STATIC_SCRATCH_BYTES
    rows = torch.empty(too_many, dtype=torch.int32, device=dev)
    with pytest.raises(sp.SpdnnError) as e:
        # the size check comes before the input is touched: a small tensor stands in for it
        sp.spdnn_infer_static(m.h, y0.data_ptr(), too_many, rows.data_ptr(), 0)
    assert e.value.code == sp.SPDNN_ESIZE and "static scratch" in str(e.value)
    m.close()
