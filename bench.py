"""Benchmark of the sparse-DNN inference hot path on one MI355X.

One step = one spdnn_infer over the whole synthetic batch (all layers: fused
SpMM+bias+clipped-ReLU, active-row compaction, buffer swap, final gather) with
inputs and weights already resident in HBM.  Prints one JSON line: value = nominal
edges (batch*N*32*L) per second; roofline = algorithmic bytes of the fused-kernel
launches (rows*N*8 + N*32*6 each) over their summed durations, against peak HBM
bandwidth; cpu_baseline = the oracle on a seeded sample of rows of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X published peak HBM3E bandwidth


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, help="benchmark configuration 0..4")
    ap.add_argument("--layers", type=int, default=None, help="override the number of layers (debug)")
    ap.add_argument("--batch", type=int, default=None, help="override the batch (debug)")
    ap.add_argument("--density", default=None, help="'mixed' = sustained-activity variant (ours)")
    ap.add_argument("--general", default=None, metavar="KMIN,KMAX",
                    help="general-layer variant (ours): neurons with KMIN..KMAX connections and varying weights, "
                         "through spdnn_create_csr; needs --layers (default 6)")
    ap.add_argument("--scatter", action="store_true",
                    help="scattered-window variant (ours): the members of every window are spread over the row by a "
                         "seeded permutation per layer")
    ap.add_argument("--out-of-core", action="store_true",
                    help="weights in pinned host memory, streamed through two device buffers (ours: the target keeps them resident)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-probe-gib", type=float, default=0.0,
                    help="also run a plain device copy of this many GiB (calibrates rocprofv3's FETCH_SIZE/WRITE_SIZE)")
    return ap.parse_args()


def measured_traffic(workload_key):
    """HBM bytes per fused-layer launch from the committed rocprofv3 counter summary
    (profiles/), if it was taken on this workload; else None."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        t = json.load(open(path)).get(workload_key)
        return float(t["hbm_bytes_per_launch"]) if t else None
    except Exception:
        return None


def algorithmic_bytes(rows, N, nnz=None):
    """Bytes one fused-layer launch must move: read and write every (active row,
    neuron) once in float32, plus the layer's weights once (u16 index + f32 value)."""
    return float(rows) * N * 8.0 + (N * 32 if nnz is None else nnz) * 6.0


def cpu_baseline(c, L, didx, dval, dbias, density, layers_run, target_s, ptr=None, edges_per_row=None):
    """The oracle as it stands, single thread, on a seeded sample of rows of the same
    workload.  Only the layers some row can reach are copied to the host."""
    import numpy as np
    import oracle
    import synth
    N, batch = c["N"], c["batch"]
    have = min(L, layers_run + 4)
    tonp = lambda a: a if isinstance(a, np.ndarray) else a.cpu().numpy()
    idx = [tonp(didx[l]) if l < have else None for l in range(L)]
    val = [tonp(dval[l]) if l < have else None for l in range(L)]
    bias = tonp(dbias)
    rng = np.random.default_rng(12345)

    def run(nrows):
        ids = np.sort(rng.choice(batch, min(nrows, batch), replace=False))
        y = synth.gen_y0(batch, N, c["seed"], density=density, rows=ids)
        t0 = time.perf_counter()
        r = oracle.infer(idx, val, bias, y, want_Y=False, ptr=ptr)
        return time.perf_counter() - t0, len(ids), r

    t, n, _ = run(16)
    rows = int(max(16, min(batch, n * target_s / max(t, 1e-6))))
    t, n, r = run(rows)
    edges = float(n) * (N * 32 * L if edges_per_row is None else edges_per_row)
    return {"value": edges / t / 1e12, "unit": "TeraEdges/s", "cores": 1, "kind": "oracle",
            "sample": "%d seeded rows of the same workload, all %d layers (%d evaluated before every "
                      "sampled row was inactive), %.2f s single-threaded" % (n, L, r.layers_evaluated, t)}


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); no multi-GPU path exists", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import synth
    import paper_2007_14152_amd as sp

    dev = "cuda:0"
    c = synth.config(a.config)
    if a.batch:
        c["batch"] = a.batch
    L = a.layers or c["L"]
    N, batch = c["N"], c["batch"]
    density = a.density if a.density else synth.DENSITY
    t_setup = time.perf_counter()
    ptr = nnz = None
    if a.general:
        kmin, kmax = (int(x) for x in a.general.split(","))
        L = a.layers or 6
        gen = [synth.gen_layer_general(N, l, c["seed"], kmin, kmax, c["window"]) for l in range(L)]
        ptr, didx, dval = [g[0] for g in gen], [g[1] for g in gen], [g[2] for g in gen]
        nnz = [int(p[N]) for p in ptr]
        dbias = synth.gen_bias(N, c["bias"])
        model = sp.Model.from_csr(ptr, didx, dval, dbias, device=dev)
    else:
        didx = torch.empty((L, N, 32), dtype=torch.int32, device=dev)
        for l in range(L):
            didx[l] = synth.gen_layer(N, l, c["seed"], c["window"], device=dev)
            if a.scatter:
                didx[l] = synth.scatter_columns(didx[l], N, l, c["seed"], device=dev)
        dval = torch.full((L, N, 32), synth.WEIGHT, dtype=torch.float32, device=dev)
        dbias = synth.gen_bias(N, c["bias"], device=dev)
        model = sp.Model([didx[l] for l in range(L)], [dval[l] for l in range(L)], dbias, device=dev,
                         out_of_core=a.out_of_core)
    y0 = synth.gen_y0(batch, N, c["seed"], density=density, device=dev)
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t_setup

    if a.copy_probe_gib > 0:
        n = int(a.copy_probe_gib * (1 << 30)) // 4
        src = torch.ones(n, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            sp.spdnn_copy_probe(dst.data_ptr(), src.data_ptr(), n * 4, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(a.warmup):
        model.infer(y0, want_Y=False)
    model.set_profiling(True)
    sum_ms = 0.0
    sum_bytes = 0.0
    launches = 0
    rows_trace = None
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        n_active, _, _ = model.infer(y0, want_Y=False)
        run, rows_in, ms = model.profile()
        sum_ms += float(ms.sum())
        sum_bytes += sum(algorithmic_bytes(r, N, nnz[l] if nnz else None) for l, r in enumerate(rows_in))
        launches += run
        rows_trace = rows_in
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    model.set_profiling(False)

    if nnz:   # general layers: an edge is a stored connection
        edges = float(batch) * sum(nnz)
        executed = float(sum(int(r) * nnz[l] for l, r in enumerate(rows_trace)))
    else:
        edges = synth.nominal_edges(N, L, batch)
        executed = float(sum(int(r) for r in rows_trace)) * N * 32
    ms_per_step = dt / a.steps * 1e3
    achieved = sum_bytes / (sum_ms * 1e-3) / 1e9 if sum_ms > 0 else 0.0
    out = {
        "metric": "TeraEdges/sec (batch*N*32*L/time) at 1 MI355X",
        "value": edges * a.steps / dt / 1e12,
        "unit": "TeraEdges/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "cfg%d: N=%d L=%d batch=%d bias=%g window=%s density=%s" % (
            a.config, N, L, batch, c["bias"], c["window"], density) + (
                " general layers %s connections per neuron, passes %s" % (
                    a.general, [model.layer_passes(l) for l in range(L)]) if a.general else "") + (
                " windows scattered" if a.scatter else "") + (
                " weights out of core (%.1f MB on the device, %.1f MB in pinned host memory)" % (
                    model.arena.numel() / 1e6, model.host_arena.numel() / 1e6) if a.out_of_core else ""),
            "layers_launched": int(launches // a.steps), "rows_in_per_layer": [int(r) for r in rows_trace[:8]],
            "n_active_final": int(n_active), "executed_TeraEdges_per_s": executed * a.steps / dt / 1e12,
            "setup_s": t_setup},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic("cfg%d_L%d_batch%d_%s" % (a.config, L, batch, density)),
                     "kernel": sp.KERNEL_NAMES[model.layer_kernel(0)], "launches": int(launches),
                     "avg_launch_ms": sum_ms / max(launches, 1),
                     "algorithmic_bytes_per_launch": sum_bytes / max(launches, 1)},
    }
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(c, L, didx, dval, dbias, density, int(launches // a.steps), a.cpu_seconds,
                                           ptr=ptr, edges_per_row=float(sum(nnz)) if nnz else None)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
