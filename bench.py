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
    ap.add_argument("--strided", default=None, metavar="S[,S...]",
                    help="strided variant (ours): neuron j reads columns (j + k*S) mod N, k = 0..31; several strides are "
                         "used by the layers in turn, as in a mixed-radix RadiX-Net")
    ap.add_argument("--out-of-core", action="store_true",
                    help="weights in pinned host memory, streamed through two device buffers (ours: the target keeps them resident)")
    ap.add_argument("--no-sustained", dest="sustained", action="store_false",
                    help="skip the second leg (same model, mixed row densities: rows alive through all layers)")
    ap.add_argument("--sustained-steps", type=int, default=2)
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stream-probe-gib", type=float, default=0.0,
                    help="instead of the benchmark: time plain streaming kernels over this many GiB (torch's fill, sum, "
                         "elementwise mul and copy: write-only, read-only, half and half) -- what the chip gives a kernel that only moves data")
    ap.add_argument("--copy-probe-gib", type=float, default=0.0,
                    help="also run a plain device copy of this many GiB (calibrates rocprofv3's FETCH_SIZE/WRITE_SIZE)")
    return ap.parse_args()


def measured_traffic(workload_key, kernel):
    """HBM bytes of one full (all rows active) launch of the dominant fused kernel, from the committed
    rocprofv3 counter summary of this workload -- a stored figure, not something this run counts, so
    it comes with its source; None if no summary exists for this workload and kernel."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        t = json.load(open(path)).get(workload_key)
    except Exception:
        return None, None
    if not t or t.get("kernel") != kernel:
        return None, None
    return float(t["hbm_bytes_full_launch"]), "stored: %s (rocprofv3 FETCH_SIZE + WRITE_SIZE of %s, scaled by a plain copy)" % (
        t["source"], t["kernel"])


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
        return time.perf_counter() - t0, len(ids), r, ids

    t, n, _, _ = run(16)
    rows = int(max(16, min(batch, n * target_s / max(t, 1e-6))))
    t, n, r, ids = run(rows)
    edges = float(n) * (N * 32 * L if edges_per_row is None else edges_per_row)
    return {"value": edges / t / 1e12, "unit": "TeraEdges/s", "cores": 1, "kind": "oracle",
            "sample": "%d seeded rows of the same workload, all %d layers (%d evaluated before every "
                      "sampled row was inactive), %.2f s single-threaded" % (n, L, r.layers_evaluated, t)}, ids, r


def parity_check(model, y0, ids, ref, final_rows):
    """Outside the timed region: the library against the oracle on the oracle's row sample.  (1) The
    final active set of the timed full-batch run, restricted to the sample, is the oracle's.  (2) The
    library run on the sampled rows alone has the oracle's active-row count on entry to every layer.
    Rows the oracle marks fragile (a pre-activation within 1e-4 of zero decides them) are excused."""
    import numpy as np
    import torch
    fragile = set(ids[ref.fragile_layer >= 0].tolist())
    want = set(ids[ref.active_rows].tolist())
    got = set(np.intersect1d(final_rows, ids).tolist())
    ok_final = not ((want ^ got) - fragile)
    model.set_profiling(True)
    n_s, rows_s, _ = model.infer(y0[torch.from_numpy(ids).to(y0.device)].contiguous(), want_Y=False)
    run, rows_in, _ = model.profile()
    model.set_profiling(False)
    apl = ref.active_per_layer
    ok_layers = all(abs(int(rows_in[l]) - int(apl[l])) <= len(fragile) for l in range(run))
    # apl[l] = rows on entry to layer l, l < L; apl[L] = rows that survive the last layer.  Layers that were
    # not launched had nothing to do; the survivors are the run's result.
    L = len(apl) - 1
    ok_layers = ok_layers and all(int(apl[l]) <= len(fragile) for l in range(run, L))
    ok_layers = ok_layers and abs(int(n_s) - int(apl[L])) <= len(fragile)
    ok_set = not ((set(ids[rows_s.cpu().numpy()].tolist()) ^ want) - fragile)
    return bool(ok_final and ok_layers and ok_set), {
        "rows_compared": int(len(ids)), "fragile_rows_excused": len(fragile), "final_set_matches": bool(ok_final),
        "per_layer_counts_match": bool(ok_layers), "sample_run_set_matches": bool(ok_set)}


def stream_probe(gib, dev):
    """GB/s of plain streaming kernels (torch's own: fill_, sum, copy_) over `gib` GiB: the rates at which
    this chip moves data when a kernel does nothing else, to set beside the fused kernel's rate."""
    import torch
    n = int(gib * (1 << 30)) // 4
    src = torch.ones(n, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    out = {"probe": "streaming kernels over %.1f GiB float32 (torch fill_, sum, elementwise mul, copy_)" % gib, "peak_GBs": HBM_PEAK_GBS}

    def rate(fn, nbytes, reps=10):
        for _ in range(3):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        e1.synchronize()
        return nbytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9

    out["write_only_GBs"] = rate(lambda: dst.fill_(1.0), n * 4)
    out["read_only_GBs"] = rate(lambda: src.sum(), n * 4)
    out["copy_GBs_read_plus_write"] = rate(lambda: torch.mul(src, 1.0, out=dst), 2 * n * 4)   # elementwise kernel
    out["device_memcpy_GBs_read_plus_write"] = rate(lambda: dst.copy_(src), 2 * n * 4)
    return out


def timed_leg(model, y0, steps, warmup, N, nnz, events_in_timed_region=True):
    """warmup + steps inferences of one resident input; HIP events on the model's stream around every
    fused launch (the library's profile).  Returns wall seconds per step and the launch statistics.
    events_in_timed_region=False: the steps are timed without the events (two per layer, 2.3 us each: a tenth of
    an inference of 120 small layers) and the launch statistics come from the same number of steps run again
    with them."""
    import numpy as np
    import torch
    for _ in range(warmup):
        model.infer(y0, want_Y=False)
    dt_plain = None
    if not events_in_timed_region:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            model.infer(y0, want_Y=False)
        torch.cuda.synchronize()
        dt_plain = time.perf_counter() - t0
    model.set_profiling(True)
    sum_ms = sum_bytes = full_ms = 0.0
    launches = full = 0
    batch = int(y0.shape[0])
    rows_trace = None
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        n_active, rows_final, _ = model.infer(y0, want_Y=False)
        run, rows_in, ms = model.profile()
        sum_ms += float(ms.sum())
        sum_bytes += sum(algorithmic_bytes(r, N, nnz[l] if nnz else None) for l, r in enumerate(rows_in))
        launches += run
        sel = rows_in == batch
        full += int(sel.sum())
        full_ms += float(ms[sel].sum())
        rows_trace = rows_in
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    model.set_profiling(False)
    if dt_plain is not None:
        dt = dt_plain
    return {"s_per_step": dt / steps, "sum_ms": sum_ms, "sum_bytes": sum_bytes, "launches": launches,
            "full_launches": full, "full_ms": full_ms, "rows_trace": np.asarray(rows_trace), "n_active": int(n_active),
            "rows_final": rows_final.cpu().numpy()}


def rows_summary(rows_trace):
    nz = [int(r) for r in rows_trace if r > 0]
    return {"layers_launched": int(len(rows_trace)), "layers_with_rows": len(nz),
            "first": int(rows_trace[0]) if len(rows_trace) else 0, "last_nonempty": nz[-1] if nz else 0,
            "head": [int(r) for r in rows_trace[:8]]}


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
    if a.stream_probe_gib > 0:
        print(json.dumps(stream_probe(a.stream_probe_gib, dev)))
        return
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
        t_create = time.perf_counter()
        model = sp.Model.from_csr(ptr, didx, dval, dbias, device=dev)
        torch.cuda.synchronize()
        t_create = time.perf_counter() - t_create
    else:
        didx = torch.empty((L, N, 32), dtype=torch.int32, device=dev)
        for l in range(L):
            didx[l] = synth.gen_layer(N, l, c["seed"], c["window"], device=dev)
            if a.scatter:
                didx[l] = synth.scatter_columns(didx[l], N, l, c["seed"], device=dev)
            if a.strided:
                strides = [int(x) for x in a.strided.split(",")]
                didx[l] = synth.gen_layer_strided(N, strides[l % len(strides)], device=dev)
        dval = torch.full((L, N, 32), synth.WEIGHT, dtype=torch.float32, device=dev)
        dbias = synth.gen_bias(N, c["bias"], device=dev)
        torch.cuda.synchronize()
        t_create = time.perf_counter()
        model = sp.Model([didx[l] for l in range(L)], [dval[l] for l in range(L)], dbias, device=dev,
                         out_of_core=a.out_of_core)
        torch.cuda.synchronize()
        t_create = time.perf_counter() - t_create
    y0 = synth.gen_y0(batch, N, c["seed"], density=density, device=dev)
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t_setup

    if a.copy_probe_gib > 0:   # a plain device copy of known size: the yardstick for the profiler's traffic counters
        n = int(a.copy_probe_gib * (1 << 30)) // 4
        src = torch.ones(n, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)    # an elementwise kernel (not a DMA copy): reads n*4 bytes, writes n*4 bytes
        torch.cuda.synchronize()
        del src, dst

    leg = timed_leg(model, y0, a.steps, a.warmup, N, nnz)
    dt = leg["s_per_step"] * a.steps
    rows_trace, launches, sum_ms, sum_bytes = leg["rows_trace"], leg["launches"], leg["sum_ms"], leg["sum_bytes"]
    n_active = leg["n_active"]

    if nnz:   # general layers: an edge is a stored connection
        edges = float(batch) * sum(nnz)
        executed = float(sum(int(r) * nnz[l] for l, r in enumerate(rows_trace)))
    else:
        edges = synth.nominal_edges(N, L, batch)
        executed = float(sum(int(r) for r in rows_trace)) * N * 32
    ms_per_step = dt / a.steps * 1e3
    achieved = sum_bytes / (sum_ms * 1e-3) / 1e9 if sum_ms > 0 else 0.0
    one_launch = model.one_launch(batch)   # small networks: every layer inside one launch of fused_chain_kernel
    kinds = {}
    for l in range(int(launches // a.steps)):
        k = "fused_chain_kernel" if one_launch else sp.KERNEL_NAMES[model.layer_kernel(l)]
        kinds[k] = kinds.get(k, 0) + 1
    kernel0 = "fused_chain_kernel" if one_launch else sp.KERNEL_NAMES[model.layer_kernel(0)]
    layers_run = int(launches // a.steps)
    if one_launch:   # the library shares the launch's duration out among the layers; the launch is the unit here
        launches = a.steps
    full_bytes = algorithmic_bytes(batch, N, nnz[0] if nnz else None)
    full_ms = leg["full_ms"] / leg["full_launches"] if leg["full_launches"] else None
    traffic, traffic_source = measured_traffic("cfg%d_batch%d_%s" % (a.config, batch, density), kernel0)
    if a.scatter or a.general or a.out_of_core or a.strided:
        traffic, traffic_source = None, None
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
                " windows scattered" if a.scatter else "") + (" strided columns, strides %s" % a.strided if a.strided else "") + (
                " weights out of core (%.1f MB on the device, %.1f MB in pinned host memory)" % (
                    model.arena.numel() / 1e6, model.host_arena.numel() / 1e6) if a.out_of_core else ""),
            "executed_TeraEdges_per_s": executed * a.steps / dt / 1e12,
            "rows_in_per_layer": rows_summary(rows_trace),
            "kernels_of_launched_layers": kinds,
            "launches_per_inference": 1 if one_launch else layers_run,
            "n_active_final": int(n_active),
            "setup_s": t_create, "generate_inputs_s": t_setup - t_create},
        # achieved = algorithmic bytes of all fused launches / their summed duration (HIP events on the
        # model's stream); full_launch_* = the launches on all `batch` rows alone
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": kernel0, "launches": int(launches),
                     "avg_launch_ms": sum_ms / max(launches, 1),
                     "algorithmic_bytes_per_launch": sum_bytes / max(launches, 1),
                     "full_launch_ms": full_ms, "full_launches": int(leg["full_launches"]),
                     "algorithmic_bytes_full_launch": full_bytes,
                     "full_launch_frac": (full_bytes / (full_ms * 1e-3) / 1e9 / HBM_PEAK_GBS) if full_ms else None},
    }
    if not a.no_cpu_baseline:
        base, ids, ref = cpu_baseline(c, L, didx, dval, dbias, density, layers_run, a.cpu_seconds,
                                      ptr=ptr, edges_per_row=float(sum(nnz)) if nnz else None)
        out["cpu_baseline"] = base
        out["parity"], out["parity_detail"] = parity_check(model, y0, ids, ref, leg["rows_final"])
    if a.sustained and density != "mixed" and not a.general:
        # Second leg (ours, labelled as such): the same model on inputs of mixed row densities, so that
        # thousands of rows stay active through all L layers -- the regime of the paper's Table I, in
        # which compaction and every layer's kernel matter.  Not part of `value`.
        del y0
        ym = synth.gen_y0(batch, N, c["seed"], density="mixed", device=dev)
        sl = timed_leg(model, ym, a.sustained_steps, 1, N, nnz, events_in_timed_region=False)
        ex = float(sum(int(r) for r in sl["rows_trace"])) * N * 32
        out["sustained_activity"] = {
            "workload": "same model, Y0 rows of mixed density (ours): every layer runs; timed without the per-layer "
                        "events, launch statistics from a second pass with them",
            "steps": a.sustained_steps, "ms_per_step": sl["s_per_step"] * 1e3,
            "nominal_TeraEdges_per_s": edges / sl["s_per_step"] / 1e12,
            "executed_TeraEdges_per_s": ex / sl["s_per_step"] / 1e12,
            "rows_in_per_layer": rows_summary(sl["rows_trace"]), "n_active_final": sl["n_active"],
            "fused_ms_per_layer": sl["sum_ms"] / max(sl["launches"], 1),
            "roofline_frac": sl["sum_bytes"] / (sl["sum_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS if sl["sum_ms"] > 0 else None}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
