#!/usr/bin/env python3
"""Benchmark of the SliceGCN hot path on one MI355X.

A step is one full-batch forward + backward pass over all k feature slices at their real
per-slice shapes: k x L layer evaluations (aggregation + dense transform), slice encoding +
concatenation, and the same chain backwards, with a seeded synthetic upstream gradient (no
optimiser step).  Inputs are resident in HBM before the timed region starts.

The headline value is the slice aggregation (SpMM) rate 2*nnz*F_s / t at the slice width
F_s, with t the average duration of that kernel measured with HIP events inside the timed
steps (the events themselves are created before the timed region); ``ms_per_step`` is the
whole fwd+bwd pass.  One JSON line is printed.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def log(msg: str):
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def spmm_bytes(n: int, nnz: int, w: int, with_add: bool = False) -> int:
    """Algorithmic HBM bytes of one aggregation call: 4 B column index + 4 B value per stored
    entry, 4 B per row pointer, each input row read once and each output row written once."""
    return 8 * nnz + 4 * (n + 1) + 8 * n * w + (4 * n * w if with_add else 0)


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(w, edges_src, edges_dst, slice_host, slices, width: int, frac: int):
    """The fp64 oracle's aggregation timed on the host: layer-1 aggregation of all k slices over the
    sub-workload made of every edge incident to the first n/frac nodes (frac = 1: the whole graph)."""
    import numpy as np
    import oracle
    n_s = max(1, w.n_nodes // frac)
    keep = (edges_src < n_s) | (edges_dst < n_s)
    s = edges_src[keep].cpu().numpy()
    d = edges_dst[keep].cpu().numpy()
    t0 = time.perf_counter()
    g = oracle.build_norm_csr(s, d, w.n_nodes)
    t_build = time.perf_counter() - t0
    t = 0.0
    for i in range(len(slices)):
        X64 = np.ascontiguousarray(slice_host(i), dtype=np.float64)
        t0 = time.perf_counter()
        oracle.spmm(g, X64)
        t += time.perf_counter() - t0
    what = "the whole graph" if frac == 1 else f"the sub-graph of all edges incident to nodes [0, {n_s})"
    return {"value": 2.0 * g.nnz * width * len(slices) / t / 1e9, "unit": "GFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle", "cpu_model": cpu_model(), "host_cpus": os.cpu_count(),
            "sample": f"fp64 oracle aggregation of all {len(slices)} slices (width {width}) over {what} "
                      f"(nnz {g.nnz} incl. self loops, {w.n_nodes} rows): {t:.2f} s in total; the oracle's own CSR "
                      f"build took {t_build:.2f} s (not in the rate)"}


def cpu_epoch(w, g, slices, hs: int, L: int):
    """One pass of the whole hot path by the fp64 oracle (all k slices x L layers forward, encoding and concat,
    and everything backward), timed with all host threads and with one.  Same seeded inputs as the GPU step."""
    import numpy as np
    import oracle
    from synth import configs, model
    k, n = len(slices), w.n_nodes
    X = configs.features(w).numpy().astype(np.float64)
    E = configs.normal_matrix(w.seed, configs.STREAM_E, k, hs, std=0.1).numpy()
    dH = configs.normal_matrix(w.seed, configs.STREAM_DH, n, k * hs).numpy().astype(np.float64)
    params = [[[t.numpy() for t in model.slice_layer_params(w, i, l, (slices[i][1] - slices[i][0]) if l == 0 else hs, hs)]
               for l in range(L)] for i in range(k)]

    def one_pass(ids):
        outs, saved = [], []
        for i in ids:
            a, b = slices[i]
            h, keep = X[:, a:b], []
            for l in range(L):
                Wa, bb, Ws, bs = params[i][l]
                hin = h
                h, Z, P = oracle.layer_fwd(g, hin, Wa, bb, Ws, bs, act=1)
                keep.append((hin, Z, P > 0))
            outs.append(h)
            saved.append(keep)
        if len(ids) == k:
            oracle.encode_concat(outs, E)
            dHs, _ = oracle.encode_concat_bwd(dH, [hs] * k, want_dE=True)
        else:
            dHs = [np.ascontiguousarray(dH[:, i * hs:(i + 1) * hs]) for i in ids]
        for j, i in enumerate(ids):
            d = dHs[j]
            for l in reversed(range(L)):
                hin, Z, mask = saved[j][l]
                d = oracle.layer_bwd(g, hin, Z, mask, params[i][l][0], params[i][l][2], d, need_dHin=l > 0).get("dHin")

    # the oracle's weight-gradient loops are slow (seconds per layer at 10^5 nodes): above 20 000 nodes the sample
    # is ONE slice model's pass, run once, and the epoch is k of them (every slice has the same shapes)
    small = n <= 20_000
    ids = list(range(k)) if small else [0]
    times = {}
    all_threads = oracle.num_threads()
    for threads in (all_threads, 1):
        oracle.set_num_threads(threads)
        reps, t0 = 0, time.perf_counter()
        if small:
            one_pass(ids)                   # untimed: page in, warm the caches
            t0 = time.perf_counter()
        while reps < (3 if small else 1) or (small and time.perf_counter() - t0 < 2.0 and reps < 50):
            one_pass(ids)
            reps += 1
        times[threads] = (time.perf_counter() - t0) / reps * (k / len(ids))
    oracle.set_num_threads(all_threads)
    return {"epochs_per_s": 1.0 / times[all_threads], "cores": all_threads,
            "epochs_per_s_one_thread": 1.0 / times[1],
            "sample": f"fp64 oracle, whole pass (forward + backward, {k} slices x {L} layers, encoding and concat)"
                      + ("" if small else f": one slice model's pass timed once, times {k}")}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg5",
                    help="cfg1..cfg5 (the benchmark workloads); comm (planted communities, for --reorder); "
                         "er:<n>:<m_und> (uniform random graph, one 32-wide slice: gather-rate probe)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-frac", type=int, default=1, help="oracle leg uses edges incident to n/frac nodes")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 4 GiB device copy (reference for HBM byte counters) and exit")
    ap.add_argument("--spmm-only", type=int, default=0, help="time only this many round-robin slice aggregations per step")
    ap.add_argument("--cache-first-agg", action="store_true",
                    help="keep the first layer's aggregation of the constant raw features across steps (the paper's "
                         "implementation recomputes it every epoch, and so does the default step)")
    ap.add_argument("--graph", action="store_true",
                    help="also capture the step into a HIP graph and time its replays (graph_ms_per_step); the "
                         "per-kernel figures still come from the eager steps")
    ap.add_argument("--ff", action="store_true",
                    help="feature-fusion variant: a shared two-layer MLP F -> F -> slice width feeds every slice model "
                         "(learned, so the first layer's input gradient and the MLP's backward join the step)")
    ap.add_argument("--classifier", action="store_true",
                    help="widen the step by the classifier MLP and the cross-entropy loss: the upstream gradient of the "
                         "slice stack then comes from the loss instead of a seeded random matrix")
    ap.add_argument("--order", choices=("aggregate", "transform", "auto"), default="aggregate",
                    help="order of the two products of every layer (SLICEGCN_LAYER_*): aggregate first (the layer as stated, "
                         "default), transform first, or transform first where the layer narrows (w_out < w_in)")
    ap.add_argument("--prescaled", action="store_true",
                    help="with --spmm-only: aggregate operands pre-scaled by D~^-1/2 (SLICEGCN_SPMM_PRESCALED: the value "
                         "stream is not read)")
    ap.add_argument("--unscaled", action="store_true",
                    help="keep the activations between the layers unscaled (every forward aggregation then reads the "
                         "stored values); by default graphs of 16 M stored entries or more keep them as D~^-1/2 H "
                         "(SLICEGCN_LAYER_IN/OUT_SCALED)")
    ap.add_argument("--streams", type=int, default=1,
                    help="slice models in flight at a time, each on its own HIP stream (default 1: one after the other); "
                         "pays on the small workloads, whose kernels leave most of the chip idle.  The per-kernel "
                         "times then overlap and say little; ms_per_step is what to read")
    ap.add_argument("--reorder", choices=("none", "degree", "bfs"), default="none",
                    help="row order of the aggregation schedule (SLICEGCN_REORDER_*): by degree, or breadth first "
                         "(pays off on graphs with communities such as --workload comm, not on R-MAT)")
    ap.add_argument("--vertex-order", choices=("permuted", "generator"), default="permuted",
                    help="'generator' keeps the R-MAT generator's own vertex numbering (low numbers are the hubs) instead "
                         "of the seeded random relabelling: a secondary data point on how much the numbering matters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (all k slices execute sequentially on it); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import synth
    from synth import configs, model
    import paper_2408_11500_amd as sg
    from paper_2408_11500_amd.stack import Classifier, FeatureFusion, GraphedStep, SliceStack

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = synth.get_workload(args.workload)

    def stream_copy():
        """A plain 4 GiB device copy with the library's copy kernel: the HBM rate this box attains."""
        rows, ld = 1 << 22, 256   # 2^30 floats = 4 GiB read + 4 GiB written by one plain copy kernel
        a = torch.ones((rows, ld), dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        for _ in range(3):
            sg.slicegcn_slice_feature(a, 0, ld, b)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5):
            sg.slicegcn_slice_feature(a, 0, ld, b)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 5
        # and a read-only pass over the same 4 GiB (the library's column sums): what a kernel that only reads attains
        ws = torch.empty(sg.slicegcn_concat_bwd_workspace_bytes(rows, [ld]), dtype=torch.uint8, device=dev)
        sums = torch.empty((1, ld), dtype=torch.float32, device=dev)
        for _ in range(3):
            sg.slicegcn_concat_bwd(a, [ld], dE=sums, ws=ws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5):
            sg.slicegcn_concat_bwd(a, [ld], dE=sums, ws=ws)
        torch.cuda.synchronize()
        dr = (time.perf_counter() - t0) / 5
        return {"copy_bytes_read": rows * ld * 4, "copy_bytes_written": rows * ld * 4, "ms": dt * 1e3,
                "GBps": 2 * rows * ld * 4 / dt / 1e9, "read_only_ms": dr * 1e3, "read_only_GBps": rows * ld * 4 / dr / 1e9}

    if args.copy_calibration:
        print(json.dumps(stream_copy()))
        return

    log(f"generating {w.name}: N={w.n_nodes} M_und={w.m_und}")
    t0 = time.perf_counter()
    src, dst = configs.edges(w, device=dev, permute=args.vertex_order == "permuted")
    torch.cuda.synchronize()
    log(f"edges in {time.perf_counter() - t0:.1f} s")
    t0 = time.perf_counter()
    build_flags = sg.SYMMETRIZE | sg.ADD_SELF_LOOPS | {"none": 0, "degree": sg.binding.REORDER_DEGREE,
                                                        "bfs": sg.binding.REORDER_BFS}[args.reorder]
    g = sg.slicegcn_build_norm_csr(src, dst, w.n_nodes, build_flags)
    torch.cuda.synchronize()
    build_ms = (time.perf_counter() - t0) * 1e3
    view = g.view()
    assert w.kind == "comm" or view.nnz == w.nnz, (view.nnz, w.nnz)
    log(f"build_norm_csr {build_ms:.1f} ms, nnz={view.nnz}")

    slices, width = sg.slicegcn_slice_strategy(w.feat, w.k)
    hs, L, k, n = w.slice_hidden, w.layers, w.k, w.n_nodes
    X = configs.features(w, device=dev)
    ff = None
    if args.ff:
        ff = FeatureFusion(n, w.feat, width, device=dev)
        ff.set_params(*model.fusion_params(w, width, device=dev))
        ff.forward(X)
    st = SliceStack(g, n, k, width, hs, L, device=dev, shared_input=ff.Xff if ff is not None else None,
                    cache_first_aggregation=args.cache_first_agg, scaled=False if args.unscaled else None, streams=args.streams,
                    order={"aggregate": 0, "transform": sg.binding.LAYER_TRANSFORM_FIRST, "auto": sg.binding.LAYER_ORDER_AUTO}[args.order])
    for i, (a, b) in enumerate(slices):
        if ff is None:
            sg.slicegcn_slice_feature(X, a, b, st.X[i])
        for l, (wi, wo) in enumerate(st.widths):
            st.set_params(i, l, *model.slice_layer_params(w, i, l, wi, wo, device=dev))
    if ff is None:
        del X
    st.E.copy_(configs.normal_matrix(w.seed, configs.STREAM_E, k, hs, device=dev, std=0.1))
    dH = configs.normal_matrix(w.seed, configs.STREAM_DH, n, k * hs, device=dev)
    cls = labels = None
    if args.classifier:
        cls = Classifier(n, k * hs, w.hidden, w.classes, device=dev)
        cls.set_params(*model.classifier_params(w, k * hs, device=dev))
        labels = configs.labels(w, device=dev).to(torch.int32)
    torch.cuda.synchronize()
    log("inputs resident")

    Yspmm = torch.empty_like(st.X[0]) if args.spmm_only else None
    Xagg = st.X
    if args.spmm_only and args.prescaled:   # D~^-1/2 X_s, made once: the raw features are constant
        Xagg = [sg.slicegcn_scale_rows(g, x[:, :width], torch.empty_like(x), width=width) for x in st.X]

    def step():
        if args.spmm_only:
            for j in range(args.spmm_only):   # round-robin over the slices, as in the real pass
                sg.slicegcn_spmm_slice(g, Xagg[j % k][:, :width], Yspmm[:, :width], prescaled=args.prescaled)
        else:
            if ff is not None:
                ff.forward(X)
            H = st.forward()
            if cls is not None:
                cls.forward_backward(H, labels, dH)
            st.backward(dH)
            if ff is not None:
                ff.backward(X, st.dXin[:, :width])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # count the kernel groups of one step, then create every event the timed steps will record beforehand
    sg.slicegcn_profile_begin()
    step()
    groups_per_step = sum(e[2] for e in sg.slicegcn_profile_end())
    sg.slicegcn_profile_reserve((args.steps + 1) * groups_per_step)
    sg.slicegcn_profile_begin()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof_full = sg.slicegcn_profile_end(with_range=True)
    prof = [e[:4] for e in prof_full]
    ms_per_step = elapsed * 1e3 / args.steps
    log(f"{args.steps} steps, {ms_per_step:.2f} ms/step")
    # the same steps once more without the per-kernel events, to show what recording them costs
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_no_events = (time.perf_counter() - t0) * 1e3 / args.steps

    graph_ms = None
    if args.graph:
        gs = GraphedStep(step)
        for _ in range(args.warmup):
            gs.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            gs.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        log(f"HIP graph replay: {graph_ms:.2f} ms/step")

    kernels = {f"{kind}_w{wd}": {"launches": cnt, "avg_ms": tot / cnt, "median_ms": med, "min_ms": lo, "max_ms": hi}
               for kind, wd, cnt, tot, lo, hi, med in prof_full}
    dom = next(((cnt, tot) for kind, wd, cnt, tot in prof if kind == "spmm" and wd == width), None)
    if dom is None:
        # this variant of the step ran no aggregation at the slice width (cached first layer, or the transform-first
        # order, which aggregates at the hidden width): time the slice-width aggregation on its own
        Y = torch.empty_like(st.X[0])
        sg.slicegcn_profile_begin()
        for j in range(2 * k):
            sg.slicegcn_spmm_slice(g, st.X[j % k][:, :width], Y[:, :width])
        extra = sg.slicegcn_profile_end()
        dom = next(((cnt, tot) for kind, wd, cnt, tot in extra if kind == "spmm" and wd == width), None)
    if dom is None:
        print("bench.py: no aggregation at the slice width was timed", file=sys.stderr)
        sys.exit(1)
    avg_s = dom[1] / dom[0] / 1e3
    nbytes = spmm_bytes(n, view.nnz, width)
    achieved = nbytes / avg_s / 1e9
    traffic = traffic_source = None
    # HBM-side bytes per aggregation call: NOT measured in this run (counters need rocprofv3); the figure is read
    # from the committed rocprofv3 --pmc summary of the same workload and launch configuration
    tfile = os.path.join(ROOT, "profiles", f"spmm_{w.name}_rocprofv3.md")
    if os.path.exists(tfile) and args.vertex_order == "permuted" and args.reorder == "none":
        import re
        # the summary holds one figure per form of the aggregation; take the one the timed launches ran in
        factored = args.prescaled if args.spmm_only else st.in_scaled
        key = "hbm_bytes_per_launch" if factored else "hbm_bytes_per_launch_with_values"
        m = re.search(rf"^{key} = (\d+)", open(tfile).read(), flags=re.M)
        traffic = int(m.group(1)) if m else None
        traffic_source = (f"profiles/spmm_{w.name}_rocprofv3.md, {key} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of "
                          "`bench.py --spmm-only`, scaled by a plain copy; a stored figure, not measured in this run)")
    out = {
        "metric": "slice_spmm_gflops", "value": 2.0 * view.nnz * width / avg_s / 1e9, "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: N={n}, nnz={view.nnz} (R-MAT, symmetrised + self loops), F={w.feat} in k={k} "
                               f"slices of {width}, {L} layers, per-slice hidden {hs}, full-batch fwd+bwd"
                               + (" [generator's vertex numbering, hubs first]" if args.vertex_order != "permuted" else "")
                               + (f" [rows visited in {args.reorder} order]" if args.reorder != "none" else "")
                               + (f" [layer order: {args.order}]" if args.order != "aggregate" else "")
                               + (" [activations kept as D~^-1/2 H between layers]" if st.scaled else "")
                               + (f" [{st.lanes} slice models in flight on streams of their own]" if st.lanes > 1 else "")
                               + (" [aggregation only]" if args.spmm_only else "")
                               + (" [operands pre-scaled by D~^-1/2]" if args.spmm_only and args.prescaled else "")

                               + (" [first-layer aggregation cached across steps]" if args.cache_first_agg and ff is None else "")
                               + (f" + feature fusion {w.feat}->{w.feat}->{width}" if ff is not None else "")
                               + (f" + classifier {k * hs}->{w.hidden}->{w.classes} and cross-entropy" if cls is not None else ""),
                   "n_nodes": n, "nnz": view.nnz, "k": k, "slice_width": width, "slice_hidden": hs, "layers": L},
        "epoch_ms": None if args.spmm_only else ms_per_step,
        "epochs_per_s": None if args.spmm_only else 1e3 / ms_per_step,
        "ms_per_step_without_events": ms_no_events, "graph_ms_per_step": graph_ms,
        "spmm_avg_ms": avg_s * 1e3, "spmm_median_ms": kernels.get(f"spmm_w{width}", {}).get("median_ms"),
        "spmm_min_ms": kernels.get(f"spmm_w{width}", {}).get("min_ms"),
        "spmm_launches_timed": dom[0], "build_norm_csr_ms": build_ms,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source, "kernel": "slice aggregation (spmm_wave_items + spmm_group_items + spmm_tiny_rows + spmm_fix kernels of one call)",
                     "algorithmic_bytes_per_launch": nbytes,
                     # what the factored form needs: no 4-byte value per stored entry, one factor per row instead
                     "algorithmic_bytes_without_values": nbytes - 4 * view.nnz + 4 * n},
        "kernels": kernels,
    }
    if traffic is not None:
        # the second bandwidth figure: bytes the memory side moved (stored counter summary) over the measured time,
        # and their ratio to the algorithmic bytes (1 = no gathered row fetched twice)
        out["roofline"]["traffic_GBps"] = traffic / avg_s / 1e9
        out["roofline"]["traffic_over_algorithmic"] = traffic / nbytes
    probe = stream_copy()   # what a plain copy and a read-only pass reach on this machine, for scale
    out["roofline"]["stream_copy_GBps"] = probe["GBps"]
    out["roofline"]["stream_read_GBps"] = probe["read_only_GBps"]
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a bounded sample")
        # the raw slice, regenerated: the stack's own copies hold the scaled layout by now
        out["cpu_baseline"] = cpu_baseline(w, src, dst,
                                           lambda i: configs.features(w, device=dev, col_start=slices[i][0],
                                                                      col_count=slices[i][1] - slices[i][0]).cpu().numpy(),
                                           slices, width, args.cpu_sample_frac)
        if n <= 200_000 and not args.spmm_only and ff is None and cls is None:
            # small workloads: the oracle's whole pass fits the time budget (seconds)
            import oracle
            og = oracle.build_norm_csr(src.cpu().numpy(), dst.cpu().numpy(), n)
            out["cpu_baseline"]["epoch"] = cpu_epoch(w, og, slices, hs, L)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
