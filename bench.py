#!/usr/bin/env python3
"""Benchmark of the cascade-selection hot path on one MI355X.

One "step" = one pass of the whole path over one synthetic sequence: full Gram-threshold selection at
layer 0 and a cascade step at each of the layers 1..L-1 (Section 4.1), all chained on the device through
ada_cascade_layers with inputs already resident in HBM.  The workload is the configuration the metric is quoted on
(GPT-J-shaped: T=2048, d=4096, 28 layers, bf16, tau=0.1, 400 centres).  The 28 layer buffers (448 MiB) exceed the 256 MB Infinity Cache, so each layer's X comes from
HBM when the step reaches it.

Prints ONE JSON line: metric / value / unit and the run's settings, `roofline` (the dominant kernel against the HBM
peak, with the hardware-counter traffic), `cpu_baseline` (the float64 oracle on the host cores), and one block per
further measurement (full selection, assignment, attention, pipeline, batches, per-head groups, other shapes).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published


def cpu_baseline(w, xs_cpu, n_cascade=3):
    """The float64 oracle, as it stands, on a bounded sample of the same workload: layer 0 (full selection)
    and the first n_cascade cascade layers; the pass rate is extrapolated as L / (t_full + (L-1) * mean t_casc)."""
    import oracle
    from paper_2605_03110_amd import workloads as wl
    t0 = time.perf_counter()
    full = oracle.select_full(wl.as_f64(xs_cpu[0]), w.tau)
    t_full = time.perf_counter() - t0
    prev = full["idx"]
    t_c = []
    for l in range(1, 1 + n_cascade):
        X = wl.as_f64(xs_cpu[l])
        t0 = time.perf_counter()
        res = oracle.cascade_step(X, w.tau, prev)
        t_c.append(time.perf_counter() - t0)
        prev = res["idx"]
    mean_c = sum(t_c) / len(t_c)
    extra = cpu_baseline_extras()
    return dict(value=w.L / (t_full + (w.L - 1) * mean_c), unit="layers/s", cores=oracle.threads(), kind="oracle", **extra,
                sample="float64 C oracle (OpenMP) on layer 0 (full, %.2f s) and layers 1-%d (cascade, mean %.2f s) of the "
                       "same sequence; extrapolated to the %d-layer pass" % (t_full, n_cascade, mean_c, w.L),
                t_full_s=t_full, t_cascade_s=mean_c)


def cpu_baseline_extras():
    """Two more samples of the oracle as it stands: the small fp32 configuration on ONE thread, and one full selection
    at the long-context shape on all cores."""
    import oracle
    from paper_2605_03110_amd import workloads as wl
    out = {}
    w0 = wl.config(0)
    xs0 = [wl.as_f64(x) for x in wl.layer_list(w0, 0, 3)]
    before = oracle.set_threads(1)
    try:
        t0 = time.perf_counter()
        f0 = oracle.select_full(xs0[0], w0.tau)
        tf = time.perf_counter() - t0
        prev, tc = f0["idx"], []
        for X in xs0[1:]:
            t0 = time.perf_counter()
            res = oracle.cascade_step(X, w0.tau, prev)
            tc.append(time.perf_counter() - t0)
            prev = res["idx"]
        th = oracle.threads()
    finally:
        oracle.set_threads(before)
    tcm = sum(tc) / len(tc)
    out["single_thread_c0"] = {"threads": th, "t_full_s": tf, "t_cascade_s": tcm,
                               "layers_per_s": w0.L / (tf + (w0.L - 1) * tcm),
                               "sample": "%s: layer 0 full + 2 cascade layers, extrapolated to %d layers" % (w0.name, w0.L)}
    w4 = wl.config(4)
    x4 = wl.as_f64(next(iter(wl.layers(w4, 0, 1))))
    t0 = time.perf_counter()
    oracle.select_full(x4, w4.tau)
    out["full_selection_c4"] = {"threads": oracle.threads(), "t_full_s": time.perf_counter() - t0,
                                "sample": "%s layer 0 of one sequence (T=%d, d=%d)" % (w4.name, w4.T, w4.d)}
    return out


def recorded_traffic(name):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of this kernel and workload (FETCH_SIZE and
    WRITE_SIZE scaled by the copy probe), or None if no summary is there."""
    import re
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None
    m = re.search(r"^traffic_bytes_per_launch\s*=\s*(\d+)", open(path).read(), flags=re.M)
    return int(m.group(1)) if m else None


def probe(pa, xs, w, ws, out, stream):
    """Short run for hardware counters: one cascade pass, full selection on four layers and twice at the long-context
    shape, two assignments and two attention launches on the last layer's set, and the 256 MiB copy probe."""
    import torch
    pa.ada_cascade_layers(xs, w.tau, ws=ws, out=out, stream=stream)
    for l in range(4):
        pa.ada_select_full(xs[l], w.tau, ws=ws, stream=stream)
    from paper_2605_03110_amd import workloads as wl
    w4 = wl.config(4)                                   # the long-context shape: two full selections of layer 0
    x4 = next(iter(wl.layers(w4, 0, 1))).to(xs[0].device)
    ws4 = pa.workspace(w4.T, xs[0].device)
    for _ in range(2):
        pa.ada_select_full(x4, w4.tau, ws=ws4, stream=stream)
    # the last layer's set: two assignment launches (the last two k_cascade_fused of the run) and two attention launches
    L = len(xs)
    if w.d % 16 == 0 and w.d // 16 in (64, 128, 256) and w.dtype == "bf16":
        last = out["idx"][L - 1]
        qd, kd, vd = (m.to(xs[0].device) for m in wl.qkv(w, 16))
        for _ in range(2):
            near = pa.ada_assign_nearest(xs[L - 1], last, r=w.T, r_dev=out["counts"][L - 1], ws=ws, stream=stream)
        for _ in range(2):
            pa.ada_attention_compressed(qd, kd, vd, 16, last, near["assign"], r=w.T, r_dev=out["counts"][L - 1], ws=ws,
                                        stream=stream)
    src = torch.empty(256 << 20, dtype=torch.uint8, device=xs[0].device).fill_(1)
    dst = torch.empty_like(src)
    for _ in range(2):
        pa.ada_profile_copy_probe(dst, src, stream=stream)
    torch.cuda.synchronize()
    print(json.dumps({"probe": "done", "copy_probe_bytes": 256 << 20}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="which of the five workload configurations, 0..4 (default 2: T=2048, d=4096, 28 layers)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the full-selection timing and the profiled pass")
    ap.add_argument("--probe", action="store_true", help="short run for rocprofv3 --pmc (no timing, no JSON result)")
    ap.add_argument("--layers", type=int, default=0, help="use only the first N layers of the configuration (0 = all); "
                    "for counter runs at the large shapes, where generating every layer on the host takes longest")
    ap.add_argument("--roofline-only", action="store_true",
                    help="the timed passes and the event-timed pass of the roofline only (for a kernel trace in which "
                         "k_cascade_fused runs this workload's cascade steps and nothing else)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (no collectives, no sharding "
              "in this library)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import __graft_entry__
    __graft_entry__.ensure_built()
    import paper_2605_03110_amd as pa
    from paper_2605_03110_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = wl.config(args.config)
    if args.layers > 0:
        w = wl.config(args.config, L=min(args.layers, w.L))
    T, d, L = w.T, w.d, w.L
    esz = 2 if w.dtype == "bf16" else 4

    xs_cpu = wl.layer_list(w, 0)
    xs = [x.to(dev) for x in xs_cpu]
    ws = pa.workspace(T, dev)
    out = dict(idx=torch.empty((L, T), dtype=torch.int32, device=dev),
               counts=torch.empty((L, 4), dtype=torch.int32, device=dev),
               gram_ops=torch.empty(L, dtype=torch.int64, device=dev))
    stream = torch.cuda.current_stream()

    def step():
        pa.ada_cascade_layers(xs, w.tau, ws=ws, out=out, stream=stream)

    if args.probe:
        probe(pa, xs, w, ws, out, stream)
        return

    out["idx"].zero_()                                   # (entries past a layer's set size are never written)
    for _ in range(max(args.warmup, 1)):
        step()
    torch.cuda.synchronize()
    first_pass = {k: out[k].clone() for k in ("idx", "counts", "gram_ops")}
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    for k, v in first_pass.items():                      # every timed pass writes the same buffers: the last equals the first
        assert torch.equal(out[k], v), "the last timed pass differs from the first in %s" % k
    ms_per_step = 1e3 * elapsed / args.steps
    layers_per_s = L * args.steps / elapsed

    counts = out["counts"].cpu()
    ops = out["gram_ops"].cpu()
    assert counts[:, 3].tolist() == [0] * L, "device status reported an error"
    rep = pa.ada_cascade_report(counts, ops, T)
    r_per_layer = counts[:, 0].tolist()
    r_prev_mean = sum(r_per_layer[:-1]) / max(L - 1, 1)

    result = {
        "metric": "cascade_select_layers_per_s", "value": layers_per_s, "unit": "layers/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": "%s: T=%d d=%d L=%d %s tau=%.2f, %d centres, noise %.3g, drift %.3g, %.0f%% reassigned "
                               "per layer (%s scale), full selection at layer 0 + cascade at layers 1..%d"
                               % (w.name, T, d, L, w.dtype, w.tau, w.K, w.sigma_n, w.sigma_c, 100 * w.p, w.scale, L - 1),
                   "T": T, "d": d, "layers": L, "batch": 1},
        "tokens_per_s": layers_per_s * T,
        "method_stats": {"gram_op_savings": rep["savings"], "mean_jaccard_cascade": sum(rep["jaccard"][1:]) / (L - 1),
                         "mean_turnover": sum(rep["turnover"][1:]) / (L - 1), "r_layer0": r_per_layer[0],
                         "mean_r_cascade": sum(r_per_layer[1:]) / (L - 1),
                         "paper_context": "paper: 22-63% savings, mean Jaccard 0.83-0.94 at T=512, tau=0.30, real "
                                          "activations, MI300X"},
    }

    # ---- per-kernel durations from HIP events on the launch stream, over a pass identical to the timed one
    kern = None
    if not args.no_extras:
        pa.ada_profile_enable(True)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        prof_elapsed = time.perf_counter() - t0
        kern = pa.ada_profile_collect()
        pa.ada_profile_enable(False)
        avg_us = {k: (1e3 * v["ms"] / v["launches"] if v["launches"] else None) for k, v in kern.items()}
        casc_s = 1e-6 * avg_us["cascade_fused"]
        # The cascade layers of a pass run in one resident launch (k_cascade_pass) when the shape allows, else one
        # launch per layer: the units of a launch are the layers it processes.
        layers_per_launch = (L - 1) * args.steps / kern["cascade_fused"]["launches"]
        # algorithmic bytes per layer: every row of X once (all T rows are tested rows, the r inherited rows are also
        # the resident operand) = T*d*e bytes; the O(T*r/8) hit words and O(T) outputs are neglected
        layer_bytes = T * d * esz
        casc_bytes = layers_per_launch * layer_bytes
        casc_flops = layers_per_launch * 2.0 * d * T * r_prev_mean   # T x r Gram entries of eq. (6), 2d flops each
        traffic_layer = recorded_traffic("cascade_fused_c%d_pmc.txt" % args.config)
        result["roofline"] = {"bound": "hbm",
                              "kernel": "k_cascade_pass (Algorithm 1, %g layers per resident launch)" % layers_per_launch
                                        if layers_per_launch > 1 else "k_cascade_fused (Algorithm 1 in one launch)",
                              "achieved": casc_bytes / casc_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                              "frac": casc_bytes / casc_s / 1e9 / HBM_PEAK_GBS,
                              "traffic": None if traffic_layer is None else int(traffic_layer * layers_per_launch),
                              "avg_launch_us": avg_us["cascade_fused"], "layers_per_launch": layers_per_launch,
                              "us_per_layer": avg_us["cascade_fused"] / layers_per_launch,
                              "bytes_per_launch": casc_bytes,
                              "mfma_tflops": casc_flops / casc_s / 1e12,
                              "mfma_frac": casc_flops / casc_s / 1e12 / MFMA_BF16_PEAK_TFLOPS}
        result["kernel_avg_us"] = avg_us
        result["ms_per_step_with_events"] = 1e3 * prof_elapsed / args.steps
    if args.roofline_only:
        print(json.dumps(result))
        return
    if not args.no_extras:

        # ---- the full T x T selection at every layer (the comparison path), same buffers
        fo = [pa.ada_select_full(xs[0], w.tau, ws=ws) for _ in range(2)]
        torch.cuda.synchronize()
        masks = torch.empty((L, T), dtype=torch.uint8, device=dev)
        idxb = torch.empty(T, dtype=torch.int32, device=dev)
        cnt = torch.empty(4, dtype=torch.int32, device=dev)
        import ctypes
        lib = pa.ada.lib()

        def full_pass():
            for l in range(L):
                rc = lib.ada_select_full(ctypes.c_void_p(xs[l].data_ptr()), T, d, xs[l].stride(0),
                                         pa.ada._dtype_code(xs[l]), float(w.tau), ctypes.c_void_p(masks[l].data_ptr()),
                                         ctypes.c_void_p(idxb.data_ptr()), ctypes.c_void_p(cnt.data_ptr()), None,
                                         ctypes.c_void_p(ws.data_ptr()), ws.numel(), ctypes.c_void_p(stream.cuda_stream), 0)
                assert rc == 0
        full_pass()
        torch.cuda.synchronize()
        n_full = max(1, args.steps // 4)
        pa.ada_profile_enable(True)
        t0 = time.perf_counter()
        for _ in range(n_full):
            full_pass()
        torch.cuda.synchronize()
        full_elapsed = time.perf_counter() - t0
        kf = pa.ada_profile_collect()
        pa.ada_profile_enable(False)
        full_us = 1e3 * kf["gram_full"]["ms"] / kf["gram_full"]["launches"]
        tri_flops = float(T) * (T - 1) * d            # strict lower triangle: T(T-1)/2 entries * 2d flops
        jac = []
        for l in range(1, L):
            o = pa.ada_set_overlap(masks[l - 1], masks[l]).cpu().tolist()
            jac.append(o[0] / o[1])
        # ---- the same pass with the cascade layers in one resident launch (ADA_FLAG_RESIDENT_PASS)
        for _ in range(2):
            pa.ada_cascade_layers(xs, w.tau, ws=ws, out=out, stream=stream, flags=pa.FLAG_RESIDENT_PASS)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            pa.ada_cascade_layers(xs, w.tau, ws=ws, out=out, stream=stream, flags=pa.FLAG_RESIDENT_PASS)
        torch.cuda.synchronize()
        res_elapsed = time.perf_counter() - t0
        assert out["counts"][:, 3].cpu().tolist() == [0] * L, "resident pass reported an error"
        result["resident_pass"] = {"ms_per_step": 1e3 * res_elapsed / args.steps,
                                   "layers_per_s": L * args.steps / res_elapsed}

        # ---- what the matrix pipes sustain on this device with realistic operands (the published peak assumes the
        # full boost clock): one workgroup per CU, matrix instructions only
        n_cu = torch.cuda.get_device_properties(dev).multi_processor_count
        pa.ada_profile_mfma_probe(n_cu, 2000, device=dev, stream=stream)
        torch.cuda.synchronize()
        pa.ada_profile_enable(True)
        probe_flops = sum(pa.ada_profile_mfma_probe(n_cu, 20000, device=dev, stream=stream) for _ in range(3))
        torch.cuda.synchronize()
        kp = pa.ada_profile_collect()
        pa.ada_profile_enable(False)
        mfma_sustained = probe_flops / (1e-3 * kp["mfma_probe"]["ms"]) / 1e12
        result["mfma_sustained_tflops"] = mfma_sustained

        result["full_select"] = {"layers_per_s": L * n_full / full_elapsed,
                                 "roofline": {"bound": "mfma", "kernel": "k_gram_dma (full lower-triangular Gram)",
                                              "achieved": tri_flops / (1e-6 * full_us) / 1e12,
                                              "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                              "frac": tri_flops / (1e-6 * full_us) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                                              "frac_of_sustained": tri_flops / (1e-6 * full_us) / 1e12 / mfma_sustained,
                                              "avg_launch_us": full_us, "flops_per_launch": tri_flops,
                                              "traffic": recorded_traffic("gram_full_c%d_pmc.txt" % args.config)},
                                 "mean_jaccard_independent": sum(jac) / len(jac)}

        # ---- nearest-representative assignment (Section 2.3) for the last layer's set: T x r products, arg max
        last = out["idx"][L - 1]
        for _ in range(2):
            pa.ada_assign_nearest(xs[L - 1], last, r=T, r_dev=out["counts"][L - 1], ws=ws, stream=stream)
        torch.cuda.synchronize()
        pa.ada_profile_enable(True)
        for l in range(L):                                   # rotate over the layer buffers: operands come from HBM
            pa.ada_assign_nearest(xs[l], last, r=T, r_dev=out["counts"][L - 1], ws=ws, stream=stream)
        torch.cuda.synchronize()
        ka = pa.ada_profile_collect()
        pa.ada_profile_enable(False)
        us_a = 1e3 * ka["assign"]["ms"] / ka["assign"]["launches"]
        result["assign_nearest"] = {"avg_launch_us": us_a, "r": r_per_layer[L - 1],
                                    "roofline": {"bound": "hbm", "kernel": "k_cascade_fused (arg-max epilogue)",
                                                 "achieved": layer_bytes / (1e-6 * us_a) / 1e9, "peak": HBM_PEAK_GBS,
                                                 "unit": "GB/s", "frac": layer_bytes / (1e-6 * us_a) / 1e9 / HBM_PEAK_GBS,
                                                 "bytes_per_launch": layer_bytes,
                                                 "traffic": recorded_traffic("assign_c%d_pmc.txt" % args.config)}}

        # ---- attention on the representative set (eq. (1)) for the last layer's set, 16 heads of d/16, with the
        # hand-over to all T tokens; synthetic Q, K, V
        # two side streams for everything below that overlaps work (a process has few hardware queues: streams beyond
        # them share one and serialise, so the same two are used throughout)
        side = [torch.cuda.Stream() for _ in range(2)]
        Hh = 16
        if d % Hh == 0 and d // Hh in ((64, 128, 256) if w.dtype == "bf16" else (64, 128)):
            qd, kd, vd = (m.to(dev) for m in wl.qkv(w, Hh))
            near = pa.ada_assign_nearest(xs[L - 1], last, r=T, r_dev=out["counts"][L - 1], ws=ws, stream=stream)
            for _ in range(2):
                pa.ada_attention_compressed(qd, kd, vd, Hh, last, near["assign"], r=T, r_dev=out["counts"][L - 1], ws=ws,
                                            stream=stream)
            torch.cuda.synchronize()
            pa.ada_profile_enable(True)
            for _ in range(10):
                att = pa.ada_attention_compressed(qd, kd, vd, Hh, last, near["assign"], r=T, r_dev=out["counts"][L - 1],
                                                  ws=ws, stream=stream)
            torch.cuda.synchronize()
            kt = pa.ada_profile_collect()
            pa.ada_profile_enable(False)
            assert att["info"].cpu().tolist()[3] == 0
            us_t = 1e3 * kt["attn"]["ms"] / kt["attn"]["launches"]
            r_last = r_per_layer[L - 1]
            att_bytes = 3 * r_last * d * esz + T * d * 4       # gathered Q, K, V rows in, fp32 rows out
            att_flops = 4.0 * r_last * r_last * d              # two r x r x d_h products per head
            result["attention_compressed"] = {
                "avg_launch_us": us_t, "r": r_last, "heads": Hh, "d_h": d // Hh,
                "roofline": {"bound": "hbm", "kernel": "k_attn_rep2 (eq. (1) + hand-over)",
                             "achieved": att_bytes / (1e-6 * us_t) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": att_bytes / (1e-6 * us_t) / 1e9 / HBM_PEAK_GBS, "bytes_per_launch": att_bytes,
                             "mfma_tflops": att_flops / (1e-6 * us_t) / 1e12,
                             "traffic": recorded_traffic("attention_c%d_pmc.txt" % args.config)}}

            # ---- every layer: selection, assignment, attention on the representative set (Section 8.4's pipeline).
            # The same synthetic Q, K, V serve all layers; the selection runs on its own stream beside the attention.
            wsp = pa.workspace_batched(T, 2, dev)
            two = side
            pipe = {}
            for name, sa, sb in (("one_stream", None, None), ("two_streams", two[0], two[1])):
                po = None
                for _ in range(2):
                    po = pa.ada_pipeline_layers(xs, [qd] * L, [kd] * L, [vd] * L, Hh, w.tau, ws=wsp, stream_sel=sa,
                                                stream_attn=sb, stream=stream, out=po)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                npipe = max(1, args.steps // 4)
                for _ in range(npipe):
                    pa.ada_pipeline_layers(xs, [qd] * L, [kd] * L, [vd] * L, Hh, w.tau, ws=wsp, stream_sel=sa,
                                           stream_attn=sb, stream=stream, out=po)
                torch.cuda.synchronize()
                pipe[name] = {"ms_per_pass": 1e3 * (time.perf_counter() - t0) / npipe}
                pi = po["info"].cpu()
                assert pi[:, 3].tolist() == [0] * L and pi[:, 7].tolist() == [0] * L, "pipeline reported an error"
                assert torch.equal(po["counts"], out["counts"]), "pipeline sets differ from the layer loop's"
            pipe["us_per_layer_two_streams"] = 1e3 * pipe["two_streams"]["ms_per_pass"] / L
            result["pipeline_select_assign_attend"] = pipe
            del wsp, po

        # ---- four independent sequences of this workload through the batched layer loop (the sequences alternate
        # between two streams, so that one sequence's set update overlaps the other's tiles)
        Bq = 4
        seqs = [xs] + [[x.to(dev) for x in wl.layers(w, b)] for b in range(1, Bq)]
        wsb = pa.workspace_batched(T, Bq, dev)
        outb = dict(idx=torch.empty((Bq, L, T), dtype=torch.int32, device=dev),
                    counts=torch.empty((Bq, L, 4), dtype=torch.int32, device=dev),
                    gram_ops=torch.empty((Bq, L), dtype=torch.int64, device=dev))
        use = [side[b % 2] for b in range(Bq)]
        for _ in range(2):
            pa.ada_cascade_layers_batched(seqs, w.tau, ws=wsb, streams=use, stream=stream, out=outb)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        nb = max(1, args.steps // 4)
        for _ in range(nb):
            pa.ada_cascade_layers_batched(seqs, w.tau, ws=wsb, streams=use, stream=stream, out=outb)
        torch.cuda.synchronize()
        b_elapsed = time.perf_counter() - t0
        assert outb["counts"][:, :, 3].cpu().flatten().tolist() == [0] * (Bq * L), "batched pass reported an error"
        assert torch.equal(outb["counts"][0], out["counts"]), "batched sequence 0 differs from the single-sequence pass"
        result["batched"] = {"sequences": Bq, "streams": 2, "ms_per_batch_pass": 1e3 * b_elapsed / nb,
                             "layers_per_s": Bq * L * nb / b_elapsed,
                             "tokens_per_s": Bq * L * nb / b_elapsed * T}
        # ---- the same four sequences stacked in one [B, T, d] tensor per layer: one launch per cascade step serves
        # all of them (ada_cascade_layers_grouped)
        xg = [torch.stack([seqs[b][l] for b in range(Bq)]) for l in range(L)]
        del seqs
        for _ in range(2):
            pa.ada_cascade_layers_grouped(xg, w.tau, ws=wsb, stream=stream, out=outb)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(nb):
            pa.ada_cascade_layers_grouped(xg, w.tau, ws=wsb, stream=stream, out=outb)
        torch.cuda.synchronize()
        g_elapsed = time.perf_counter() - t0
        assert torch.equal(outb["counts"][0], out["counts"]), "grouped sequence 0 differs from the single-sequence pass"
        pa.ada_profile_enable(True)
        pa.ada_cascade_layers_grouped(xg, w.tau, ws=wsb, stream=stream, out=outb)
        torch.cuda.synchronize()
        kg = pa.ada_profile_collect()
        pa.ada_profile_enable(False)
        result["batched"]["stacked_one_launch_per_step"] = {
            "ms_per_batch_pass": 1e3 * g_elapsed / nb, "layers_per_s": Bq * L * nb / g_elapsed,
            "tokens_per_s": Bq * L * nb / g_elapsed * T,
            "cascade_launch_us": 1e3 * kg["cascade_fused"]["ms"] / kg["cascade_fused"]["launches"]}
        del xg
        # ---- sixteen stacked sequences (four layers each): the regime in which a launch's fixed chain of memory round
        # trips is shared by enough tiles to matter little, i.e. what the tile engine itself sustains
        B16, L16 = 16, 4
        per16 = [list(wl.layers(w, b, L16)) for b in range(B16)]
        x16 = [torch.stack([per16[b][l] for b in range(B16)]).to(dev) for l in range(L16)]
        del per16
        ws16 = pa.workspace_batched(T, B16, dev)
        o16 = None
        for _ in range(2):
            o16 = pa.ada_cascade_layers_grouped(x16, w.tau, ws=ws16, stream=stream, out=o16)
        torch.cuda.synchronize()
        pa.ada_profile_enable(True)
        for _ in range(5):
            pa.ada_cascade_layers_grouped(x16, w.tau, ws=ws16, stream=stream, out=o16)
        torch.cuda.synchronize()
        k16 = pa.ada_profile_collect()
        pa.ada_profile_enable(False)
        us16 = 1e3 * k16["cascade_fused"]["ms"] / k16["cascade_fused"]["launches"]
        r16 = float(o16["counts"][:, :-1, 0].float().mean())
        result["batched"]["stacked_16_sequences"] = {
            "sequences": B16, "layers": L16, "cascade_launch_us": us16, "us_per_layer_and_sequence": us16 / B16,
            "roofline": {"bound": "hbm", "kernel": "k_cascade_fused (16 problems per launch)",
                         "achieved": B16 * layer_bytes / (1e-6 * us16) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": B16 * layer_bytes / (1e-6 * us16) / 1e9 / HBM_PEAK_GBS,
                         "bytes_per_launch": B16 * layer_bytes,
                         "mfma_frac": B16 * 2.0 * d * T * r16 / (1e-6 * us16) / 1e12 / MFMA_BF16_PEAK_TFLOPS}}
        del x16, ws16, o16
        # ---- a representative set per head (Section 8.5): the H column blocks of X as H problems in one launch
        Hh = 16 if d % 16 == 0 else 1
        hv = [pa.heads_view(x, Hh) for x in xs]
        wsh = pa.workspace_batched(T, Hh, dev)
        outh = dict(idx=torch.empty((Hh, L, T), dtype=torch.int32, device=dev),
                    counts=torch.empty((Hh, L, 4), dtype=torch.int32, device=dev),
                    gram_ops=torch.empty((Hh, L), dtype=torch.int64, device=dev))
        for _ in range(2):
            pa.ada_cascade_layers_grouped(hv, w.tau, ws=wsh, stream=stream, out=outh)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(nb):
            pa.ada_cascade_layers_grouped(hv, w.tau, ws=wsh, stream=stream, out=outh)
        torch.cuda.synchronize()
        h_elapsed = time.perf_counter() - t0
        pa.ada_profile_enable(True)
        pa.ada_cascade_layers_grouped(hv, w.tau, ws=wsh, stream=stream, out=outh)
        torch.cuda.synchronize()
        kh = pa.ada_profile_collect()
        pa.ada_profile_enable(False)
        ch = outh["counts"].cpu()
        assert ch[:, :, 3].flatten().tolist() == [0] * (Hh * L), "per-head pass reported an error"
        result["per_head"] = {"heads": Hh, "d_h": d // Hh, "ms_per_pass": 1e3 * h_elapsed / nb,
                              "layers_per_s": L * nb / h_elapsed,
                              "cascade_launch_us_all_heads": 1e3 * kh["cascade_fused"]["ms"] / kh["cascade_fused"]["launches"],
                              "mean_r_h": float(ch[:, 1:, 0].float().mean())}
        del wsb, outb, hv, wsh, outh

        # ---- the cascade step at the two other d=4096 shapes (first six layers of configs[3] and configs[4]), where
        # the wider tiles take over: 64 x 128 at r ~ 920, 128 x 128 at T = 8192
        other = {}
        for ci in (3, 4):
            if ci == args.config:
                continue
            wo = wl.config(ci)
            xo = [x.to(dev) for x in wl.layers(wo, 0, 6)]
            wso = pa.workspace(wo.T, dev)
            for _ in range(2):
                oo = pa.ada_cascade_layers(xo, wo.tau, ws=wso, stream=stream, want_lists=False)
            torch.cuda.synchronize()
            pa.ada_profile_enable(True)
            for _ in range(5):
                oo = pa.ada_cascade_layers(xo, wo.tau, ws=wso, stream=stream, want_lists=False)
            torch.cuda.synchronize()
            ko = pa.ada_profile_collect()
            pa.ada_profile_enable(False)
            us_o = 1e3 * ko["cascade_fused"]["ms"] / ko["cascade_fused"]["launches"]
            by = wo.T * wo.d * (2 if wo.dtype == "bf16" else 4)
            r_in = float(oo["counts"][:-1, 0].float().mean())         # the sets the timed steps inherited
            fl = 2.0 * wo.d * wo.T * r_in                             # T x r Gram entries of eq. (6), 2 d flops each
            other[wo.name] = {"T": wo.T, "d": wo.d, "mean_r": float(oo["counts"][1:, 0].float().mean()),
                              "mean_r_inherited": r_in, "cascade_launch_us": us_o,
                              "hbm_frac": by / (1e-6 * us_o) / 1e9 / HBM_PEAK_GBS,
                              "mfma_tflops": fl / (1e-6 * us_o) / 1e12,
                              "mfma_frac": fl / (1e-6 * us_o) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                              "bound": "mfma" if fl / (MFMA_BF16_PEAK_TFLOPS * 1e12) > by / (HBM_PEAK_GBS * 1e9) else "hbm",
                              "traffic": recorded_traffic("cascade_fused_c%d_pmc.txt" % ci)}
            del xo, wso, oo
        # configs[4] as the configuration states it: a batch of four sequences, here stacked in one tensor with one
        # launch per step for all four (three layers of each)
        if args.config != 4:
            w4b = wl.config(4)
            B4, L4 = 4, 5
            per4 = [list(wl.layers(w4b, b, L4)) for b in range(B4)]
            x4g = [torch.stack([per4[b][l] for b in range(B4)]).to(dev) for l in range(L4)]
            del per4
            ws4g = pa.workspace_batched(w4b.T, B4, dev)
            o4 = None
            for _ in range(2):
                o4 = pa.ada_cascade_layers_grouped(x4g, w4b.tau, ws=ws4g, stream=stream, want_lists=False, out=o4)
            torch.cuda.synchronize()
            pa.ada_profile_enable(True)
            for _ in range(4):
                pa.ada_cascade_layers_grouped(x4g, w4b.tau, ws=ws4g, stream=stream, want_lists=False, out=o4)
            torch.cuda.synchronize()
            k4g = pa.ada_profile_collect()
            pa.ada_profile_enable(False)
            us_g = 1e3 * k4g["cascade_fused"]["ms"] / k4g["cascade_fused"]["launches"]
            by4 = B4 * w4b.T * w4b.d * 2
            r4 = float(o4["counts"][:, :-1, 0].float().mean())
            fl4 = 2.0 * w4b.d * w4b.T * r4 * B4
            other[w4b.name + "_batch4_stacked"] = {"T": w4b.T, "d": w4b.d, "sequences": B4,
                                                   "mean_r": float(o4["counts"][:, 1:, 0].float().mean()),
                                                   "cascade_launch_us": us_g, "us_per_layer_and_sequence": us_g / B4,
                                                   "hbm_frac": by4 / (1e-6 * us_g) / 1e9 / HBM_PEAK_GBS,
                                                   "mfma_frac": fl4 / (1e-6 * us_g) / 1e12 / MFMA_BF16_PEAK_TFLOPS}
            # the configuration's own schedule on these layers: the cascade at every layer, and the full T x T selection
            # of all four sequences at layer 0 and at every 8th layer (here: layers 0 and L4 - 1 stand for 0 and 8)
            m4 = torch.empty((B4, w4b.T), dtype=torch.uint8, device=dev)
            i4 = torch.empty((B4, w4b.T), dtype=torch.int32, device=dev)
            c4 = torch.empty((B4, 4), dtype=torch.int32, device=dev)

            def schedule_pass():
                pa.ada_cascade_layers_grouped(x4g, w4b.tau, ws=ws4g, stream=stream, want_lists=False, out=o4)
                pa.ada_select_full_grouped(x4g[L4 - 1], w4b.tau, ws=ws4g, stream=stream,
                                           out=dict(mask=m4, idx=i4, counts=c4))
            schedule_pass()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(3):
                schedule_pass()
            torch.cuda.synchronize()
            sched_ms = 1e3 * (time.perf_counter() - t0) / 3
            other[w4b.name + "_schedule"] = {
                "what": "four stacked sequences: full selection at layer 0, cascade at layers 1..%d, full selection "
                        "again at the last of them (the configuration repeats this every 8 layers)" % (L4 - 1),
                "layers": L4, "sequences": B4, "ms_per_pass": sched_ms,
                "layers_per_s": B4 * L4 / (1e-3 * sched_ms), "tokens_per_s": B4 * L4 * w4b.T / (1e-3 * sched_ms)}
            del x4g, ws4g, o4
        result["cascade_other_shapes"] = other

        # ---- the greedy covering of Section 2.5 on layer 0 (pair bits from the register-staged Gram tiles, then the
        # sequential resolution by one workgroup)
        if T <= 16384:
            for _ in range(2):
                gsel = pa.ada_select_full(xs[0], w.tau, ws=ws, stream=stream, flags=pa.FLAG_GREEDY_COVER)
            torch.cuda.synchronize()
            pa.ada_profile_enable(True)
            for _ in range(5):
                gsel = pa.ada_select_full(xs[0], w.tau, ws=ws, stream=stream, flags=pa.FLAG_GREEDY_COVER)
            torch.cuda.synchronize()
            kgr = pa.ada_profile_collect()
            pa.ada_profile_enable(False)
            result["greedy_cover"] = {"r": int(gsel["counts"][0]),
                                      "gram_us": 1e3 * kgr["gram_full"]["ms"] / kgr["gram_full"]["launches"],
                                      "resolve_us": 1e3 * kgr["update"]["ms"] / kgr["update"]["launches"]}

        # ---- the same selection at the long-context shape (configs[4]: T=8192, d=4096, one sequence), where the
        # triangle has enough tiles to fill the chip and the kernel is bound by the matrix pipes
        w4 = wl.config(4)
        x4 = next(iter(wl.layers(w4, 0, 1))).to(dev)
        ws4 = pa.workspace(w4.T, dev)
        for _ in range(2):
            pa.ada_select_full(x4, w4.tau, ws=ws4, stream=stream)
        torch.cuda.synchronize()
        pa.ada_profile_enable(True)
        for _ in range(5):
            pa.ada_select_full(x4, w4.tau, ws=ws4, stream=stream)
        torch.cuda.synchronize()
        k4 = pa.ada_profile_collect()
        pa.ada_profile_enable(False)
        us4 = 1e3 * k4["gram_full"]["ms"] / k4["gram_full"]["launches"]
        flops4 = float(w4.T) * (w4.T - 1) * w4.d
        result["full_select_long"] = {"workload": "%s layer 0: T=%d d=%d %s, one sequence" % (w4.name, w4.T, w4.d, w4.dtype),
                                      "roofline": {"bound": "mfma", "kernel": "k_gram_dma (full lower-triangular Gram)",
                                                   "achieved": flops4 / (1e-6 * us4) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
                                                   "unit": "TFLOP/s", "frac": flops4 / (1e-6 * us4) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                                                   "frac_of_sustained": flops4 / (1e-6 * us4) / 1e12 / mfma_sustained,
                                                   "avg_launch_us": us4, "flops_per_launch": flops4,
                                                   "traffic": recorded_traffic("gram_full_c4_pmc.txt")}}

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, xs_cpu)

    print(json.dumps(result))


if __name__ == "__main__":
    main()
