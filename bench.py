#!/usr/bin/env python3
"""Benchmark of the H-BitLinear forward path on one MI355X.

A step = one pass of the whole hot path over one batch: the FWHT+quantiser launch
(Eq. 3-6) followed by the ternary-GEMM+dequant launch (Eq. 7) - exactly the two
launches hbl_hbitlinear_forward() makes - on the 7B-shaped prefill W_down site:
X bf16 [8192 x 16384] -> 4096, INT4 activations (configuration 4, the shape the
target "% of INT8 MFMA peak" is quoted on).  Inputs are resident in HBM before
the timed region, which is K calls of hbl_hbitlinear_forward after W warm-up calls.
One JSON line is printed; it also carries the roofline of the dominant kernel (the
GEMM; per-kernel durations come from K more calls of the same public function, every
launch timed by an event pair of its own through hbl_trace_begin / hbl_trace_end), the
other prefill configurations, the oracle timed on the host cores on a bounded sample,
and the batched-decode layer figures (configuration 5).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0   # MI355X published dense int8 (5.0 POP/s)
F6F4_MFMA_PEAK_TOPS = 10100.0  # MI355X published dense fp6 / fp4 (10.1 PFLOP/s)
HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--site", default="wdown_7b", choices=["wdown_7b", "wo_7b"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--decode-layers", type=int, default=24)
    return ap.parse_args()


def setup_site(hbl, synth, torch, site, eps):
    """Weights: draw -> ternarise per scale group -> pack (all on the GPU path)."""
    W = synth.make_w(site)
    rows = site.N // site.groups
    codes, alphas = [], []
    for g in range(site.groups):
        c, a = hbl.ternarize_weights_absmean(torch.from_numpy(W[g * rows:(g + 1) * rows]).cuda(), eps)
        codes.append(c)
        alphas.append(a)
    packed = hbl.pack_ternary_2bit(torch.cat(codes, 0).contiguous())
    return packed, torch.cat(alphas).contiguous(), W


def to_dev(torch, np, x):
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(x).cuda()


def timed_calls(torch, fn, steps, warmup):
    """ms per call of fn(): `warmup` untimed calls, then `steps` calls bracketed by synchronisation."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def wake_device(torch, fn, seconds=0.06):
    """An idle MI355X takes ~25 ms of work to reach its steady clocks (measured on this workload: 0.66, 0.37,
    0.35, 0.34, 0.335 ms per call over the first five groups of 20 calls, 0.333 from there on).  Untimed calls of
    fn() for `seconds`, ahead of the contract's warm-up steps, so that the timed steps see the steady state the
    kernels run in when the GPU is busy."""
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(10):
            fn()
        torch.cuda.synchronize()


def traced_calls(torch, hbl, fn, steps):
    """Per-kernel durations of `steps` more calls of fn(): every launch carries its own start / stop event pair
    (hbl_trace_begin / hbl_trace_end: the dispatch's device timestamps, no marker packets between the kernels),
    so the launches overlap their dispatch with the previous kernel as in the untraced loop.
    -> {kernel name: mean ms per launch}, launches per call."""
    torch.cuda.synchronize()
    with hbl.trace(16 * steps) as tr:
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
    names = sorted({n for n, _ in tr.launches})
    return {n: tr.mean_ms(n) for n in names}, tr.seen / steps


def bench_prefill(args, hbl, synth, torch, np):
    site = {s.name: s for s in synth.config_sites(4)}[args.site]
    T, K, N, bits, eps = site.T, site.K, site.N, 4, hbl.EPS
    x_host = synth.make_x(site)
    x = to_dev(torch, np, x_host)
    packed, alphas, W_host = setup_site(hbl, synth, torch, site, eps)
    y = torch.empty((T, N), dtype=torch.bfloat16, device="cuda")
    ws = hbl.alloc_workspace(T, K, N, bits)

    def step():
        hbl.hbitlinear_forward(x, packed, N, alphas, bits, eps, y=y, workspace=ws)

    # THE timed region: K calls of the public function after W warm-up calls, bracketed by synchronisation
    wake_device(torch, step)
    ms_per_step = timed_calls(torch, step, args.steps, args.warmup)
    # the same K calls once more with every launch timed by its own event pair: the per-kernel durations
    kernel_ms, launches_per_step = traced_calls(torch, hbl, step, args.steps)

    # INT8 activations (the paper's first training stage) on the same site: int8 matrix cores, byte codes
    ms_int8 = timed_calls(torch, lambda: hbl.hbitlinear_forward(x, packed, N, alphas, 8, eps, y=y, workspace=ws),
                          args.steps, 3)
    # INT4 activations kept on the int8 matrix cores (codes + 8 in bytes) through the stage-level calls: what the
    # fp6 x fp4 path is measured against
    codes = torch.empty((T, K), dtype=torch.int8, device="cuda")
    sd = torch.empty(T, dtype=torch.float32, device="cuda")
    cs = torch.empty(T, dtype=torch.int32, device="cuda")

    def step_int8_cores():
        hbl.fwht_quant_into(x, bits, site.hadamard, codes, sd, cs, eps, code_offset=hbl.CODES_UINT4_PLUS8)
        hbl.gemm_dequant_bf16(codes, sd, cs, packed, N, alphas, y=y, code_offset=hbl.CODES_UINT4_PLUS8)

    ms_i8cores = timed_calls(torch, step_int8_cores, args.steps, 3)
    i8_kernel_ms, _ = traced_calls(torch, hbl, step_int8_cores, args.steps)
    del codes

    ops = 2.0 * T * K * N
    t_gemm = kernel_ms.get("ternary_gemm_f6f4_kernel", float("nan"))
    t_quant = kernel_ms.get("fwht_quant_bigrow_kernel", float("nan"))
    out = {
        "T": T, "K": K, "N": N, "ms_per_step": ms_per_step, "kernel_ms": kernel_ms,
        "launches_per_step": launches_per_step, "ms_fwht_quant": t_quant, "ms_gemm": t_gemm,
        "tops_end_to_end": ops / (ms_per_step * 1e-3) / 1e12,
        "tops_gemm": ops / (t_gemm * 1e-3) / 1e12,
        # bytes the quantiser launch moves: bf16 in, code records out (0.75 byte per feature + padding, as stored), scales
        "fwht_quant_bytes": 2.0 * T * K + hbl.code_bytes(T, K, hbl.CODES_BF6) + 4.0 * T,
        "int8_activations": {"ms_per_step": ms_int8, "TOPS": ops / (ms_int8 * 1e-3) / 1e12,
                             "frac_int8_mfma_peak": ops / (ms_int8 * 1e-3) / 1e12 / INT8_MFMA_PEAK_TOPS},
        "int4_on_int8_cores": {"ms_per_step": ms_i8cores, "TOPS": ops / (ms_i8cores * 1e-3) / 1e12,
                               "frac_int8_mfma_peak": ops / (ms_i8cores * 1e-3) / 1e12 / INT8_MFMA_PEAK_TOPS,
                               "kernel_ms": i8_kernel_ms,
                               "note": "stage-level calls with HBL_CODES_UINT4_PLUS8: same results, int8 MFMA"},
    }
    out["fwht_quant_gbs"] = out["fwht_quant_bytes"] / (t_quant * 1e-3) / 1e9
    return out, site, x_host, W_host


def bench_other_prefill_configs(args, hbl, synth, torch, np):
    """Whole forward call (both launches) on the other prefill configurations: 2 (INT4 and INT8), 3 and the
    W_o site of 4 - with the input recipe of each configuration."""
    eps, out = hbl.EPS, {}
    cases = [("config2_wo_1p3b_int4", synth.config_sites(2)[0], 4), ("config2_wo_1p3b_int8", synth.config_sites(2)[0], 8),
             ("config3_wdown_3b_int4", synth.config_sites(3)[0], 4), ("config4_wo_7b_int4", synth.config_sites(4)[0], 4)]
    for name, site, bits in cases:
        x = to_dev(torch, np, synth.make_x(site))
        packed, alphas, _ = setup_site(hbl, synth, torch, site, eps)
        y = torch.empty((site.T, site.N), dtype=torch.bfloat16, device="cuda")
        ws = hbl.alloc_workspace(site.T, site.K, site.N, bits)

        def step():
            hbl.hbitlinear_forward(x, packed, site.N, alphas, bits, eps, y=y, workspace=ws)

        wake_device(torch, step, 0.03)
        ms = timed_calls(torch, step, args.steps, args.warmup)
        kernel_ms, _ = traced_calls(torch, hbl, step, args.steps)
        ops = 2.0 * site.T * site.K * site.N
        out[name] = {"T": site.T, "K": site.K, "N": site.N, "bits": bits, "ms_per_step": ms,
                     "TOPS": ops / (ms * 1e-3) / 1e12, "frac_int8_mfma_peak": ops / (ms * 1e-3) / 1e12 / INT8_MFMA_PEAK_TOPS,
                     "kernel_ms": kernel_ms}
        del x, packed, y, ws
        torch.cuda.empty_cache()
    return out


def cpu_baseline(site, x_host, W_host, synth, np, budget_s=15.0):
    """The oracle as it stands, on a bounded sample of token rows of the same workload."""
    from oracle import hbl_oracle as O
    wc, alpha = O.ternarize_weights_absmean(W_host, 1e-5)
    rows = min(site.T, 4 * O.num_threads())   # probe: a few rows per thread, so that the estimate sees every core busy
    t0 = time.perf_counter()
    O.bitlinear_forward(np.ascontiguousarray(x_host[:rows]), wc, alpha, 4, site.hadamard, 1e-5)
    dt = time.perf_counter() - t0
    rows2 = int(max(rows, min(site.T, rows * budget_s / max(dt, 1e-3))))
    rows2 = min(site.T, max(O.num_threads(), rows2 // O.num_threads() * O.num_threads()))
    t0 = time.perf_counter()
    O.bitlinear_forward(np.ascontiguousarray(x_host[:rows2]), wc, alpha, 4, site.hadamard, 1e-5)
    dt = time.perf_counter() - t0
    t0 = time.perf_counter()
    O.fwht_quant(np.ascontiguousarray(x_host[:rows2]), 4, hadamard=site.hadamard, eps=1e-5)
    dt_quant = time.perf_counter() - t0   # the front end alone, on the same rows (not part of `value`)
    return {
        "value": 2.0 * rows2 * site.K * site.N / dt / 1e12, "unit": "TOPS", "cores": O.num_threads(),
        "kind": "oracle", "seconds": dt, "seconds_fwht_quant": dt_quant, "seconds_gemm_dequant": max(dt - dt_quant, 0.0),
        "sample": f"first {rows2} of {site.T} token rows of the same X, all {site.N} outputs "
                  f"(FWHT + INT4 quantiser + int32 GEMM + bf16 dequant)",
    }


def bench_prefill_layer(args, hbl, synth, torch, np):
    """All four projections of the 7B layer at the prefill batch (T = 8192): the two H-BitLinear sites of
    configuration 4 plus the plain QKV and up/gate projections with configuration 5's shapes."""
    T, bits, eps = 8192, 4, hbl.EPS
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    out, total_ms, total_ops = {}, 0.0, 0.0
    for s in synth.config_sites(5, batch=T):
        x = torch.randn((T, s.K), device="cuda", generator=g).to(torch.bfloat16)
        c = torch.randint(-1, 2, (s.N, s.K), dtype=torch.int8, device="cuda", generator=g)
        packed = hbl.pack_ternary_2bit(c)
        del c
        al = torch.full((s.groups,), 0.016, dtype=torch.float32, device="cuda")
        y = torch.empty((T, s.N), dtype=torch.bfloat16, device="cuda")
        ws = hbl.alloc_workspace(T, s.K, s.N, bits)
        fn = hbl.hbitlinear_forward if s.hadamard else hbl.plain_bitlinear_forward
        wake_device(torch, lambda: fn(x, packed, s.N, al, bits, eps, y=y, workspace=ws), 0.03)
        ms = timed_calls(torch, lambda: fn(x, packed, s.N, al, bits, eps, y=y, workspace=ws), 10, 3)
        ops = 2.0 * T * s.K * s.N
        out[s.name.replace("dec_", "")] = {"K": s.K, "N": s.N, "hadamard": s.hadamard, "ms": ms,
                                           "TOPS": ops / (ms * 1e-3) / 1e12}
        total_ms += ms
        total_ops += ops
        del x, packed, y, ws
    out["layer"] = {"ms": total_ms, "TOPS": total_ops / (total_ms * 1e-3) / 1e12,
                    "frac_int8_mfma_peak": total_ops / (total_ms * 1e-3) / 1e12 / INT8_MFMA_PEAK_TOPS}
    return out


def bench_decode(args, hbl, synth, torch, np):
    """Configuration 5: one 7B decoder layer's four projections, weights cycled over `layers`
    independent copies (1.6 GB at 24) so that they stream from HBM rather than from cache."""
    eps, bits = hbl.EPS, 4
    layers = args.decode_layers
    base = synth.config_sites(5, batch=64)
    # independent packed weights per layer: drawn once on the GPU (uniform ternary codes are enough
    # for timing: the kernels' work does not depend on the weight values)
    g = torch.Generator(device="cuda")
    g.manual_seed(4)
    packed = []
    for _ in range(layers):
        per = []
        for s in base:
            c = torch.randint(-1, 2, (s.N, s.K), dtype=torch.int8, device="cuda", generator=g)
            per.append(hbl.pack_ternary_2bit(c))
            del c
        packed.append(per)
    alphas = [torch.full((s.groups,), 0.016, dtype=torch.float32, device="cuda") for s in base]
    w_bytes = sum(s.N * s.K // 4 + 4 * s.N for s in base)   # the 2-bit form a decode call streams, + row sums
    res = {}
    for B in (1, 8, 32, 64):
        sites = synth.config_sites(5, batch=B)
        xs = [to_dev(torch, np, synth.make_x(s)) for s in sites]
        ys = [torch.empty((B, s.N), dtype=torch.bfloat16, device="cuda") for s in sites]
        wss = [hbl.alloc_workspace(B, s.K, s.N, bits) for s in sites]
        # grouped form: the four projections of a layer (independent inputs here) in one call
        items = [[(xs[i], packed[l][i], s.N, alphas[i], bits, s.hadamard, ys[i]) for i, s in enumerate(sites)]
                 for l in range(layers)]
        probs = [hbl.make_problems(it) for it in items]
        gws = torch.empty(hbl.grouped_workspace_bytes(probs[0], len(sites)), dtype=torch.uint8, device="cuda")

        def layer_sequential(l):
            for i, s in enumerate(sites):
                fn = hbl.hbitlinear_forward if s.hadamard else hbl.plain_bitlinear_forward
                fn(xs[i], packed[l][i], s.N, alphas[i], bits, eps, y=ys[i], workspace=wss[i])

        def layer_grouped(l):
            hbl.bitlinear_forward_grouped(items[l], eps, workspace=gws, problems=probs[l])

        io_bytes = sum(2 * B * s.K + 2 * B * s.N for s in sites)
        entry = {}
        y_first = None
        for mode, layer in (("sequential", layer_sequential), ("grouped", layer_grouped)):
            for l in range(layers):
                layer(l)
            torch.cuda.synchronize()
            # one HIP graph of all layers (kernel nodes only, no memset nodes), replayed
            graph = torch.cuda.CUDAGraph()
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                with torch.cuda.graph(graph, stream=side):
                    for l in range(layers):
                        layer(l)
            torch.cuda.synchronize()
            y_eager = [y.clone() for y in ys]
            graph.replay()
            torch.cuda.synchronize()
            assert all(torch.equal(a.view(torch.int16), b.view(torch.int16)) for a, b in zip(y_eager, ys)), \
                "graph replay differs from eager"
            if y_first is None:
                y_first = y_eager
            else:   # both forms end on the last layer's weights: identical outputs
                assert all(torch.equal(a.view(torch.int16), b.view(torch.int16)) for a, b in zip(y_first, ys)), \
                    "grouped call differs from the per-projection calls"
            reps = 5
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                graph.replay()
            e1.record()
            torch.cuda.synchronize()
            us_layer = e0.elapsed_time(e1) * 1e3 / (reps * layers)
            e0.record()
            for l in range(layers):
                layer(l)
            e1.record()
            torch.cuda.synchronize()
            us_layer_eager = e0.elapsed_time(e1) * 1e3 / layers
            gbs = (w_bytes + io_bytes) / (us_layer * 1e-6) / 1e9
            entry[mode] = {"us_per_layer": us_layer, "us_per_layer_eager": us_layer_eager, "GBps": gbs,
                           "frac_hbm_peak": gbs / HBM_PEAK_GBS}
        # each projection by itself (one forward call per layer's weights)
        per_site = {}
        for i, s in enumerate(sites):
            fn = hbl.hbitlinear_forward if s.hadamard else hbl.plain_bitlinear_forward

            def one_site():
                for l in range(layers):
                    fn(xs[i], packed[l][i], s.N, alphas[i], bits, eps, y=ys[i], workspace=wss[i])

            one_site()
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                with torch.cuda.graph(graph, stream=side):
                    one_site()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(5):
                graph.replay()
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / (5 * layers)
            nbytes = s.N * s.K // 4 + 4 * s.N + 2 * B * s.K + 2 * B * s.N
            per_site[s.name] = {"us": us, "GBps": nbytes / (us * 1e-6) / 1e9}
        entry["per_projection"] = per_site
        res[str(B)] = entry
    best = max(res, key=lambda b: res[b]["grouped"]["GBps"])
    roofline = {"kernel": "quant_grouped_kernel + decode_gemm_kernel (one grouped call per layer, batch %s)" % best,
                "bound": "hbm", "achieved": res[best]["grouped"]["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": res[best]["grouped"]["GBps"] / HBM_PEAK_GBS,
                # FETCH_SIZE + WRITE_SIZE of the layer's GEMM launch at batch <= 8 (profiles/hbm_traffic_counters.txt)
                "traffic": measured_traffic("decode_gemm_kernel", "layer_7b_batch8"),
                "note": "call level: both launches of the grouped call; the GEMM launch alone streams the layer's "
                        "67.1 MB in 13-14 us (profiles/decode_layer_kernels_config5.txt)"}
    return {"layers_cycled": layers, "weight_bytes_per_layer": w_bytes, "roofline": roofline,
            "launch": "one HIP graph of all layers; sequential = four forward calls per layer in model order "
                      "(2 kernel nodes each), grouped = one hbl_bitlinear_forward_grouped call per layer "
                      "(one quantiser launch, one weight-streaming GEMM launch)",
            "batch": res}


def measured_traffic(kernel, workload):
    """HBM bytes one launch moves, from the rocprofv3 --pmc passes recorded in profiles/hbm_traffic_counters.txt
    (its `@traffic kernel workload FETCH_KIB WRITE_KIB` lines; FETCH_SIZE and WRITE_SIZE scaled by the `@scale`
    factors a copy kernel of known size gave).  Counters cannot be read from inside this process; a workload
    the passes did not cover has no figure (None)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_counters.txt")
    scale, rows = {}, {}
    try:
        with open(path) as fh:
            for line in fh:
                f = line.split()
                if len(f) == 3 and f[0] == "@scale":
                    scale[f[1]] = float(f[2])
                elif len(f) == 5 and f[0] == "@traffic":
                    rows[(f[1], f[2])] = (float(f[3]), float(f[4]))
    except OSError:
        return None
    if (kernel, workload) not in rows or "FETCH_SIZE" not in scale or "WRITE_SIZE" not in scale:
        return None
    fetch, write = rows[(kernel, workload)]
    return int(fetch * scale["FETCH_SIZE"] * 1024 + write * scale["WRITE_SIZE"] * 1024)


def bench_kv_quant(hbl, torch):
    """Per-head absmax quantiser of the attention states (Section 3.1) on the K (or V) states of the 7B prefill
    batch: 8192 tokens x 32 heads of 128, bf16 in, packed codes + one fp32 scale per head out.  HBM-bound:
    algorithmic bytes = 2 per value in, bits/8 per value + 4 per row out."""
    rows, d, nbuf = 8192 * 32, 128, 6   # six distinct 67 MB inputs: more than the 256 MB memory-side cache holds
    g = torch.Generator(device="cuda")
    g.manual_seed(11)
    xs = [torch.randn((rows, d), device="cuda", generator=g).to(torch.bfloat16) for _ in range(nbuf)]
    backs = [torch.empty_like(x) for x in xs]
    out = {"workload": f"{rows} head rows of {d} (8192 tokens x 32 heads), bf16, {nbuf} buffers in rotation"}
    for bits in (8, 4, 3):
        ps = [hbl.kv_quant_absmax(x, bits) for x in xs]
        res = {}
        for name, fn, nbytes in (
                ("quant", lambda i: hbl.kv_quant_absmax(xs[i], bits, packed=ps[i][0], scales=ps[i][1]),
                 rows * d * 2 + rows * d * bits // 8 + rows * 4),
                ("dequant", lambda i: hbl.kv_dequant(ps[i][0], ps[i][1], d, bits, out=backs[i]),
                 rows * d * bits // 8 + rows * 4 + rows * d * 2)):
            for i in range(nbuf):
                fn(i)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = 4 * nbuf
            e0.record()
            for r in range(reps):
                fn(r % nbuf)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / reps
            res[name] = {"us": us, "GBps": nbytes / us / 1e3, "frac_hbm_peak": nbytes / us / 1e3 / 8000.0}
        out[str(bits)] = res
    return out


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.stderr.write("bench.py: this build runs on ONE GPU only (the hot path is a single-GPU kernel pair; "
                         "tokens shard trivially across GPUs with no exchange). Use --gpus 1.\n")
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2504_18415_amd import hbl, synth
    hbl.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    pre, site, x_host, W_host = bench_prefill(args, hbl, synth, torch, np)
    result = {
        "metric": "H-BitLinear TOPS (INT4 acts)", "value": pre["tops_end_to_end"], "unit": "TOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": pre["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf6 x fp4 (exact small integers), fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": f"config 4 (7B prefill) {site.name}: X bf16 [{site.T}x{site.K}] -> {site.N}, "
                               f"Hadamard n={site.K}, INT4 activations, 2-bit packed ternary W",
                   "T": site.T, "K": site.K, "N": site.N, "bits": 4},
        "frac_int8_mfma_peak_end_to_end": pre["tops_end_to_end"] / INT8_MFMA_PEAK_TOPS,
        # the GEMM's own dtype sets its roofline; the benchmark's target is quoted against the int8 peak,
        # so that fraction is given too
        "roofline": {"kernel": "ternary_gemm_f6f4_kernel (fp6 x fp4 MFMA, GEMM + dequant epilogue)",
                     "bound": "mfma", "achieved": pre["tops_gemm"], "peak": F6F4_MFMA_PEAK_TOPS, "unit": "TOP/s",
                     "frac": pre["tops_gemm"] / F6F4_MFMA_PEAK_TOPS,
                     "traffic": measured_traffic("ternary_gemm_f6f4_kernel", site.name),
                     "traffic_unit": "bytes per launch (FETCH_SIZE + WRITE_SIZE, profiles/hbm_traffic_counters.txt)",
                     "algorithmic_bytes": hbl.code_bytes(site.T, site.K, hbl.CODES_BF6) + site.N * site.K // 4
                                          + 2 * site.T * site.N,
                     "avg_kernel_ms": pre["ms_gemm"],
                     "timing": "mean over the launches of K calls of the public function, each launch with an event "
                               "pair of its own (hbl_trace_begin / hbl_trace_end)",
                     "frac_of_int8_mfma_peak": pre["tops_gemm"] / INT8_MFMA_PEAK_TOPS},
        "fwht_quant": {"avg_kernel_ms": pre["ms_fwht_quant"], "bound": "hbm", "achieved": pre["fwht_quant_gbs"],
                       "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": pre["fwht_quant_gbs"] / HBM_PEAK_GBS,
                       "algorithmic_bytes": pre["fwht_quant_bytes"]},
        "kernel_ms": pre["kernel_ms"], "launches_per_step": pre["launches_per_step"],
        "int8_activations": pre["int8_activations"], "int4_on_int8_cores": pre["int4_on_int8_cores"],
    }
    if not args.no_decode:
        torch.cuda.empty_cache()
        result["other_prefill_configs"] = bench_other_prefill_configs(args, hbl, synth, torch, np)
        torch.cuda.empty_cache()
        result["prefill_layer_7b"] = bench_prefill_layer(args, hbl, synth, torch, np)
        torch.cuda.empty_cache()
        result["decode"] = bench_decode(args, hbl, synth, torch, np)
        result["kv_quant"] = bench_kv_quant(hbl, torch)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(site, x_host, W_host, synth, np)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
