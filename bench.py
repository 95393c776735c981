#!/usr/bin/env python3
"""Benchmark of the libentro hot path on one MI355X.

A step is one entro_decode_dequant pass (-> bf16) over the whole mistral-7B-shaped
8-bit weight set (32 layers x 7 linears = 224 tensors, one prepared launch), with
the compressed streams and offset tables already resident in HBM.  The same run
also times the two other sinks of the path on the same compressed set -- integer
output (entro_decode -> u8) and the fused batch-1 GEMV (entro_decode_gemv, four
launches per layer as the layer's data dependencies allow, eagerly and as one
captured HIP graph; and all products in one launch) -- and reports them as extra
fields.  The memory probe and the plain uint8 GEMV it is compared with come from
bench_kernels/ (their own shared object, not the library).  One JSON line is
printed at the end.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published peak
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "k_batch_bf16_mistral7b_pmc_hbm_bytes.txt")


def profiled_traffic():
    """(HBM bytes per launch of the headline kernel, where that number comes from): the rocprofv3 byte
    counters (FETCH_SIZE + WRITE_SIZE, scaled by a copy of known size) are taken in runs of their own,
    so this is read from the committed summary, which names the commit it was taken at; (None, None)
    when no summary is there."""
    value, commit = None, "unknown"
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch"):
                    value = int(line.split("=")[1])
                if line.startswith("commit"):
                    commit = line.split("=")[1].strip()
    except OSError:
        pass
    if value is None:
        return None, None
    return value, f"not measured in this run: copied from profiles/{os.path.basename(TRAFFIC_FILE)}, taken at commit {commit}"


def log(msg):
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--layers", type=int, default=32, help="layers of the mistral-7B-shaped set (32 = the full workload)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the u8 and GEMV legs")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the legs on configs[0..2]")
    ap.add_argument("--no-limited", action="store_true", help="skip the leg with length-limited codebooks")
    ap.add_argument("--no-compress", action="store_true", help="skip the compression kernels' leg")
    ap.add_argument("--sub-symbols", type=int, default=256,
                    help="entry points inside the segments every this many symbols (0: none)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain device copy of known size (reference for rocprofv3 --pmc byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (segments decode independently, the path needs no collectives); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synth
    import paper_2505_02380_amd as E
    from paper_2505_02380_amd.workload import prepare_config, default_threads
    import bench_kernels

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if not os.path.exists(E.library_path()):                # the library is used as built; none at all: build it
        from paper_2505_02380_amd import build as lib_build
        lib_build.build(force=True)
    E.lib()
    if not os.path.exists(bench_kernels.LIB):
        bench_kernels.build(force=True)
    bench_kernels.lib()

    # ------------------------------------------------------------------ inputs
    t0 = time.time()
    done = [0]

    def progress(i, total):
        done[0] += 1
        if done[0] % 28 == 0 or done[0] == total:
            log(f"encoded {done[0]}/{total} tensors ({time.time() - t0:.0f} s)")

    log(f"preparing mistral-7B-shaped set, {args.layers} layers, {default_threads()} host threads")
    encs = prepare_config(4, layers=args.layers, progress=progress, sub_symbols=args.sub_symbols)
    n_sym = sum(e.n for e in encs)
    stream_bytes = sum(e.stream.size for e in encs)
    offset_bytes = sum(e.offsets.size * 8 for e in encs)
    sub_bytes = sum(e.sub_bits.size * 2 for e in encs if e.sub_symbols)
    total_bits = sum(e.total_bits for e in encs)
    mean_len = total_bits / n_sym
    log(f"{n_sym} symbols, {stream_bytes / 1e9:.3f} GB compressed, mean code length {mean_len:.3f} bits, "
        f"prepared in {time.time() - t0:.0f} s")

    dts = [E.to_device(e, dev) for e in encs]
    out_bf16 = torch.empty(n_sym, dtype=torch.bfloat16, device=dev)
    views, pos = [], 0
    for e in encs:
        views.append(out_bf16[pos:pos + e.n])
        pos += e.n
    ts = [d.ctensor(v) for d, v in zip(dts, views)]
    ws = torch.zeros(E.entro_workspace_bytes(ts, E.ENTRO_OP_DEQUANT), dtype=torch.uint8, device=dev)
    plan = E.entro_plan_init(ts, E.ENTRO_OP_DEQUANT, E.ENTRO_BF16, ws)

    def timed(fn, steps, warmup):
        """(wall ms per step, event ms per step) over exactly `steps` calls after `warmup` calls."""
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        t_start = time.perf_counter()
        for a, b in ev:
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t_start) * 1e3 / steps
        return wall, sum(a.elapsed_time(b) for a, b in ev) / steps

    # ------------------------------------------------- headline: decode + dequant -> bf16
    log("timing entro_decode_dequant -> bf16")
    wall_ms, kern_ms = timed(lambda: E.entro_plan_run(plan), args.steps, args.warmup)
    out_bytes = n_sym * 2
    algo_bytes = stream_bytes + offset_bytes + out_bytes
    decoded_gbps = out_bytes / (wall_ms * 1e-3) / 1e9
    achieved = algo_bytes / (kern_ms * 1e-3) / 1e9
    log(f"dequant: {wall_ms:.3f} ms/step wall, {kern_ms:.3f} ms kernel, {achieved:.0f} GB/s algorithmic")

    # ------------------------- check against the oracle: whole tensors of every kind, sampled segments of the rest
    import oracle
    from concurrent.futures import ThreadPoolExecutor

    def oracle_symbols(e):
        return oracle.decode(e.stream, e.offsets, e.n, e.chunk_symbols, e.cb.lengths(), e.cb.codes())

    def check_whole(enc_list, idx, got_of, ref_of, what):
        """Every element of the tensors `idx` of enc_list: got_of(i) is the GPU's output as a numpy array,
        ref_of(e, q) the oracle's from the oracle-decoded symbols q (one oracle call per tensor and thread)."""
        with ThreadPoolExecutor(default_threads()) as pool:
            qs = list(pool.map(lambda i: oracle_symbols(enc_list[i]), idx))
        for i, q in zip(idx, qs):
            if not np.array_equal(got_of(i), ref_of(enc_list[i], q)):
                print(f"bench.py: GPU output ({what}) differs from the oracle in tensor {enc_list[i].name}", file=sys.stderr)
                sys.exit(1)
        return len(idx)

    def check_segments(enc_list, count, seed, got_of, ref_of, what):
        """`count` segments drawn over all tensors: got_of(i, lo, hi) the GPU's output for symbols [lo, hi)."""
        rng_s = np.random.default_rng(seed)
        for _ in range(count):
            i = int(rng_s.integers(0, len(enc_list)))
            e = enc_list[i]
            k = int(rng_s.integers(0, e.offsets.size - 1))
            lo, hi = k * e.chunk_symbols, min((k + 1) * e.chunk_symbols, e.n)
            q = oracle.decode_chunks(e.stream, e.offsets, e.n, e.chunk_symbols, e.cb.lengths(), e.cb.codes(), k, 1,
                                     out=np.zeros(e.n, np.uint8))[lo:hi]
            if not np.array_equal(got_of(i, lo, hi), ref_of(e, q)):
                print(f"bench.py: GPU output ({what}) differs from the oracle in tensor {e.name} segment {k}", file=sys.stderr)
                sys.exit(1)
        return count

    def bf16_ref(e, q):
        return oracle.dequant_bf16(q, e.qp.scale, e.qp.zero_point)

    def kinds_idx(enc_list):
        """The first tensor of every kind (name without the layer) and the last tensor of the set."""
        first = {}
        for i, e in enumerate(enc_list):
            first.setdefault(e.name.split(".", 1)[1], i)
        return sorted(set(first.values()) | {len(enc_list) - 1})

    whole_idx = kinds_idx(encs)
    whole = check_whole(encs, whole_idx, lambda i: views[i].view(torch.int16).cpu().numpy().view(np.uint16), bf16_ref, "bf16")
    checked = check_segments(encs, 24, 2024, lambda i, lo, hi: views[i][lo:hi].view(torch.int16).cpu().numpy().view(np.uint16),
                             bf16_ref, "bf16")
    log(f"{whole} whole tensors ({sum(encs[i].n for i in whole_idx)} elements) and {checked} sampled segments match the oracle")

    # ------------------------- batch > 1 ("pre-fill"): the weights are decoded once, then multiplied as dense matrices
    prefill = None
    if not args.no_extras:
        batch = 256
        gen = torch.Generator(device=dev)
        gen.manual_seed(7)
        n0 = min(7, len(encs))
        xs_b = {c: torch.randn(batch, c, device=dev, generator=gen).to(torch.bfloat16) for c in sorted({e.cols for e in encs[:n0]})}
        w0 = [views[i].view(encs[i].rows, encs[i].cols) for i in range(n0)]

        def layer_gemms():
            return [torch.matmul(xs_b[w.shape[1]], w.t()) for w in w0]            # library GEMMs on the decoded bf16 weights

        wpf, kpf = timed(layer_gemms, args.steps, args.warmup)
        ys_b = layer_gemms()
        # one token's row of two products against the oracle's GEMV on the exact weights (the dense path multiplies
        # weights rounded to bf16 and rounds y to bf16: 2^-8 relative per factor, averaged over the row)
        for i in (0, n0 - 1):
            e = encs[i]
            q = oracle_symbols(e)
            xb = xs_b[e.cols][5].view(torch.int16).cpu().numpy().view(np.uint16)
            y_ref, _ = oracle.gemv(q, e.rows, e.cols, e.qp.scale, e.qp.zero_point, xb)
            yh = ys_b[i][5].float().cpu().numpy().astype(np.float64)
            if np.max(np.abs(yh - y_ref)) > 1e-2 * max(np.max(np.abs(y_ref)), 1e-30):
                print(f"bench.py: dense product on the decoded weights of {e.name} differs from the oracle", file=sys.stderr)
                sys.exit(1)
        prefill = {"workload": f"layer 0 at batch {batch}: entro_decode_dequant -> bf16 once, then the layer's seven products as "
                               "library GEMMs (torch.matmul) on the decoded weights",
                   "decode_ms_per_layer": round(wall_ms / args.layers, 4), "dense_gemms_ms_per_layer": round(kpf, 4),
                   "decode_share_of_a_prefill_layer": round((wall_ms / args.layers) / (wall_ms / args.layers + kpf), 3),
                   "verified_rows": 2}
        log(f"pre-fill: decode {wall_ms / args.layers:.3f} ms per layer, dense GEMMs at batch {batch} {kpf:.3f} ms per layer")
        del xs_b, w0, ys_b

    # ------------------------- what this GPU's memory takes of a plain stream with the same read/write mix
    rb = (stream_bytes + offset_bytes + 15) // 16 * 16
    probe_src = torch.zeros(rb, dtype=torch.uint8, device=dev)
    probe_scratch = torch.zeros(16, dtype=torch.uint8, device=dev)
    wp, kp = timed(lambda: bench_kernels.stream_probe(probe_src, rb, out_bf16, out_bytes, probe_scratch), args.steps, args.warmup)
    ceiling = (rb + out_bytes) / (kp * 1e-3) / 1e9
    log(f"stream probe with the same byte counts: {kp:.3f} ms, {ceiling:.0f} GB/s")
    del probe_src

    traffic, traffic_source = profiled_traffic() if args.layers == 32 else (None, None)
    result = {
        "metric": "decoded weights GB/s (entro_decode_dequant -> bf16, mistral-7B-shaped 8-bit set)",
        "value": round(decoded_gbps, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8",
        "data": "synthetic",
        "config": {"workload": f"configs[3]: mistral-7B-shaped, {args.layers} layers x 7 linears, Student-t(5)*0.02, "
                               "asymmetric 8-bit, chunks of 4096 symbols, decode+dequant to bf16",
                   "symbols": n_sym, "tensors": len(encs), "compressed_bytes": stream_bytes,
                   "mean_code_len_bits": round(mean_len, 4),
                   "offset_table_bits_per_symbol": round(offset_bytes * 8 / n_sym, 4),
                   "entry_points_inside_segments": {"every_symbols": args.sub_symbols,
                                                    "bits_per_symbol": round(sub_bytes * 8 / n_sym, 4),
                                                    "read_by": "launches too small to fill the device with whole segments "
                                                               "(the dependent GEMV step) in full; large launches for the units "
                                                               "left over behind a workgroup's last whole round"},
                   "bits_saved": round(E.entro_bits_saved(8, mean_len), 4),
                   "theoretical_speedup": round(E.entro_theoretical_speedup(8, mean_len), 4)},
        "symbols_per_s": round(n_sym / (wall_ms * 1e-3), 0),
        "compressed_GBps": round(stream_bytes / (wall_ms * 1e-3) / 1e9, 2),
        "hbm_fraction_wall": round(algo_bytes / (wall_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "verified_whole_tensors": whole, "verified_segments": checked,
        "roofline": {"bound": "hbm", "kernel": "k_batch<3> (entro_decode_dequant_batch -> bf16)", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "algorithmic_bytes_per_launch": algo_bytes, "kernel_ms": round(kern_ms, 4),
                     "traffic": traffic, "traffic_source": traffic_source},
        # a coalesced kernel that reads and writes the same byte counts, reads and writes interleaved in
        # their ratio: the rate memory takes a plain stream of this mix at, and the launch against it
        "stream_ceiling": {"GBps": round(ceiling, 1), "kernel_ms": round(kp, 4), "frac_of_peak": round(ceiling / HBM_PEAK_GBPS, 4),
                           "launch_frac_of_ceiling": round(achieved / ceiling, 4)},
    }

    if prefill:
        result["prefill"] = prefill

    # ------------------------------------------------------------ extra legs: u8 and GEMV
    if not args.no_extras:
        log("timing entro_decode -> u8")
        out_u8 = torch.empty(n_sym, dtype=torch.uint8, device=dev)
        v8, pos = [], 0
        for e in encs:
            v8.append(out_u8[pos:pos + e.n])
            pos += e.n
        ts8 = [d.ctensor(v) for d, v in zip(dts, v8)]
        ws8 = torch.zeros(E.entro_workspace_bytes(ts8, E.ENTRO_OP_DECODE), dtype=torch.uint8, device=dev)
        plan8 = E.entro_plan_init(ts8, E.ENTRO_OP_DECODE, E.ENTRO_U8, ws8)
        w8, k8 = timed(lambda: E.entro_plan_run(plan8), args.steps, args.warmup)
        result["decode_u8"] = {"ms_per_step": round(w8, 4), "kernel_ms": round(k8, 4),
                               "symbols_per_s": round(n_sym / (w8 * 1e-3), 0),
                               "hbm_frac": round((stream_bytes + offset_bytes + n_sym) / (k8 * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}
        whole8 = check_whole(encs, whole_idx, lambda i: v8[i].cpu().numpy(), lambda e, q: q, "u8")
        result["decode_u8"]["verified_whole_tensors"] = whole8
        # the product on those plain bytes: the uint8 model that the entropy-coded one is compared with,
        # all 224 products in one launch
        log("timing the plain uint8 GEMV on the decoded bytes (comparison)")
        xs_p = {c: torch.from_numpy(synth.make_x_bf16(0, c % 7, c).view(np.int16)).to(dev).view(torch.bfloat16)
                for c in sorted({e.cols for e in encs})}
        ys_p = [torch.zeros(e.rows, dtype=torch.float32, device=dev) for e in encs]
        plain = bench_kernels.PlainGemv([(v, e.rows, e.cols, e.qp.scale, e.qp.zero_point, xs_p[e.cols], y)
                                         for e, v, y in zip(encs, v8, ys_p)], dev)
        wpl, kpl = timed(plain.run, args.steps, args.warmup)
        rngp = np.random.default_rng(99)
        for _ in range(8):
            i = int(rngp.integers(0, len(encs)))
            e = encs[i]
            r = int(rngp.integers(0, e.rows))
            k0, k1 = (r * e.cols) // e.chunk_symbols, ((r + 1) * e.cols - 1) // e.chunk_symbols
            q = oracle.decode_chunks(e.stream, e.offsets, e.n, e.chunk_symbols, e.cb.lengths(), e.cb.codes(), k0, k1 - k0 + 1)
            xh = xs_p[e.cols].view(torch.int16).cpu().numpy().view(np.uint16)
            y_ref, _ = oracle.gemv(q[r * e.cols:(r + 1) * e.cols], 1, e.cols, e.qp.scale, e.qp.zero_point, xh)
            yh = ys_p[i].cpu().numpy().astype(np.float64)
            if abs(yh[r] - y_ref[0]) > 1e-3 * max(abs(y_ref[0]), np.sqrt(np.mean(yh ** 2))):
                print(f"bench.py: plain uint8 GEMV differs from the oracle, tensor {e.name} row {r}", file=sys.stderr)
                sys.exit(1)
        result["gemv_plain_uint8"] = {"workload": "the same 224 products on the decoded weights stored one byte each (what the "
                                                  "entropy-coded model is compared with), all in one launch "
                                                  "(bench_kernels/, not part of the library)",
                                      "us_per_layer": round(wpl * 1e3 / args.layers, 2),
                                      "kernel_us_per_layer": round(kpl * 1e3 / args.layers, 2),
                                      "weight_GBps": round(n_sym / (kpl * 1e-3) / 1e9, 1),
                                      "hbm_frac": round(n_sym / (kpl * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4), "verified_rows": 8}
        log(f"plain uint8 gemv: {kpl * 1e3 / args.layers:.1f} us/layer")
        del out_u8, v8, ts8, plan8, xs_p, ys_p, plain

        log("timing entro_decode_gemv (batch-1 token step, 4 launches per layer)")
        groups = [(0, 3), (3, 4), (4, 6), (6, 7)]          # q,k,v | o | gate,up | down
        layers = args.layers
        plans = []
        keep = []
        for layer in range(layers):
            base = 7 * layer
            for a, b in groups:
                tl = []
                for j in range(a, b):
                    e = encs[base + j]
                    xb = synth.make_x_bf16(layer, j, e.cols)
                    x = torch.from_numpy(xb.view(np.int16)).to(dev).view(torch.bfloat16)
                    y = torch.zeros(e.rows, dtype=torch.float32, device=dev)
                    keep.append((x, y, base + j, xb))
                    tl.append(dts[base + j].ctensor(y, x))
                wsg = torch.zeros(E.entro_workspace_bytes(tl, E.ENTRO_OP_GEMV), dtype=torch.uint8, device=dev)
                keep.append(wsg)
                plans.append(E.entro_plan_init(tl, E.ENTRO_OP_GEMV, E.ENTRO_F32, wsg))

        def token_step():
            for p in plans:
                E.entro_plan_run(p)

        wg, kg = timed(token_step, args.steps, args.warmup)
        # the same launches recorded once into a HIP graph and replayed (plan runs only enqueue kernels)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            token_step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            token_step()
        wgr, kgr = timed(graph.replay, args.steps, args.warmup)

        def check_gemv(what):
            """A few rows of the first layer's `q` and the last layer's `down` against the oracle."""
            for (x, y, idx, xb) in [k for k in keep if isinstance(k, tuple)][:1] + [k for k in keep if isinstance(k, tuple)][-1:]:
                e = encs[idx]
                yh = y.cpu().numpy().astype(np.float64)
                rows = [0, e.rows // 2, e.rows - 1]
                sub = np.empty((len(rows), e.cols), np.uint8)
                for j, r in enumerate(rows):
                    k0, k1 = (r * e.cols) // e.chunk_symbols, ((r + 1) * e.cols - 1) // e.chunk_symbols
                    q = oracle.decode_chunks(e.stream, e.offsets, e.n, e.chunk_symbols, e.cb.lengths(), e.cb.codes(),
                                             k0, k1 - k0 + 1)
                    sub[j] = q[r * e.cols:(r + 1) * e.cols]
                y_ref, _ = oracle.gemv(sub, len(rows), e.cols, e.qp.scale, e.qp.zero_point, xb)
                rms = np.sqrt(np.mean(yh ** 2))
                if np.max(np.abs(yh[rows] - y_ref) / np.maximum(np.abs(y_ref), rms)) > 1e-3:
                    print(f"bench.py: GEMV output ({what}) differs from the oracle in tensor {e.name}", file=sys.stderr)
                    sys.exit(1)

        check_gemv("dependent launches, graph replay")
        result["gemv"] = {"us_per_layer": round(wg * 1e3 / layers, 2), "kernel_us_per_layer": round(kg * 1e3 / layers, 2),
                          "hip_graph_us_per_layer": round(wgr * 1e3 / layers, 2),
                          "launches_per_layer": len(groups), "wide_tables": bool(plans[0].wide_tables),
                          "compressed_GBps": round(stream_bytes / (wg * 1e-3) / 1e9, 2),
                          "effective_uint8_GBps": round(n_sym / (wg * 1e-3) / 1e9, 2),
                          "hbm_frac": round((stream_bytes + offset_bytes) / (kg * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}
        log(f"gemv: {result['gemv']['us_per_layer']} us/layer")

        # the same 224 products as one launch (no dependencies between them): what the kernel sustains
        # when the whole chip has work, against the latency-bound step above
        log("timing entro_decode_gemv, all layers in one launch")
        pairs = [k for k in keep if isinstance(k, tuple)]
        tl_all = [dts[idx].ctensor(y, x) for (x, y, idx, xb) in pairs]
        ws_all = torch.zeros(E.entro_workspace_bytes(tl_all, E.ENTRO_OP_GEMV), dtype=torch.uint8, device=dev)
        plan_all = E.entro_plan_init(tl_all, E.ENTRO_OP_GEMV, E.ENTRO_F32, ws_all)
        for (x, y, idx, xb) in pairs:
            y.zero_()
        wa, ka = timed(lambda: E.entro_plan_run(plan_all), args.steps, args.warmup)
        check_gemv("one launch")
        result["gemv_one_launch"] = {"us_per_layer": round(wa * 1e3 / layers, 2), "kernel_us_per_layer": round(ka * 1e3 / layers, 2),
                                     "compressed_GBps": round(stream_bytes / (wa * 1e-3) / 1e9, 2),
                                     "effective_uint8_GBps": round(n_sym / (wa * 1e-3) / 1e9, 2),
                                     "hbm_frac": round((stream_bytes + offset_bytes) / (ka * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}
        log(f"gemv, one launch: {result['gemv_one_launch']['us_per_layer']} us/layer")

    # ------------------------------------------------ the headline set again with length-limited codebooks
    if not args.no_extras and not args.no_limited:
        # no code longer than the decoder's first-level table is wide: the slow path for long codes never
        # runs; what it costs in bits is reported beside what it gains
        log("preparing the headline set with codes of at most 14 bits")
        encs_l = prepare_config(4, layers=args.layers, max_len=14)
        dts_l = [E.to_device(e, dev) for e in encs_l]
        ts_l = [d.ctensor(v) for d, v in zip(dts_l, views)]
        ws_l = torch.zeros(E.entro_workspace_bytes(ts_l, E.ENTRO_OP_DEQUANT), dtype=torch.uint8, device=dev)
        plan_l = E.entro_plan_init(ts_l, E.ENTRO_OP_DEQUANT, E.ENTRO_BF16, ws_l)
        wl, kl = timed(lambda: E.entro_plan_run(plan_l), args.steps, args.warmup)
        rngl = np.random.default_rng(14)
        for _ in range(12):
            i = int(rngl.integers(0, len(encs_l)))
            e = encs_l[i]
            k = int(rngl.integers(0, e.offsets.size - 1))
            lo, hi = k * e.chunk_symbols, min((k + 1) * e.chunk_symbols, e.n)
            q = oracle.decode_chunks(e.stream, e.offsets, e.n, e.chunk_symbols, e.cb.lengths(), e.cb.codes(), k, 1,
                                     out=np.zeros(e.n, np.uint8))[lo:hi]
            ref = oracle.dequant_bf16(q, e.qp.scale, e.qp.zero_point)
            got = views[i][lo:hi].view(torch.int16).cpu().numpy().view(np.uint16)
            if not np.array_equal(got, ref):
                print(f"bench.py: length-limited leg differs from the oracle in tensor {e.name} segment {k}", file=sys.stderr)
                sys.exit(1)
        tl_l = [dts_l[idx].ctensor(y, x) for (x, y, idx, xb) in pairs]
        ws_lg = torch.zeros(E.entro_workspace_bytes(tl_l, E.ENTRO_OP_GEMV), dtype=torch.uint8, device=dev)
        plan_lg = E.entro_plan_init(tl_l, E.ENTRO_OP_GEMV, E.ENTRO_F32, ws_lg)
        y_before = torch.cat([y for (x, y, idx, xb) in pairs]).clone()
        wlg, klg = timed(lambda: E.entro_plan_run(plan_lg), args.steps, args.warmup)
        y_after = torch.cat([y for (x, y, idx, xb) in pairs])
        # same symbols, same x, same summation order: the products must not change at all
        if not torch.equal(y_before, y_after):
            print("bench.py: GEMV over length-limited streams differs from the unrestricted run", file=sys.stderr)
            sys.exit(1)
        bits_l = sum(e.total_bits for e in encs_l) / n_sym
        sb_l = sum(e.stream.size for e in encs_l)
        result["length_limited_14"] = {
            "mean_code_len_bits": round(bits_l, 4), "extra_bits_per_symbol": round(bits_l - mean_len, 5),
            "max_code_len": max(e.cb.max_len for e in encs_l), "max_code_len_unrestricted": max(e.cb.max_len for e in encs),
            "dequant_bf16_ms": round(wl, 4), "dequant_bf16_kernel_ms": round(kl, 4),
            "dequant_bf16_hbm_frac": round((sb_l + offset_bytes + 2 * n_sym) / (kl * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
            "gemv_one_launch_us_per_layer": round(wlg * 1e3 / layers, 2), "verified_segments": 12}
        log(f"length-limited: {wl:.3f} ms/step, gemv {wlg * 1e3 / layers:.1f} us/layer, +{bits_l - mean_len:.5f} bits/symbol")
        del encs_l, dts_l, ts_l, plan_l, tl_l, plan_lg, ws_l, ws_lg

    # ------------------------------------------------ the other workloads: integer decode
    if not args.no_other_configs:
        del out_bf16, views, ts, plan
        others = {}
        for cfg, label, dtype_out in ((1, "configs[0]: one 2048x2048 tensor, round trip -> u8", E.ENTRO_U8),
                                      (2, "configs[1]: smolLM-1.7B-shaped, 24 layers + norm gains -> u8", E.ENTRO_U8),
                                      (3, "configs[2]: phi3-mini-shaped, 32 layers, 4-bit -> packed u4", E.ENTRO_U4_PACKED)):
            log(f"preparing and timing {label}")
            sub_c = args.sub_symbols * (2 if cfg == 3 else 1)        # segments of 8192 symbols hold at most 16 pieces
            enc_c = prepare_config(cfg, sub_symbols=sub_c)
            dts_c = [E.to_device(e, dev) for e in enc_c]
            packed = dtype_out == E.ENTRO_U4_PACKED
            sizes = [(e.n + 1) // 2 if packed else e.n for e in enc_c]
            pad = [(-sz) % 16 for sz in sizes]                       # keep every tensor's output 16-byte aligned
            out_c = torch.zeros(sum(sizes) + sum(pad), dtype=torch.uint8, device=dev)
            v_c, pos = [], 0
            for sz, pd in zip(sizes, pad):
                v_c.append(out_c[pos:pos + sz])
                pos += sz + pd
            ts_c = [d.ctensor(v) for d, v in zip(dts_c, v_c)]
            ws_c = torch.zeros(E.entro_workspace_bytes(ts_c, E.ENTRO_OP_DECODE), dtype=torch.uint8, device=dev)
            plan_c = E.entro_plan_init(ts_c, E.ENTRO_OP_DECODE, dtype_out, ws_c)
            wc, kc = timed(lambda: E.entro_plan_run(plan_c), args.steps, args.warmup)
            # whole tensors of every kind and sampled segments of the rest against the oracle
            idx_c = kinds_idx(enc_c)
            if packed:
                whole_c = check_whole(enc_c, idx_c, lambda i: v_c[i].cpu().numpy(), lambda e, q: oracle.pack_u4(q), label)
                n_checks = check_segments(enc_c, 12, cfg, lambda i, lo, hi: v_c[i][lo // 2:(hi + 1) // 2].cpu().numpy(),
                                          lambda e, q: oracle.pack_u4(q), label)
            else:
                whole_c = check_whole(enc_c, idx_c, lambda i: v_c[i].cpu().numpy(), lambda e, q: q, label)
                n_checks = check_segments(enc_c, 12, cfg, lambda i, lo, hi: v_c[i][lo:hi].cpu().numpy(), lambda e, q: q, label)
            n_c = sum(e.n for e in enc_c)
            sb_c = sum(e.stream.size for e in enc_c)
            ob_c = sum(e.offsets.size * 8 for e in enc_c)
            bits_c = sum(e.total_bits for e in enc_c) / n_c
            others[f"config{cfg}"] = {"workload": label, "symbols": n_c, "tensors": len(enc_c), "entry_points_every_symbols": sub_c,
                                      "mean_code_len_bits": round(bits_c, 4), "ms_per_step": round(wc, 4),
                                      "kernel_ms": round(kc, 4), "symbols_per_s": round(n_c / (wc * 1e-3), 0),
                                      "decoded_GBps": round(sum(sizes) / (wc * 1e-3) / 1e9, 2),
                                      "compressed_GBps": round(sb_c / (wc * 1e-3) / 1e9, 2),
                                      "hbm_frac": round((sb_c + ob_c + sum(sizes)) / (kc * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                                      "verified_whole_tensors": whole_c, "verified_segments": n_checks}
            log(f"config {cfg}: {wc:.3f} ms/step")
            if cfg == 3:
                # the same 4-bit set dequantized to bf16 (what an inference engine asks for), sampled like the rest
                out_b = torch.zeros(n_c, dtype=torch.bfloat16, device=dev)
                v_b, pos = [], 0
                for e in enc_c:
                    v_b.append(out_b[pos:pos + e.n])
                    pos += e.n
                ts_b = [d.ctensor(v) for d, v in zip(dts_c, v_b)]
                ws_b = torch.zeros(E.entro_workspace_bytes(ts_b, E.ENTRO_OP_DEQUANT), dtype=torch.uint8, device=dev)
                plan_b = E.entro_plan_init(ts_b, E.ENTRO_OP_DEQUANT, E.ENTRO_BF16, ws_b)
                wb, kb = timed(lambda: E.entro_plan_run(plan_b), args.steps, args.warmup)
                whole_b = check_whole(enc_c, idx_c, lambda i: v_b[i].view(torch.int16).cpu().numpy().view(np.uint16), bf16_ref,
                                      "configs[2] -> bf16")
                check_segments(enc_c, 12, 33, lambda i, lo, hi: v_b[i][lo:hi].view(torch.int16).cpu().numpy().view(np.uint16),
                               bf16_ref, "configs[2] -> bf16")
                others["config3_bf16"] = {"workload": "configs[2] tensors, entro_decode_dequant -> bf16", "symbols": n_c,
                                          "ms_per_step": round(wb, 4), "kernel_ms": round(kb, 4),
                                          "symbols_per_s": round(n_c / (wb * 1e-3), 0),
                                          "decoded_GBps": round(2 * n_c / (wb * 1e-3) / 1e9, 2),
                                          "hbm_frac": round((sb_c + ob_c + 2 * n_c) / (kb * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                                          "verified_whole_tensors": whole_b, "verified_segments": 12}
                log(f"config 3 -> bf16: {wb:.3f} ms/step")
                del out_b, v_b, ts_b, plan_b, ws_b
                # and multiplied into activation vectors (4-bit token generation; segments of 8192 symbols
                # hold two and two thirds matrix rows here), all products in one launch
                xs_g, ys_g, ts_g = [], [], []
                for i, e in enumerate(enc_c):
                    xb = synth.make_x_bf16(i // 4, i % 4, e.cols)
                    xs_g.append(xb)
                    x = torch.from_numpy(xb.view(np.int16)).to(dev).view(torch.bfloat16)
                    y = torch.zeros(e.rows, dtype=torch.float32, device=dev)
                    ys_g.append((x, y))
                    ts_g.append(dts_c[i].ctensor(y, x))
                ws_g = torch.zeros(max(256, E.entro_workspace_bytes(ts_g, E.ENTRO_OP_GEMV)), dtype=torch.uint8, device=dev)
                plan_g = E.entro_plan_init(ts_g, E.ENTRO_OP_GEMV, E.ENTRO_F32, ws_g)
                wg3, kg3 = timed(lambda: E.entro_plan_run(plan_g), args.steps, args.warmup)
                rngc = np.random.default_rng(cfg)
                for _ in range(8):
                    i = int(rngc.integers(0, len(enc_c)))
                    e = enc_c[i]
                    r = int(rngc.integers(0, e.rows))
                    k0, k1 = (r * e.cols) // e.chunk_symbols, ((r + 1) * e.cols - 1) // e.chunk_symbols
                    q = oracle.decode_chunks(e.stream, e.offsets, e.n, e.chunk_symbols, e.cb.lengths(), e.cb.codes(),
                                             k0, k1 - k0 + 1)
                    y_ref, _ = oracle.gemv(q[r * e.cols:(r + 1) * e.cols], 1, e.cols, e.qp.scale, e.qp.zero_point, xs_g[i])
                    yh = ys_g[i][1].cpu().numpy().astype(np.float64)
                    rms = np.sqrt(np.mean(yh ** 2))
                    if abs(yh[r] - y_ref[0]) / max(abs(y_ref[0]), rms) > 1e-3:
                        print(f"bench.py: GEMV output differs from the oracle in {label}, tensor {e.name} row {r}", file=sys.stderr)
                        sys.exit(1)
                n_layers3 = len(enc_c) // 4
                others["config3_gemv"] = {"workload": "configs[2] tensors, entro_decode_gemv, all products in one launch",
                                          "us_per_layer": round(wg3 * 1e3 / n_layers3, 2),
                                          "symbols_per_s": round(n_c / (wg3 * 1e-3), 0),
                                          "effective_uint4_GBps": round(n_c / 2 / (wg3 * 1e-3) / 1e9, 2),
                                          "verified_rows": 8}
                log(f"config 3 gemv: {wg3 * 1e3 / n_layers3:.1f} us/layer")
                del xs_g, ys_g, ts_g, plan_g, ws_g
            del enc_c, dts_c, out_c, v_c, ts_c, plan_c
        result["other_configs"] = others

    # ------------------------------------------------ the steps before the path, on the GPU
    if not args.no_extras and not args.no_compress:
        log("timing the compression kernels on layer 0's fp32 weights")
        specs0 = synth.config_tensors(4, layers=1)
        comp = {"workload": "layer 0 of the mistral-7B-shaped set, fp32 weights resident in HBM: range, quantise + count, "
                            "encode (kernels; the (s, z) and codebook steps between them run on the host and are not timed)",
                "tensors": {}}
        k_total, n_total, host_s = 0.0, 0, 0.0
        for spec, e in zip(specs0, encs):
            assert e.name == f"L{spec.layer}.{spec.name}" and e.n == spec.rows * spec.cols
            w_host = synth.make_tensor(spec).ravel()
            t_h = time.perf_counter()
            E.encode_tensor(w_host, 8, E.ENTRO_ASYMMETRIC, e.chunk_symbols)
            host_s += time.perf_counter() - t_h
            w = torch.from_numpy(w_host).to(dev)
            small = torch.empty(8, dtype=torch.int32, device=dev)
            counts = torch.empty(256, dtype=torch.int64, device=dev)
            qd = torch.empty(w.numel(), dtype=torch.uint8, device=dev)
            _, k_r = timed(lambda: E.entro_range_device(w, small), 5, 1)
            r = small[:4].cpu().numpy()
            mn, mx = r[:2].view(np.float32)
            qp = E.entro_qparams_from_range(float(mn), float(mx), int(r[2]), 8, E.ENTRO_ASYMMETRIC)
            _, k_q = timed(lambda: E.entro_quantize_device(w, qp, qd, counts), 5, 1)
            cnt = counts.cpu().numpy().view(np.uint64)
            cb = E.entro_codebook_from_counts(cnt, 8)
            st_d = torch.empty(E.entro_encoded_bytes(cnt, cb), dtype=torch.uint8, device=dev)
            off_d = torch.empty(E.entro_num_chunks(w.numel(), e.chunk_symbols) + 1, dtype=torch.int64, device=dev)
            status = small[4:5]
            _, k_e = timed(lambda: E.entro_encode_device(qd, cb, e.chunk_symbols, st_d, off_d, status), 5, 1)
            # the host library encoded the same weights for the decode legs: the two streams must be identical
            same = (int(status.item()) == 0 and np.float32(qp.scale) == np.float32(e.qp.scale)
                    and qp.zero_point == e.qp.zero_point and np.array_equal(st_d.cpu().numpy(), e.stream)
                    and np.array_equal(off_d.cpu().numpy().view(np.uint64), e.offsets))
            if not same:
                print(f"bench.py: device-side compression of {e.name} differs from the host library's", file=sys.stderr)
                sys.exit(1)
            nn = w.numel()
            comp["tensors"][e.name] = {"symbols": nn, "range_us": round(k_r * 1e3, 1), "quantize_us": round(k_q * 1e3, 1),
                                       "encode_us": round(k_e * 1e3, 1)}
            k_total += k_r + k_q + k_e
            n_total += nn
            del w, qd, st_d, off_d
        # algorithmic bytes: 4 (range) + 4 + 1 (quantise) + 1 + 1 + stream + offsets (encode: two passes over the symbols)
        comp_bytes = n_total * 11 + sum(e.stream.size + e.offsets.size * 8 for e in encs[: len(specs0)])
        comp.update({"kernel_ms_per_layer": round(k_total, 4), "symbols_per_s": round(n_total / (k_total * 1e-3), 0),
                     "algorithmic_GBps": round(comp_bytes / (k_total * 1e-3) / 1e9, 1),
                     "hbm_frac": round(comp_bytes / (k_total * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                     "identical_to_host_encoder": True,
                     "host_library_ms_per_layer": round(host_s * 1e3, 1), "host_threads": default_threads()})
        result["compress_device"] = comp
        log(f"compression kernels: {k_total:.3f} ms per layer, {n_total / (k_total * 1e-3) / 1e9:.0f} G symbols/s")

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        wc, kc = timed(lambda: dst.copy_(src), 3, 1)
        result["copy_calibration"] = {"bytes_each_way": 1 << 30, "kernel_ms": round(kc, 4),
                                      "GBps_read_plus_write": round(2 * (1 << 30) / (kc * 1e-3) / 1e9, 1)}

    # -------------------------------------------------------------- oracle on the host cores
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a bounded sample")
        budget_syms = 1_500_000_000      # about 15 s of one core
        t_cpu, syms = 0.0, 0
        sample = []
        for e in encs:
            if syms + e.n > budget_syms and syms > 0:
                break
            ln, code = e.cb.lengths(), e.cb.codes()
            t1 = time.perf_counter()
            q = oracle.decode(e.stream, e.offsets, e.n, e.chunk_symbols, ln, code)
            oracle.dequant_bf16(q, e.qp.scale, e.qp.zero_point)
            t_cpu += time.perf_counter() - t1
            syms += e.n
            sample.append(e.name)
        result["cpu_baseline"] = {"value": round(syms * 2 / t_cpu / 1e9, 4), "unit": "GB/s", "cores": 1,
                                  "kind": "oracle",
                                  "sample": f"{len(sample)} tensors ({sample[0]}..{sample[-1]}), {syms} symbols, "
                                            f"{t_cpu:.1f} s: bit-at-a-time tree-walk decode + (q-z)*s -> bf16",
                                  "symbols_per_s": round(syms / t_cpu, 0)}
        # the paper's own scheme on the host: threads over independently decodable pieces (here: the
        # sample's tensors), the same oracle calls, as many threads as the box gives this process
        from concurrent.futures import ThreadPoolExecutor
        n_thr = default_threads()

        def one(e):
            q = oracle.decode(e.stream, e.offsets, e.n, e.chunk_symbols, e.cb.lengths(), e.cb.codes())
            oracle.dequant_bf16(q, e.qp.scale, e.qp.zero_point)

        t1 = time.perf_counter()
        with ThreadPoolExecutor(n_thr) as pool:
            list(pool.map(one, encs[: len(sample)]))
        t_par = time.perf_counter() - t1
        result["cpu_baseline_threads"] = {"value": round(syms * 2 / t_par / 1e9, 4), "unit": "GB/s", "cores": n_thr,
                                          "kind": "oracle", "sample": "the same tensors, one oracle call per tensor and thread",
                                          "symbols_per_s": round(syms / t_par, 0)}
    # the paper's own figures, from another machine: context beside the numbers above, not a target
    result["paper_context"] = {"hardware": "NVIDIA Jetson P3450, Huffman decode on 4 Cortex-A57 threads (Table 3)",
                               "decode_whole_model_s": {"uint8": 6.66, "uint4": 1.66, "params": 3.8e9},
                               "decode_G_symbols_per_s": {"uint8": 0.57, "uint4": 2.29},
                               "token_generation_speedup": {"uint8": 1.32, "uint4": 2.47},
                               "effective_bits": {"uint8": 5.58, "uint4": 1.39}}
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
