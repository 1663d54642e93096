#!/usr/bin/env python3
"""Benchmark of the BitLinear hot path on one MI355X.

Default workload (the largest single-GPU configuration): the 100B-shape model's token decode at M=1 -- 80 layers
with hidden 12288 and FFN 33792, 7 ternary x int8 GEMVs per layer, all 36.99 GB of 2-bit packed weights resident in
HBM.  One "step" is one token: 80 launches of the fused kernel (bl_decode_batch: the per-token absmax int8
quantization of a layer's four inputs and its 7 GEMVs in one launch), captured as ONE HIP graph and replayed; every
layer has its own weights, so every step streams all of them from HBM.  Inputs are resident in HBM before the timed
region starts.

Prints ONE JSON line: metric = packed-weight GB/s of the decode GEMVs, with the dominant kernel's roofline and the
CPU oracle timed beside it (one full layer on the host cores, all cores and one thread; the whole token is that
times 80, stated as extrapolated).  The other benchmark configurations (1536^2 matrix, 3B-shape layer, 7B-shape
layer at M = 1, 4, 8, the prefill products, the paper's own 100B shape) are nested under "extra", each with its own
roofline and cpu_baseline; so are the measured ceilings (a register-only MFMA loop, a read-only streaming kernel)
and the whole-model token loop in the paper's unit.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E, published
INT8_PEAK_TOPS = 5000.0     # MI355X dense int8 MFMA, published


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100, help="timed steps (tokens of the 100B-shape model)")
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--layers", type=int, default=40, help="distinct 3B-shape layers to rotate through (extra.config2)")
    ap.add_argument("--model-layers", type=int, default=80, help="layers of the headline model (80 = the configuration)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-extra", action="store_true", help="skip the extra sections")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--cpu-seconds", type=float, default=8.0, help="CPU work of the headline's oracle baseline")
    ap.add_argument("--profiler-run", action="store_true",
                    help="few launches per measurement (no clock ramp, no spread): for a profiler that collects counters "
                         "and slows every dispatch; the times such a run prints are not results")
    ap.add_argument("--models", default="", help="with --only tokens: comma-separated Appendix-A model names (default: all 12)")
    ap.add_argument("--only", default="", help="run only one extra section (copy|ceilings|prefill|config1|config2|config3|decode100b|paper100b|appendixa|tokens|tokens8k|prompt|prompt2k|tl2) and print it")
    return ap.parse_args()


def timed(torch, fn):
    """Run fn() bracketed by synchronize + events on the current stream; returns (event ms, wall ms)."""
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    fn()
    e1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3
    return e0.elapsed_time(e1), wall


PROFILER_RUN = False   # --profiler-run: at most 100 steps, one untimed replay and one timed one per measurement, no spread


def run_steps(torch, step_fns, count, use_graph, stats=None):
    """Time exactly `count` steps (step i = step_fns[i % len]).  With use_graph the steps are
    captured once into a HIP graph (one replay = all `count` steps) so that host launch overhead
    is out of the timed region; the replay itself is what is timed."""
    n = len(step_fns)
    scale = 1.0
    if PROFILER_RUN and count > 100:    # the caller divides by its own count
        scale, count = count / 100.0, 100

    def eager():
        for i in range(count):
            step_fns[i % n]()

    if not use_graph:
        ms, wall = timed(torch, eager)
        return ms * scale, wall, "eager"
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            eager()
    torch.cuda.synchronize()
    # untimed replays: the first pays one-time upload costs, and the GPU needs some tens of milliseconds of
    # sustained work to reach its steady clocks (a 2 ms burst of the prefill kernel measures 25 % slower)
    t0 = time.perf_counter()
    for _ in range(1 if PROFILER_RUN else 50):
        g.replay()
        torch.cuda.synchronize()
        if time.perf_counter() - t0 > 0.05:
            break
    ms, wall = timed(torch, g.replay)
    if stats is not None and not PROFILER_RUN:   # further replays of the same K steps: spread of the per-step time
        more = sorted([ms] + [timed(torch, g.replay)[0] for _ in range(4)])
        stats.update({"replays": len(more), "ms_per_step_min": round(more[0] / count, 6),
                      "ms_per_step_median": round(more[len(more) // 2] / count, 6),
                      "ms_per_step_max": round(more[-1] / count, 6)})
    del g
    return ms * scale, wall, "hip-graph"


def check_layer_against_oracle(torch, np, oracle, layer, host):
    """Fused launch of one layer vs the oracle: bit-exact q / scales / acc, outputs within 1e-6."""
    from paper_2410_16144_amd import ops
    from paper_2410_16144_amd.decode_layer import INPUT_OF
    in_x = [layer.xs[INPUT_OF[p.name]] for p in layer.projs]
    grp = ops.DecodeGroup(layer.weights, in_x, want_acc=True, want_quant=True)
    outs = grp.launch()
    layer.step_fused()
    torch.cuda.synchronize()
    refs_q = [oracle.quant_act(b) for b in host["x_bits"]]
    for i, p in enumerate(layer.projs):
        q, a, s = refs_q[INPUT_OF[p.name]]
        assert np.array_equal(grp.quants[i].q.cpu().numpy()[:, :p.K], q), "q mismatch " + p.name
        assert np.array_equal(grp.quants[i].a_scale.cpu().numpy(), a), "a_scale mismatch " + p.name
        acc_ref = oracle.matmul_i32(q, host["w"][i])
        assert np.array_equal(grp.accs[i].cpu().numpy(), acc_ref), "acc mismatch " + p.name
        ref = oracle.dequant(acc_ref, host["w_scale"][i], a)
        for got in (outs[i].cpu().numpy(), layer.outs[i].cpu().numpy()):
            assert np.all(np.abs(got - ref) <= 1e-6 * np.abs(ref)), "out mismatch " + p.name


def _passes(fn, seconds):
    """Repeat fn() for about `seconds` (at least once); returns (count, elapsed seconds)."""
    n, t0 = 0, time.perf_counter()
    while True:
        fn()
        n += 1
        dt = time.perf_counter() - t0
        if dt >= seconds:
            return n, dt


def cpu_layer_baseline(oracle, host, projs, packed_bytes, seconds, what, model_layers=None):
    """The oracle as it stands, timed on the host cores on repeated passes over ONE layer (its 4 quantizations, 7
    integer products and 7 dequantizations, whatever M the inputs have): all cores first, then one thread.  The rate
    is quoted on the packed 2-bit byte count, like the GPU value (the oracle itself reads unpacked int8 weights)."""
    from paper_2410_16144_amd.decode_layer import INPUT_OF

    def one_pass():
        qs = [oracle.quant_act(b) for b in host["x_bits"]]
        for i, p in enumerate(projs):
            q, a, _ = qs[INPUT_OF[p.name]]
            acc = oracle.matmul_i32(q, host["w"][i])
            oracle.dequant(acc, host["w_scale"][i], a)

    cores = oracle.num_threads()
    one_pass()                                   # pages the weights in
    n, dt = _passes(one_pass, seconds)
    res = {"value": round(packed_bytes * n / dt / 1e9, 3), "unit": "GB/s", "cores": cores, "kind": "oracle",
           "ms_per_layer": round(dt / n * 1e3, 3),
           "sample": "%d full passes over one %s (4 quantizations + 7 products), %.1f s of CPU work on %d threads; the "
                     "oracle reads unpacked int8 weights, the rate is quoted on the same packed 2-bit byte count as "
                     "the GPU value" % (n, what, dt, cores)}
    oracle.set_num_threads(1)
    try:
        n1, dt1 = _passes(one_pass, max(1.0, seconds / 4))
    finally:
        oracle.set_num_threads(cores)
    res["one_thread"] = {"value": round(packed_bytes * n1 / dt1 / 1e9, 3), "unit": "GB/s", "cores": 1,
                         "ms_per_layer": round(dt1 / n1 * 1e3, 3), "passes": n1}
    if model_layers:
        res["ms_per_step"] = round(dt / n * 1e3 * model_layers, 1)
        res["one_thread"]["ms_per_step"] = round(dt1 / n1 * 1e3 * model_layers, 1)
        res["sample"] += "; ONE layer timed, the %d-layer token is that x %d, extrapolated" % (model_layers, model_layers)
    else:
        res["ms_per_step"] = res["ms_per_layer"]
    return res


def cpu_prefill_baseline(np, oracle, M, K, N):
    """The oracle on one prefill product of the benchmark's shape (host-drawn operands of the same distributions):
    quantization + integer product + dequantization.  All cores on the full M (once); one thread on a sample of 32
    token rows, scaled to M (the oracle's work is linear in the rows)."""
    from paper_2410_16144_amd import synth
    rng = synth.rng_for(synth.seed_for(4, 1, 0 if K == 4096 else 1))
    w = synth.ternary_weights(rng, N, K)
    bits = synth.to_bf16_bits(synth.activations(rng, M, K))

    def product(b):
        q, a, _ = oracle.quant_act(b)
        oracle.dequant(oracle.matmul_i32(q, w), np.float32(0.02), a)

    cores = oracle.num_threads()
    product(bits[:16])
    t0 = time.perf_counter()
    product(bits)
    dt = time.perf_counter() - t0
    ops = 2.0 * M * K * N
    rows1 = 32
    oracle.set_num_threads(1)
    try:
        t0 = time.perf_counter()
        product(bits[:rows1])
        dt1 = (time.perf_counter() - t0) * M / rows1
    finally:
        oracle.set_num_threads(cores)
    return {"value": round(ops / dt / 1e12, 4), "unit": "TOP/s", "cores": cores, "kind": "oracle", "ms_per_step": round(dt * 1e3, 1),
            "sample": "the whole product once (M=%d K=%d N=%d: quantization, integer product, dequantization), %.1f s on "
                      "%d threads" % (M, K, N, dt, cores),
            "one_thread": {"value": round(ops / dt1 / 1e12, 4), "unit": "TOP/s", "cores": 1, "ms_per_step": round(dt1 * 1e3, 1),
                           "sample": "%d of the %d token rows timed, scaled to all rows" % (rows1, M)}}


def hbm_roofline(kernel, bytes_per_launch, launch_us, traffic=None):
    gbs = bytes_per_launch / launch_us / 1e3
    return {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": traffic, "kernel": kernel,
            "avg_launch_us": round(launch_us, 3), "bytes_per_launch": int(bytes_per_launch)}


def last_kernel():
    from paper_2410_16144_amd import binding
    return binding.bl_last_kernel()


def extra_copy(torch):
    """A plain device-to-device copy of known size (torch's copy kernel): the practical HBM rate
    of this box, and the calibration launch for the FETCH_SIZE / WRITE_SIZE counters."""
    dev = torch.device("cuda:0")
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device=dev).fill_(3)
    dst = torch.empty_like(src)
    for _ in range(2):
        dst.copy_(src)
    ms, _ = timed(torch, lambda: [dst.copy_(src) for _ in range(10)])
    us = ms * 1e3 / 10
    return {"bytes_read": n, "bytes_written": n, "us": round(us, 1), "GBps_read_plus_write": round(2 * n / us / 1e3, 1)}


def extra_prefill(torch, M, K, N, use_graph=True, iters=100):
    from paper_2410_16144_amd import ops, synth
    dev = torch.device("cuda:0")
    w = synth.ternary_weights_device(4000 + M + K, N, K, dev)
    pw = ops.pack_ternary(w, 0.02)
    del w
    g = torch.Generator(device=dev)
    g.manual_seed(4001)
    x = torch.randn((M, K), device=dev, dtype=torch.float32, generator=g).to(torch.bfloat16)
    qa = ops.quant_act(x)
    out = torch.empty((M, N), dtype=torch.float32, device=dev)
    # the quantizer first: timed behind the matrix-core kernel it reads several microseconds slower for a while
    msq, _, _ = run_steps(torch, [lambda: ops.quant_act(x, qa)], iters, use_graph)
    usq = msq * 1e3 / iters
    for _ in range(3):
        ops.gemm(pw, qa, out)
    kernel = last_kernel()
    ms, _, mode = run_steps(torch, [lambda: ops.gemm(pw, qa, out)], iters, use_graph)
    us = ms * 1e3 / iters
    tops = 2.0 * M * K * N / us / 1e6
    # the same launch on all-zero activations: identical instruction stream and memory traffic, only the operand
    # bits stop toggling.  The gap to the real-data time is what the chip's power limit (lower sustained clock)
    # costs this kernel; it is reported beside the headline, never instead of it
    us_zero = None
    if True:
        qz = ops.quant_act(torch.zeros_like(x))
        ops.gemm(pw, qz, out)
        msz, _, _ = run_steps(torch, [lambda: ops.gemm(pw, qz, out)], iters, use_graph)
        us_zero = round(msz * 1e3 / iters, 2)
        ops.gemm(pw, qa, out)
    # context only: the vendor library's dense int8 x int8 -> int32 product of the same shape (weights as int8,
    # four times the bytes, no dequantization), through torch._int_mm
    lib_us = None
    try:
        a8 = qa.q[:, :K].contiguous()
        b8 = torch.randint(-1, 2, (N, K), device=dev, dtype=torch.int8).t()
        torch._int_mm(a8, b8)
        msl, _, _ = run_steps(torch, [lambda: torch._int_mm(a8, b8)], iters, False)
        lib_us = round(msl * 1e3 / iters, 2)
    except Exception:   # not every build of the framework has it
        pass
    return {"workload": "prefill M=%d K=%d N=%d" % (M, K, N), "gemm_us": round(us, 2), "quant_act_us": round(usq, 2),
            "launch": mode, "gemm_us_on_all_zero_activations": us_zero, "vendor_library_dense_int8_gemm_us": lib_us,
            "roofline": {"bound": "mfma", "achieved": round(tops / 1e3, 4), "peak": INT8_PEAK_TOPS / 1e3,
                         "unit": "POP/s", "frac": round(tops / INT8_PEAK_TOPS, 4), "traffic": None, "kernel": kernel,
                         "avg_launch_us": round(us, 2), "ops_per_launch": 2 * M * K * N},
            "tops_including_quant_act": round(2.0 * M * K * N / (us + usq) / 1e6, 1)}


def extra_decode_shape(torch, name, hidden, ffn, M, layers, steps, use_graph, config=5, p_zero=None, outliers=0.0,
                       cpu_seconds=0.0, dependency_ordered=False):
    """Layer decode on one model shape, `layers` distinct layers rotated so that every launch reads HBM.  Variants:
    the fused launch (quantize + 7 products in one kernel), one grouped quantization launch + one grouped product
    launch, four quantization launches + one grouped product launch, and the grouped product launch alone.  The
    `roofline` block is the best variant that INCLUDES the quantization (the hot path is both steps), quoted on its
    product kernel; cpu_seconds > 0 adds the oracle on the same layer (layer 0 is then drawn on the host)."""
    from paper_2410_16144_amd.decode_layer import make_layer
    dev = torch.device("cuda:0")
    host = None
    ls = []
    for i in range(layers):
        l, h = make_layer(config, i, hidden, ffn, M, dev, p_zero, outliers, host=(i == 0 and cpu_seconds > 0))
        ls.append(l)
        host = h if i == 0 else host
    pb = ls[0].packed_bytes
    res = {"workload": "%s layer decode M=%d (hidden %d, ffn %d), %d distinct layers rotated"
                       % (name, M, hidden, ffn, layers), "packed_bytes_per_layer": pb}
    variants = [("fused_1_launch", "step_fused"), ("grouped_quant_plus_grouped_gemv", "step_two_launches"),
                ("quant_x4_plus_grouped_gemv", "step_single_launch"), ("grouped_gemv_only", None)]
    if dependency_ordered:
        variants.append(("fused_dependency_ordered_4_launches", "step_fused_dependency_ordered"))
    best = None
    for label, attr in variants:
        fns = [getattr(l, attr) if attr else l.group_all.launch for l in ls]
        for f in fns[:2]:
            f()
        kernel = last_kernel()
        ms, _, mode = run_steps(torch, fns, steps, use_graph)
        us = ms * 1e3 / steps
        res[label] = {"us_per_layer": round(us, 2), "GBps": round(pb / us / 1e3, 1),
                      "frac_of_hbm_peak": round(pb / us / 1e3 / HBM_PEAK_GBS, 4), "product_kernel": kernel}
        if attr in ("step_fused", "step_two_launches") and (best is None or us < best[1]):
            best = (label, us, kernel)
    res["launch"] = mode
    res["roofline"] = hbm_roofline(best[2], pb, best[1])
    res["roofline"]["sequence"] = best[0] + " (quantization included; avg_launch_us is the whole sequence)"
    if cpu_seconds > 0:
        import oracle
        res["cpu_baseline"] = cpu_layer_baseline(oracle, host, ls[0].projs, pb, cpu_seconds, "%s layer at M=%d" % (name, M))
    return res


def extra_tl2(torch, use_graph):
    """The 1.78-bit layout on the paper's TL2 code beside the 2-bit layout: one-token decode product of single
    matrices (bl_tl2_gemv has no grouped launch), copies rotated so that every launch reads HBM.  Both kernels
    compute the same bits; the time ratio is the answer to whether 11 % fewer bytes outweigh the extra table
    lookups."""
    from paper_2410_16144_amd import ops, synth
    dev = torch.device("cuda:0")
    rows = []
    for K, N, copies in ((12288, 32768, 6), (16384, 32768, 4), (12288, 33792, 6), (8192, 45568, 6), (4096, 11008, 40)):
        ws = [synth.ternary_weights_device(900 + i, N, K, dev) for i in range(2)]
        two = [ops.pack_ternary(ws[i % 2], 0.02) for i in range(2)]
        tl2 = [ops.tl2_pack(ws[i % 2], 0.02) for i in range(2)]
        two = [ops.PackedWeight(two[i % 2].blob.clone(), two[i % 2].desc) for i in range(copies)]
        tl2 = [ops.PackedWeight(tl2[i % 2].blob.clone(), tl2[i % 2].desc) for i in range(copies)]
        del ws
        x = torch.randn((1, K), device=dev, dtype=torch.float32).to(torch.bfloat16)
        qa2 = ops.quant_act(x)
        qa3 = ops.quant_act(x, ops.tl2_quant_buffer(K, dev))
        out = torch.empty((1, N), dtype=torch.float32, device=dev)
        same = torch.equal(ops.gemv(two[0], qa2), ops.tl2_gemv(tl2[0], qa3))
        groups = [ops.GemvGroup([p], [qa2], [out]) for p in two]
        steps = 40 * copies
        ms2, _, _ = run_steps(torch, [g.launch for g in groups], steps, use_graph)
        groups3 = [ops.Tl2GemvGroup([p], [qa3], [out]) for p in tl2]
        ms3, _, mode = run_steps(torch, [g.launch for g in groups3], steps, use_graph)
        us2, us3 = ms2 * 1e3 / steps, ms3 * 1e3 / steps
        rows.append({"K": K, "N": N, "bytes_2bit": N * K // 4, "bytes_tl2": int(tl2[0].desc.bytes),
                     "us_2bit": round(us2, 2), "us_tl2": round(us3, 2), "tl2_speedup": round(us2 / us3, 3),
                     "GBps_2bit": round(N * K / 4 / us2 / 1e3, 1), "GBps_tl2_own_bytes": round(tl2[0].desc.bytes / us3 / 1e3, 1),
                     "outputs_bit_identical": bool(same), "launch": mode})
        del two, tl2, groups, groups3
    # a whole decoder layer per launch (7 matrices, plain form: quantized activations given), both layouts
    from paper_2410_16144_amd import decode_layer
    layers = []
    for name, hidden, ffn, count in (("3B-shape", 3200, 8640, 30), ("7B-shape", 4096, 11008, 20), ("100B-shape", 12288, 33792, 4)):
        projs = synth.layer_projections(hidden, ffn)
        xs = {K: torch.randn((1, K), device=dev, dtype=torch.float32).to(torch.bfloat16) for K in (hidden, ffn)}
        qa2 = {K: ops.quant_act(x) for K, x in xs.items()}
        qa3 = {K: ops.quant_act(x, ops.tl2_quant_buffer(K, dev)) for K, x in xs.items()}
        g2, g3 = [], []
        for c in range(count):
            ws = [synth.ternary_weights_device(950 + 7 * (c % 2) + i, p.N, p.K, dev) for i, p in enumerate(projs)]
            outs = [torch.empty((1, p.N), dtype=torch.float32, device=dev) for p in projs]
            g2.append(ops.GemvGroup([ops.pack_ternary(w, 0.02) for w in ws], [qa2[p.K] for p in projs], outs))
            g3.append(ops.Tl2GemvGroup([ops.tl2_pack(w, 0.02) for w in ws], [qa3[p.K] for p in projs], outs))
            del ws
        same = all(torch.equal(a.clone(), b) for a, b in zip([o.clone() for o in g2[0].launch()], g3[0].launch()))
        steps = 20 * count
        ms2, _, _ = run_steps(torch, [g.launch for g in g2], steps, use_graph)
        ms3, _, mode = run_steps(torch, [g.launch for g in g3], steps, use_graph)
        b2 = sum(p.N * p.K // 4 for p in projs)
        b3 = sum(int(w.desc.bytes) for w in g3[0].weights)
        layers.append({"layer": name, "bytes_2bit": b2, "bytes_tl2": b3, "us_2bit": round(ms2 * 1e3 / steps, 2),
                       "us_tl2": round(ms3 * 1e3 / steps, 2), "tl2_speedup": round(ms2 / ms3, 3),
                       "GBps_2bit": round(b2 / (ms2 * 1e3 / steps) / 1e3, 1),
                       "GBps_tl2_own_bytes": round(b3 / (ms3 * 1e3 / steps) / 1e3, 1),
                       "outputs_bit_identical": bool(same), "launch": mode})
        del g2, g3
    return {"single_matrices": rows, "layers_one_launch": layers}


def extra_config1(torch, use_graph, cpu_seconds=1.0):
    """The smallest case: one 1536x1536 matrix (0.59 MB packed), fp32 activations, M=1, uniform ternary weights with
    scale 0.02.  Launch-latency bound; reported cold (rotating through 1 GiB of copies) and cache-resident (one copy)."""
    import numpy as np
    from paper_2410_16144_amd import ops, synth
    dev = torch.device("cuda:0")
    N = K = 1536
    nb = N * K // 4
    copies = (1 << 30) // nb // 8 + 1    # 8 distinct matrices, each stored this many times: over 1 GiB in all
    rng = synth.rng_for(synth.seed_for(1))
    w0 = synth.ternary_weights(rng, N, K)
    x0 = synth.activations(rng, 1, K)
    base = [ops.pack_ternary(torch.from_numpy(w0).to(dev), 0.02)]
    base += [ops.pack_ternary(synth.ternary_weights_device(100 + i, N, K, dev), 0.02) for i in range(1, 8)]
    pws = [ops.PackedWeight(b.blob.clone(), b.desc) for _ in range(copies) for b in base]
    x = torch.from_numpy(x0).to(dev)
    qa = ops.quant_act(x)
    out = torch.empty((1, N), dtype=torch.float32, device=dev)
    plain = [ops.GemvGroup([pw], [qa], [out]) for pw in pws]
    fused = [ops.DecodeGroup([pw], [x], [out]) for pw in pws]
    res = {"workload": "one 1536x1536 matrix, M=1, fp32 activations (%d copies = %.1f GiB rotated when cold)"
                       % (len(pws), len(pws) * nb / 2**30), "packed_bytes": nb}
    steps = 2 * len(pws)
    kernels = {}
    for label, fns in (("gemv_cold", [g.launch for g in plain]), ("gemv_cache_resident", [plain[0].launch]),
                       ("fused_cold", [g.launch for g in fused]), ("fused_cache_resident", [fused[0].launch])):
        fns[0]()
        kernels[label] = last_kernel()
        ms, _, _ = run_steps(torch, fns, steps, use_graph)
        us = ms * 1e3 / steps
        res[label] = {"us": round(us, 2), "GBps": round(nb / us / 1e3, 1)}
    res["roofline"] = hbm_roofline(kernels["fused_cold"], nb, res["fused_cold"]["us"])
    res["roofline"]["sequence"] = "fused_cold (quantize + product in one launch, weights from HBM)"
    if cpu_seconds > 0:
        import oracle

        def one_pass():
            q, a, _ = oracle.quant_act(x0)
            oracle.dequant(oracle.matmul_i32(q, w0), np.float32(0.02), a)

        cores = oracle.num_threads()
        one_pass()
        n, dt = _passes(one_pass, cpu_seconds)
        oracle.set_num_threads(1)
        try:
            n1, dt1 = _passes(one_pass, cpu_seconds)
        finally:
            oracle.set_num_threads(cores)
        res["cpu_baseline"] = {"value": round(nb * n / dt / 1e9, 3), "unit": "GB/s", "cores": cores, "kind": "oracle",
                               "ms_per_step": round(dt / n * 1e3, 4),
                               "sample": "%d full passes (quantization + product + dequantization), %.1f s" % (n, dt),
                               "one_thread": {"value": round(nb * n1 / dt1 / 1e9, 3), "unit": "GB/s", "cores": 1,
                                              "ms_per_step": round(dt1 / n1 * 1e3, 4)}}
    return res


class PowerSampler:
    """Samples the board's socket power (hwmon power1_input, microwatts) from a thread while GPU work runs."""

    def __init__(self, period=0.02):
        import glob
        import threading
        paths = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input"))
        self.path = paths[0] if paths else None
        self.period, self.samples, self._stop = period, [], threading.Event()
        self._thread = threading.Thread(target=self._run, daemon=True)

    def read(self):
        try:
            with open(self.path) as f:
                return int(f.read()) / 1e6
        except (OSError, ValueError, TypeError):
            return None

    def _run(self):
        while not self._stop.is_set():
            w = self.read()
            if w is not None:
                self.samples.append(w)
            time.sleep(self.period)

    def __enter__(self):
        self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop.set()
        self._thread.join()


def energy_per_token(torch, fns, tokens_per_replay, seconds=3.0, graph=True):
    """Section 3's energy metric on this board: mean socket power while whole tokens are decoded back to back
    for `seconds`, times the time per token.  Returns None where the power sensor is not readable.  graph=False:
    `fns` are called as they are (e.g. one function that replays a captured token)."""
    idle = PowerSampler().read()
    if idle is None:
        return None
    g = None
    if graph:
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                for f in fns:
                    f()
        torch.cuda.synchronize()
        fns = [g.replay]
    for f in fns:
        f()
    torch.cuda.synchronize()
    with PowerSampler() as ps:
        t0 = time.perf_counter()
        n = 0
        while time.perf_counter() - t0 < seconds:
            for _ in range(20):
                for f in fns:
                    f()
            torch.cuda.synchronize()
            n += 20
        dt = time.perf_counter() - t0
    del g
    if not ps.samples:
        return None
    watts = sum(ps.samples) / len(ps.samples)
    per_token = dt / (n * tokens_per_replay)
    return {"socket_power_W_mean": round(watts, 1), "socket_power_W_max": round(max(ps.samples), 1),
            "socket_power_W_idle_before": round(idle, 1), "power_samples": len(ps.samples),
            "ms_per_token_wall": round(per_token * 1e3, 4), "J_per_token": round(watts * per_token, 4),
            "note": "whole-board socket power (hwmon power1_input) x wall time per token; BitLinear products only"}


def extra_appendix_a(torch, use_graph):
    """Token rate of the BitLinear products alone on the 12 model shapes of Appendix A (the paper's own unit,
    tokens/s, on dummy weights as in the paper): one token = n_layers x 7 GEMVs with their 4 quantizations, timed
    (a) as one fused launch per layer and (b) as the four fused launches a real layer's data dependencies allow
    (QKV, O, gate/up, down).  Attention, norms and sampling are not part of this build and not in the figure."""
    from paper_2410_16144_amd import synth
    from paper_2410_16144_amd.decode_layer import make_layer
    dev = torch.device("cuda:0")
    rows = []
    for name, (hidden, ffn, n_layers) in synth.PAPER_MODELS.items():
        layer_bytes = sum(p.packed_bytes for p in synth.layer_projections(hidden, ffn))
        count = max(2, min(n_layers, (1 << 30) // layer_bytes + 1))
        ls = [make_layer(6, i, hidden, ffn, 1, dev, None, 0.0)[0] for i in range(count)]
        steps = max(4 * count, 200)
        row = {"model": name, "hidden": hidden, "ffn": ffn, "layers": n_layers, "packed_GB": round(layer_bytes * n_layers / 1e9, 3),
               "distinct_layers_rotated": count}
        for label, attr in (("one_launch_per_layer", "step_fused"), ("dependency_ordered", "step_fused_dependency_ordered")):
            fns = [getattr(l, attr) for l in ls]
            for f in fns[:2]:
                f()
            ms, _, _ = run_steps(torch, fns, steps, use_graph)
            us = ms * 1e3 / steps
            row[label] = {"us_per_layer": round(us, 2), "ms_per_token": round(us * n_layers / 1e3, 4),
                          "tokens_per_s": round(1e6 / (us * n_layers), 1),
                          "GBps": round(layer_bytes / us / 1e3, 1)}
        rows.append(row)
        del ls
        torch.cuda.empty_cache()
    return rows


def extra_decoder_tokens(torch, models, max_pos=512, tokens=64):
    """Whole-model token rate in the paper's own unit (Section 3's tables: tokens/s) on Appendix A's shapes with
    dummy weights as in the paper: every token passes through ALL layers -- norms, the seven products, rotary
    embedding, attention over the bf16 cache, gate, residuals -- as ONE captured graph per token (10 launches
    per layer).  No embedding lookup, output head or sampling: the paper gives no vocabulary.  Timed at a short
    context (positions 0 .. tokens-1) and at a longer one (the last `tokens` positions below max_pos)."""
    from paper_2410_16144_amd import decoder, synth
    dev = torch.device("cuda:0")
    rows = []
    for name in models or list(synth.PAPER_MODELS):
        hidden, ffn, n_layers = synth.PAPER_MODELS[name]
        stack = decoder.make_stack(name, max_pos, dev)
        stack.capture()
        x = torch.randn((tokens, 1, hidden), device=dev, generator=torch.Generator(device=dev).manual_seed(1))
        row = {"model": name, "hidden": hidden, "ffn": ffn, "layers": n_layers, "heads": synth.PAPER_HEADS[name],
               "packed_GB": round(sum(p.packed_bytes for p in synth.layer_projections(hidden, ffn)) * n_layers / 1e9, 3)}
        for label, start in (("context_0", 0), ("context_%d" % (max_pos - tokens), max_pos - tokens)):
            def run():
                for t in range(tokens):
                    stack.h.copy_(x[t])
                    stack.step()
            stack.set_position(start)
            run()                      # untimed pass (also brings the clocks up)
            stack.set_position(start)
            ms, _ = timed(torch, run)
            assert int(stack.pos[0]) == start + tokens and bool(torch.isfinite(stack.y).all())
            row[label] = {"ms_per_token": round(ms / tokens, 4), "tokens_per_s": round(tokens * 1e3 / ms, 1),
                          "us_per_layer": round(ms * 1e3 / tokens / n_layers, 2)}
        if name in ("700M", "7B", "70B") and PowerSampler().read() is not None:
            # the sizes of the paper's energy table (Section 3): socket power while tokens are decoded back to back
            with PowerSampler() as ps:
                t0, n = time.perf_counter(), 0
                while time.perf_counter() - t0 < 2.0:
                    stack.set_position(0)
                    run()
                    torch.cuda.synchronize()
                    n += tokens
                dt = time.perf_counter() - t0
            if ps.samples:
                watts = sum(ps.samples) / len(ps.samples)
                row["energy"] = {"socket_power_W_mean": round(watts, 1), "ms_per_token_wall": round(dt / n * 1e3, 4),
                                 "J_per_token": round(watts * dt / n, 4),
                                 "note": "whole-board socket power x wall time per token, positions 0..%d, host launch gaps included" % (tokens - 1)}
        rows.append(row)
        del stack
        torch.cuda.empty_cache()
    return rows


def extra_prompt(torch, models, M=512, max_pos=1024):
    """Prompt processing through the same decoder block: M tokens at once, the products as bl_gemm / bl_gemm_batch over
    the M rows, attention as bl_attn_prefill (eager launches).  Prompt tokens per second, first at positions 0..M-1,
    then for a second piece at M..2M-1."""
    from paper_2410_16144_amd import decoder, synth
    dev = torch.device("cuda:0")
    rows = []
    for name in models or ["700M", "7B"]:
        hidden, ffn, n_layers = synth.PAPER_MODELS[name]
        stack = decoder.make_stack(name, max_pos, dev, gated=False)
        x = torch.randn((2 * M, hidden), device=dev, generator=torch.Generator(device=dev).manual_seed(2))
        row = {"model": name, "hidden": hidden, "ffn": ffn, "layers": n_layers, "prompt_tokens": M}
        for label, start in (("positions_0", 0), ("positions_%d" % M, M)):
            piece = x[start:start + M].contiguous()
            stack.set_position(start)
            stack.prefill(piece)           # untimed pass
            stack.set_position(start)
            ms, wall = timed(torch, lambda: stack.prefill(piece))
            assert bool(torch.isfinite(stack.layers[-1].attn.v_cache[start + M - 1].float()).all())
            row[label] = {"ms": round(ms, 3), "prompt_tokens_per_s": round(M * 1e3 / ms, 1),
                          "us_per_layer": round(ms * 1e3 / n_layers, 1), "wall_ms": round(wall, 3)}
        rows.append(row)
        del stack
        torch.cuda.empty_cache()
    return rows


def decoder_cpu_baseline(name="700M", seconds=5.0):
    """The decoder oracle as it stands (numpy fp64 around the C oracle's products), timed on the host on ONE layer of
    the `name` shape, token after token for about `seconds`; the whole model is that times its layer count."""
    import numpy as np
    import oracle
    from oracle import decoder as D
    from paper_2410_16144_amd import synth
    hidden, ffn, n_layers = synth.PAPER_MODELS[name]
    r = synth.rng_for(synth.seed_for(7, 0, 0))
    layer = {}
    for p in synth.layer_projections(hidden, ffn):
        layer[p.name] = synth.ternary_weights(r, p.N, p.K)
        layer["s_" + p.name] = synth.draw_w_scale(r)
    for g, k in (("g_in", hidden), ("g_attn", hidden), ("g_post", hidden), ("g_ffn", ffn)):
        layer[g] = r.uniform(0.5, 1.5, k)
    max_pos = 64
    kc, vc = np.zeros((max_pos, hidden)), np.zeros((max_pos, hidden))
    h = r.standard_normal(hidden)
    D.decoder_layer_step(h, 0, layer, kc, vc, synth.PAPER_HEADS[name])
    n, t0 = 0, time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        D.decoder_layer_step(h, 1 + n % (max_pos - 1), layer, kc, vc, synth.PAPER_HEADS[name])
        n += 1
    dt = time.perf_counter() - t0
    return {"model": name, "kind": "oracle", "cores": oracle.num_threads(), "ms_per_layer": round(dt / n * 1e3, 3),
            "tokens_per_s_whole_model": round(n / dt / n_layers, 2),
            "sample": "%d tokens through one %s-shape layer (positions 1..%d, again and again), %.1f s of CPU work; x %d "
                      "layers" % (n, name, max_pos - 1, dt, n_layers)}


def extra_ceilings(torch, use_graph):
    """The two measured denominators beside the published peaks: a register-only loop of v_mfma_i32_32x32x32_i8 (what the
    matrix cores deliver with nothing in the way, with and without the prefill kernel's in-register code expansion, at
    one and two waves per SIMD), and a read-only 128-bit streaming kernel over buffers of the decode launches' sizes,
    each launch on a buffer that was not read recently (HBM, not the memory-side cache).  The probes are a library of
    their own (tests/ceilings), not part of libbitlinear.so."""
    import ctypes
    path = os.path.join(ROOT, "tests", "ceilings", "libceilings.so")
    if not os.path.exists(path):
        raise RuntimeError("tests/ceilings/libceilings.so is not built: run __graft_entry__.build()")
    lib = ctypes.CDLL(path)
    vp = ctypes.c_void_p
    lib.ceil_mfma_loop.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, vp]
    lib.ceil_stream_read.argtypes = [vp, ctypes.c_int64, vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp]
    dev = torch.device("cuda:0")
    cus = torch.cuda.get_device_properties(dev).multi_processor_count
    sink = torch.zeros(1024, dtype=torch.int32, device=dev)

    def stream():
        return int(torch.cuda.current_stream().cuda_stream)

    def check(rc):
        if rc != 0:
            raise RuntimeError("ceilings probe launch failed: hipError %d" % rc)

    res = {"mfma_loop": [], "stream_read": []}
    ops_iter = lib.ceil_mfma_ops_per_wave_iter()
    for expand in (0, 1):
        for waves_per_simd in (1, 2):
            blocks, iters = cus * waves_per_simd, 4000
            fn = lambda: check(lib.ceil_mfma_loop(expand, blocks, iters, sink.data_ptr(), stream()))
            fn()
            ms, _, _ = run_steps(torch, [fn], 20, use_graph)       # ~0.1 s sustained before the timed replay
            pops = ops_iter * 4.0 * blocks * iters * 20 / (ms * 1e-3) / 1e15
            res["mfma_loop"].append({"operands": "expanded from 2-bit codes in registers (7 VALU ops per operand)" if expand
                                     else "loop constants", "waves_per_simd": waves_per_simd, "POPs": round(pops, 3),
                                     "frac_of_published_peak": round(pops * 1e3 / INT8_PEAK_TOPS, 4)})
    for label, nbytes, copies in (("3B-shape layer", 30976000, 40), ("7B-shape layer", 50593792, 24),
                                  ("100B-shape layer", 462422016, 6), ("1 GiB", 1 << 30, 3)):
        nbytes = nbytes // 1024 * 1024
        bufs = [torch.empty(nbytes, dtype=torch.uint8, device=dev).fill_(i + 1) for i in range(copies)]
        row = {"buffer": label, "bytes": nbytes, "copies_rotated": copies}
        for loads, flag_sets in (("ordinary_loads", (0, 2)), ("streaming_loads", (1, 3))):
            best = None
            for flags in flag_sets:
                for wgs_per_cu, threads, unroll in ((1, 1024, 8), (2, 1024, 8), (2, 1024, 4), (4, 512, 8), (8, 256, 8), (16, 256, 8)):
                    fns = [(lambda b=b: check(lib.ceil_stream_read(b.data_ptr(), nbytes, sink.data_ptr(), cus * wgs_per_cu, threads,
                                                                   unroll, flags, stream()))) for b in bufs]
                    fns[0]()
                    steps = max(2 * copies, int(1e9 // nbytes))
                    ms, _, _ = run_steps(torch, fns, steps, use_graph)
                    us = ms * 1e3 / steps
                    if best is None or us < best[0]:
                        best = (us, wgs_per_cu, threads, unroll, flags)
            us, wgs_per_cu, threads, unroll, flags = best
            row[loads] = {"us": round(us, 2), "GBps": round(nbytes / us / 1e3, 1),
                          "frac_of_published_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4),
                          "launch": "%d workgroups per CU x %d threads, %d loads in flight, %s" % (
                              wgs_per_cu, threads, unroll, "one range per wave" if flags & 2 else "chunks dealt round-robin")}
        res["stream_read"].append(row)
        del bufs
        torch.cuda.empty_cache()
    return res


def headline_100b(torch, np, args, use_graph):
    """The timed region of the default run: the 100B-shape model, all layers resident, one token per step."""
    import oracle
    from paper_2410_16144_amd.decode_layer import make_layer
    dev = torch.device("cuda:0")
    hidden, ffn, n_layers = 12288, 33792, args.model_layers
    t_build = time.perf_counter()
    # layer 0 is drawn on the host so that the oracle sees the same bits; the rest on the device
    layer0, host = make_layer(5, 0, hidden, ffn, 1, dev, None, 0.0, host=True)
    layers = [layer0]
    for i in range(1, n_layers):
        layers.append(make_layer(5, i, hidden, ffn, 1, dev, None, 0.0)[0])
        if i % 10 == 9:
            torch.cuda.synchronize()
            print("bench: %d of %d layers packed (%.0f s)" % (i + 1, n_layers, time.perf_counter() - t_build), file=sys.stderr, flush=True)
    torch.cuda.synchronize()
    layer_bytes = layer0.packed_bytes
    total = layer_bytes * n_layers
    check_layer_against_oracle(torch, np, oracle, layer0, host)
    print("bench: layer 0 agrees with the oracle (bit-exact q / acc, out within 1e-6)", file=sys.stderr, flush=True)

    fns = [l.step_fused for l in layers]

    def token():
        for f in fns:
            f()

    for _ in range(args.warmup):
        token()
    kernel = last_kernel()
    torch.cuda.synchronize()
    if use_graph:
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                token()
        torch.cuda.synchronize()
        step, mode = g.replay, "hip-graph (one graph of %d launches per token)" % n_layers
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < 0.05:      # untimed replays: one-time upload costs, clocks
            g.replay()
            torch.cuda.synchronize()
    else:
        step, mode = token, "eager"

    def run(count):
        for _ in range(count):
            step()

    ms, wall_ms = timed(torch, lambda: run(args.steps))
    ms_per_step = ms / args.steps
    more = sorted([ms_per_step] + [timed(torch, lambda: run(min(args.steps, 20)))[0] / min(args.steps, 20) for _ in range(4)])
    spread = {"replays": len(more), "ms_per_step_min": round(more[0], 5), "ms_per_step_median": round(more[len(more) // 2], 5),
              "ms_per_step_max": round(more[-1], 5)}
    value = total / (ms_per_step * 1e-3) / 1e9
    launch_us = ms_per_step * 1e3 / n_layers      # the step is n_layers launches of ONE kernel, back to back
    result = {
        "metric": "ternary x int8 GEMV packed-weight GB/s", "value": round(value, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "100B-shape full-model token decode, M=1: %d layers (hidden 12288, ffn 33792), per layer the "
                               "absmax int8 quantization of its 4 inputs + 7 ternary GEMVs in one fused launch; "
                               "%.2f GB of 2-bit packed weights resident, every layer its own; one step = one token"
                               % (n_layers, total / 1e9),
                   "launch": mode, "packed_bytes_per_step": total, "tokens_per_s_gemv_only": round(1e3 / ms_per_step, 1),
                   "frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4), "wall_ms_timed_region": round(wall_ms, 3),
                   "spread_over_replays": spread, "build_s": round(time.perf_counter() - t_build, 1)},
        "roofline": hbm_roofline(kernel, layer_bytes, launch_us, load_traffic("decode_kernel_100b_layer_m1_fused")),
    }
    result["roofline"]["launches_per_step"] = n_layers
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_layer_baseline(oracle, host, layer0.projs, layer_bytes, args.cpu_seconds,
                                                    "100B-shape layer at M=1", model_layers=n_layers)
    energy = None
    if use_graph and not args.no_extra:
        energy = energy_per_token(torch, [g.replay], 1, graph=False)
    del layers, fns, layer0, host
    if use_graph:
        del g
    torch.cuda.empty_cache()
    return result, energy


def load_traffic(kernel_key):
    """HBM traffic per launch measured offline with rocprofv3 --pmc (see profiles/): committed numbers."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        return json.load(f).get(kernel_key)


def sections(torch, np, args, use_graph):
    """The extra sections by name (each is also `--only <name>`)."""
    models = args.models.split(",") if args.models else None
    cpu = 0.0 if args.no_cpu else 2.0

    def prefill():
        rows = []
        for m in (512, 2048):
            for (k, n) in ((4096, 11008), (11008, 4096)):
                row = extra_prefill(torch, m, k, n, use_graph)
                if not args.no_cpu:
                    import oracle
                    row["cpu_baseline"] = cpu_prefill_baseline(np, oracle, m, k, n)
                rows.append(row)
        return rows

    return {
        "copy": lambda: extra_copy(torch),
        "ceilings": lambda: extra_ceilings(torch, use_graph),
        "config1": lambda: extra_config1(torch, use_graph, cpu_seconds=cpu / 2),
        "config2": lambda: extra_decode_shape(torch, "3B-shape", 3200, 8640, 1, args.layers, 2000, use_graph, config=2, p_zero=0.4,
                                              outliers=0.01, cpu_seconds=cpu, dependency_ordered=True),
        "config3": lambda: [extra_decode_shape(torch, "7B-shape", 4096, 11008, m, 24, 480, use_graph, config=3, cpu_seconds=cpu)
                            for m in (1, 4, 8)],
        "prefill": prefill,
        "decode100b": lambda: extra_decode_shape(torch, "100B-shape", 12288, 33792, 1, 6, 120, use_graph),
        "paper100b": lambda: extra_decode_shape(torch, "Appendix-A 100B", 8192, 45568, 1, 6, 120, use_graph),
        "appendixa": lambda: extra_appendix_a(torch, use_graph),
        "tokens": lambda: {"gpu": extra_decoder_tokens(torch, models),
                           "cpu_baseline": None if args.no_cpu else decoder_cpu_baseline()},
        "tokens8k": lambda: extra_decoder_tokens(torch, models or ["7B"], max_pos=8192),
        "prompt": lambda: extra_prompt(torch, models),
        "prompt2k": lambda: extra_prompt(torch, models or ["7B"], M=2048, max_pos=4096),
        "tl2": lambda: extra_tl2(torch, use_graph),
    }


def against_measured_ceilings(result, extra):
    """Beside every roofline's `frac` (of the PUBLISHED peak): `frac_of_measured_ceiling`, the same launch against what the
    committed probes reached in this run -- the read-only streaming kernel on a buffer of the same size (decode) or the
    register-only matrix-core loop with in-register expansion at two waves per SIMD (prefill)."""
    c = extra.get("ceilings")
    if not c:
        return
    read_us = {r["buffer"]: r["streaming_loads"]["us"] for r in c["stream_read"]}
    mfma = max(r["POPs"] for r in c["mfma_loop"] if r["operands"].startswith("expanded"))

    def decode(block, buffer):
        r = block.get("roofline")
        if r and buffer in read_us:
            r["frac_of_measured_ceiling"] = round(read_us[buffer] / r["avg_launch_us"], 4)
            r["measured_ceiling"] = "read-only streaming kernel over %s: %.2f us" % (buffer, read_us[buffer])

    decode(result, "100B-shape layer")
    decode(extra.get("config2_3b_layer", {}), "3B-shape layer")
    for block in extra.get("config3_7b_layer", []):
        decode(block, "7B-shape layer")
    for row in extra.get("config4_prefill", []):
        r = row["roofline"]
        r["frac_of_measured_ceiling"] = round(r["achieved"] / mfma, 4)
        r["measured_ceiling"] = "register-only MFMA loop with in-register expansion: %.2f POP/s" % mfma


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (--gpus 1); multi-GPU sharding is a design note, "
              "not code. Refusing --gpus %d." % args.gpus, file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2410_16144_amd import binding

    binding.lib()  # raises if the HIP library is not built; there is no fallback
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    use_graph = not args.no_graph
    global PROFILER_RUN
    PROFILER_RUN = args.profiler_run
    sect = sections(torch, np, args, use_graph)

    if args.only:
        print(json.dumps({args.only: sect[args.only]()}))
        return

    # ---- the timed region: exactly --steps tokens of the 100B-shape model after --warmup untimed ones
    result, energy = headline_100b(torch, np, args, use_graph)

    if not args.no_extra:
        extra = {}
        if energy is not None:
            extra["energy_100b_token"] = energy
        # the other benchmark configurations, each with its own roofline and cpu_baseline; then the measured ceilings,
        # the paper's own 100B shape, and the whole-model token loop in the paper's unit on three of Appendix A's shapes
        for name, key in (("config1", "config1_1536"), ("config2", "config2_3b_layer"), ("config3", "config3_7b_layer"),
                          ("prefill", "config4_prefill"), ("ceilings", "ceilings"), ("copy", "copy_1GiB"),
                          ("paper100b", "decode_paper_100b_layer")):
            t0 = time.perf_counter()
            extra[key] = sect[name]()
            torch.cuda.empty_cache()
            print("bench: section %s done (%.0f s)" % (name, time.perf_counter() - t0), file=sys.stderr, flush=True)
        extra["decoder_tokens"] = extra_decoder_tokens(torch, ["700M", "7B", "30B"])
        torch.cuda.empty_cache()
        against_measured_ceilings(result, extra)
        result["extra"] = extra

    print(json.dumps(result))


if __name__ == "__main__":
    main()
