#!/usr/bin/env python3
"""Benchmark of the BitLinear W1.58A8 hot path on one MI355X.

Headline workload (config 1 of the benchmark spec): decode at M=1 over the four
BitLinear shapes of a 2B-style layer, for 30 distinct layers (521 MB of packed
weights, more than L2 + Infinity Cache, so everything streams from HBM).  A
"step" is one pass of the hot path over those 30 layers = 120 BitLinears: for
each, per-token absmax int8 quantisation of its bf16 activations, the
packed-ternary product with int32 accumulation, and the fp32 rescale - all in
ONE launch of the persistent streaming kernel (bl_stack_run).  Launches are
replayed from a HIP graph; inputs are resident in HBM.

    value = packed weight bytes per step / time per step   [GB/s]

Also reported in the same JSON line: the same work as one launch per layer
(the previous headline), the measured achievable roofs (plain streaming read,
register-resident int8 MFMA loop), the prefill product (config 3: M=2048, int8
matrix-core TOPS), batched decode (config 2), the chained stack (config 4) and
the CPU oracle timed on the host cores (baseline only).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
INT8_PEAK_TOPS = 5000.0      # MI355X dense int8 MFMA, published (5.0 POP/s)
SHAPE_ORDER = ["qkv", "o", "gate_up", "down"]


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def profiled_traffic(key):
    """HBM bytes per launch (read + written) of a kernel/workload, from the rocprofv3 --pmc
    FETCH_SIZE / WRITE_SIZE summary committed in profiles/hbm_traffic.txt (lines
    `key read_bytes write_bytes`, counters already scaled by the plain-copy calibration).
    None if the file or the key is missing: the bench line then says so instead of guessing."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    try:
        for line in open(path):
            f = line.split()
            if len(f) >= 3 and f[0] == key:
                return float(f[1]) + float(f[2])
    except OSError:
        pass
    return None


class Layer:
    """Device-resident packed weights and decode/prefill buffers of one layer."""
    pass


def build_layers(bl, torch, synth, n_layers, layout, dev):
    layers = []
    t0 = time.time()
    for l in range(n_layers):
        L = Layer()
        L.packed, L.beta = {}, {}
        for name in SHAPE_ORDER:
            N, K = synth.LAYER_SHAPES[name]
            W = torch.from_numpy(synth.latent_weights(0, N, K, layer=l, matrix=name)).to(dev)
            L.packed[name], L.beta[name] = bl.bl_pack_ternary(W, layout)
            del W
        layers.append(L)
        if l % 10 == 9:
            torch.cuda.synchronize()
            log("[bench] packed %d/%d layers (%.1fs)" % (l + 1, n_layers, time.time() - t0))
    torch.cuda.synchronize()
    return layers


def make_decode_buffers(bl, torch, synth, M, dev):
    import numpy as np
    buf = {}
    for name in SHAPE_ORDER:
        N, K = synth.LAYER_SHAPES[name]
        X = synth.activations_bf16(0, M, K, layer=0, matrix=name, relu2=(name == "down"))
        b = Layer()
        b.X = torch.from_numpy(X.view(np.int16)).to(dev).view(torch.bfloat16)
        b.q = torch.empty((M, K), dtype=torch.int8, device=dev)
        b.scale = torch.empty(M, dtype=torch.float32, device=dev)
        b.rowsum = torch.empty(M, dtype=torch.int32, device=dev)
        b.y = torch.empty((M, N), dtype=torch.float32, device=dev)
        b.N, b.K, b.M = N, K, M
        buf[name] = b
    return buf


def decode_step(lib, stream, L, buf, layout, with_quant=True):
    """Per-call path: for each of the four BitLinears, bl_quant_act_int8 then
    bl_gemv_w158a8 (8 launches per layer)."""
    for name in SHAPE_ORDER:
        b = buf[name]
        if with_quant:
            rc = lib.bl_quant_act_int8(b.X.data_ptr(), b.M, b.K, b.q.data_ptr(), b.scale.data_ptr(),
                                       b.rowsum.data_ptr(), stream)
            assert rc == 0, rc
        rc = lib.bl_gemv_w158a8(L.packed[name].data_ptr(), L.beta[name].data_ptr(), layout, b.q.data_ptr(),
                                b.scale.data_ptr(), b.rowsum.data_ptr(), b.M, b.N, b.K, None, b.y.data_ptr(),
                                None, stream)
        assert rc == 0, rc


def decode_step_fused(lib, stream, L, buf, layout):
    """Fused path: bl_bitlinear_decode per shape (quantiser inside the product kernel, 4 launches)."""
    for name in SHAPE_ORDER:
        b = buf[name]
        rc = lib.bl_bitlinear_decode(L.packed[name].data_ptr(), L.beta[name].data_ptr(), layout, b.X.data_ptr(),
                                     b.M, b.N, b.K, None, b.y.data_ptr(), None, None, stream)
        assert rc == 0, rc


def make_group_descs(bl, layers, buf, fused=True):
    """One bl_decode_desc array per layer: the four shapes, fp32 outputs; inputs bf16
    (fused quantiser) or already quantised int8 with scales and row sums."""
    out = []
    for L in layers:
        items = []
        for n in SHAPE_ORDER:
            it = dict(packed=L.packed[n], beta=L.beta[n], N=buf[n].N, K=buf[n].K, y=buf[n].y)
            if fused:
                it["X"] = buf[n].X
            else:
                it.update(q=buf[n].q, scale=buf[n].scale, rowsum=buf[n].rowsum)
            items.append(it)
        out.append(bl.make_decode_descs(items))
    return out


def capture(torch, fn):
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    return g


def time_graph_steps(torch, graphs_and_counts, total_steps):
    """Replay graphs covering exactly total_steps steps; returns seconds."""
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    done = 0
    for g, cnt, reps in graphs_and_counts:
        for _ in range(reps):
            g.replay()
            done += cnt
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    assert done == total_steps, (done, total_steps)
    return e0.elapsed_time(e1) * 1e-3, t1 - t0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3000)
    ap.add_argument("--warmup", type=int, default=300)
    ap.add_argument("--layers", type=int, default=30, help="distinct layers rotated through (30 = 521 MB)")
    ap.add_argument("--layout", type=int, default=1)
    ap.add_argument("--no-prefill", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-chain", action="store_true")
    ap.add_argument("--no-batched", action="store_true")
    ap.add_argument("--prefill-m", type=int, default=2048)
    ap.add_argument("--no-large-m", action="store_true", help="leave out the prefill layer at M = 8192 (profile runs: its launches share grids with M = 2048)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (reference for scaling HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")
        sys.exit(2)

    import numpy as np
    import torch
    import synth
    from paper_2504_12285_amd import binding as bl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    lib = bl.load()
    layout = args.layout
    nl = args.layers
    layers = build_layers(bl, torch, synth, nl, layout, dev)
    layer_bytes = sum(n * k // 4 for n, k in synth.LAYER_SHAPES.values())

    # ------------------------------------------------------------ decode, M=1
    M = 1
    buf = make_decode_buffers(bl, torch, synth, M, dev)
    side = torch.cuda.Stream()
    K_steps, W_steps = args.steps, args.warmup
    stack_bytes = nl * layer_bytes
    sink = torch.zeros(64, dtype=torch.int32, device=dev)
    with torch.cuda.stream(side):
        st = torch.cuda.current_stream().cuda_stream
        for l in range(min(nl, 4)):
            decode_step(lib, st, layers[l], buf, layout)
        torch.cuda.synchronize()

        # headline: the 120 BitLinears of the 30 layers in one streamed launch, quantiser inside
        items = []
        ys = []
        for L in layers:
            for n in SHAPE_ORDER:
                y = torch.empty((1, buf[n].N), dtype=torch.float32, device=dev)
                ys.append(y)
                items.append(dict(packed=L.packed[n], beta=L.beta[n], N=buf[n].N, K=buf[n].K, X=buf[n].X, y=y))
        stack = bl.Stack(items, layout, 1, dev)
        assert stack.plan.packed_bytes == stack_bytes and stack.plan.prep_count == 0
        stack.run()
        torch.cuda.synchronize()
        per_graph = 10
        g_stack = capture(torch, lambda: [stack.run() for _ in range(per_graph)])
        plan = [(g_stack, per_graph, K_steps // per_graph)] if K_steps >= per_graph else []
        if K_steps % per_graph:
            g_rem = capture(torch, lambda: [stack.run() for _ in range(K_steps % per_graph)])
            plan.append((g_rem, K_steps % per_graph, 1))
        for _ in range(max(1, W_steps // per_graph)):
            g_stack.replay()
        torch.cuda.synchronize()
        t_gpu, t_wall = time_graph_steps(torch, plan, K_steps)
        ms_per_step = t_gpu * 1e3 / K_steps
        value = stack_bytes / (t_gpu / K_steps) / 1e9
        # the timed region consists of launches of the streaming kernel only (the quantiser runs
        # inside it), so the same HIP-event interval gives that kernel's average launch duration
        stream_avg_s = t_gpu / K_steps

        # the same work as one launch per layer (bl_bitlinear_decode_group: four shapes, fused quantiser)
        descs = make_group_descs(bl, layers, buf)

        def run_steps(first, count, mode="group"):
            s = torch.cuda.current_stream().cuda_stream
            for i in range(first, first + count):
                L = layers[i % nl]
                if mode == "group":          # the whole layer: one launch, quantiser fused
                    rc = lib.bl_bitlinear_decode_group(descs[i % nl], 4, layout, M, s)
                    assert rc == 0, rc
                elif mode == "fused":
                    decode_step_fused(lib, s, L, buf, layout)
                elif mode == "calls":
                    decode_step(lib, s, L, buf, layout, True)
                else:                        # products only, activations already quantised
                    decode_step(lib, s, L, buf, layout, False)

        reps = max(1, min(K_steps, 20))
        alt = {}
        for mode, launches in (("group", 1), ("fused", 4), ("calls", 8), ("gemv_only", 4)):
            g = capture(torch, lambda: run_steps(0, nl, mode))
            for _ in range(2):
                g.replay()
            t_alt, _ = time_graph_steps(torch, [(g, nl, reps)], nl * reps)
            alt[mode] = {"us_per_layer": round(t_alt / (nl * reps) * 1e6, 3), "launches_per_layer": launches,
                         "GBps": round(layer_bytes / (t_alt / (nl * reps)) / 1e9, 1)}
        one_layer_s = alt["group"]["us_per_layer"] * 1e-6
        # the streaming kernel on one layer per launch and on one very large product
        st1 = [bl.Stack(items[4 * l:4 * l + 4], layout, 1, dev) for l in range(nl)]
        g = capture(torch, lambda: [s_.run() for s_ in st1])
        g.replay()
        t_alt, _ = time_graph_steps(torch, [(g, nl, reps)], nl * reps)
        alt["stream_one_layer_per_launch"] = {"us_per_layer": round(t_alt / (nl * reps) * 1e6, 3), "launches_per_layer": 1,
                                              "GBps": round(layer_bytes / (t_alt / (nl * reps)) / 1e9, 1)}
        del st1
        big_n = 30 * 13824
        big = torch.randint(0, 256, (big_n * 2560 // 4,), dtype=torch.uint8, device=dev)
        yb = torch.empty((1, big_n), dtype=torch.float32, device=dev)
        stb = bl.Stack([dict(packed=big, beta=layers[0].beta["gate_up"], N=big_n, K=2560, X=buf["gate_up"].X, y=yb)],
                       layout, 1, dev)
        g = capture(torch, stb.run)
        g.replay()
        t_big, _ = time_graph_steps(torch, [(g, 1, 10)], 10)
        alt["large_n"] = {"shape": "N=%d K=2560 M=1, one streamed launch" % big_n, "us": round(t_big / 10 * 1e6, 2),
                          "GBps": round(big_n * 2560 / 4 / (t_big / 10) / 1e9, 1)}
        del big, yb, stb

        # the same 120 BitLinears with five weights per byte (layout 2: a fifth fewer bytes, three times
        # the decode arithmetic per weight): repacked on the GPU from the 2-bit form
        items5, keep5 = [], []
        for L in layers:
            for n in SHAPE_ORDER:
                Wt, _bad = bl.bl_unpack_ternary(L.packed[n], buf[n].N, buf[n].K, layout)
                p5, _ = bl.bl_pack_ternary(Wt, bl.BL_LAYOUT_TRIT5, beta=L.beta[n])
                keep5.append(p5)
                items5.append(dict(packed=p5, beta=L.beta[n], N=buf[n].N, K=buf[n].K, X=buf[n].X,
                                   y=torch.empty((1, buf[n].N), dtype=torch.float32, device=dev)))
                del Wt
        st5 = bl.Stack(items5, bl.BL_LAYOUT_TRIT5, 1, dev)
        st5.run()
        torch.cuda.synchronize()
        assert all(torch.equal(a["y"], y) for a, y in zip(items5, ys)), "five-per-byte form disagrees with the 2-bit form"
        g = capture(torch, lambda: [st5.run() for _ in range(10)])
        g.replay()
        t5, _ = time_graph_steps(torch, [(g, 10, 5)], 50)
        alt["stream_five_weights_per_byte"] = {
            "us_per_step": round(t5 / 50 * 1e6, 2), "packed_bytes_per_step": int(st5.plan.packed_bytes),
            "GBps_of_its_own_bytes": round(st5.plan.packed_bytes / (t5 / 50) / 1e9, 1),
            "GBps_in_2bit_bytes": round(stack_bytes / (t5 / 50) / 1e9, 1)}
        del st5, items5, keep5

        # the 30 down projections as one table: dense (layout 1) against the k-major form (layout 3), which
        # does not read the weights of zero activations; with the squared-ReLU inputs as generated and with
        # ordinary activations of which a seeded half is set to zero
        def down_tables(Xs):
            dense, sparse, keep = [], [], []
            for L, X in zip(layers, Xs):
                Wt, _bad = bl.bl_unpack_ternary(L.packed["down"], 2560, 6912, layout)
                pk, _ = bl.bl_pack_ternary(Wt, bl.BL_LAYOUT_KMAJOR, beta=L.beta["down"])
                del Wt
                keep.append(pk)
                for lst, pw in ((dense, L.packed["down"]), (sparse, pk)):
                    lst.append(dict(packed=pw, beta=L.beta["down"], N=2560, K=6912, X=X,
                                    y=torch.empty((1, 2560), dtype=torch.float32, device=dev)))
            return dense, sparse, keep
        rng_s = np.random.default_rng(11)
        x_gen = [torch.from_numpy(synth.activations_bf16(0, 1, 6912, layer=l, matrix="down", relu2=True).view(np.int16))
                 .to(dev).view(torch.bfloat16) for l in range(nl)]
        x_half = []
        for l in range(nl):
            xb = synth.activations_bf16(0, 1, 6912, layer=l, matrix="down", relu2=False)
            xb = np.where(rng_s.random(xb.shape) < 0.5, xb, np.uint16(0)).astype(np.uint16)
            x_half.append(torch.from_numpy(xb.view(np.int16)).to(dev).view(torch.bfloat16))
        sparsity = {}
        for tag, Xs in (("squared_relu_inputs_as_generated", x_gen), ("half_of_the_inputs_zero", x_half)):
            dense, sparse, keep = down_tables(Xs)
            qs = [bl.bl_quant_act_int8(X)[0] for X in Xs]
            nz = float(np.mean([float((q != 0).float().mean().item()) for q in qs]))
            res = {"nonzero_fraction_of_q": round(nz, 4)}
            outs = {}
            for name, tab, lay in (("dense_layout1", dense, layout), ("k_major", sparse, bl.BL_LAYOUT_KMAJOR)):
                st_ = bl.Stack(tab, lay, 1, dev)
                st_.run()
                torch.cuda.synchronize()
                outs[name] = [t_["y"].clone() for t_ in tab]
                g = capture(torch, lambda: [st_.run() for _ in range(10)])
                g.replay()
                tt, _ = time_graph_steps(torch, [(g, 10, 5)], 50)
                res[name] = {"us_per_30_products": round(tt / 50 * 1e6, 2), "packed_bytes": int(st_.plan.packed_bytes)}
                del st_
            assert all(torch.equal(a, b) for a, b in zip(outs["dense_layout1"], outs["k_major"]))
            res["k_major"]["weight_bytes_of_nonzero_rows"] = int(res["k_major"]["packed_bytes"] * nz)
            sparsity[tag] = res
            del dense, sparse, keep
        alt["down_projection_sparsity"] = sparsity
        log("[bench] down projection, 30 layers per launch: %s" % sparsity)

        # achievable roof: a plain 128-bit streaming read (same slicing, no arithmetic) of 2 GiB, and
        # of as many bytes as one step streams, at the stream kernel's occupancy and at the best one
        probe = torch.randint(0, 256, (2 << 30,), dtype=torch.uint8, device=dev)

        def probe_rate(nbytes, per_cu):
            def fn():
                rc = lib.bl_probe_stream_read(probe.data_ptr(), nbytes, per_cu, sink.data_ptr(),
                                              torch.cuda.current_stream().cuda_stream)
                assert rc == 0, rc
            fn()
            g_ = capture(torch, fn)
            g_.replay()
            t_, _ = time_graph_steps(torch, [(g_, 1, 10)], 10)
            return nbytes / (t_ / 10) / 1e9
        read_roof = {"bytes_2GiB_8wg_per_cu": round(probe_rate(2 << 30, 8), 1),
                     "bytes_2GiB_4wg_per_cu": round(probe_rate(2 << 30, 4), 1),
                     "bytes_of_one_step_4wg_per_cu": round(probe_rate(stack_bytes, 4), 1)}
        del probe
        achievable = max(read_roof.values())
    log("[bench] decode M=1, 120 BitLinears per streamed launch: %.2f us/step, %.1f GB/s (%.3f of %.0f); "
        "one launch per layer: %s; read roof %s"
        % (ms_per_step * 1e3, value, value / HBM_PEAK_GBS, HBM_PEAK_GBS, alt, read_roof))

    out = {
        "metric": "W1.58A8 GEMV HBM GB/s at M=1 (decode) + int8 TOPS at M=2048 (prefill)",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": K_steps, "warmup": W_steps,
        "ms_per_step": round(ms_per_step, 6), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "config 1: decode M=1 over the four BitLinear shapes of a 2B-style layer (qkv 3840x2560, "
                               "o 2560x2560, gate_up 13824x2560, down 2560x6912), %d distinct layers = %d BitLinears per "
                               "step, quantise+product+rescale of every one" % (nl, 4 * nl),
                   "packed_bytes_per_step": stack_bytes, "layout": layout,
                   "launch": "hip graph; one bl_stack_run launch per step (persistent streaming kernel over a device "
                             "table of %d products, absmax int8 quantiser inside the launch)" % (4 * nl)},
        "roofline": {"bound": "hbm", "achieved": round(value, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(value / HBM_PEAK_GBS, 4), "traffic": profiled_traffic("bl_stream_m1:30_layers"),
                     "kernel": "bl_stream_m1", "bytes_per_launch": float(stack_bytes),
                     "avg_launch_us": round(stream_avg_s * 1e6, 3),
                     "achievable": achievable, "frac_of_achievable": round(value / achievable, 4),
                     "achievable_detail": read_roof},
        "roofline_one_layer_per_launch": {
            "bound": "hbm", "achieved": round(layer_bytes / one_layer_s / 1e9, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(layer_bytes / one_layer_s / 1e9 / HBM_PEAK_GBS, 4),
            "traffic": profiled_traffic("bl_gemv_rows:one_layer"), "kernel": "bl_gemv_rows",
            "bytes_per_launch": float(layer_bytes), "avg_launch_us": round(one_layer_s * 1e6, 3),
            "note": "the same 120 BitLinears as 30 launches of bl_bitlinear_decode_group (17.4 MB each): launch and "
                    "ramp bound, a plain read of 17.4 MB takes about 7 us"},
        "decode_alternatives": alt,
    }

    if args.calibrate_copy:
        ca = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        cb = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        for _ in range(5):
            cb.copy_(ca)
        torch.cuda.synchronize()
        del ca, cb

    # ------------------------------------------------------- prefill, M=2048
    if not args.no_prefill:
        Mp = args.prefill_m
        pre = {}
        for name in SHAPE_ORDER:
            N, K = synth.LAYER_SHAPES[name]
            X = synth.activations_bf16(0, Mp, K, layer=0, matrix=name, relu2=(name == "down"))
            Xd = torch.from_numpy(X.view(np.int16)).to(dev).view(torch.bfloat16)
            b = Layer()
            b.q, b.scale, b.rowsum = bl.bl_quant_act_int8(Xd)
            b.y = torch.empty((Mp, N), dtype=torch.float32, device=dev)
            b.N, b.K = N, K
            pre[name] = b
        torch.cuda.synchronize()

        def prefill_layer(l):
            s = torch.cuda.current_stream().cuda_stream
            for name in SHAPE_ORDER:
                b = pre[name]
                rc = lib.bl_gemm_w158a8(layers[l].packed[name].data_ptr(), layers[l].beta[name].data_ptr(), layout,
                                        b.q.data_ptr(), b.scale.data_ptr(), b.rowsum.data_ptr(), Mp, b.N, b.K,
                                        None, b.y.data_ptr(), None, s)
                assert rc == 0, rc

        for l in range(2):
            prefill_layer(l)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n_pre = 2 * nl
        e0.record()
        for i in range(n_pre):
            prefill_layer(i % nl)
        e1.record()
        torch.cuda.synchronize()
        t_pre = e0.elapsed_time(e1) * 1e-3 / n_pre
        ops = sum(2.0 * Mp * n * k for n, k in synth.LAYER_SHAPES.values())
        tops = ops / t_pre / 1e12
        per_shape = {}
        for name in SHAPE_ORDER:
            b = pre[name]
            e0.record()
            for i in range(nl):
                rc = lib.bl_gemm_w158a8(layers[i].packed[name].data_ptr(), layers[i].beta[name].data_ptr(), layout,
                                        b.q.data_ptr(), b.scale.data_ptr(), b.rowsum.data_ptr(), Mp, b.N, b.K,
                                        None, b.y.data_ptr(), None, torch.cuda.current_stream().cuda_stream)
            e1.record()
            torch.cuda.synchronize()
            dt = e0.elapsed_time(e1) * 1e-3 / nl
            per_shape[name] = {"us": round(dt * 1e6, 2), "tops": round(2.0 * Mp * b.N * b.K / dt / 1e12, 1)}
        # the same four launches at M = 8192 (not the headline size: what the tile kernel does once a
        # workgroup has several tiles and its stores travel during the next tile)
        large_m = None
        if Mp == 2048 and not args.no_large_m:
            Ml = 8192
            ql = {K: torch.randint(-127, 128, (Ml, K), dtype=torch.int8, device=dev) for K in (2560, 6912)}
            sl = torch.rand(Ml, device=dev) * 0.01 + 0.01
            rl = {K: ql[K].to(torch.int32).sum(1).to(torch.int32) for K in ql}
            yl = torch.empty((Ml, 13824), dtype=torch.float32, device=dev)

            def large_layer(l):
                s_ = torch.cuda.current_stream().cuda_stream
                for name in SHAPE_ORDER:
                    N, K = synth.LAYER_SHAPES[name]
                    rc = lib.bl_gemm_w158a8(layers[l].packed[name].data_ptr(), layers[l].beta[name].data_ptr(), layout,
                                            ql[K].data_ptr(), sl.data_ptr(), rl[K].data_ptr(), Ml, N, K, None,
                                            yl.data_ptr(), None, s_)
                    assert rc == 0, rc
            for i in range(4):
                large_layer(i % nl)
            torch.cuda.synchronize()
            e0.record()
            for i in range(16):
                large_layer(i % nl)
            e1.record()
            torch.cuda.synchronize()
            t_l = e0.elapsed_time(e1) * 1e-3 / 16
            ops_l = sum(2.0 * Ml * n * k for n, k in synth.LAYER_SHAPES.values())
            large_m = {"M": Ml, "us_per_layer": round(t_l * 1e6, 1), "tops": round(ops_l / t_l / 1e12, 1),
                       "frac_of_int8_peak": round(ops_l / t_l / 1e12 / INT8_PEAK_TOPS, 4),
                       "data": "uniform random int8 activations (timing only)"}
            del ql, rl, yl
        # what the memory system takes when every workgroup stores its tile at once: the epilogue's
        # store pattern alone, on a matrix of the size of the widest output (3 workgroups per CU)
        wr = torch.empty((Mp, 13824), dtype=torch.float32, device=dev)
        for _ in range(2):
            assert lib.bl_probe_stream_write(wr.data_ptr(), Mp, 13824, 3, torch.cuda.current_stream().cuda_stream) == 0
        torch.cuda.synchronize()
        e0.record()
        for _ in range(10):
            lib.bl_probe_stream_write(wr.data_ptr(), Mp, 13824, 3, torch.cuda.current_stream().cuda_stream)
        e1.record()
        torch.cuda.synchronize()
        write_roof = Mp * 13824 * 4 / (e0.elapsed_time(e1) * 1e-3 / 10) / 1e9
        out_bytes = sum(Mp * n * 4 for n, _ in synth.LAYER_SHAPES.values())
        del wr
        # the clock the tile kernel actually runs at: workgroup 0 of every launch counts shader
        # clocks and ticks of the constant-rate wall clock (the chip lowers its clock under the
        # power this kernel draws, so the datasheet peak at 2.4 GHz is not what it is offered)
        wall_khz = lib.bl_probe_wall_clock_khz()
        stamps = torch.zeros(2, dtype=torch.int64, device=dev)
        if wall_khz > 0:
            assert lib.bl_debug_clock_stamps(stamps.data_ptr()) == 0
            for name in SHAPE_ORDER:
                b = pre[name]
                mhz = []
                for i in range(nl):
                    rc = lib.bl_gemm_w158a8(layers[i].packed[name].data_ptr(), layers[i].beta[name].data_ptr(), layout,
                                            b.q.data_ptr(), b.scale.data_ptr(), b.rowsum.data_ptr(), Mp, b.N, b.K,
                                            None, b.y.data_ptr(), None, torch.cuda.current_stream().cuda_stream)
                    assert rc == 0, rc
                    if i >= nl // 2:
                        c, w = stamps.tolist()
                        if w > 0:
                            mhz.append(c / (w / (wall_khz * 1e3)) / 1e6)
                per_shape[name]["clock_mhz"] = round(float(np.median(mhz)), 0) if mhz else None
            assert lib.bl_debug_clock_stamps(None) == 0
        # achievable roof of the matrix cores: a register-resident loop of the same MFMA instruction
        import ctypes
        mops = ctypes.c_double(0)
        rc = lib.bl_probe_mfma_i8(20000, sink.data_ptr(), ctypes.byref(mops), torch.cuda.current_stream().cuda_stream)
        assert rc == 0, rc
        torch.cuda.synchronize()
        e0.record()
        for _ in range(3):
            lib.bl_probe_mfma_i8(20000, sink.data_ptr(), None, torch.cuda.current_stream().cuda_stream)
        e1.record()
        torch.cuda.synchronize()
        mfma_roof = mops.value / (e0.elapsed_time(e1) * 1e-3 / 3) / 1e12
        # the same loop on random int8 operands (the activations of this workload for one operand
        # and ternary codes for the other would sit between the two), with the clock it ran at
        rnd = torch.randint(-127, 128, (65536,), dtype=torch.int8, device=dev)
        lib.bl_probe_mfma_i8_ex(20000, rnd.data_ptr(), stamps.data_ptr(), sink.data_ptr(), None,
                                torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(3):
            lib.bl_probe_mfma_i8_ex(20000, rnd.data_ptr(), stamps.data_ptr(), sink.data_ptr(), None,
                                    torch.cuda.current_stream().cuda_stream)
        e1.record()
        torch.cuda.synchronize()
        mfma_roof_rnd = mops.value / (e0.elapsed_time(e1) * 1e-3 / 3) / 1e12
        c, w = stamps.tolist()
        mfma_rnd_mhz = round(c / (w / (wall_khz * 1e3)) / 1e6, 0) if wall_khz > 0 and w > 0 else None
        clocks = [v.get("clock_mhz") for v in per_shape.values() if v.get("clock_mhz")]
        kernel_mhz = float(np.mean(clocks)) if clocks else None
        log("[bench] prefill M=%d: %.1f us/layer, %.1f TOPS (MFMA-only loop: %.0f, on random operands %.0f at %s MHz; tile kernel at %s MHz); %s"
            % (Mp, t_pre * 1e6, tops, mfma_roof, mfma_roof_rnd, mfma_rnd_mhz, kernel_mhz, per_shape))
        out["prefill"] = {"workload": "config 3: M=%d, four layer shapes, int8 q + per-row scales -> fp32 y" % Mp,
                          "tops": round(tops, 2), "unit": "TOP/s", "us_per_layer": round(t_pre * 1e6, 2),
                          "per_shape": per_shape, "same_layer_at_large_m": large_m,
                          "output_stores": {"bytes_per_layer": out_bytes, "store_pattern_alone_GBps": round(write_roof, 1),
                                            "us_per_layer_at_that_rate": round(out_bytes / write_roof / 1e3, 1)},
                          "roofline": {"bound": "mfma", "achieved": round(tops, 2), "peak": INT8_PEAK_TOPS,
                                       "unit": "TOP/s", "frac": round(tops / INT8_PEAK_TOPS, 4),
                                       "traffic": profiled_traffic("bl_gemm_tile256:layer_m2048") if Mp == 2048 else None,
                                       "kernel": "bl_gemm_tile256", "achievable": round(mfma_roof, 1),
                                       "frac_of_achievable": round(tops / mfma_roof, 4),
                                       "achievable_random_operands": round(mfma_roof_rnd, 1),
                                       "achievable_random_operands_clock_mhz": mfma_rnd_mhz,
                                       "frac_of_achievable_random_operands": round(tops / mfma_roof_rnd, 4),
                                       "kernel_clock_mhz": round(kernel_mhz, 0) if kernel_mhz else None,
                                       "peak_at_kernel_clock": round(INT8_PEAK_TOPS * kernel_mhz / 2400.0, 1) if kernel_mhz else None,
                                       "frac_at_kernel_clock": round(tops / (INT8_PEAK_TOPS * kernel_mhz / 2400.0), 4) if kernel_mhz else None}}

    # ------------------------------------------- config 2: batched decode, M in {8, 32, 64}
    if not args.no_batched:
        cfg2 = {}
        for Mb in (8, 32, 64):
            bb = make_decode_buffers(bl, torch, synth, Mb, dev)
            for name in SHAPE_ORDER:
                b = bb[name]
                lib.bl_quant_act_int8(b.X.data_ptr(), Mb, b.K, b.q.data_ptr(), b.scale.data_ptr(), b.rowsum.data_ptr(),
                                      torch.cuda.current_stream().cuda_stream)
            ws = torch.empty(4096, dtype=torch.uint8, device=dev)
            torch.cuda.synchronize()

            def run_b():
                s = torch.cuda.current_stream().cuda_stream
                for l in range(nl):
                    for name in SHAPE_ORDER:
                        b = bb[name]
                        rc = lib.bl_gemv_w158a8(layers[l].packed[name].data_ptr(), layers[l].beta[name].data_ptr(),
                                                layout, b.q.data_ptr(), b.scale.data_ptr(), b.rowsum.data_ptr(), Mb,
                                                b.N, b.K, None, b.y.data_ptr(), ws.data_ptr(), s)
                        assert rc == 0, rc
            descs_q = make_group_descs(bl, layers, bb, fused=False)

            def run_g():
                s = torch.cuda.current_stream().cuda_stream
                for l in range(nl):
                    rc = lib.bl_bitlinear_decode_group(descs_q[l], 4, layout, Mb, s)
                    assert rc == 0, rc
            variants = {"calls": run_b, "grouped": run_g}
            if Mb * (6912 + 16) <= 96 * 1024:
                descs_x = make_group_descs(bl, layers, bb, fused=True)

                def run_f():
                    s = torch.cuda.current_stream().cuda_stream
                    for l in range(nl):
                        rc = lib.bl_bitlinear_decode_group(descs_x[l], 4, layout, Mb, s)
                        assert rc == 0, rc
                variants["grouped_fused"] = run_f
            ops2 = sum(2.0 * Mb * n * k for n, k in synth.LAYER_SHAPES.values())
            res = {}
            with torch.cuda.stream(side):
                for vname, fn in variants.items():
                    fn()
                    torch.cuda.synchronize()
                    g = capture(torch, fn)
                    g.replay()
                    t_b, _ = time_graph_steps(torch, [(g, nl, 5)], 5 * nl)
                    t_b /= 5 * nl
                    res[vname] = {"us_per_layer": round(t_b * 1e6, 2), "GBps_packed": round(layer_bytes / t_b / 1e9, 1),
                                  "tops": round(ops2 / t_b / 1e12, 2)}
            # one streamed launch over all layers (bl_stack_* in its batched form: the token rows of a
            # product in LDS, the weights streamed once through the matrix cores)
            if layout == 1:
                items_b = [dict(packed=layers[l].packed[name], beta=layers[l].beta[name], q=bb[name].q,
                                scale=bb[name].scale, rowsum=bb[name].rowsum, N=bb[name].N, K=bb[name].K, y=bb[name].y)
                           for l in range(nl) for name in SHAPE_ORDER]
                stb = bl.Stack(items_b, layout, Mb, dev)
                with torch.cuda.stream(side):
                    stb.run()
                    torch.cuda.synchronize()
                    g = capture(torch, stb.run)
                    g.replay()
                    t_s, _ = time_graph_steps(torch, [(g, 1, 30)], 30)
                    t_s /= 30 * nl
                res["streamed"] = {"us_per_layer": round(t_s * 1e6, 2), "GBps_packed": round(layer_bytes / t_s / 1e9, 1),
                                   "frac_of_hbm_peak": round(layer_bytes / t_s / 1e9 / HBM_PEAK_GBS, 4),
                                   "tops": round(ops2 / t_s / 1e12, 2), "launches_per_%d_layers" % nl: 1 if stb.plan.prep_count == 0 else 2,
                                   "table_entries": int(stb.plan.entries)}
                del stb, items_b
            cfg2["M=%d" % Mb] = res
            del bb
        out["config2_batched_decode"] = cfg2
        log("[bench] config 2 (calls: 4 bl_gemv_w158a8 launches per layer, int8 inputs; grouped: one "
            "bl_bitlinear_decode_group launch, int8 inputs; grouped_fused: one launch, bf16 inputs; streamed: one "
            "bl_stack_run launch over all layers, int8 inputs): %s" % cfg2)

    # ------------------------------------------- config 4: the chained 30-layer stack
    if not args.no_chain:
        from paper_2504_12285_amd import chain
        wts = [{n: (L.packed[n], L.beta[n]) for n in SHAPE_ORDER} for L in layers]
        x0 = torch.from_numpy(synth.bf16_bits_to_f32(synth.activations_bf16(0, 1, 2560, layer=100))).to(dev)
        Bd = chain.ChainBuffers(1, dev)
        xa, xb = x0.clone(), torch.empty_like(x0)

        def decode_token():
            x, Bd.x_next = xa, xb
            for w in wts:
                nxt = chain.layer_decode(w, layout, x, Bd)
                Bd.x_next, x = x, nxt
        with torch.cuda.stream(side):
            decode_token()
            torch.cuda.synchronize()
            g = capture(torch, decode_token)
            g.replay()
            n_tok = 50
            t_tok, _ = time_graph_steps(torch, [(g, 1, n_tok)], n_tok)
        t_tok /= n_tok
        # the same chain with the RMS normalisation in front of every quantiser (gains: ones
        # perturbed by a seeded 5 %; no trained gains exist here) and the true absmax/127 rescale
        rng = np.random.default_rng(7)
        gains = {n: torch.from_numpy((1.0 + 0.05 * rng.standard_normal(synth.LAYER_SHAPES[n][1])).astype(np.float32)).to(dev)
                 for n in SHAPE_ORDER}

        def decode_token_norm():
            x, Bd.x_next = xa, xb
            for w in wts:
                nxt = chain.layer_decode(w, layout, x, Bd, gains=gains)
                Bd.x_next, x = x, nxt
        with torch.cuda.stream(side):
            decode_token_norm()
            torch.cuda.synchronize()
            g = capture(torch, decode_token_norm)
            g.replay()
            t_tokn, _ = time_graph_steps(torch, [(g, 1, n_tok)], n_tok)
        t_tokn /= n_tok
        Mc = 4096
        xp = torch.from_numpy(synth.bf16_bits_to_f32(synth.activations_bf16(0, Mc, 2560, layer=101))).to(dev)
        Bp = chain.ChainBuffers(Mc, dev)
        chain.run_chain(wts[:2], layout, xp, mode="prefill")
        torch.cuda.synchronize()
        def prefill_chain_time(step):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            Bp.q_valid_for = None
            e0.record()
            x = xp
            for w in wts:
                nxt = step(w, layout, x, Bp)
                Bp.x_next, x = x, nxt
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e-3
        t_stack = min(prefill_chain_time(chain.layer_prefill) for _ in range(2))
        t_stack_unfused = min(prefill_chain_time(chain._layer_prefill_unfused) for _ in range(2))
        ops_stack = nl * sum(2.0 * Mc * n * k for n, k in synth.LAYER_SHAPES.values())
        out["config4"] = {
            "decode_chain": {"workload": "%d chained layers, M=1, 4 fused launches per layer (producer+quantiser+"
                                         "product+rescale+residual), hip graph" % nl,
                             "us_per_token": round(t_tok * 1e6, 1), "us_per_launch": round(t_tok * 1e6 / (4 * nl), 2),
                             "GBps": round(nl * layer_bytes / t_tok / 1e9, 1)},
            "decode_chain_rmsnorm": {"workload": "the same with the RMS normalisation fused in front of each quantiser",
                                     "us_per_token": round(t_tokn * 1e6, 1),
                                     "us_per_launch": round(t_tokn * 1e6 / (4 * nl), 2)},
            "prefill_chain": {"workload": "%d chained layers, M=%d, elementwise glue + bf16 rounding + row maximum in the "
                                          "products' epilogues, one-pass quantiser between products" % (nl, Mc),
                              "ms": round(t_stack * 1e3, 3), "tops_products_only_ops": round(ops_stack / t_stack / 1e12, 1),
                              "ms_producer_kernel_in_front_of_every_product": round(t_stack_unfused * 1e3, 3)}}
        log("[bench] config 4: %s" % out["config4"])
        del xp, Bp

    # ------------------------------------------------------ CPU oracle baseline
    if not args.no_cpu:
        import oracle
        prep = {}
        for name in SHAPE_ORDER:
            N, K = synth.LAYER_SHAPES[name]
            W = synth.latent_weights(0, N, K, layer=0, matrix=name)
            beta = oracle.absmean_beta(W)
            prep[name] = (oracle.ternarize(W, beta), beta,
                          synth.activations_bf16(0, 1, K, layer=0, matrix=name, relu2=(name == "down")))
        t0 = time.perf_counter()
        reps = 0
        while True:
            for name in SHAPE_ORDER:
                Wt, beta, X = prep[name]
                r = oracle.bitlinear(X, Wt, beta)
            reps += 1
            if time.perf_counter() - t0 > 10.0 or reps >= 100000:
                break
        dt = (time.perf_counter() - t0) / reps
        # spot-check the GPU result of layer 0 against the oracle while we are here
        rc = lib.bl_bitlinear_decode_group(descs[0], 4, layout, 1, torch.cuda.current_stream().cuda_stream)
        assert rc == 0, rc
        torch.cuda.synchronize()
        yd = buf["down"].y.cpu().numpy()
        assert np.allclose(yd, r["y"], rtol=1e-6, atol=0), "GPU result differs from the oracle"
        stack.run()                      # and the streamed launch: layer 0, down projection
        torch.cuda.synchronize()
        assert np.allclose(ys[3].cpu().numpy(), r["y"], rtol=1e-6, atol=0), "streamed result differs from the oracle"
        out["cpu_baseline"] = {"value": round(layer_bytes / dt / 1e9, 3), "unit": "GB/s",
                               "cores": oracle.omp_threads(), "kind": "oracle",
                               "sample": "layer 0 of the same workload (4 shapes, M=1, quantise+product+rescale), "
                                         "%d repetitions, %.2f ms each" % (reps, dt * 1e3)}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
