#!/usr/bin/env python3
"""Benchmark of the integer-only fused attention forward pass on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--kv-tile T] [--per-head]
                    [--no-cpu-baseline] [--no-others] [--no-peaks]

One step = one pass of the whole hot path (a single fused kernel launch: both int8 matmuls, the
integer online softmax, normalisation and the int8 store) over one batch of the workload.  Inputs
are seeded synthetic tensors already resident in HBM.  To keep the 256 MB last-level cache from
serving the (39 MB) inputs of the headline workload, consecutive steps rotate over enough distinct
input/output sets to exceed it; ``hot_cache`` reports the same measurement on one set.

Prints ONE JSON line.  ``value`` is algorithmic int8 TOPS: 4*N^2*d*B*H operations (two matmuls,
2 ops per multiply-add, no padding counted) per second.

``roofline`` is priced against the binding one of the two published roofs the method is judged by
(HBM 8 TB/s, dense int8 matrix rate 5.0 POP/s): HBM for every workload here.  ``roofline_mfma`` and
``roofline_alu`` stand beside it; the latter counts the vector-ALU lane-operations the kernel
actually executed (SQ_INSTS_VALU x 64 of the committed rocprofv3 run of this workload, if that run
belongs to the present kernel sources) against the chip's plain integer rate.  ``peak_measured`` is
what the chip sustains in the same run on a register-only int8 MFMA loop and on a 256 MiB copy.
``other_workloads`` times the four remaining benchmark configurations the same way (fewer steps)
and checks each against the oracle.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0            # MI355X HBM3E
PEAK_MFMA_INT8_TOPS = 5000.0     # dense int8 MFMA
CUS, LANES_PER_CU_CLK, CLOCK_GHZ = 256, 64, 2.4
PEAK_ALU_TOPS = CUS * LANES_PER_CU_CLK * CLOCK_GHZ / 1000.0    # 39.3 T integer lane-ops/s
ALU_OPS_PER_SCORE = 14.0         # algorithmic integer lane-operations per score element (the paper's steps)
LLC_BYTES = 256 << 20
KERNEL_SOURCES = ["qflash_kernels.hip", "qflash_resident.h", "qflash_cu.hip", "qflash_win.hip", "qflash_ring.hip", "qflash_qmax.hip",
                  "qflash_tile.h", "qflash_device.h", "qflash_internal.h", "qflash_dynamic.hip", "qflash_api.cpp",
                  "qflash_plan.cpp", "qflash_derive.h"]


def kernel_source_digest():
    """Identifies the kernel sources a stored counter reading belongs to."""
    h = hashlib.sha256()
    for f in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2604_25306_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def stored_counters(key):
    """HBM bytes and executed vector instructions per launch of a workload, from the committed
    rocprofv3 runs (profiles/counters.json) -- only if they were taken with the present sources."""
    path = os.path.join(ROOT, "profiles", "counters.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        c = json.load(f)
    if c.get("kernel_source_digest") != kernel_source_digest():
        return None
    return c.get("workloads", {}).get(key)


def measure(qf, torch, np, args, name, steps, warmup, cpu_baseline, batch=None):
    from workloads import make_workload
    wl = make_workload(name, batch=batch, per_head=args.per_head)
    B, H, N, d = wl.shape
    tile = args.kv_tile or wl.kv_tiles[0]
    if args.per_head:
        params = [qf.qflash_params_from_scales(wl.sQ[h], wl.sK[h], wl.sV[h], d) for h in range(H)]
        params_c = qf.params_array(params)          # built once: the timed loop only passes it on
    else:
        params = qf.qflash_params_from_scales(wl.sQ, wl.sK, wl.sV, d)
    dev = torch.device("cuda:0")

    io_bytes = 4 * B * H * N * d                       # Q, K, V read once, O written once
    bias_bytes = wl.bias.nbytes if wl.bias is not None else 0
    if args.dynamic:
        # float32 Q, K, V read twice (abs-max, quantise), int8 copies written and read, O written
        from workloads import make_float_qkv, make_float_window_bias
        floats = make_float_qkv(name, batch=batch)
        io_bytes = (2 * 12 + 3 + 3 + 1) * B * H * N * d
        # windowed workloads: the bias arrives in real units with an exclusion mask and is converted
        # on the GPU with the scales found on the fly (read 5 B, written and read 4 B per element)
        dyn_bias = make_float_window_bias(name) if wl.bias is not None else None
    n_sets = max(1, -(-int(LLC_BYTES * 1.25) // io_bytes))
    src = floats if args.dynamic else (wl.Q, wl.K, wl.V)
    base = [torch.from_numpy(x).to(dev) for x in src]
    sets = []
    for r in range(n_sets):
        q, k, v = (torch.roll(t, shifts=r, dims=0).contiguous() if r else t for t in base)
        sets.append((q, k, v, torch.empty(q.shape, dtype=torch.int8, device=dev)))
    bias = torch.from_numpy(wl.bias).to(dev) if wl.bias is not None else None
    ctx = qf.Context(0)
    if args.no_table:
        ctx.configure(qf.CFG_EXP_TABLE, 0)
    if args.quantised_max:
        ctx.configure(qf.CFG_QUANTISED_MAX, 1)
    # The bias of a windowed layer is a constant of the layer: packed once, outside the timed region.
    packed = ctx.pack_bias(bias) if bias is not None and not args.plain_bias else None
    if packed is not None:
        bias_bytes = packed.numel() * 4
    if args.dynamic:
        packed = None
        if dyn_bias is not None:
            dbias, dmask = (torch.from_numpy(x).to(dev) for x in dyn_bias)
            bias_bytes = 13 * dbias.numel()
            ws = torch.empty(qf.qflash_dynamic_bias_workspace_bytes(B, H, N, d, dbias.shape[0], dbias.shape[1]),
                             dtype=torch.uint8, device=dev)
        else:
            dbias = dmask = None
            ws = torch.empty(qf.qflash_dynamic_workspace_bytes(B, H, N, d), dtype=torch.uint8, device=dev)

    def step(i):
        q, k, v, o = sets[i % len(sets)]
        if args.dynamic:
            ctx.attention_dynamic(q, k, v, o, tile, ws, bias_real=dbias, excluded=dmask)
        elif packed is not None:
            ctx.attention_packed_bias(q, k, v, o, params_c if args.per_head else params, tile, packed,
                                      bias.shape[0], bias.shape[1])
        else:
            ctx.attention(q, k, v, o, params_c if args.per_head else params, tile, bias=bias)

    GRAPH_STEPS = 50
    graphs = {}
    # A launch shorter than the Python call that enqueues it (about 10 us) is timed from a graph.
    use_graph = args.graph or 4.0 * B * H * N * N * d < 2e9

    def graph_for(rotate):
        # one graph of GRAPH_STEPS consecutive steps, captured after a warm-up on the capture stream
        if rotate not in graphs:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                for i in range(len(sets) + 2):
                    step(i)
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                for i in range(GRAPH_STEPS):
                    step(i if rotate else 0)
            graphs[rotate] = g
        return graphs[rotate]

    def timed(n_steps, rotate=True):
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g = graph_for(rotate) if use_graph else None
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record()
        if g is not None:
            for _ in range(n_steps // GRAPH_STEPS):
                g.replay()
        else:
            for i in range(n_steps):
                step(i if rotate else 0)
        ev1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return wall, ev0.elapsed_time(ev1) * 1e-3

    if use_graph:
        steps = max(GRAPH_STEPS, steps // GRAPH_STEPS * GRAPH_STEPS)
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    wall, ev_s = timed(steps, rotate=True)
    _, ev_hot = timed(steps, rotate=False)

    sec_per_step = wall / steps
    kern_s = ev_s / steps                             # HIP events on the launch stream
    ops = 4.0 * N * N * d * B * H
    scores = float(B) * H * N * N
    tops = ops / sec_per_step / 1e12

    key = "%s/kv%d%s" % (name, tile, "/dynamic" if args.dynamic else "/per_head" if args.per_head else
                         "/plain_bias" if bias is not None and packed is None else "")
    cnt = stored_counters(key) if batch is None and not args.no_table and not args.quantised_max else None
    traffic = cnt.get("hbm_bytes") if cnt else None

    def roof(bound, achieved, peak, unit, **extra):
        r = {"bound": bound, "achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak,
             "traffic": traffic}
        r.update(extra)
        return r

    res = {
        "workload": name, "value": tops, "ms_per_step": sec_per_step * 1e3, "us_per_layer": sec_per_step * 1e6,
        "steps": steps,
        "config": {"workload": name, "B": B, "H": H, "N": N, "d": d, "kv_tile": tile,
                   "bias": None if wl.bias is None else "real units + mask, converted on the GPU" if args.dynamic
                   else "packed" if packed is not None else "plain",
                   "scales": "dynamic" if args.dynamic else "per_head" if args.per_head else "per_tensor",
                   "weights": "arithmetic" if args.no_table else "table where it fits",
                   "algorithm": "quantised-maximum variant (not the paper's)" if args.quantised_max else "Algorithm 1",
                   "input_sets_rotated": len(sets), "launch": "hip_graph" if use_graph else "eager"},
        "kernel_us_events": kern_s * 1e6,
        "hot_cache": {"kernel_us_events": ev_hot / steps * 1e6, "tops": ops / (ev_hot / steps) / 1e12},
        # The binding one of the two published roofs: HBM (Q, K, V read once, O written once).
        "roofline": roof("hbm", (io_bytes + bias_bytes) / kern_s / 1e9, PEAK_HBM_GBS, "GB/s"),
        "roofline_mfma": roof("mfma", ops / kern_s / 1e12, PEAK_MFMA_INT8_TOPS, "TOP/s"),
    }
    # The third resource, plain integer vector ALUs: executed lane-operations where the committed
    # counter run belongs to these sources, else the count of the method's definition.
    if cnt and cnt.get("valu_insts"):
        lane_ops = 64.0 * cnt["valu_insts"]
        res["roofline_alu"] = roof("alu", lane_ops / kern_s / 1e12, PEAK_ALU_TOPS, "TOP/s",
                                   lane_ops_per_score=lane_ops / scores, source="SQ_INSTS_VALU x 64, profiles/counters.json")
    else:
        res["roofline_alu"] = roof("alu", ALU_OPS_PER_SCORE * scores / kern_s / 1e12, PEAK_ALU_TOPS, "TOP/s",
                                   lane_ops_per_score=ALU_OPS_PER_SCORE, source="nominal count of the method's steps")

    ref = None
    if cpu_baseline:
        import oracle
        if args.dynamic:
            t0 = time.perf_counter()
            ref, _ = oracle.qflash_attention_dynamic(*floats, tile, bias_real=dyn_bias[0] if dyn_bias else None,
                                                     excluded=dyn_bias[1] if dyn_bias else None)
            t_cpu, reps = time.perf_counter() - t0, 1
            po = None
        elif args.per_head:
            po = [oracle.derive_params(wl.sQ[h], wl.sK[h], d) for h in range(H)]
            assert all(a.astuple() == b.astuple() for a, b in zip(po, params))
        else:
            po = oracle.derive_params(wl.sQ, wl.sK, d)
            assert po.astuple() == params.astuple()
        if not args.dynamic:
            reps, t_cpu = 0, 0.0
        budget = 3.0 if cpu_baseline == "full" else 0.0          # "check": a single pass, for the comparison only
        while not args.dynamic and (reps == 0 or (t_cpu < budget and reps < 20)):
            t0 = time.perf_counter()
            ref = (oracle.qflash_attention_qmax if args.quantised_max else oracle.qflash_attention)(
                wl.Q, wl.K, wl.V, po, tile, bias=wl.bias)
            t_cpu += time.perf_counter() - t0
            reps += 1
        same = bool(np.array_equal(ref, sets[0][3].cpu().numpy()))
        res["gpu_output_matches"] = same
        res["cpu_baseline"] = {"value": ops * reps / t_cpu / 1e12, "unit": "TOPS",
                               "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": "%d full passes of %s (all %d heads), %.2f s per pass"
                                         % (reps, name, B * H, t_cpu / reps),
                               "gpu_output_matches": same}
    else:
        # without the oracle the only check is that the launch wrote something
        res["gpu_output_matches"] = None
        assert int(sets[0][3].to(torch.int32).abs().sum().item()) > 0
    ctx.close()
    return res


def measure_peaks(qf, torch):
    """What the chip sustains: register-only int8 MFMA loop, 256 MiB device copy (same run, same clocks)."""
    dev = torch.device("cuda:0")
    wgs, iters = 512, 4096                         # two workgroups of four wavefronts per compute unit
    out = torch.zeros(2 * wgs + 2, dtype=torch.int64, device=dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    qf.qflash_peaks_mfma_i8(wgs, 64, out)          # warm-up
    torch.cuda.synchronize()
    e0.record()
    ops = qf.qflash_peaks_mfma_i8(wgs, iters, out)
    e1.record()
    torch.cuda.synchronize()
    t = e0.elapsed_time(e1) * 1e-3
    o = out.cpu().numpy()[:2 * wgs].reshape(wgs, 2).astype("float64")
    clock_ghz = float((o[:, 0] / (o[:, 1] * 10.0)).mean())         # cycles per 10 ns tick
    src = torch.empty(256 << 20, dtype=torch.int8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    qf.qflash_peaks_copy(src, dst)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(4):
        qf.qflash_peaks_copy(src, dst)
    e1.record()
    torch.cuda.synchronize()
    tc = e0.elapsed_time(e1) * 1e-3 / 4
    # vector integer issue: one workgroup of 16 wavefronts per compute unit (4 per SIMD, as the attention kernels run)
    vout = torch.zeros(2 * CUS + 2, dtype=torch.int64, device=dev)
    qf.qflash_peaks_valu(CUS, 256, vout)           # warm-up
    torch.cuda.synchronize()
    e0.record()
    lane_ops = qf.qflash_peaks_valu(CUS, 16384, vout)
    e1.record()
    torch.cuda.synchronize()
    tv = e0.elapsed_time(e1) * 1e-3
    vo = vout.cpu().numpy()[:2 * CUS].reshape(CUS, 2).astype("float64")
    vclock = float((vo[:, 0] / (vo[:, 1] * 10.0)).mean())
    return {"valu_lane_tops": lane_ops / tv / 1e12, "valu_clock_ghz": vclock,
            "valu_cycles_per_instruction_simd": (vclock * 1e9) * tv / (lane_ops / 64.0 / (CUS * 4)),
            "mfma_int8_tops": ops / t / 1e12, "mfma_int8_ops_per_clk_cu": ops / t / (clock_ghz * 1e9) / CUS,
            "mfma_clock_ghz": clock_ghz, "hbm_copy_gbs": 2.0 * (256 << 20) / tc / 1e9,
            "how": "512 workgroups x 4 wavefronts x 4096 x 4 independent v_mfma_i32_32x32x32_i8; 256 MiB copy, read + write; "
                   "256 workgroups x 16 wavefronts x 16384 x 16 independent 32-bit integer vector instructions"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default=None)
    ap.add_argument("--kv-tile", type=int, default=None)
    ap.add_argument("--batch", type=int, default=None,
                    help="run the named workload at another batch size (its B; for the windowed "
                         "workloads: number of windows); the stored counter figures are then omitted")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="only the named (or headline) workload")
    ap.add_argument("--no-peaks", action="store_true", help="skip the MFMA and copy micro-benchmarks")
    ap.add_argument("--graph", action="store_true",
                    help="replay the launches from a captured HIP graph of 50 steps (for workloads so "
                         "small that the Python call per launch, about 10 us, is what the eager loop measures)")
    ap.add_argument("--dynamic", action="store_true",
                    help="start from float32 Q, K, V: abs-max, scales, constants and quantisation on "
                         "the GPU in front of the attention kernel (qflash_attention_dynamic); one "
                         "step is the whole pipeline")
    ap.add_argument("--per-head", action="store_true",
                    help="per-head variant of the workload: heads of different range, one set of "
                         "integer constants per head (qflash_attention_per_head)")
    ap.add_argument("--plain-bias", action="store_true",
                    help="workloads with a bias: hand it over in the plain [N,N] layout on every call "
                         "instead of packing it once before the timed region (qflash_pack_bias)")
    ap.add_argument("--no-table", action="store_true",
                    help="evaluate the weight of every score arithmetically (Algorithm 2 in the vector ALUs) "
                         "instead of reading it from the table in LDS; same bits")
    ap.add_argument("--quantised-max", action="store_true",
                    help="time the quantised-maximum variant (QFLASH_CFG_QUANTISED_MAX: NOT the paper's "
                         "Algorithm 1, different results; checked against its own oracle)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 256 MiB device-to-device copy, so that a rocprofv3 --pmc "
                         "trace of this command holds a kernel of known HBM traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path shards over batch*heads with no "
              "collectives; nothing here uses a second GPU). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2604_25306_amd as qf
    from workloads import HEADLINE, BASELINE_CONFIGS, CONFIGS

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    qf.load_library()           # fails loudly when the HIP library is missing
    name = args.workload or HEADLINE

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.int8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    head = measure(qf, torch, np, args, name, args.steps, args.warmup,
                   None if args.no_cpu_baseline else "full", batch=args.batch)
    out = {
        "metric": "int8 attention TOPS + us/layer, ViT-B/16 B=64 (H=12,N=197,d=64)",
        "value": head["value"], "unit": "TOPS", "n_gpus": 1, "steps": head["steps"], "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "us_per_layer": head["us_per_layer"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8/int32",
        "data": "synthetic", "config": head["config"], "kernel_us_events": head["kernel_us_events"],
        "hot_cache": head["hot_cache"],
        "roofline": head["roofline"], "roofline_mfma": head["roofline_mfma"], "roofline_alu": head["roofline_alu"],
        "gpu_output_matches": head["gpu_output_matches"],
    }
    if "cpu_baseline" in head:
        out["cpu_baseline"] = head["cpu_baseline"]

    if not args.no_peaks:
        pk = measure_peaks(qf, torch)
        out["peak_measured"] = pk
        out["roofline"]["frac_of_measured_copy"] = out["roofline"]["achieved"] / pk["hbm_copy_gbs"]
        out["roofline_mfma"]["frac_of_measured_mfma"] = out["roofline_mfma"]["achieved"] / pk["mfma_int8_tops"]
        out["roofline_alu"]["peak_at_measured_clock"] = CUS * LANES_PER_CU_CLK * pk["mfma_clock_ghz"] / 1000.0
        out["roofline_alu"]["frac_of_measured_valu"] = out["roofline_alu"]["achieved"] / pk["valu_lane_tops"]

    # The other benchmark configurations, timed the same way with fewer steps, each checked against
    # the oracle (one pass) unless the baseline is switched off.
    if not args.no_others and args.workload is None and args.batch is None and not (args.dynamic or args.per_head or args.quantised_max):
        others = {}
        for wname in BASELINE_CONFIGS:
            for tile in CONFIGS[wname][4]:
                if wname == name and tile == head["config"]["kv_tile"]:
                    continue
                a2 = argparse.Namespace(**vars(args))
                a2.kv_tile = tile
                r = measure(qf, torch, np, a2, wname, max(100, args.steps // 5), max(20, args.warmup // 5),
                            None if args.no_cpu_baseline else "check")
                label = wname if len(CONFIGS[wname][4]) == 1 else "%s/kv%d" % (wname, tile)
                others[label] = {k: r[k] for k in ("kernel_us_events", "value", "us_per_layer", "roofline",
                                                   "roofline_mfma", "roofline_alu", "gpu_output_matches", "config")}
        out["other_workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
