#!/usr/bin/env python3
"""Benchmark: decode MoE-layer latency of the bit-sliced expert FFN on one MI355X.

A step is one pass of the whole hot path (cache-aware route -> precision select -> gate/up +
SwiGLU -> down + combine) for ONE token through the DeepSeek-V2-Lite-shaped layer: 64 routed
experts of 2048x1408 (top-6, 8-bit AMAT, group 128, MSB/LSB nibble planes) + 2 shared experts
always high-bit; router logits ~ N(0,1) with +1.0 on 32 'cached' experts of which 16 hold both
slices.  All inputs are synthetic, seeded, and resident in HBM before the timed region.

Prints ONE JSON line.  `value` is microseconds per token-layer; `roofline` prices the same
launches against the 8 TB/s HBM peak using ALGORITHMIC bytes (only the planes the mask selects);
`cpu_baseline` is the unmodified CPU oracle timed on a few steps of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


PLANE_BITS = 4      # bits per code in a plane: 4 for the 8/4 nest, 3 for 6/3 (--nest 63), 2 for 4/2 (--nest 42)


def slot_bytes(d, f, group, prec, scale_bytes=2):
    """Algorithmic bytes one expert moves at a precision: planes read + metadata."""
    planes = 2 if prec else 1
    gu = planes * (2 * f * d * PLANE_BITS // 8) + 2 * f * (-(-d // group)) * (scale_bytes + 1)
    dn = planes * (d * f * PLANE_BITS // 8) + d * (-(-f // group)) * (scale_bytes + 1)
    return gu, dn


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1024)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-steps", type=int, default=40)
    ap.add_argument("--workload", choices=["decode", "prefill", "stack-qwen", "stack-dsv2"], default="decode",
                    help="decode (default, the headline metric) or the prefill grouped GEMM of one Qwen-shaped layer")
    ap.add_argument("--group", type=int, default=0, choices=[0, 32, 64, 128],
                    help="decode: quantisation group of the expert weights (default: the workload's 128; 32 is the "
                         "paper's expert format, with four times the scales and zero-points)")
    ap.add_argument("--shape", choices=["dsv2", "qwen", "wide", "tiny"], default="dsv2",
                    help="decode: dsv2 = the headline DeepSeek-V2-Lite-shaped layer; qwen = one Qwen1.5-MoE-shaped layer "
                         "(60 experts top-4, one shared expert of d_ff 5632 behind a sigmoid gate, 18 experts HIGH, all "
                         "MSB slices resident), reported as its own line; wide = d_model 4096 (16 experts of d_ff 2048, top-4, one "
                         "shared expert: rows of two 64-chunk k-slices, the wide gate/up kernel); tiny = the fp32 correctness "
                         "layer (BASELINE configs[0]: d_model 256, 8 experts of d_ff 128, top-2, group 64), launch-bound")
    ap.add_argument("--router-matvec", action="store_true",
                    help="decode (one token per step): logits from the router mat-vec W_r x (a third launch) instead of "
                         "supplied logits")
    ap.add_argument("--nest", choices=["84", "63", "42"], default="84",
                    help="decode: bit nest of the expert weights: 84 = 8-bit codes / 4-bit low-bit model (headline), "
                         "63 = 6-bit codes / 3-bit, 42 = 4-bit codes / 2-bit low-bit model (3/4 and 1/2 of the plane bytes)")
    ap.add_argument("--tokens", type=int, default=1,
                    help="decode: tokens per step that pass the layer together in one pair of launches (1 = the headline "
                         "single-batch workload; 2-16 = smoe_decode_layer_multi, reported per token)")
    ap.add_argument("--prefill-tokens", type=int, default=0,
                    help="prefill: tokens of the prompt (default: the workload's 2048)")
    ap.add_argument("--with-shared", action="store_true",
                    help="prefill: add the Qwen-shaped shared expert (d_ff 5632 behind a sigmoid gate) that every "
                         "token passes through; reported as its own line, not the headline")
    ap.add_argument("--launch", choices=["graph", "eager"], default="graph",
                    help="decode: how the timed steps are launched: replayed from a captured HIP graph (default; the eager "
                         "figure is reported beside it) or as eager calls only")
    ap.add_argument("--single-launch", action="store_true",
                    help="decode: also time the same steps with one kernel launch per call (smoe_ctx_single_launch)")
    ap.add_argument("--replicas", type=int, default=4,
                    help="decode: layer replicas of the cold-weights figure (0 or 1: skip it)")
    ap.add_argument("--no-stream-floor", action="store_true",
                    help="decode: skip the plain-streaming reference measurement")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="after the timed passes, copy this many MiB device-to-device four times (a kernel of known "
                         "traffic, used to scale the HBM byte counters of a profiler run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (the decode layer of one token has no second-GPU path); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2512_12990_amd import binding as B, synth

    if not os.path.exists(B.LIB_PATH):
        from paper_2512_12990_amd import build as _b
        _b.build()
    assert torch.cuda.is_available(), "bench.py needs the GPU (there is no CPU fallback)"
    if args.workload == "prefill":
        return prefill_bench(args)
    if args.workload in ("stack-qwen", "stack-dsv2"):
        return stack_bench(args)
    global PLANE_BITS
    bh, bl = {"84": (8, 4), "63": (6, 3), "42": (4, 2)}[args.nest]
    PLANE_BITS = bl
    wl = synth.DSV2_LAYER
    if args.shape == "qwen":
        import dataclasses
        wl = dataclasses.replace(synth.QWEN_STACK, n_layers=1, steps=1024)
    if args.shape == "tiny":
        wl = synth.TINY
    if args.shape == "wide":
        wl = synth.Workload("wide-layer", synth.LayerShape(4096, 16, 2048, 4, 128, n_shared=1, shared_d_ff=2048), steps=256)
    if args.group:
        import dataclasses
        wl = dataclasses.replace(wl, layer=dataclasses.replace(wl.layer, group=args.group))
    shp = wl.layer
    dev = "cuda:0"
    # everything runs on one side stream: the context launches on it, the events are recorded on it,
    # and a HIP graph can be captured from it
    side = torch.cuda.Stream()
    torch.cuda.set_stream(side)
    ctx = B.Ctx(0, stream=side)
    adt = shp.act                                   # activation and scale dtype of the workload
    ADT, asz = B._DT[adt], (4 if adt == "f32" else 2)

    def build_layer(replica):
        """One layer's banks; replica r > 0 draws different weights of the same shape."""
        routed = B.Bank(ctx, shp.n_experts, shp.d_model, shp.d_ff, shp.group, adt, adt, bh, bl)
        shared = B.Bank(ctx, shp.n_shared, shp.d_model, shp.shared_d_ff, shp.group, adt, adt, bh, bl) if shp.n_shared else None
        for e in range(shp.n_experts):
            wg, wu, wd = synth.expert_weights(wl.seed, replica, e, shp.d_model, shp.d_ff, adt, dev)
            B.smoe_quantize_slice(ctx, routed, e, wg[None], wu[None], wd[None])
        for i in range(shp.n_shared):
            wg, wu, wd = synth.expert_weights(wl.seed, replica, 1000 + i, shp.d_model, shp.shared_d_ff, adt, dev)
            B.smoe_quantize_slice(ctx, shared, i, wg[None], wu[None], wd[None])
        return routed, shared

    routed, shared = build_layer(0)
    n_in = wl.steps
    x_all = synth.activations(wl.seed, n_in, shp.d_model, adt).to(dev)
    z_all = synth.normal_logits(wl.seed, n_in, shp.n_experts).to(dev)
    if args.shape == "qwen":
        mask_np = synth.fraction_masks(wl.seed, 1, 0, shp.n_experts, 0.3)[0]
        bias_np = np.zeros(shp.n_experts, np.float32)
    elif args.shape == "wide":
        mask_np, bias_np = synth.cached_set_mask(wl.seed, shp.n_experts, 8, 4, 1.0)
    elif args.shape == "tiny":
        mask_np = synth.bernoulli_masks(wl.seed, 1, shp.n_experts)[0]
        bias_np = np.zeros(shp.n_experts, np.float32)
    else:
        mask_np, bias_np = synth.cached_set_mask(wl.seed, shp.n_experts, 32, 16, 1.0)
    mask = torch.from_numpy(mask_np).to(dev)
    bias = torch.from_numpy(bias_np).to(dev)
    wsg = synth.shared_gate_weight(wl.seed, 0, shp.d_model, adt).to(dev) if shp.shared_gate else None
    y = torch.empty((n_in, shp.d_model), dtype=x_all.dtype, device=dev)
    prec = torch.zeros((n_in, shp.top_k), dtype=torch.uint8, device=dev)
    idx = torch.zeros((n_in, shp.top_k), dtype=torch.int32, device=dev)
    torch.cuda.synchronize()

    # argument lists are marshalled once; the timed loop only makes the C calls
    import ctypes as C
    vp = lambda t: C.c_void_p(t.data_ptr())
    TT = args.tokens
    wr = synth.router_weight(wl.seed, 0, shp.n_experts, shp.d_model).to(dev) if args.router_matvec else None

    def make_calls(routed, shared):
        sh = shared.h if shared is not None else None
        if TT == 1:
            return B.lib().smoe_decode_layer, [
                (ctx.h, routed.h, sh, vp(x_all[i]), C.c_int(ADT), C.c_int(shp.top_k),
                 None if wr is not None else vp(z_all[i]), vp(wr) if wr is not None else None,
                 vp(bias), C.c_int(0), C.c_float(1.0), vp(mask), C.c_float(0.0), vp(wsg) if wsg is not None else None,
                 C.c_int(0), vp(y[i]), vp(idx[i]), None, vp(prec[i])) for i in range(n_in)]
        # step t takes the TT consecutive tokens that start at row (t * TT) mod n_in
        assert 2 <= TT <= 16 and n_in % TT == 0
        return B.lib().smoe_decode_layer_multi, [
            (ctx.h, routed.h, sh, C.c_int(TT), vp(x_all[i]), C.c_int(ADT), C.c_int(shp.top_k), vp(z_all[i]),
             vp(bias), C.c_int(0), C.c_float(1.0), vp(mask), C.c_float(0.0), vp(wsg) if wsg is not None else None,
             C.c_int(0), vp(y[i]), vp(idx[i]), None, vp(prec[i])) for i in range(0, n_in, TT)]

    fn, calls = make_calls(routed, shared)
    n_calls = len(calls)

    def make_step(fn, call_lists):
        """Step t makes call t of layer replica t mod R (R = 1: the one layer every step)."""
        R = len(call_lists)

        def step(t):
            rc = fn(*call_lists[t % R][t % n_calls])
            if rc != 0:
                raise B.SmoeError("decode call failed: %d" % rc)
        return step

    def timed(run):
        """GPU time of run() between two events on the launch stream, and the host's wall time, in ms."""
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(side)
        run()
        e1.record(side)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1), (time.perf_counter() - t0) * 1e3

    def measure(step):
        """ms per step of exactly args.steps steps after args.warmup warm-up steps: eager launches, and the
        same steps replayed from a captured HIP graph (a serving loop records its decode calls once)."""
        for t in range(args.warmup):
            step(t)
        eager_ms, eager_wall = timed(lambda: [step(t) for t in range(args.warmup, args.warmup + args.steps)])
        res = {"eager_ms_per_step": eager_ms / args.steps, "eager_host_wall_ms_per_step": eager_wall / args.steps}
        if args.launch == "graph":
            G = min(args.steps, 256)
            while args.steps % G:
                G -= 1
            graphs = []
            for g0 in range(args.warmup, args.warmup + args.steps, G):      # the same steps, in the same order
                gr = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gr, stream=side):
                    for t in range(g0, g0 + G):
                        step(t)
                graphs.append(gr)
            for gr in graphs[:1]:
                gr.replay()                                                   # untimed first replay (upload)
            graph_ms, graph_wall = timed(lambda: [gr.replay() for gr in graphs])
            res.update({"graph_ms_per_step": graph_ms / args.steps, "graph_host_wall_ms_per_step": graph_wall / args.steps,
                        "graph_steps_per_graph": G})
            res["windows"] = sorted(timed(lambda: [gr.replay() for gr in graphs])[0] / args.steps for _ in range(5))
            res["graphs"] = graphs
        else:
            res["windows"] = sorted(timed(lambda: [step(t) for t in range(args.warmup, args.warmup + args.steps)])[0] / args.steps
                                    for _ in range(5))
        res["ms_per_step"] = res["graph_ms_per_step"] if args.launch == "graph" else res["eager_ms_per_step"]
        return res

    step = make_step(fn, [calls])
    m = measure(step)
    ms_per_step = m["ms_per_step"]
    windows = [w * 1e3 / TT for w in m["windows"]]

    # The same steps with one kernel launch per call instead of two (smoe_ctx_single_launch; an option, slower here)
    one = None
    if TT == 1 and args.single_launch:
        m["graphs"] = None
        ctx.single_launch(True)
        m1 = measure(step)
        calls1, timeouts1 = ctx.single_launch_status()
        ctx.single_launch(False)
        one = {"us_per_token": m1["ms_per_step"] * 1e3, "eager_us_per_token": m1["eager_ms_per_step"] * 1e3,
               "calls_that_took_it": calls1, "work_groups_timed_out": timeouts1,
               "note": "same steps, same launch mode as value, one kernel launch per call (gate/up phase, in-kernel hand-over of h, "
                       "down phase); bit-identical results"}
        del m1

    # A plain device-to-device copy of 256 MiB, for scale: what this machine's HBM delivers to a streaming
    # kernel (bytes read + bytes written per second).
    csrc = torch.full((256 << 20,), 7, dtype=torch.uint8, device=dev)
    cdst = torch.empty_like(csrc)
    cdst.copy_(csrc)
    copy_ms, _ = timed(lambda: [cdst.copy_(csrc) for _ in range(4)])
    copy_gbps = 4 * 2 * csrc.numel() / (copy_ms * 1e-3) / 1e9
    del csrc, cdst

    # Dominant kernel (gate/up streams 2/3 of the bytes): a second pass over the SAME steps with
    # a start and a stop event attached by the library to each of the two dispatches of a call.
    ctx.timing(True)
    for t in range(args.warmup, args.warmup + args.steps):
        step(t)
    gu_us, dn_us, n_timed = ctx.timing_read()
    ctx.timing(False)
    gu_us /= n_timed
    dn_us /= n_timed

    # algorithmic bytes of exactly the timed steps, from the precision flags the kernels reported
    prec_np = prec.cpu().numpy()
    idx_np = idx.cpu().numpy()
    hi_gu, hi_dn = slot_bytes(shp.d_model, shp.d_ff, shp.group, 1, asz)
    lo_gu, lo_dn = slot_bytes(shp.d_model, shp.d_ff, shp.group, 0, asz)
    sh_gu, sh_dn = slot_bytes(shp.d_model, shp.shared_d_ff, shp.group, 1, asz) if shp.n_shared else (0, 0)
    sh_gu, sh_dn = sh_gu * shp.n_shared, sh_dn * shp.n_shared
    total_bytes = gu_bytes = 0
    high_slots = timed_rows = 0
    for t in range(args.warmup, args.warmup + args.steps):
        r0 = (t % n_calls) * TT
        high_slots += int(prec_np[r0:r0 + TT].sum())
        timed_rows += TT
        if TT == 1:
            nh = int(prec_np[r0].sum())
            nl = shp.top_k - nh
        else:
            # what the step must move: every expert some token of the step selected once, with its LSB
            # plane if some token runs it HIGH
            need = {}
            for tt in range(r0, r0 + TT):
                for e, p in zip(idx_np[tt], prec_np[tt]):
                    need[int(e)] = max(need.get(int(e), 0), int(p))
            nh = sum(need.values())
            nl = len(need) - nh
        gu = sh_gu + nh * hi_gu + nl * lo_gu + TT * (shp.d_model * asz + shp.n_experts * 9)
        dn = sh_dn + nh * hi_dn + nl * lo_dn + TT * shp.d_model * asz
        gu_bytes += gu
        total_bytes += gu + dn
    bytes_per_step = total_bytes / args.steps
    gu_bytes_per_launch = gu_bytes / args.steps
    achieved = bytes_per_step / (ms_per_step * 1e-3) / 1e9
    gu_achieved = gu_bytes_per_launch / (gu_us * 1e-6) / 1e9

    # HBM bytes per gate/up launch as the FETCH_SIZE / WRITE_SIZE counters read them: only for the one
    # configuration the committed counter runs cover (profiles/...hbm_traffic.txt); any other run prints null
    traffic = traffic_src = None
    key = (args.shape, args.nest, shp.group, TT, bool(args.router_matvec))
    if key in MEASURED_TRAFFIC:
        traffic, traffic_src = MEASURED_TRAFFIC[key]

    # hot set of the one-layer workload: the experts the mask marks resident (what the steps keep selecting)
    hot_experts = int((mask_np & 1).sum()) or shp.n_experts
    hot_bytes = sh_gu + sh_dn + int((mask_np == 3).sum()) * (hi_gu + hi_dn) + (hot_experts - int((mask_np == 3).sum())) * (lo_gu + lo_dn)

    out = {
        "metric": "decode MoE-layer us/token (+ achieved HBM GB/s as a fraction of MI355X peak)",
        "value": ms_per_step * 1e3 / TT, "unit": "us/token", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": ("u%d+u%d bit-sliced weights, bf16 activations rewritten per 32-chunk as 3 balanced hex digits, signed 4-bit dot products, int32/fp32 accumulate" % (bl, bl)
                  if adt == "bf16" else "u%d+u%d bit-sliced weights, fp32 activations and scales, fp32 multiply-add" % (bl, bl)),
        "data": "synthetic",
        "config": {"workload": ("DeepSeek-V2-Lite-shaped MoE layer decode, %d token%s/step (BASELINE configs[1])" if args.shape == "dsv2" else
                                "d_model-4096 MoE layer decode, %d token%s/step (no BASELINE config: the wide-row kernel)" if args.shape == "wide" else
                                "tiny fp32 MoE layer decode, %d token%s/step (BASELINE configs[0]; launch-bound)" if args.shape == "tiny" else
                                "Qwen1.5-MoE-shaped MoE layer decode, %d token%s/step (one layer of BASELINE configs[2])") % (TT, "" if TT == 1 else "s"),
                   "d_model": shp.d_model, "n_experts": shp.n_experts, "d_ff": shp.d_ff, "top_k": shp.top_k,
                   "n_shared": shp.n_shared, "shared_d_ff": shp.shared_d_ff, "group": shp.group, "nest": "%d/%d" % (bh, bl),
                   "cached": int((mask_np & 1).sum()), "cached_high": int((mask_np == 3).sum()),
                   "mean_high_slots": high_slots / timed_rows, "launches_per_step": 3 if wr is not None else 2,
                   "tokens_per_step": TT,
                   "launch_mode": ("HIP graph replay (%d steps per graph, the same %d steps in order)" % (m["graph_steps_per_graph"], args.steps)
                                   if args.launch == "graph" else "eager launches"),
                   "weights_resident": "one layer of %.0f MB in HBM, re-read every step; the hot set the steps select from (%d resident "
                                       "experts + %d shared) is about %.0f MB, which fits the 256 MB memory-side cache -- see "
                                       "cold_weights for the same steps over rotating layer replicas" %
                                       ((routed.nbytes + (shared.nbytes if shared else 0)) / 1e6, hot_experts, shp.n_shared, hot_bytes / 1e6)},
        "hbm_gbps": achieved, "hbm_frac": achieved / HBM_PEAK_GBPS, "bytes_per_token": bytes_per_step / TT,
        "eager_us_per_token": m["eager_ms_per_step"] * 1e3 / TT,
        "host_wall_ms_per_step": m["graph_host_wall_ms_per_step"] if args.launch == "graph" else m["eager_host_wall_ms_per_step"],
        "eager_host_wall_ms_per_step": m["eager_host_wall_ms_per_step"],
        "repeat_windows_us_per_token": {"median": windows[2], "min": windows[0], "max": windows[-1], "n": 5},
        "copy_256mib_gbps": copy_gbps,
        "roofline": {"bound": "hbm", "kernel": "gateup_kernel<%s> (route + gate/up + SwiGLU of all %d slots)" % (adt, shp.top_k + shp.n_shared),
                     "achieved": gu_achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": gu_achieved / HBM_PEAK_GBPS,
                     "bytes_per_launch": gu_bytes_per_launch, "avg_launch_us": gu_us,
                     "other_kernel": {"kernel": "down_kernel<%s>" % adt, "avg_launch_us": dn_us,
                                      "bytes_per_launch": bytes_per_step - gu_bytes_per_launch,
                                      "achieved": (bytes_per_step - gu_bytes_per_launch) / (dn_us * 1e-6) / 1e9},
                     "timing": "start/stop HIP events attached to every dispatch on the launch stream, eager pass over the same steps",
                     "traffic": traffic, "traffic_source": traffic_src,
                     "traffic_over_algorithmic": (traffic / gu_bytes_per_launch) if traffic else None},
    }

    if one is not None:
        out["single_launch"] = one

    # A practical roof measured in the same run: the same two launch shapes doing nothing but streaming the
    # step's algorithmic bytes (gate/up bytes on the gate/up grid, down bytes on the down grid) out of the
    # bank's store, windows rotating through it so that nothing is re-read from a cache; and one launch
    # over the sum.
    if TT == 1 and args.shape == "dsv2" and not args.no_stream_floor:
        m["graphs"] = None
        sread = B.lib().smoe_stream_read
        sink = torch.zeros(64, dtype=torch.uint8, device=dev)
        base = routed._base
        gub, dnb = int(gu_bytes_per_launch) & ~255, int(bytes_per_step - gu_bytes_per_launch) & ~255
        span = (routed.nbytes - gub - dnb - 4096) & ~255

        def floor_step(two):
            def step(t):
                off = (t * (gub + dnb)) % span
                if two:
                    rc = sread(ctx.h, C.c_void_p(base + off), C.c_size_t(gub), C.c_int(512), vp(sink))
                    rc = rc or sread(ctx.h, C.c_void_p(base + off + gub), C.c_size_t(dnb), C.c_int(256), vp(sink))
                else:
                    rc = sread(ctx.h, C.c_void_p(base + off), C.c_size_t(gub + dnb), C.c_int(768), vp(sink))
                if rc != 0:
                    raise B.SmoeError("stream read failed: %d" % rc)
            return step
        f2 = measure(floor_step(True))
        f1 = measure(floor_step(False))
        out["stream_floor"] = {"two_launches_us_per_step": f2["ms_per_step"] * 1e3, "one_launch_us_per_step": f1["ms_per_step"] * 1e3,
                               "bytes": [gub, dnb], "work_groups": [512, 256],
                               "value_over_two_launch_floor": ms_per_step / f2["ms_per_step"],
                               "note": "plain 16-byte-per-lane streaming reads of the step's algorithmic bytes from the bank store "
                                       "(no routing, no arithmetic, no dependency between the two launches' data), same launch "
                                       "mode as value"}
        del f1, f2

    # The same steps with the weights cold: R replicas of the layer (different weights, same shape), step t
    # on replica t mod R, so that the bytes a step reads were last touched R steps -- R times the hot set -- ago
    # and cannot come from the memory-side cache.
    if args.replicas > 1:
        m["graphs"] = None                                      # release the first measurement's graphs
        layers = [(routed, shared)] + [build_layer(r) for r in range(1, args.replicas)]
        lists = [make_calls(rt, sh)[1] for rt, sh in layers]
        mc = measure(make_step(fn, lists))
        cold_gbps = bytes_per_step / (mc["ms_per_step"] * 1e-3) / 1e9
        out["cold_weights"] = {"replicas": args.replicas, "working_set_mb": args.replicas * hot_bytes / 1e6,
                               "us_per_token": mc["ms_per_step"] * 1e3 / TT, "eager_us_per_token": mc["eager_ms_per_step"] * 1e3 / TT,
                               "hbm_gbps": cold_gbps, "hbm_frac": cold_gbps / HBM_PEAK_GBPS,
                               "note": "same inputs and routing, hence the same algorithmic bytes per step; step t reads "
                                       "replica t mod %d" % args.replicas}
        del layers, lists, mc

    if args.calib_copy_mib:
        src = torch.full((args.calib_copy_mib << 20,), 7, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
    if not args.no_cpu_baseline and args.shape == "dsv2" and args.nest == "84":      # the oracle leg times the headline workload only
        out["cpu_baseline"] = cpu_baseline(wl, args.cpu_steps, idx_np, prec_np)
    print(json.dumps(out))


# HBM bytes per gate/up launch from rocprofv3 counter runs of exactly this command line, keyed by
# (shape, nest, group, tokens per step, router mat-vec): value, where it was recorded
MEASURED_TRAFFIC = {
    ("dsv2", "84", 128, 1, False): (39.54e6 + 0.36e6, "profiles/decode_dsv2lite_gateup_down_hbm_traffic.txt "
                                    "(FETCH_SIZE and WRITE_SIZE runs of this command, scaled by a 256 MiB copy)"),
}


def prefill_bench(args):
    """One Qwen1.5-MoE-shaped layer, 2048 tokens, 60 experts top-4, all high-bit: route + histogram +
    grouped expert GEMMs on MFMA + combine.  A step is one such layer pass."""
    import torch
    from paper_2512_12990_amd import binding as B, synth
    wl = synth.QWEN_PREFILL
    shp = wl.layer
    T, dev = args.prefill_tokens or wl.prefill_tokens, "cuda:0"
    ctx = B.Ctx(0)
    routed = B.Bank(ctx, shp.n_experts, shp.d_model, shp.d_ff, shp.group, "bf16", "bf16")
    for e in range(shp.n_experts):
        wg, wu, wd = synth.expert_weights(wl.seed, 0, e, shp.d_model, shp.d_ff, "bf16", dev)
        B.smoe_quantize_slice(ctx, routed, e, wg[None], wu[None], wd[None])
    x = synth.activations(wl.seed, T, shp.d_model, "bf16").to(dev)
    wr = synth.router_weight(wl.seed, 0, shp.n_experts, shp.d_model).to(dev)
    shared, wsg, f_s = None, None, 0
    if args.with_shared:
        f_s = synth.QWEN_STACK.layer.shared_d_ff
        shared = B.Bank(ctx, 1, shp.d_model, f_s, shp.group, "bf16", "bf16")
        wg, wu, wd = synth.expert_weights(wl.seed, 0, 1000, shp.d_model, f_s, "bf16", dev)
        B.smoe_quantize_slice(ctx, shared, 0, wg[None], wu[None], wd[None])
        wsg = synth.shared_gate_weight(wl.seed, 0, shp.d_model, "bf16").to(dev)
    scratch = torch.empty(B.smoe_prefill_bytes(T, shp.n_experts, shp.top_k, shp.d_model, shp.d_ff, f_s), dtype=torch.uint8,
                          device=dev)
    steps = min(args.steps, 50)
    for _ in range(3):
        B.smoe_prefill_histogram(ctx, routed, shared, x, shp.top_k, w_router=wr, shared_gate_w=wsg, add_residual=True,
                                 scratch=scratch)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(steps):
        B.smoe_prefill_histogram(ctx, routed, shared, x, shp.top_k, w_router=wr, shared_gate_w=wsg, add_residual=True,
                                 scratch=scratch)
    ev1.record()
    torch.cuda.synchronize()
    ms = ev0.elapsed_time(ev1) / steps
    flops = 2.0 * T * shp.top_k * 3 * shp.d_model * shp.d_ff + 2.0 * T * 3 * shp.d_model * f_s
    y_g, idx_g, w_g, _ = B.smoe_prefill_histogram(ctx, routed, shared, x, shp.top_k, w_router=wr, shared_gate_w=wsg,
                                                  add_residual=True, scratch=scratch)
    torch.cuda.synchronize()
    wbytes = shp.n_experts * sum(slot_bytes(shp.d_model, shp.d_ff, shp.group, 1))
    if f_s:
        wbytes += sum(slot_bytes(shp.d_model, f_s, shp.group, 1))
    out = ({
        "metric": "prefill MoE-layer ms (%d tokens, grouped expert GEMM + histogram)" % T, "value": ms, "unit": "ms/layer",
        "n_gpus": 1, "steps": steps, "warmup": 3, "ms_per_step": ms, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16 MFMA, fp32 accumulate, u4+u4 sliced weights", "data": "synthetic",
        "config": {"workload": "Qwen1.5-MoE-shaped prefill layer (BASELINE configs[4], one layer)", "tokens": T,
                   "n_experts": shp.n_experts, "top_k": shp.top_k, "d_model": shp.d_model, "d_ff": shp.d_ff,
                   "shared_d_ff": f_s},
        "tokens_per_s": T / (ms * 1e-3),
        "roofline": {"bound": "mfma", "achieved": flops / (ms * 1e-3) / 1e12, "peak": 2500.0, "unit": "TFLOP/s",
                     "frac": flops / (ms * 1e-3) / 1e12 / 2500.0, "flops_per_step": flops,
                     "weight_bytes_per_step": wbytes, "weight_gbps": wbytes / (ms * 1e-3) / 1e9, "traffic": None,
                     "kernel": "whole layer pass (route_batch, group, grouped_gemm<0>, grouped_gemm<1>, combine)"}})
    if not args.no_cpu_baseline and not args.with_shared:
        out["cpu_baseline"] = cpu_baseline_prefill(wl, T, min(args.cpu_steps, 16), idx_g.cpu().numpy(), w_g.cpu().numpy())
    print(json.dumps(out))


def stack_bench(args):
    """Whole decode steps of the multi-layer workloads (BASELINE configs[2] and configs[3]): a step sends
    one token through every layer.  The MoE layers' outputs feed the next layer directly (add_residual);
    the attention / normalisation blocks between MoE layers are outside the path and left out, so the
    numbers are the MoE layers alone.  stack-dsv2 keeps its per-step host work inside the window: masks
    and routing bias come from the slice LRU (25 % of the slices), which is fed the step's selections."""
    import ctypes as C
    import numpy as np
    import torch
    from paper_2512_12990_amd import binding as B, synth
    qwen = args.workload == "stack-qwen"
    wl = synth.QWEN_STACK if qwen else synth.DSV2_STACK
    shp = wl.layer
    dev = "cuda:0"
    d, E, k = shp.d_model, shp.n_experts, shp.top_k
    LM = wl.n_layers if qwen else wl.n_layers - 1
    ctx = B.Ctx(0)

    def bank(n, f, l, tag0):
        b = B.Bank(ctx, n, d, f, shp.group, "bf16", "bf16")
        for e in range(n):
            wg, wu, wd = synth.expert_weights(wl.seed, l, tag0 + e, d, f, "bf16", dev)
            B.smoe_quantize_slice(ctx, b, e, wg[None], wu[None], wd[None])
        return b

    routed = [bank(E, shp.d_ff, l, 0) for l in range(LM)]
    shared = [bank(shp.n_shared, shp.shared_d_ff, l, 1000) for l in range(LM)]
    dense = None if qwen else bank(1, wl.dense_first_d_ff, 2000, 1000)
    steps = min(args.steps, wl.steps)
    warm = min(args.warmup, 10)
    n_in = steps + warm
    x0 = synth.activations(wl.seed, n_in, d, "bf16").to(dev)
    vp = lambda t: C.c_void_p(t.data_ptr())
    xs = torch.empty((wl.n_layers + 1, d), dtype=torch.bfloat16, device=dev)       # layer inputs of the current step
    idx_o = torch.zeros((LM, 16), dtype=torch.int32, device=dev)            # (rows padded to 64 bytes)
    prec_o = torch.zeros((LM, 16), dtype=torch.uint8, device=dev)             # 16-byte rows keep every pointer aligned
    lib = B.lib()
    if qwen:
        wr = [synth.router_weight(wl.seed, l, E, d).to(dev) for l in range(LM)]
        wsg = [synth.shared_gate_weight(wl.seed, l, d, "bf16").to(dev) for l in range(LM)]
        masks = torch.zeros((LM, E), dtype=torch.uint8, device=dev)
        calls = [(ctx.h, routed[l].h, shared[l].h, vp(xs[l]), C.c_int(B.BF16), C.c_int(k), None, vp(wr[l]), None, C.c_int(0),
                  C.c_float(1.0), vp(masks[l]), C.c_float(0.0), vp(wsg[l]), C.c_int(1), vp(xs[l + 1]), vp(idx_o[l]), None,
                  vp(prec_o[l])) for l in range(LM)]
    else:
        z = [synth.zipf_logits(wl.seed, l + 1, n_in, E).to(dev) for l in range(LM)]
        masks = torch.zeros((LM, E), dtype=torch.uint8, device=dev)
        bias = torch.zeros((LM, E), dtype=torch.float32, device=dev)
        cache = B.Cache(LM, E, (2 * LM * E) // 4)
        dense_call = (ctx.h, None, dense.h, vp(xs[0]), C.c_int(B.BF16), C.c_int(0), None, None, None, C.c_float(0.0), None,
                      C.c_int(1), vp(xs[1]), None)
        host_masks = torch.zeros((LM, E), dtype=torch.uint8).pin_memory()
        host_bias = torch.zeros((LM, E), dtype=torch.float32).pin_memory()
        host_idx = torch.zeros((LM, 16), dtype=torch.int32).pin_memory()
        want = np.ones((LM, k), np.uint8)
        hm_np, hb_np, hi_np = host_masks.numpy(), host_bias.numpy(), host_idx.numpy()

    def step(t):
        xs[0].copy_(x0[t])
        if qwen:
            if t % 32 == 0:
                masks.copy_(torch.from_numpy(synth.fraction_masks(wl.seed, LM, t // 32, E, 0.3)))
            for l in range(LM):
                rc = lib.smoe_decode_layer(*calls[l])
                if rc:
                    raise B.SmoeError("decode call failed: %d" % rc)
        else:
            cache.snapshot_all(1.0, hm_np, hb_np)      # straight into the pinned staging buffers
            masks.copy_(host_masks, non_blocking=True)
            bias.copy_(host_bias, non_blocking=True)
            rc = lib.smoe_expert_ffn(*dense_call)
            for l in range(LM):
                rc = rc or lib.smoe_decode_layer(ctx.h, routed[l].h, shared[l].h, vp(xs[l + 1]), C.c_int(B.BF16), C.c_int(k),
                                                 vp(z[l][t]), None, vp(bias[l]), C.c_int(0), C.c_float(1.0), vp(masks[l]),
                                                 C.c_float(0.0), None, C.c_int(1), vp(xs[l + 2]), vp(idx_o[l]), None,
                                                 vp(prec_o[l]))
            if rc:
                raise B.SmoeError("decode call failed: %d" % rc)
            host_idx.copy_(idx_o)                       # synchronises: the LRU needs this step's selections
            if t % 16 == 0:                             # HIGH slots of a sampled step: selected experts with both slices resident
                high_sum[0] += int((hm_np[lrange, hi_np[:, :k]] == 3).sum())
                high_sum[1] += 1
            cache.access_all(hi_np, k, want)

    high_sum = [0, 0]
    lrange = np.arange(LM)[:, None]
    for t in range(warm):
        step(t)
    torch.cuda.synchronize()
    high_sum[0] = high_sum[1] = 0
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for t in range(warm, warm + steps):
        step(t)
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms = ev0.elapsed_time(ev1) / steps
    assert bool(torch.isfinite(xs.float()).all())
    # algorithmic bytes of the last step (the precision flags of its layers), as a sample of the mix
    pr = prec_o.cpu().numpy()[:, :k]
    hi_b = sum(slot_bytes(d, shp.d_ff, shp.group, 1)); lo_b = sum(slot_bytes(d, shp.d_ff, shp.group, 0))
    sh_b = shp.n_shared * sum(slot_bytes(d, shp.shared_d_ff, shp.group, 1))
    step_bytes = float(sum(sh_b + int(p.sum()) * hi_b + int(k - p.sum()) * lo_b for p in pr))
    if not qwen:
        step_bytes += sum(slot_bytes(d, wl.dense_first_d_ff, shp.group, 1))
    out = {
        "metric": "decode us/token per MoE layer over the whole %d-layer stack" % wl.n_layers,
        "value": ms * 1e3 / wl.n_layers, "unit": "us/token-layer", "n_gpus": 1, "steps": steps, "warmup": warm,
        "ms_per_step": ms, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "u4+u4 bit-sliced weights, bf16 activations, signed 4-bit dot products, int32/fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": ("Qwen1.5-MoE-shaped 24-layer decode stack (BASELINE configs[2]): router mat-vec, one gated wide "
                                "shared expert, masks redrawn every 32 steps" if qwen else
                                "DeepSeek-V2-Lite-shaped 26-layer decode stack (BASELINE configs[3]): dense first layer, Zipf-skewed "
                                "logits, masks and bias from the host slice LRU (25 % of the slices) inside the timed window"),
                   "layers": wl.n_layers, "d_model": d, "n_experts": E, "d_ff": shp.d_ff, "top_k": k,
                   "n_shared": shp.n_shared, "shared_d_ff": shp.shared_d_ff, "group": shp.group,
                   "mean_high_slots_last_step": float(pr.sum() / LM),
                   "mean_high_slots_sampled_steps": (high_sum[0] / (high_sum[1] * LM)) if high_sum[1] else None},
        "us_per_step": ms * 1e3, "host_wall_ms_per_step": wall_ms / steps,
        "bytes_last_step": step_bytes, "hbm_gbps": step_bytes / (ms * 1e-3) / 1e9,
        "hbm_frac": step_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "roofline": {"bound": "hbm", "kernel": "whole step (all layers: router mat-vec where used, gate/up, down)",
                     "achieved": step_bytes / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": step_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, "traffic": None},
    }
    if not qwen:
        out["lru_stats"] = cache.stats()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_stack(wl, qwen, 4)
    print(json.dumps(out))


def cpu_baseline(wl, n_steps, idx_np, prec_np):
    """The CPU oracle, as it stands, on the first n_steps tokens of the same workload (quantised
    experts prepared outside the timed region, like the GPU's)."""
    import numpy as np
    from oracle import slicemoe_oracle as O
    from paper_2512_12990_amd import synth
    shp = wl.layer
    x_all = synth.activations(wl.seed, wl.steps, shp.d_model, "bf16").float().numpy()
    z_all = synth.normal_logits(wl.seed, wl.steps, shp.n_experts).numpy()
    mask, bias = synth.cached_set_mask(wl.seed, shp.n_experts, 32, 16, 1.0)
    need = sorted({int(e) for t in range(n_steps) for e in O.route(z_all[t][None], bias, shp.top_k)[0][0]})
    gen_dev = "cuda:0"
    experts = {}
    for tag in need + [1000 + i for i in range(shp.n_shared)]:
        f = shp.shared_d_ff if tag >= 1000 else shp.d_ff
        wg, wu, wd = (w.float().cpu().numpy() for w in synth.expert_weights(wl.seed, 0, tag, shp.d_model, f, "bf16", gen_dev))
        experts[tag] = O.quantize_expert(wg, wu, wd, shp.group, scale_dtype="bf16")
    sharedl = [experts[1000 + i] for i in range(shp.n_shared)]
    c0, t0 = time.process_time(), time.perf_counter()
    for t in range(n_steps):
        idx, w = O.route(z_all[t][None], bias, shp.top_k)
        prec = O.precision_select(idx[0], w[0], mask)
        O.moe_layer(x_all[t].astype(np.float64), experts, idx[0], w[0], prec, sharedl)
    wall = time.perf_counter() - t0
    cpu = time.process_time() - c0
    return {"value": wall / n_steps * 1e6, "unit": "us/token", "cores": max(1, int(round(cpu / wall))),
            "kind": "oracle", "sample": "first %d of the 1024 decode steps (route + 6 routed + 2 shared experts each), "
            "numpy fp64; expert quantisation outside the timed region" % n_steps,
            "host_cpus": os.cpu_count()}


def cpu_baseline_prefill(wl, T, n_tok, idx_np, w_np):
    """The CPU oracle on the first n_tok tokens of the prefill layer (its routed experts, all high-bit), with the
    routing the GPU pass produced; scaled to the layer's T tokens."""
    import numpy as np
    from oracle import slicemoe_oracle as O
    from paper_2512_12990_amd import synth
    shp = wl.layer
    x = synth.activations(wl.seed, T, shp.d_model, "bf16").float().numpy()[:n_tok]
    need = sorted({int(e) for e in idx_np[:n_tok].ravel()})
    experts = {}
    for e in need:
        wg, wu, wd = (w.float().cpu().numpy() for w in synth.expert_weights(wl.seed, 0, e, shp.d_model, shp.d_ff, "bf16", "cuda:0"))
        experts[e] = O.quantize_expert(wg, wu, wd, shp.group, scale_dtype="bf16")
    c0, t0 = time.process_time(), time.perf_counter()
    O.prefill_layer(x.astype(np.float64), experts, idx_np[:n_tok], w_np[:n_tok].astype(np.float64))
    wall = time.perf_counter() - t0
    cpu = time.process_time() - c0
    return {"value": wall / n_tok * T * 1e3, "unit": "ms/layer", "cores": max(1, int(round(cpu / wall))), "kind": "oracle",
            "sample": "first %d of the %d tokens through the layer's routed experts (numpy fp64), scaled by %d/%d; expert "
                      "quantisation outside the timed region" % (n_tok, T, T, n_tok), "host_cpus": os.cpu_count()}


def cpu_baseline_stack(wl, qwen, n_layers):
    """The CPU oracle on one token through the first n_layers MoE layers of the stack (each layer's input drawn
    as the workload's activations: the layers are timed, not chained), scaled to us per token-layer."""
    import numpy as np
    from oracle import slicemoe_oracle as O
    from paper_2512_12990_amd import synth
    shp = wl.layer
    d, E, k = shp.d_model, shp.n_experts, shp.top_k
    x = synth.activations(wl.seed, n_layers, d, "bf16").float().numpy().astype(np.float64)
    jobs = []
    for l in range(n_layers):
        if qwen:
            z = O.router_logits(x[l][None].astype(np.float32), synth.router_weight(wl.seed, l, E, d).numpy())
            mask = synth.fraction_masks(wl.seed, n_layers, 0, E, 0.3)[l]
            bias = None
            wsg = synth.shared_gate_weight(wl.seed, l, d, "bf16").float().numpy()
        else:
            z = synth.zipf_logits(wl.seed, l + 1, 1, E).numpy()
            mask, bias = synth.cached_set_mask(wl.seed + l, E, E // 4, E // 8, 1.0)
            wsg = None
        idx, w = O.route(z, bias, k)
        experts = {}
        for tag in [int(e) for e in idx[0]] + [1000 + i for i in range(shp.n_shared)]:
            f = shp.shared_d_ff if tag >= 1000 else shp.d_ff
            wg, wu, wd = (t.float().cpu().numpy() for t in synth.expert_weights(wl.seed, l, tag, d, f, "bf16", "cuda:0"))
            experts[tag] = O.quantize_expert(wg, wu, wd, shp.group, scale_dtype="bf16")
        jobs.append((x[l], experts, idx[0], w[0], O.precision_select(idx[0], w[0], mask),
                     [experts[1000 + i] for i in range(shp.n_shared)], wsg))
    c0, t0 = time.process_time(), time.perf_counter()
    for xl, experts, idx, w, prec, sh, wsg in jobs:
        O.moe_layer(xl, experts, idx, w, prec, sh, wsg, True)
    wall = time.perf_counter() - t0
    cpu = time.process_time() - c0
    return {"value": wall / n_layers * 1e6, "unit": "us/token-layer", "cores": max(1, int(round(cpu / wall))), "kind": "oracle",
            "sample": "one token through %d MoE layers of the stack (route + %d routed + %d shared experts each), numpy fp64; "
                      "expert quantisation outside the timed region" % (n_layers, k, shp.n_shared), "host_cpus": os.cpu_count()}


if __name__ == "__main__":
    main()
