"""Slice-cache policy report on a synthetic decode trace (paper Sections 4.1, 4.3, 5 and 6).

    python -m paper_2512_12990_amd.dbsc_report [--model dsv2lite|qwen] [--steps N] [--beta B]

Routes a popularity-skewed synthetic trace through the library's router (`smoe_route`, on the GPU),
feeds the decisions to the library's slice LRU (`smoe_cache_*`, host) and prints, per cache size and
criticality threshold, the slice miss rates, the high-bit-normalised miss rate and the modeled
energy and latency per token on the paper's device (`smoe_cost_model`); then the cold misses of the
first decode steps for a cache warmed from prefill access counts (`smoe_topn_slices`,
`smoe_cache_init_order`) against an empty one.  All numbers describe synthetic traces: they show
how the policy behaves, not the paper's measured gains.
"""
import argparse

import numpy as np
import torch

from . import binding as B
from . import synth

MODELS = {
    # MoE layers, experts, top-k, d_model, d_ff, group
    "dsv2lite": (25, 64, 6, 2048, 1408, 128),
    "qwen": (24, 60, 4, 2048, 1408, 128),
}


def slice_bytes(d, f, group):
    """(MSB slice, LSB slice) of one 8/4 expert: a nibble plane of the three matrices each; the MSB
    slice also carries zero-points and bf16 scales (the low-bit model needs them)."""
    plane = 3 * d * f // 2
    meta = 3 * (2 * f * -(-d // group) + d * -(-f // group))
    return plane + meta, plane


def route_trace(ctx, seed, L, E, k, steps, period, beta, cache):
    """idx [steps, L, k] int32, w [steps, L, k] fp32.  beta = 0: every layer's steps in one call.
    beta > 0: cache-aware routing (Section 2.1) in closed loop with `cache`: the bias of a step comes
    from the slice state left by the previous step, and every decision is fed back at once (all
    slots ask for both slices)."""
    z = [synth.zipf_logits(seed, l, steps, E, period=period).to("cuda:%d" % ctx.device) for l in range(L)]
    idx = np.empty((steps, L, k), np.int32)
    w = np.empty((steps, L, k), np.float32)
    if beta <= 0.0:
        for l in range(L):
            i, ww = B.smoe_route(ctx, k, logits=z[l])
            idx[:, l], w[:, l] = i.cpu().numpy(), ww.cpu().numpy()
        return idx, w
    mask = np.empty((L, E), np.uint8)
    bias = np.empty((L, E), np.float32)
    for t in range(steps):
        cache.snapshot_all(beta, mask, bias)
        bd = torch.from_numpy(bias).to(z[0].device)
        for l in range(L):
            i, ww = B.smoe_route(ctx, k, logits=z[l][t:t + 1], bias=bd[l])
            idx[t, l], w[t, l] = i.cpu().numpy()[0], ww.cpu().numpy()[0]
        cache.access_all(np.ascontiguousarray(idx[t]), k, np.ones((L, k), np.uint8))
    return idx, w


def replay(cache, idx, w, tau, first=None):
    n = idx.shape[0] if first is None else first
    k = idx.shape[2]
    for t in range(n):
        want = np.ascontiguousarray((w[t] >= tau).astype(np.uint8))      # tau = 0: every slot asks for its LSB slice
        cache.access_all(np.ascontiguousarray(idx[t]), k, want)
    return cache.stats()


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--model", choices=sorted(MODELS), default="dsv2lite")
    ap.add_argument("--steps", type=int, default=512, help="decode steps of the trace")
    ap.add_argument("--prefill", type=int, default=512, help="prompt tokens whose routing fills the warm-up histogram")
    ap.add_argument("--period", type=int, default=64, help="steps between redraws of the popularity permutation")
    ap.add_argument("--beta", type=float, default=0.0, help="cache-aware routing bias (0: routing ignores the cache)")
    ap.add_argument("--tau-warm", type=float, default=0.2, help="criticality threshold used in the warm-up comparison")
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()
    if not torch.cuda.is_available():
        raise SystemExit("dbsc_report routes its trace with the HIP library: it needs the GPU")
    L, E, k, d, f, G = MODELS[args.model]
    bm, bl = slice_bytes(d, f, G)
    spec = B.smoe_system_spec_paper()
    ctx = B.Ctx(0)
    ops_hi = 2.0 * 3 * d * f            # multiply-adds x 2 of one expert, per requested expert
    n_slices = 2 * L * E
    print("model %s: %d MoE layers x %d experts, top-%d; MSB slice %.2f MB, LSB slice %.2f MB; trace: Zipf(1.1) logits, "
          "%d steps, permutation redrawn every %d, beta %.2f" % (args.model, L, E, k, bm / 1e6, bl / 1e6, args.steps,
                                                                   args.period, args.beta))
    print()
    print("| cache (slices) | tau_head | MSB miss | LSB miss | LSB requests | high-bit-normalised miss | mJ/token | ms/token |")
    print("|---|---|---|---|---|---|---|---|")
    for frac in (0.125, 0.25, 0.5):
        cap = int(n_slices * frac)
        if args.beta > 0.0:
            idx, w = route_trace(ctx, args.seed, L, E, k, args.steps, args.period, args.beta, B.Cache(L, E, cap))
        elif frac == 0.125:
            idx, w = route_trace(ctx, args.seed, L, E, k, args.steps, args.period, 0.0, None)
        for tau in (0.0, 0.1, 0.2, 0.3):
            st = replay(B.Cache(L, E, cap), idx, w, tau)
            req_m, req_l = st["msb_hit"] + st["msb_miss"], st["lsb_hit"] + st["lsb_miss"]
            c = B.smoe_cost_model(spec, st, bm, bl, ops_hi * req_m)
            print("| %d (%.1f %%) | %.1f | %.3f | %.3f | %.2f of MSB | %.3f | %.2f | %.2f |" % (
                cap, 100 * frac, tau, st["msb_miss"] / max(req_m, 1), st["lsb_miss"] / max(req_l, 1), req_l / max(req_m, 1),
                c["miss_rate_high"], 1e3 * c["energy_j"] / args.steps, 1e3 * c["latency_s"] / args.steps))
    # ---- Predictive Cache Warmup: prompt and early decode share one popularity permutation
    print()
    n_pre, first = args.prefill, 16
    idx, w = route_trace(ctx, args.seed + 1, L, E, k, n_pre + first, max(args.period, n_pre + first), 0.0, None)
    hist = np.zeros((L, E), np.uint32)
    for l in range(L):
        hist[l] = np.bincount(idx[:n_pre, l].reshape(-1), minlength=E)
    print("first %d decode steps after a %d-token prompt, tau_head %.1f (a warmed cache holds MSB slices only, so LSB slices "
          "fetched for critical experts are the first to leave again):" % (first, n_pre, args.tau_warm))
    print()
    print("| cache (slices) | initial state | MSB misses | Flash MB | mJ/token | ms/token |")
    print("|---|---|---|---|---|---|")
    for frac in (0.125, 0.25, 0.5):
        cap = int(n_slices * frac)
        for name in ("empty", "warmed from prefill counts"):
            cache = B.Cache(L, E, cap)
            if name != "empty":
                cache.init_order(B.smoe_topn_slices(hist, cap))
            st = replay(cache, idx[n_pre:], w[n_pre:], args.tau_warm)
            c = B.smoe_cost_model(spec, st, bm, bl, ops_hi * (st["msb_hit"] + st["msb_miss"]))
            print("| %d (%.1f %%) | %s | %d of %d | %.1f | %.2f | %.2f |" % (
                cap, 100 * frac, name, st["msb_miss"], st["msb_hit"] + st["msb_miss"], c["flash_bits"] / 8e6,
                1e3 * c["energy_j"] / first, 1e3 * c["latency_s"] / first))
    ctx.close()


if __name__ == "__main__":
    main()
