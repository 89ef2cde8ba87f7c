"""GPU parity of the prefill path: routing indices and the per-expert histogram bit-exact,
grouped-GEMM outputs within the bf16 tolerance, top-N retention order from the GPU histogram."""
import sys

import numpy as np
import pytest
import torch

from oracle import slicemoe_oracle as O
from paper_2512_12990_amd import binding as B
from paper_2512_12990_amd import synth
from helpers import LayerPair, t2np

pytestmark = pytest.mark.gpu
TOL = 2e-2


def say(*a):
    print(*a, flush=True)


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available()
    c = B.Ctx(0)
    yield c
    torch.cuda.synchronize()
    c.close()


def _check_routing(ctx, x, wr, k, idx, w, hist, E):
    _, _, z = B.smoe_route(ctx, k, x=x, w_router=wr, want_logits=True)
    ridx, rw = O.route(z.cpu().numpy(), None, k)          # top-k of the GPU's own fp32 logits
    assert np.array_equal(idx.cpu().numpy(), ridx)
    np.testing.assert_allclose(w.cpu().numpy(), rw, rtol=2e-5, atol=1e-7)
    h = hist.cpu().numpy().view(np.uint32)
    assert np.array_equal(h, O.histogram(ridx, E)) and int(h.sum()) == ridx.size
    zr = O.router_logits(t2np(x), t2np(wr))
    np.testing.assert_allclose(z.cpu().numpy(), zr, rtol=0, atol=2e-5 * np.abs(zr).max())
    return ridx, rw


@pytest.mark.parametrize("T,E,k,d,f,G", [(200, 6, 2, 256, 128, 64), (37, 5, 3, 128, 192, 32), (450, 3, 1, 128, 64, 64),
                                          (70, 4, 2, 4096, 128, 128)])
def test_prefill_small_all_tokens(ctx, T, E, k, d, f, G):
    # 200 tokens over 6 experts: one expert tile is ragged; 37 tokens: a single partial fragment;
    # 450 tokens over 3 experts top-1: some expert gets more than one 192-row tile; d_model 4096: the
    # router's activations need more than 64 KB of LDS
    say("prefill small", T, E, k, d, f, G)
    shp = synth.LayerShape(d, E, f, k, G, act="bf16")
    pair = LayerPair(ctx, shp, seed=21)
    x = synth.activations(21, T, d, "bf16").cuda()
    wr = synth.router_weight(21, 0, E, d, std=0.05).cuda()
    for resid in (False, True):
        y, idx, w, hist = B.smoe_prefill_histogram(ctx, pair.routed, None, x, k, w_router=wr, add_residual=resid)
        ridx, rw = _check_routing(ctx, x, wr, k, idx, w, hist, E)
        yref = O.prefill_layer(t2np(x).astype(np.float64), pair.oracle_routed(), ridx,
                               rw.astype(np.float32).astype(np.float64), add_residual=resid)
        yg = t2np(y)
        for t in range(T):
            assert O.max_abs_rel(yg[t], yref[t]) <= TOL, t
        assert O.max_abs_rel(yg, yref) <= TOL


@pytest.mark.parametrize("n_shared,f_s,gate", [(1, 320, True), (2, 128, False)])
def test_prefill_with_shared_experts(ctx, n_shared, f_s, gate):
    # the shared-expert group sees every token (dense GEMMs over the token rows): one wide shared expert
    # behind a sigmoid gate (Qwen shape) or two plain ones (DeepSeek shape); 230 tokens = one full
    # 192-row tile and a ragged one; 320 = 2.5 column tiles of the gate/up GEMM
    T, E, k, d, f, G = 230, 6, 2, 256, 128, 64
    say("prefill with shared experts", n_shared, f_s, gate)
    shp = synth.LayerShape(d, E, f, k, G, n_shared=n_shared, shared_d_ff=f_s, shared_gate=gate, act="bf16")
    pair = LayerPair(ctx, shp, seed=23)
    x = synth.activations(23, T, d, "bf16").cuda()
    wr = synth.router_weight(23, 0, E, d, std=0.05).cuda()
    wsg = synth.shared_gate_weight(23, 0, d, "bf16", std=0.05).cuda() if gate else None
    for resid in (False, True):
        y, idx, w, hist = B.smoe_prefill_histogram(ctx, pair.routed, pair.shared, x, k, w_router=wr, shared_gate_w=wsg,
                                                   add_residual=resid)
        ridx, rw = _check_routing(ctx, x, wr, k, idx, w, hist, E)
        yref = O.prefill_layer(t2np(x).astype(np.float64), pair.oracle_routed(), ridx,
                               rw.astype(np.float32).astype(np.float64), pair.oracle_shared(),
                               None if wsg is None else t2np(wsg), add_residual=resid)
        yg = t2np(y)
        for t in range(T):
            assert O.max_abs_rel(yg[t], yref[t]) <= TOL, t
    # a prefill layer and the decode layer agree on a token (both HIGH): same semantics on both paths
    t = 7
    mask = np.full(E, 3, np.uint8)
    yd = B.smoe_expert_ffn(ctx, pair.routed, pair.shared, x[t].clone(), idx[t].clone(), w[t].clone(),
                           torch.from_numpy(mask).cuda(), shared_gate_w=wsg, add_residual=True)
    assert O.max_abs_rel(t2np(yd), t2np(y[t])) <= TOL


@pytest.mark.parametrize("nest", [(4, 2), (6, 3)])
@pytest.mark.parametrize("G,sdt", [(64, "bf16"), (32, "bf16")])
def test_prefill_lower_nests(ctx, G, sdt, nest):
    # the 4/2 nest (4-bit codes in 2-bit planes) and the 6/3 nest (6-bit codes in 3-bit planes) through
    # the prefill path, with a gated shared expert
    T, E, k, d, f = 230, 6, 2, 256, 192
    say("prefill lower nest", nest, G)
    shp = synth.LayerShape(d, E, f, k, G, n_shared=1, shared_d_ff=128, shared_gate=True, act=sdt, b_high=nest[0],
                           b_low=nest[1])
    pair = LayerPair(ctx, shp, seed=41)
    x = synth.activations(41, T, d, "bf16").cuda()
    wr = synth.router_weight(41, 0, E, d, std=0.05).cuda()
    wsg = synth.shared_gate_weight(41, 0, d, "bf16", std=0.05).cuda()
    y, idx, w, hist = B.smoe_prefill_histogram(ctx, pair.routed, pair.shared, x, k, w_router=wr, shared_gate_w=wsg,
                                               add_residual=True)
    ridx, rw = _check_routing(ctx, x, wr, k, idx, w, hist, E)
    yref = O.prefill_layer(t2np(x).astype(np.float64), pair.oracle_routed(), ridx,
                           rw.astype(np.float32).astype(np.float64), pair.oracle_shared(), t2np(wsg), add_residual=True)
    yg = t2np(y)
    for t in range(T):
        assert O.max_abs_rel(yg[t], yref[t]) <= TOL, t
    # and it agrees with the decode path on one token (both HIGH)
    t = 3
    yd = B.smoe_expert_ffn(ctx, pair.routed, pair.shared, x[t].clone(), idx[t].clone(), w[t].clone(),
                           torch.from_numpy(np.full(E, 3, np.uint8)).cuda(), shared_gate_w=wsg, add_residual=True)
    assert O.max_abs_rel(t2np(yd), t2np(y[t])) <= TOL


def test_prefill_empty_expert_and_given_logits(ctx):
    say("prefill with an expert nobody selects")
    T, E, k, d, f, G = 64, 4, 2, 128, 64, 32
    shp = synth.LayerShape(d, E, f, k, G, act="bf16")
    pair = LayerPair(ctx, shp, seed=22)
    x = synth.activations(22, T, d, "bf16").cuda()
    z = synth.normal_logits(22, T, E)
    z[:, 2] = -30.0
    y, idx, w, hist = B.smoe_prefill_histogram(ctx, pair.routed, None, x, k, logits=z.cuda(), norm_topk=True)
    ridx, rw = O.route(z.numpy(), None, k, norm_topk=True)
    assert np.array_equal(idx.cpu().numpy(), ridx)
    h = hist.cpu().numpy().view(np.uint32)
    assert h[2] == 0 and np.array_equal(h, O.histogram(ridx, E))
    yref = O.prefill_layer(t2np(x).astype(np.float64), pair.oracle_routed(), ridx, rw)
    assert O.max_abs_rel(t2np(y), yref) <= TOL


def test_prefill_qwen_layer_full_size_sampled_tokens(ctx):
    """2048 tokens through one Qwen1.5-MoE-shaped layer (60 experts of 2048x1408, top-4, all
    high-bit): every index and the histogram exactly, sampled token rows against the oracle."""
    wl = synth.QWEN_PREFILL
    shp = wl.layer
    T = wl.prefill_tokens
    say("qwen prefill layer: quantising 60 experts")
    pair = LayerPair(ctx, shp, seed=wl.seed, gen_device="cuda:0", keep_dense=False)
    x = synth.activations(wl.seed, T, shp.d_model, "bf16").cuda()
    wr = synth.router_weight(wl.seed, 0, shp.n_experts, shp.d_model).cuda()
    y, idx, w, hist = B.smoe_prefill_histogram(ctx, pair.routed, None, x, shp.top_k, w_router=wr, add_residual=False)
    torch.cuda.synchronize()
    say("  prefill done; checking routing of all tokens")
    ridx, rw = _check_routing(ctx, x, wr, shp.top_k, idx, w, hist, shp.n_experts)
    hist_np = hist.cpu().numpy().view(np.uint32)
    ids = B.smoe_topn_slices(hist_np[None, :], 30)
    assert np.array_equal(ids, O.topn_slices(hist_np[None, :], 30))
    yg = t2np(y)
    assert np.isfinite(yg).all()
    xs = t2np(x).astype(np.float64)
    for t in (0, 1031, 2047):
        say("  oracle token", t)
        prec = np.ones(shp.top_k, np.uint8)
        yref = O.moe_layer(xs[t], pair.oracle_routed(), ridx[t], rw[t].astype(np.float32).astype(np.float64), prec)
        err = O.max_abs_rel(yg[t], yref)
        say("    max-abs-rel", err)
        assert err <= TOL


def test_prefill_more_pairs_than_the_grouping_registers_hold(ctx):
    # 4100 tokens top-3 = 12300 (token, slot) pairs: every thread of the grouping kernel owns a run of 13,
    # more than the eight it keeps in registers, so the pairs are read one by one in both passes; every
    # expert gets a dozen 192-row tiles.  (8192 tokens top-4, the long-prompt bench line, runs the same path.)
    T, E, k, d, f, G = 4100, 5, 3, 128, 64, 32
    say("prefill, long pair list", T, E, k)
    shp = synth.LayerShape(d, E, f, k, G, n_shared=1, shared_d_ff=64, act="bf16")
    pair = LayerPair(ctx, shp, seed=27)
    x = synth.activations(27, T, d, "bf16").cuda()
    wr = synth.router_weight(27, 0, E, d, std=0.05).cuda()
    y, idx, w, hist = B.smoe_prefill_histogram(ctx, pair.routed, pair.shared, x, k, w_router=wr, add_residual=True)
    ridx, rw = _check_routing(ctx, x, wr, k, idx, w, hist, E)
    assert int(hist.cpu().numpy().view(np.uint32).max()) > 192 * 8
    yref = O.prefill_layer(t2np(x).astype(np.float64), pair.oracle_routed(), ridx, rw.astype(np.float32).astype(np.float64),
                           pair.oracle_shared(), None, add_residual=True)
    yg = t2np(y)
    for t in range(T):
        assert O.max_abs_rel(yg[t], yref[t]) <= TOL, t


def test_prefill_qwen_24_layer_chain(ctx):
    """The prefill workload as stated: 2048 tokens through 24 Qwen1.5-MoE-shaped layers, each layer's output
    (plus residual, rescaled to unit RMS per token in place of the attention / normalisation blocks that are
    outside the path) feeding the next.  Per layer: every routing index and the histogram exactly; at the
    end the top-N slice order over the [24, 60] histogram; sampled tokens of sampled layers against the oracle,
    which is handed the GPU's own layer input (teacher-forced)."""
    wl = synth.QWEN_PREFILL
    shp = wl.layer
    T, L, E, k, d = wl.prefill_tokens, wl.n_layers, shp.n_experts, shp.top_k, shp.d_model
    say("qwen prefill chain: quantising %d x %d experts" % (L, E))
    layers = [LayerPair(ctx, shp, seed=wl.seed, layer=l, gen_device="cuda:0", keep_dense=False) for l in range(L)]
    wr = [synth.router_weight(wl.seed, l, E, d).cuda() for l in range(L)]
    x = synth.activations(wl.seed, T, d, "bf16").cuda()
    scratch = torch.empty(B.smoe_prefill_bytes(T, E, k, d, shp.d_ff), dtype=torch.uint8, device="cuda:0")
    samples = {0: (0, 2047), 11: (5, 1033), 23: (1, 700, 2046)}
    hists = np.zeros((L, E), np.uint32)
    kept = {}
    for l in range(L):
        y, idx, w, hist = B.smoe_prefill_histogram(ctx, layers[l].routed, None, x, k, w_router=wr[l], add_residual=True,
                                                   scratch=scratch)
        ridx, rw = _check_routing(ctx, x, wr[l], k, idx, w, hist, E)
        hists[l] = hist.cpu().numpy().view(np.uint32)
        if l in samples:
            # the MoE term on its own (no residual) is what the oracle is compared with: next to x it is
            # small, and a comparison of x + MoE(x) would mostly compare x with itself
            y_moe = B.smoe_prefill_histogram(ctx, layers[l].routed, None, x, k, w_router=wr[l], add_residual=False,
                                             scratch=scratch)[0]
            kept[l] = (t2np(x), t2np(y_moe), ridx, rw)
            resid = t2np(y) - (t2np(x) + t2np(y_moe))
            assert np.abs(resid).max() <= 2.0 ** -7 * np.abs(t2np(y)).max()      # y = bf16(x + MoE(x)), two roundings apart
        yf = y.float()
        x = (yf * torch.rsqrt((yf * yf).mean(dim=1, keepdim=True) + 1e-6)).to(torch.bfloat16)
    assert hists.sum() == L * T * k
    n_keep = (2 * L * E) // 4
    assert np.array_equal(B.smoe_topn_slices(hists, n_keep), O.topn_slices(hists, n_keep))
    for l, toks in samples.items():
        xin, yg, ridx, rw = kept[l]
        for t in toks:
            say("  oracle layer", l, "token", t)
            yref = O.moe_layer(xin[t].astype(np.float64), layers[l].oracle_routed(), ridx[t],
                               rw[t].astype(np.float32).astype(np.float64), np.ones(k, np.uint8))
            err = O.max_abs_rel(yg[t], yref)
            say("    max-abs-rel", err)
            assert err <= TOL


def test_prefill_random_small_shapes(ctx):
    # a seeded sweep over prefill shapes: token counts around the 192-row tile, d_model and d_ff any
    # multiple of 64 (ragged column tiles), every group size, with and without shared experts
    rng = np.random.default_rng(77)
    for case in range(8):
        T = int(rng.choice([1, 3, 31, 64, 190, 193, 260, 400]))
        d = int(rng.choice([64, 128, 192, 320]))
        f = int(rng.integers(1, 6)) * 64
        G = int(rng.choice([32, 64, 128]))
        E = int(rng.integers(1, 9))
        k = int(rng.integers(1, min(E, 4) + 1))
        n_sh = int(rng.integers(0, 3))
        f_s = int(rng.integers(1, 5)) * 64 if n_sh else 0
        gate = bool(n_sh and rng.random() < 0.5)
        say("random prefill shape", case, dict(T=T, d=d, f=f, G=G, E=E, k=k, n_sh=n_sh, f_s=f_s, gate=gate))
        shp = synth.LayerShape(d, E, f, k, G, n_shared=n_sh, shared_d_ff=f_s, shared_gate=gate, act="bf16")
        pair = LayerPair(ctx, shp, seed=300 + case)
        x = synth.activations(300 + case, T, d, "bf16").cuda()
        wr = synth.router_weight(300 + case, 0, E, d, std=0.05).cuda()
        wsg = synth.shared_gate_weight(300 + case, 0, d, "bf16", std=0.05).cuda() if gate else None
        y, idx, w, hist = B.smoe_prefill_histogram(ctx, pair.routed, pair.shared, x, k, w_router=wr, shared_gate_w=wsg,
                                                   add_residual=bool(case & 1))
        ridx, rw = _check_routing(ctx, x, wr, k, idx, w, hist, E)
        yref = O.prefill_layer(t2np(x).astype(np.float64), pair.oracle_routed(), ridx,
                               rw.astype(np.float32).astype(np.float64), pair.oracle_shared(),
                               None if wsg is None else t2np(wsg), add_residual=bool(case & 1))
        yg = t2np(y)
        for t in range(T):
            assert O.max_abs_rel(yg[t], yref[t]) <= TOL, (case, t)
