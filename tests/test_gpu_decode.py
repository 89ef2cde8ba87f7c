"""GPU parity: HIP path (through the C ABI) against the CPU oracle, same seeded inputs.

Integer results (codes, planes, zero-points, scale bits, top-k indices, precision flags) must be
bit-exact; FFN outputs within max-abs-rel 1e-4 (fp32 activations) / 2e-2 (bf16)."""
import sys

import numpy as np
import pytest
import torch

from oracle import slicemoe_oracle as O
from paper_2512_12990_amd import binding as B
from paper_2512_12990_amd import synth
from helpers import LayerPair, t2np

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    c = B.Ctx(0)
    yield c
    torch.cuda.synchronize()
    c.close()


def dev(a, dtype=None):
    t = torch.as_tensor(a)
    if dtype is not None:
        t = t.to(dtype)
    return t.to("cuda:0").contiguous()


# ------------------------------------------------------------------------------ quantise / slice
@pytest.mark.parametrize("d,f,G,dt", [(256, 128, 64, "f32"), (256, 160, 64, "bf16"), (2048, 1408, 128, "bf16"),
                                      (96, 64, 32, "f32")])
def test_quantize_slice_bit_exact(ctx, d, f, G, dt):
    say("quantize", d, f, G, dt)
    shape = synth.LayerShape(d, 2, f, 1, G, act=dt)
    pair = LayerPair(ctx, shape, seed=3)
    for e in range(2):
        ex = pair.oracle_expert(e)
        for mi, qm in enumerate((ex.gate, ex.up, ex.down)):
            got = B.smoe_export_codes(ctx, pair.routed, e, mi)
            assert np.array_equal(got["q"], qm.q)
            assert np.array_equal(got["msb"], qm.msb()) and np.array_equal(got["lsb"], qm.lsb())
            assert np.array_equal(got["zp"], qm.zp)
            assert np.array_equal(got["scale"].view(np.uint32), qm.scale.view(np.uint32))


@pytest.mark.parametrize("nest", [(4, 2), (6, 3)])
@pytest.mark.parametrize("d,f,G,dt", [(256, 160, 64, "bf16"), (96, 64, 32, "f32"), (2048, 1408, 32, "bf16")])
def test_quantize_slice_lower_nests_bit_exact(ctx, d, f, G, dt, nest):
    # the 4/2 nest: 4-bit codes whose upper two bits are the low-bit model, 2-bit planes;
    # the 6/3 nest: 6-bit codes, upper three bits, 3-bit planes of twelve bytes per 32 columns
    bh, bl = nest
    say("quantize", nest, d, f, G, dt)
    shape = synth.LayerShape(d, 2, f, 1, G, act=dt, b_high=bh, b_low=bl)
    pair = LayerPair(ctx, shape, seed=3)
    full = B.smoe_bank_bytes(B.BankDesc(2, d, f, G, 8, 4, B._DT[dt], B._DT[dt]))
    assert pair.routed.nbytes < (0.6 if bl == 2 else 0.85) * full
    for e in range(2):
        ex = pair.oracle_expert(e)
        for mi, qm in enumerate((ex.gate, ex.up, ex.down)):
            got = B.smoe_export_codes(ctx, pair.routed, e, mi)
            assert int(got["q"].max()) <= (1 << bh) - 1 and int(got["msb"].max()) <= (1 << bl) - 1
            assert np.array_equal(got["q"], qm.q)
            assert np.array_equal(got["msb"], qm.msb()) and np.array_equal(got["lsb"], qm.lsb())
            assert np.array_equal(got["zp"], qm.zp)
            assert np.array_equal(got["scale"].view(np.uint32), qm.scale.view(np.uint32))


@pytest.mark.parametrize("nest", [(8, 4), (6, 3), (4, 2)])
@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_quantize_symmetric_bit_exact(ctx, dt, nest):
    # the symmetric quantiser of the non-expert weights (Section 6.1 item 1) in the same store
    bh, bl = nest
    say("quantize symmetric", nest, dt)
    shape = synth.LayerShape(256, 2, 96, 1, 128, act=dt, b_high=bh, b_low=bl, symmetric=True)
    pair = LayerPair(ctx, shape, seed=11)
    for e in range(2):
        ex = pair.oracle_expert(e)
        for mi, qm in enumerate((ex.gate, ex.up, ex.down)):
            got = B.smoe_export_codes(ctx, pair.routed, e, mi)
            assert np.all(got["zp"] == 1 << (bh - 1)) and int(got["q"].min()) >= 1
            assert np.array_equal(got["q"], qm.q)
            assert np.array_equal(got["msb"], qm.msb()) and np.array_equal(got["lsb"], qm.lsb())
            assert np.array_equal(got["scale"].view(np.uint32), qm.scale.view(np.uint32))


def test_quantize_special_groups_bit_exact(ctx):
    # flat groups, one-sided groups, exact zeros, a huge and a tiny group next to each other
    say("quantize special")
    d, f, G = 128, 64, 32
    rng = np.random.default_rng(0)
    wg = (rng.standard_normal((1, f, d)) * 0.02).astype(np.float32)
    wg[0, 0, :32] = 0.0
    wg[0, 1, :32] = np.abs(wg[0, 1, :32]) + 0.1
    wg[0, 2, :32] = -np.abs(wg[0, 2, :32]) - 0.1
    wg[0, 3, 32:64] *= 1e4
    wg[0, 3, 64:96] *= 1e-6
    wg[0, 4, ::5] = 0.0
    wu = (rng.standard_normal((1, f, d)) * 0.02).astype(np.float32)
    wd = (rng.standard_normal((1, d, f)) * 0.02).astype(np.float32)
    for dt in ("f32", "bf16"):
        bank = B.Bank(ctx, 1, d, f, G, "f32", dt)
        B.smoe_quantize_slice(ctx, bank, 0, dev(wg), dev(wu), dev(wd))
        for mi, w in enumerate((wg, wu, wd)):
            ref = O.quantize(w[0], G, scale_dtype=dt)
            got = B.smoe_export_codes(ctx, bank, 0, mi)
            assert np.array_equal(got["q"], ref.q) and np.array_equal(got["zp"], ref.zp)
            assert np.array_equal(got["scale"].view(np.uint32), ref.scale.view(np.uint32))


# ------------------------------------------------------------------------------ route
@pytest.mark.parametrize("E,k,T", [(8, 2, 16), (64, 6, 200), (60, 4, 64), (256, 16, 8), (5, 5, 3)])
def test_route_given_logits(ctx, E, k, T):
    say("route logits", E, k, T)
    z = synth.normal_logits(7, T, E)
    z[0, : min(E, 4)] = 0.25                      # ties
    z[1 % T, :] = -0.0
    bias = torch.zeros(E)
    bias[torch.randperm(E, generator=torch.Generator().manual_seed(1))[: E // 2]] = 1.0
    for b, norm, rs in [(None, False, 1.0), (bias, False, 1.0), (bias, True, 2.5)]:
        idx, w = B.smoe_route(ctx, k, logits=dev(z), bias=None if b is None else dev(b), norm_topk=norm, routed_scale=rs)
        ridx, rw = O.route(z.numpy(), None if b is None else b.numpy(), k, norm, rs)
        assert np.array_equal(idx.cpu().numpy(), ridx)
        np.testing.assert_allclose(w.cpu().numpy(), rw, rtol=2e-5, atol=1e-7)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_route_from_activations(ctx, dt):
    say("route from x", dt)
    T, E, d, k = 33, 60, 2048, 4
    x = synth.activations(5, T, d, dt)
    wr = synth.router_weight(5, 0, E, d)
    idx, w, z = B.smoe_route(ctx, k, x=dev(x), w_router=dev(wr), want_logits=True)
    zg = z.cpu().numpy()
    zr = O.router_logits(t2np(x), wr.numpy())
    np.testing.assert_allclose(zg, zr, rtol=0, atol=2e-5 * np.abs(zr).max())
    # indices are a function of an fp32 logits array: the oracle's top-k runs on the GPU's logits
    ridx, rw = O.route(zg, None, k)
    assert np.array_equal(idx.cpu().numpy(), ridx)
    np.testing.assert_allclose(w.cpu().numpy(), rw, rtol=2e-5, atol=1e-7)


# ------------------------------------------------------------------------------ expert FFN
def _run_layer_steps(ctx, wl: synth.Workload, pair: LayerPair, steps, masks, bias, logits, x_all, use_fused, wr=None,
                     wsg=None, add_residual=False, tau=0.0, norm_topk=False, routed_scale=1.0):
    shp = wl.layer
    tol = TOL[shp.act]
    worst = 0.0
    for t in steps:
        x = x_all[t]
        mask = masks[t] if masks.ndim == 2 else masks
        xd = dev(x)
        md = dev(mask)
        if use_fused:
            idx_o = torch.empty(shp.top_k, dtype=torch.int32, device="cuda:0")
            w_o = torch.empty(shp.top_k, dtype=torch.float32, device="cuda:0")
            p_o = torch.empty(shp.top_k, dtype=torch.uint8, device="cuda:0")
            y = B.smoe_decode_layer(ctx, pair.routed, pair.shared, xd, shp.top_k,
                                    logits=None if logits is None else dev(logits[t]),
                                    w_router=None if wr is None else dev(wr), bias=None if bias is None else dev(bias),
                                    norm_topk=norm_topk, routed_scale=routed_scale, slice_mask=md, tau_head=tau, shared_gate_w=None if wsg is None else dev(wsg),
                                    add_residual=add_residual, idx_out=idx_o, w_out=w_o, prec_out=p_o)
            idx, w, prec = idx_o.cpu().numpy(), w_o.cpu().numpy(), p_o.cpu().numpy()
            if logits is not None:
                ridx, rw = O.route(logits[t].numpy()[None], None if bias is None else bias.numpy(), shp.top_k, norm_topk,
                                   routed_scale)
            else:
                _, _, zg = B.smoe_route(ctx, shp.top_k, x=xd[None], w_router=dev(wr), want_logits=True)
                ridx, rw = O.route(zg.cpu().numpy(), None if bias is None else bias.numpy(), shp.top_k, norm_topk, routed_scale)
            assert np.array_equal(idx, ridx[0]), (t, idx, ridx)
            np.testing.assert_allclose(w, rw[0], rtol=2e-5, atol=1e-7)
        else:
            z = logits[t].numpy()[None] if logits is not None else O.router_logits(t2np(x), wr.numpy())
            ridx, rw = O.route(z, None if bias is None else bias.numpy(), shp.top_k, norm_topk, routed_scale)
            p_o = torch.empty(shp.top_k, dtype=torch.uint8, device="cuda:0")
            y = B.smoe_expert_ffn(ctx, pair.routed, pair.shared, xd, dev(ridx[0]), dev(rw[0].astype(np.float32)), md,
                                  tau_head=tau, shared_gate_w=None if wsg is None else dev(wsg),
                                  add_residual=add_residual, prec_out=p_o)
            prec = p_o.cpu().numpy()
        # the oracle uses the gate weights the GPU path was given / produced in fp32: the threshold
        # decision is taken on the very fp32 weight the kernel compares (checked against the oracle's
        # weight above), so a weight that sits on the threshold cannot fall on different sides
        w_used = (w if use_fused else rw[0]).astype(np.float32).astype(np.float64)
        rprec = O.precision_select(ridx[0], w_used, mask, tau)
        assert np.array_equal(prec, rprec), (t, prec, rprec)
        yref = O.moe_layer(t2np(x).astype(np.float64), pair.oracle_routed(), ridx[0], w_used, rprec,
                           pair.oracle_shared(), None if wsg is None else t2np(wsg), add_residual)
        err = O.max_abs_rel(t2np(y), yref)
        worst = max(worst, err)
        assert err <= tol, (t, err)
        assert np.abs(yref).max() > 0, t          # a comparison against an all-zero reference would prove nothing
    return worst


@pytest.mark.parametrize("use_fused", [False, True])
def test_tiny_fp32_layer_all_steps(ctx, use_fused):
    wl = synth.TINY
    say("tiny fp32 layer, fused =", use_fused)
    shp = wl.layer
    pair = LayerPair(ctx, shp, seed=wl.seed)
    x_all = synth.activations(wl.seed, wl.steps, shp.d_model, shp.act)
    masks = synth.bernoulli_masks(wl.seed, wl.steps, shp.n_experts)
    wr = synth.router_weight(wl.seed, 0, shp.n_experts, shp.d_model)
    worst = _run_layer_steps(ctx, wl, pair, range(wl.steps), masks, None, None, x_all, use_fused, wr=wr)
    say("  worst max-abs-rel", worst)


def test_medium_bf16_layer_ragged(ctx):
    # several row tiles, a ragged chunk count (d_ff = 352 -> 11 chunks, 3 groups of 128 with a
    # 96-wide tail), shared expert wider than routed ones with a sigmoid gate, residual, threshold
    say("medium bf16 ragged layer")
    shp = synth.LayerShape(512, 12, 352, 3, 128, n_shared=1, shared_d_ff=2144, shared_gate=True, act="bf16")
    wl = synth.Workload("medium", shp, steps=6, seed=11)
    pair = LayerPair(ctx, shp, seed=wl.seed)
    x_all = synth.activations(wl.seed, wl.steps, shp.d_model, shp.act)
    masks = synth.bernoulli_masks(wl.seed, wl.steps, shp.n_experts)
    masks[2, :] = 0          # everything missing: all LOW
    masks[3, :] = 3          # everything resident: all HIGH
    wr = synth.router_weight(wl.seed, 0, shp.n_experts, shp.d_model, std=0.05)
    wsg = synth.shared_gate_weight(wl.seed, 0, shp.d_model, shp.act)
    for fused in (False, True):
        worst = _run_layer_steps(ctx, wl, pair, range(wl.steps), masks, None, None, x_all, fused, wr=wr, wsg=wsg,
                                 add_residual=True, tau=0.0 if fused else 0.34)
        say("  fused", fused, "worst max-abs-rel", worst)


@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_group32_layer(ctx, dt):
    # the paper's expert format: groups of 32 (Section 6.1 item 1 and Table 1 note 1, "G32 asymmetric"): one scale and one
    # zero-point per 32-chunk of every row; d_ff = 416 leaves a ragged chunk count (13)
    say("group-32 layer", dt)
    shp = synth.LayerShape(512, 10, 416, 3, 32, n_shared=1, shared_d_ff=224, act=dt)
    wl = synth.Workload("g32", shp, steps=5, seed=17)
    pair = LayerPair(ctx, shp, seed=wl.seed)
    x_all = synth.activations(wl.seed, wl.steps, shp.d_model, shp.act)
    masks = synth.bernoulli_masks(wl.seed, wl.steps, shp.n_experts)
    masks[1, :] = 3
    logits = synth.normal_logits(wl.seed, wl.steps, shp.n_experts)
    for fused in (False, True):
        worst = _run_layer_steps(ctx, wl, pair, range(wl.steps), masks, None, logits, x_all, fused, add_residual=fused)
        say("  fused", fused, "worst max-abs-rel", worst)


# (down work-groups of 8 output rows at 2 tokens, 16 at 5, 32 at 8, 64 at 12 and 16)
@pytest.mark.parametrize("T,dt", [(2, "f32"), (5, "bf16"), (8, "bf16"), (12, "f32"), (16, "bf16")])
def test_multi_token_layer(ctx, T, dt):
    # T tokens through one layer in one pair of launches: every token must come out exactly as from
    # its own smoe_decode_layer call (bit for bit: same kernels, same order of operations) and
    # within tolerance of the oracle; routing outputs row by row
    say("multi-token layer", T, dt)
    shp = synth.LayerShape(512, 12, 352, 3, 128, n_shared=1, shared_d_ff=608, shared_gate=True, act=dt)
    pair = LayerPair(ctx, shp, seed=19)
    k, E, d = shp.top_k, shp.n_experts, shp.d_model
    x = synth.activations(19, T, d, dt).cuda()
    z = synth.normal_logits(19, T, E)
    mask_np = synth.bernoulli_masks(19, 1, E)[0]
    bias_np = np.where(mask_np & 1, np.float32(0.5), np.float32(0)).astype(np.float32)
    wsg = synth.shared_gate_weight(19, 0, d, dt)
    idx = torch.empty((T, k), dtype=torch.int32, device="cuda:0")
    w = torch.empty((T, k), dtype=torch.float32, device="cuda:0")
    prec = torch.empty((T, k), dtype=torch.uint8, device="cuda:0")
    y = B.smoe_decode_layer_multi(ctx, pair.routed, pair.shared, x, k, z.cuda(), bias=dev(bias_np), slice_mask=dev(mask_np),
                                  tau_head=0.3, shared_gate_w=dev(wsg), add_residual=True, idx_out=idx, w_out=w,
                                  prec_out=prec)
    idx_np, w_np, prec_np = idx.cpu().numpy(), w.cpu().numpy(), prec.cpu().numpy()
    for t in range(T):
        y1 = B.smoe_decode_layer(ctx, pair.routed, pair.shared, x[t].clone(), k, logits=z[t].cuda(), bias=dev(bias_np),
                                 slice_mask=dev(mask_np), tau_head=0.3, shared_gate_w=dev(wsg), add_residual=True)
        assert torch.equal(y1, y[t]), t
        ridx, rw = O.route(z[t].numpy()[None], bias_np, k)
        assert np.array_equal(idx_np[t], ridx[0]), t
        np.testing.assert_allclose(w_np[t], rw[0], rtol=2e-5, atol=1e-7)
        w_used = w_np[t].astype(np.float64)
        rprec = O.precision_select(ridx[0], w_used, mask_np, 0.3)
        assert np.array_equal(prec_np[t], rprec), t
        yref = O.moe_layer(t2np(x[t]).astype(np.float64), pair.oracle_routed(), ridx[0], w_used, rprec,
                           pair.oracle_shared(), t2np(wsg), True)
        assert O.max_abs_rel(t2np(y[t]), yref) <= TOL[dt], t
    # argument checks: too many tokens, missing logits
    lib = B.lib()
    import ctypes as C
    assert lib.smoe_decode_layer_multi(ctx.h, pair.routed.h, None, 17, C.c_void_p(x.data_ptr()), B._DT[x.dtype], k,
                                       C.c_void_p(z.cuda().data_ptr()), None, 0, C.c_float(1.0), None, C.c_float(0.0), None, 0,
                                       C.c_void_p(y.data_ptr()), None, None, None) == -2
    assert lib.smoe_decode_layer_multi(ctx.h, pair.routed.h, None, 2, C.c_void_p(x.data_ptr()), B._DT[x.dtype], k,
                                       None, None, 0, C.c_float(1.0), None, C.c_float(0.0), None, 0,
                                       C.c_void_p(y.data_ptr()), None, None, None) == -1


@pytest.mark.parametrize("nest", [(4, 2), (6, 3)])
@pytest.mark.parametrize("dt,G", [("bf16", 128), ("bf16", 32), ("f32", 64)])
def test_lower_nest_layer(ctx, dt, G, nest):
    # the 4/2 nest (4-bit codes, 2-bit planes): LOW = upper two bits with the zero-point shifted by
    # two, HIGH = both planes; the 6/3 nest likewise with three bits; ragged chunk counts, a shared
    # expert, masks of every kind
    bh, bl = nest
    say("lower nest layer", nest, dt, G)
    shp = synth.LayerShape(512, 10, 416, 3, G, n_shared=1, shared_d_ff=224, act=dt, b_high=bh, b_low=bl)
    wl = synth.Workload("mat42", shp, steps=5, seed=37)
    pair = LayerPair(ctx, shp, seed=wl.seed)
    x_all = synth.activations(wl.seed, wl.steps, shp.d_model, shp.act)
    masks = synth.bernoulli_masks(wl.seed, wl.steps, shp.n_experts)
    masks[1, :] = 3
    masks[2, :] = 1
    logits = synth.normal_logits(wl.seed, wl.steps, shp.n_experts)
    for fused in (False, True):
        worst = _run_layer_steps(ctx, wl, pair, range(wl.steps), masks, None, logits, x_all, fused, add_residual=fused)
        say("  fused", fused, "worst max-abs-rel", worst)
    # HIGH and LOW differ, and a full-size layer shape runs too (one step, against the oracle)
    shp2 = synth.LayerShape(2048, 8, 1408, 2, 128, n_shared=1, shared_d_ff=1408, act=dt, b_high=bh, b_low=bl)
    if dt == "bf16" and G == 128:
        wl2 = synth.Workload("mat42-full", shp2, steps=1, seed=38)
        pair2 = LayerPair(ctx, shp2, seed=wl2.seed)
        x2 = synth.activations(wl2.seed, 1, 2048, dt)
        m2 = synth.bernoulli_masks(wl2.seed, 1, 8)
        z2 = synth.normal_logits(wl2.seed, 1, 8)
        _run_layer_steps(ctx, wl2, pair2, range(1), m2, None, z2, x2, True)


@pytest.mark.parametrize("d,dt,G,nest", [(4096, "bf16", 128, (8, 4)), (2560, "bf16", 32, (8, 4)), (2112, "f32", 64, (8, 4)),
                                         (8192, "bf16", 128, (8, 4)), (4096, "bf16", 128, (6, 3)), (2560, "f32", 128, (4, 2))])
def test_wide_rows_layer(ctx, d, dt, G, nest):
    # d_model above 2048: a row of the gate/up matrices spans several 64-chunk k-slices (2112 and 2560:
    # a ragged last slice; 8192: four full ones); shared expert with its sigmoid gate, router mat-vec,
    # residual, masks of every kind
    bh, bl = nest
    say("wide rows", d, dt, G, nest)
    shp = synth.LayerShape(d, 6, 96, 2, G, n_shared=1, shared_d_ff=160, shared_gate=True, act=dt, b_high=bh, b_low=bl)
    wl = synth.Workload("wide", shp, steps=3, seed=41)
    pair = LayerPair(ctx, shp, seed=wl.seed)
    x_all = synth.activations(wl.seed, wl.steps, d, dt)
    masks = synth.bernoulli_masks(wl.seed, wl.steps, shp.n_experts)
    masks[1, :] = 3
    masks[2, :] = 1
    logits = synth.normal_logits(wl.seed, wl.steps, shp.n_experts)
    wsg = synth.shared_gate_weight(wl.seed, 0, d, dt)
    wr = synth.router_weight(wl.seed, 0, shp.n_experts, d)
    for fused in (False, True):
        worst = _run_layer_steps(ctx, wl, pair, range(wl.steps), masks, None, logits, x_all, fused, wsg=wsg, add_residual=fused)
        say("  fused", fused, "worst max-abs-rel", worst)
    worst = _run_layer_steps(ctx, wl, pair, range(1), masks, None, None, x_all, True, wr=wr, wsg=wsg, tau=0.4)
    say("  router mat-vec, tau 0.4: worst", worst)
    # several tokens per step agree with the one-token entry point
    T, k = 3, shp.top_k
    x = dev(x_all[:T])
    z = dev(logits[:T])
    y = B.smoe_decode_layer_multi(ctx, pair.routed, pair.shared, x, k, z, slice_mask=dev(masks[0]), shared_gate_w=dev(wsg))
    for t in range(T):
        y1 = B.smoe_decode_layer(ctx, pair.routed, pair.shared, x[t].clone(), k, logits=z[t].clone(), slice_mask=dev(masks[0]),
                                 shared_gate_w=dev(wsg))
        assert torch.equal(y[t], y1), t


def test_dense_ffn_through_shared_bank(ctx):
    # no routed bank at all: a dense SwiGLU run HIGH; K of the down projection is not a multiple
    # of the group (416 = 3*128 + 32)
    say("dense FFN via shared bank")
    shp = synth.LayerShape(256, 0, 0, 0, 128, n_shared=1, shared_d_ff=416, act="bf16")
    pair = LayerPair(ctx, shp, seed=5, routed=False)
    x = synth.activations(5, 2, 256, "bf16")
    for t in range(2):
        y = B.smoe_expert_ffn(ctx, None, pair.shared, dev(x[t]), None, None, None)
        yref = O.moe_layer(t2np(x[t]).astype(np.float64), [], [], [], [], pair.oracle_shared())
        assert O.max_abs_rel(t2np(y), yref) <= TOL["bf16"]


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_symmetric_store_layer(ctx, dt):
    # a layer whose banks were filled by the symmetric quantiser: the dense FFN through the shared bank
    # (how the symmetric INT8 non-expert weights of the paper's set-up run) and a routed mix of HIGH / LOW
    say("symmetric store", dt)
    shp = synth.LayerShape(256, 4, 128, 2, 128, n_shared=1, shared_d_ff=416, act=dt, symmetric=True)
    pair = LayerPair(ctx, shp, seed=6)
    x = synth.activations(6, 2, 256, dt)
    for t in range(2):
        y = B.smoe_expert_ffn(ctx, None, pair.shared, dev(x[t]), None, None, None)
        yref = O.moe_layer(t2np(x[t]).astype(np.float64), [], [], [], [], pair.oracle_shared())
        assert O.max_abs_rel(t2np(y), yref) <= TOL[dt]
    idx = np.array([2, 0], np.int32)
    w = np.array([0.7, 0.3], np.float32)
    mask = np.array([3, 1, 1, 3], np.uint8)
    prec = torch.zeros(2, dtype=torch.uint8, device="cuda:0")
    y = B.smoe_expert_ffn(ctx, pair.routed, pair.shared, dev(x[0]), dev(idx), dev(w), dev(mask), prec_out=prec)
    assert t2np(prec).tolist() == [0, 1]
    yref = O.moe_layer(t2np(x[0]).astype(np.float64), pair.oracle_routed(), idx, w, [0, 1], pair.oracle_shared())
    assert O.max_abs_rel(t2np(y), yref) <= TOL[dt]


def test_determinism_and_high_low_differ(ctx):
    say("determinism")
    shp = synth.LayerShape(256, 4, 128, 2, 64, act="f32")
    pair = LayerPair(ctx, shp, seed=2)
    x = dev(synth.activations(2, 1, 256, "f32")[0])
    idx = dev(np.array([1, 3], np.int32))
    w = dev(np.array([0.6, 0.4], np.float32))
    hi = dev(np.full(4, 3, np.uint8))
    lo = dev(np.full(4, 1, np.uint8))
    y1 = B.smoe_expert_ffn(ctx, pair.routed, None, x, idx, w, hi).clone()
    y2 = B.smoe_expert_ffn(ctx, pair.routed, None, x, idx, w, hi).clone()
    y3 = B.smoe_expert_ffn(ctx, pair.routed, None, x, idx, w, lo).clone()
    assert torch.equal(y1, y2)
    assert O.max_abs_rel(t2np(y3), t2np(y1)) > 1e-3


def test_argument_errors_on_device(ctx):
    say("argument errors")
    import ctypes as C
    lib = B.lib()
    shp = synth.LayerShape(256, 4, 128, 2, 64, act="f32")
    pair = LayerPair(ctx, shp, seed=2)
    x = dev(synth.activations(2, 1, 256, "f32")[0])
    y = torch.empty_like(x)
    idx = dev(np.array([1, 3], np.int32))
    w = dev(np.array([0.6, 0.4], np.float32))
    p = lambda t: C.c_void_p(t.data_ptr())
    call = lambda k, xx, yy, ii: lib.smoe_expert_ffn(ctx.h, pair.routed.h, None, xx, 0, k, ii, p(w), None,
                                                     C.c_float(0), None, 0, yy, None)
    assert call(2, p(x), p(x), p(idx)) == -1                      # y aliases x
    assert call(5, p(x), p(y), p(idx)) == -2                      # k > E
    assert call(2, C.c_void_p(x.data_ptr() + 4), p(y), p(idx)) == -3
    assert call(2, p(x), p(y), None) == -1
    assert lib.smoe_route(ctx.h, 1, 300, 2, 0, p(x), None, 0, None, None, 0, C.c_float(1), None, p(idx), p(w)) == -2
    assert lib.smoe_quantize_slice(ctx.h, pair.routed.h, 3, 2, p(x), p(x), p(x)) == -2
    # a row of more than four 64-chunk k-slices: valid, not implemented by the decode kernels (no launch)
    big = B.Bank(ctx, 2, 8192 + 32, 32, 32, "f32", "f32")
    xb = torch.zeros(8192 + 32, dtype=torch.float32, device="cuda:0")
    yb = torch.empty_like(xb)
    assert lib.smoe_expert_ffn(ctx.h, big.h, None, p(xb), 0, 2, p(idx), p(w), None, C.c_float(0), None, 0, p(yb), None) == -6


# ------------------------------------------------------------------------------ full-size layer
def test_dsv2lite_layer_full_size_sampled_steps(ctx):
    """The benchmark workload (64 experts of 2048x1408, top-6, 2 shared, bf16) in the launch
    configuration the bench times; the oracle recomputes sampled steps and sampled experts."""
    wl = synth.DSV2_LAYER
    shp = wl.layer
    say("dsv2-lite layer: quantising 66 experts on the GPU")
    pair = LayerPair(ctx, shp, seed=wl.seed, gen_device="cuda:0", keep_dense=False)
    x_all = synth.activations(wl.seed, wl.steps, shp.d_model, shp.act)
    logits = synth.normal_logits(wl.seed, wl.steps, shp.n_experts)
    mask, bias = synth.cached_set_mask(wl.seed, shp.n_experts, 32, 16, 1.0)
    bias_t = torch.from_numpy(bias)
    # routing decisions for every step: bit-exact
    idx, w = B.smoe_route(ctx, shp.top_k, logits=dev(logits), bias=dev(bias_t))
    ridx, rw = O.route(logits.numpy(), bias, shp.top_k)
    assert np.array_equal(idx.cpu().numpy(), ridx)
    np.testing.assert_allclose(w.cpu().numpy(), rw, rtol=2e-5, atol=1e-7)
    say("  routing of 1024 steps matches; checking 33 steps spread over the run")
    steps = list(range(0, 1024, 32)) + [1023]
    worst = _run_layer_steps(ctx, wl, pair, steps, mask, bias_t, logits, x_all, True)
    say("  fused worst", worst)
    # codes of one sampled routed expert and one shared expert: bit-exact at full size
    for bank, slot, tag in ((pair.routed, int(ridx[0, 0]), int(ridx[0, 0])), (pair.shared, 1, 1001)):
        ex = pair.oracle_expert(tag)
        for mi, qm in enumerate((ex.gate, ex.up, ex.down)):
            got = B.smoe_export_codes(ctx, bank, slot, mi)
            assert np.array_equal(got["q"], qm.q) and np.array_equal(got["zp"], qm.zp)
            assert np.array_equal(got["scale"].view(np.uint32), qm.scale.view(np.uint32))


def test_random_small_shapes(ctx):
    # a seeded sweep over layer shapes: ragged d_ff (any multiple of 32), every group size, both
    # activation dtypes, with and without shared experts, a sigmoid gate, a residual and a threshold;
    # one step per shape through the fused call and through route + expert_ffn
    rng = np.random.default_rng(2024)
    for case in range(14):
        d = int(rng.choice([64, 96, 256, 544, 1024, 2048]))
        G = int(rng.choice([32, 64, 128]))
        f = int(rng.integers(1, 12)) * 32
        E = int(rng.integers(2, 20))
        k = int(rng.integers(1, min(E, 6) + 1))
        n_sh = int(rng.integers(0, 3))
        f_s = int(rng.integers(1, 9)) * 32 if n_sh else 0
        dt = "bf16" if rng.random() < 0.6 else "f32"
        gate = bool(n_sh and rng.random() < 0.5)
        say("random shape", case, dict(d=d, G=G, f=f, E=E, k=k, n_sh=n_sh, f_s=f_s, dt=dt, gate=gate))
        shp = synth.LayerShape(d, E, f, k, G, n_shared=n_sh, shared_d_ff=f_s, shared_gate=gate, act=dt)
        wl = synth.Workload("rand%d" % case, shp, steps=2, seed=100 + case)
        pair = LayerPair(ctx, shp, seed=wl.seed)
        x_all = synth.activations(wl.seed, wl.steps, d, dt)
        masks = synth.bernoulli_masks(wl.seed, wl.steps, E)
        logits = synth.normal_logits(wl.seed, wl.steps, E)
        wsg = synth.shared_gate_weight(wl.seed, 0, d, dt, std=0.05) if gate else None
        tau = float(rng.choice([0.0, 0.25]))
        for fused in (False, True):
            _run_layer_steps(ctx, wl, pair, range(wl.steps), masks, None, logits, x_all, fused, wsg=wsg,
                             add_residual=bool(case & 1), tau=tau)


def test_random_wide_shapes(ctx):
    # the same kind of sweep over rows of more than 64 chunks (two to four k-slices, the last one ragged
    # or full), both nests' plane widths included
    rng = np.random.default_rng(2025)
    for case in range(8):
        d = int(rng.choice([2080, 3072, 4128, 5120, 6176, 8192]))
        G = int(rng.choice([32, 64, 128]))
        f = int(rng.integers(1, 5)) * 32
        E = int(rng.integers(2, 9))
        k = int(rng.integers(1, min(E, 4) + 1))
        n_sh = int(rng.integers(0, 3))
        f_s = int(rng.integers(1, 4)) * 32 if n_sh else 0
        dt = "bf16" if rng.random() < 0.6 else "f32"
        gate = bool(n_sh and rng.random() < 0.5)
        bh, bl = [(8, 4), (6, 3), (4, 2)][int(rng.integers(0, 3))]
        say("random wide shape", case, dict(d=d, G=G, f=f, E=E, k=k, n_sh=n_sh, f_s=f_s, dt=dt, gate=gate, nest=(bh, bl)))
        shp = synth.LayerShape(d, E, f, k, G, n_shared=n_sh, shared_d_ff=f_s, shared_gate=gate, act=dt, b_high=bh, b_low=bl)
        wl = synth.Workload("randw%d" % case, shp, steps=2, seed=300 + case)
        pair = LayerPair(ctx, shp, seed=wl.seed)
        x_all = synth.activations(wl.seed, wl.steps, d, dt)
        masks = synth.bernoulli_masks(wl.seed, wl.steps, E)
        logits = synth.normal_logits(wl.seed, wl.steps, E)
        wsg = synth.shared_gate_weight(wl.seed, 0, d, dt, std=0.05) if gate else None
        tau = float(rng.choice([0.0, 0.25]))
        for fused in (False, True):
            _run_layer_steps(ctx, wl, pair, range(wl.steps), masks, None, logits, x_all, fused, wsg=wsg,
                             add_residual=bool(case & 1), tau=tau)


def test_decode_steps_replay_from_a_hip_graph():
    # a serving loop can record its decode calls once and replay them: every call only enqueues two
    # kernels on the context's stream.  Four steps are captured on a side stream, replayed three times
    # with eager calls and synchronisations between the replays, and every replay must reproduce the
    # eager outputs bit for bit.
    say("graph capture of decode steps")
    side = torch.cuda.Stream()
    gctx = B.Ctx(0, stream=side)
    shp = synth.LayerShape(512, 12, 352, 3, 128, n_shared=1, shared_d_ff=608, act="bf16")
    pair = LayerPair(gctx, shp, seed=29)
    k, E, d, n = shp.top_k, shp.n_experts, shp.d_model, 4
    x = synth.activations(29, n, d, "bf16").cuda()
    z = synth.normal_logits(29, n, E).cuda()
    mask = dev(synth.bernoulli_masks(29, 1, E)[0])
    side.wait_stream(torch.cuda.current_stream())

    def steps(y, idx):
        for i in range(n):
            B.smoe_decode_layer(gctx, pair.routed, pair.shared, x[i], k, logits=z[i], slice_mask=mask, add_residual=True,
                                y=y[i], idx_out=idx[i])

    y_e = torch.zeros((n, d), dtype=torch.bfloat16, device="cuda:0")
    idx_e = torch.zeros((n, 4), dtype=torch.int32, device="cuda:0")      # 16-byte rows
    y_g, idx_g = torch.zeros_like(y_e), torch.zeros_like(idx_e)
    with torch.cuda.stream(side):
        steps(y_e, idx_e)                       # eager reference (also the warm-up before the capture)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        steps(y_g, idx_g)
    for rep in range(3):
        y_g.fill_(0)
        idx_g.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y_g, y_e) and torch.equal(idx_g[:, :k], idx_e[:, :k]), rep
        with torch.cuda.stream(side):           # eager work between the replays
            steps(y_e, idx_e)
        side.synchronize()
    gctx.close()
