"""GPU parity of decode paths that the layer tests in test_gpu_decode.py do not reach: routed banks of
more than 64 experts in the fused prologue (four experts per lane), top-k up to 16, tied and -0.0
logits through the fused selection, normalised / scaled gate weights through the fused calls, many
tokens per step with wide d_ff (the entry -> slot division of the gate/up split), activations with
outliers and degenerate chunks, and the documented clamp of out-of-range expert indices."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import slicemoe_oracle as O
from paper_2512_12990_amd import binding as B
from paper_2512_12990_amd import synth
from helpers import LayerPair, t2np
from test_gpu_decode import TOL, _run_layer_steps, ctx, dev, say      # noqa: F401  (ctx is a fixture)

pytestmark = pytest.mark.gpu


def _tricky_logits(seed, steps, E):
    """N(0,1) logits with exact ties across lanes and across the 64-expert register groups, rows of
    -0.0 / +0.0, and a row that is constant (every pick is a tie)."""
    z = synth.normal_logits(seed, steps, E)
    z[0, :] = -0.0
    z[0, ::3] = 0.0                       # +0.0 and -0.0 compare equal: ties go to the lower index
    z[1, :] = 0.25
    if steps > 2:
        top = float(z[2].max()) + 1.0
        for e in (E - 1, E // 2, 3, 64 % E, (64 + 3) % E, (128 + 3) % E):
            z[2, e] = top                 # tied maxima in different lanes and register groups
    if steps > 3:
        z[3, 1::2] = z[3, 0::2][: z[3, 1::2].numel()]      # every score appears twice
    return z


@pytest.mark.parametrize("E,k,dt", [(96, 8, "bf16"), (160, 16, "f32"), (256, 5, "bf16"), (256, 16, "bf16"), (65, 3, "f32")])
def test_large_banks_fused_and_split(ctx, E, k, dt):
    # more than 64 experts: four experts per lane in the fused top-k, selection and weights; the
    # given-decision path (route + expert_ffn) picks the mask of experts 64.. by lane exchange
    say("large bank", E, k, dt)
    shp = synth.LayerShape(256, E, 64, k, 64, n_shared=1, shared_d_ff=96, act=dt)
    wl = synth.Workload("bank%d" % E, shp, steps=5, seed=50 + E)
    pair = LayerPair(ctx, shp, seed=wl.seed)
    x_all = synth.activations(wl.seed, wl.steps, shp.d_model, dt)
    masks = synth.bernoulli_masks(wl.seed, wl.steps, E)
    masks[1, ::2] = 0
    logits = _tricky_logits(wl.seed, wl.steps, E)
    bias = torch.zeros(E)
    bias[torch.randperm(E, generator=torch.Generator().manual_seed(E))[: E // 2]] = 1.0
    for fused in (False, True):
        for b, norm, rs, tau in [(None, False, 1.0, 0.0), (bias, False, 1.0, 0.0), (bias, True, 2.5, 0.0), (bias, True, 1.0, 0.2)]:
            worst = _run_layer_steps(ctx, wl, pair, range(wl.steps), masks, b, logits, x_all, fused, add_residual=fused,
                                     tau=tau, norm_topk=norm, routed_scale=rs)
            say("  fused", fused, "bias", b is not None, "norm", norm, "scale", rs, "tau", tau, "worst", worst)


@pytest.mark.parametrize("E,k", [(64, 6), (60, 4), (8, 8), (33, 16)])
def test_fused_topk_ties_signed_zero_norm_scale(ctx, E, k):
    # one expert per lane: ties, signed zeros, a bias, normalised and scaled weights through
    # smoe_decode_layer and smoe_decode_layer_multi
    say("fused top-k ties", E, k)
    dt = "bf16"
    shp = synth.LayerShape(256, E, 96, k, 32, n_shared=0, act=dt)
    wl = synth.Workload("ties%d" % E, shp, steps=4, seed=70 + E)
    pair = LayerPair(ctx, shp, seed=wl.seed)
    x_all = synth.activations(wl.seed, wl.steps, shp.d_model, dt)
    masks = synth.bernoulli_masks(wl.seed, wl.steps, E)
    logits = _tricky_logits(wl.seed, wl.steps, E)
    bias = torch.zeros(E)
    bias[::2] = 0.5
    for b, norm, rs in [(None, True, 1.0), (bias, False, 0.5), (bias, True, 16.0)]:
        worst = _run_layer_steps(ctx, wl, pair, range(wl.steps), masks, b, logits, x_all, True, norm_topk=norm, routed_scale=rs)
        say("  one-token: bias", b is not None, "norm", norm, "scale", rs, "worst", worst)
    # the same through the multi-token entry point (one mask for all tokens)
    T = wl.steps
    idx = torch.empty((T, k), dtype=torch.int32, device="cuda:0")
    w = torch.empty((T, k), dtype=torch.float32, device="cuda:0")
    prec = torch.empty((T, k), dtype=torch.uint8, device="cuda:0")
    y = B.smoe_decode_layer_multi(ctx, pair.routed, None, dev(x_all), k, dev(logits), bias=dev(bias), norm_topk=True,
                                  routed_scale=2.5, slice_mask=dev(masks[0]), idx_out=idx, w_out=w, prec_out=prec)
    ridx, rw = O.route(logits.numpy(), bias.numpy(), k, True, 2.5)
    assert np.array_equal(idx.cpu().numpy(), ridx)
    np.testing.assert_allclose(w.cpu().numpy(), rw, rtol=2e-5, atol=1e-7)
    for t in range(T):
        w_used = rw[t].astype(np.float32).astype(np.float64)
        rprec = O.precision_select(ridx[t], w_used, masks[0])
        assert np.array_equal(prec.cpu().numpy()[t], rprec)
        yref = O.moe_layer(t2np(x_all[t]).astype(np.float64), pair.oracle_routed(), ridx[t], w_used, rprec, [])
        assert O.max_abs_rel(t2np(y[t]), yref) <= TOL[dt], t


@pytest.mark.parametrize("T,f,k,f_s,dt", [(9, 3584, 8, 0, "bf16"), (12, 448, 3, 8224, "bf16"), (16, 2720, 10, 96, "f32"),
                                          (10, 3584, 8, 8224, "bf16")])
def test_many_tokens_wide_d_ff(ctx, T, f, k, f_s, dt):
    # nine or more tokens per step leave 32 gate/up work-groups per token, so a work-group owns
    # ceil(d_ff / 32) row pairs of every slot (112 for d_ff 3584, 257 for the 8224-wide shared expert, 85
    # for 2720): the entry -> (slot, row pair) division has to be exact for these counts too
    say("many tokens, wide d_ff", T, f, k, f_s, dt)
    d, E = 128, 12
    shp = synth.LayerShape(d, E, f, k, 32, n_shared=1 if f_s else 0, shared_d_ff=f_s, act=dt)
    pair = LayerPair(ctx, shp, seed=90 + T)
    x = synth.activations(90 + T, T, d, dt)
    z = synth.normal_logits(90 + T, T, E)
    mask_np = synth.bernoulli_masks(90 + T, 1, E)[0]
    need = B.smoe_workspace_bytes(T, k, f, shp.n_shared, f_s)
    big = B.Ctx(0, workspace_bytes=max(need, 4 << 20))
    idx = torch.empty((T, k), dtype=torch.int32, device="cuda:0")
    w = torch.empty((T, k), dtype=torch.float32, device="cuda:0")
    prec = torch.empty((T, k), dtype=torch.uint8, device="cuda:0")
    y = B.smoe_decode_layer_multi(big, pair.routed, pair.shared, dev(x), k, dev(z), slice_mask=dev(mask_np), idx_out=idx,
                                  w_out=w, prec_out=prec)
    torch.cuda.synchronize()
    ridx, rw = O.route(z.numpy(), None, k)
    assert np.array_equal(idx.cpu().numpy(), ridx)
    w_np = w.cpu().numpy()
    for t in range(T):
        y1 = B.smoe_decode_layer(big, pair.routed, pair.shared, dev(x[t]), k, logits=dev(z[t]), slice_mask=dev(mask_np))
        assert torch.equal(y1, y[t]), t
        w_used = w_np[t].astype(np.float64)
        rprec = O.precision_select(ridx[t], w_used, mask_np)
        assert np.array_equal(prec.cpu().numpy()[t], rprec), t
        if t in (0, T // 2, T - 1):
            yref = O.moe_layer(t2np(x[t]).astype(np.float64), pair.oracle_routed(), ridx[t], w_used, rprec, pair.oracle_shared())
            assert O.max_abs_rel(t2np(y[t]), yref) <= TOL[dt], t
    # a workspace that is too small for the step is refused, not overrun
    small = B.Ctx(0, workspace_bytes=need - 256)
    with pytest.raises(B.SmoeError):
        B.smoe_decode_layer_multi(small, pair.routed, pair.shared, dev(x), k, dev(z), slice_mask=dev(mask_np))
    torch.cuda.synchronize()
    small.close()
    big.close()


@pytest.mark.parametrize("dt", ["bf16", "f32"])
@pytest.mark.parametrize("d,f", [(2048, 352), (512, 1408)])
def test_heavy_tailed_activations(ctx, dt, d, f):
    # hidden states are not N(0,1): outlier channels, all-zero chunks, chunks that span many binades.
    # The bf16 path re-expresses each 32-chunk of x (and of h) as block integers; the stated tolerance
    # must hold on such inputs too, with the oracle computing on the exact inputs in fp64
    say("heavy-tailed activations", dt, d, f)
    E, k = 8, 3
    shp = synth.LayerShape(d, E, f, k, 128, n_shared=1, shared_d_ff=f, shared_gate=True, act=dt)
    wl = synth.Workload("heavy", shp, steps=6, seed=120)
    pair = LayerPair(ctx, shp, seed=wl.seed)
    x_all = synth.heavy_tailed_activations(wl.seed, wl.steps, d, dt)
    masks = synth.bernoulli_masks(wl.seed, wl.steps, E)
    logits = synth.normal_logits(wl.seed, wl.steps, E)
    wsg = synth.shared_gate_weight(wl.seed, 0, d, dt, std=0.002)
    for fused in (False, True):
        worst = _run_layer_steps(ctx, wl, pair, range(wl.steps), masks, None, logits, x_all, fused, wsg=wsg, add_residual=False)
        say("  fused", fused, "worst max-abs-rel", worst)
    # an all-zero token: exact zeros out (every chunk scale is zero), not NaN
    y = B.smoe_decode_layer(ctx, pair.routed, pair.shared, torch.zeros(d, dtype=x_all.dtype, device="cuda:0"), k,
                            logits=dev(logits[0]), slice_mask=dev(masks[0]))
    assert float(y.float().abs().max()) == 0.0


def test_out_of_range_expert_index_is_clamped(ctx):
    # smoe_expert_ffn takes the decision from device memory, so the host cannot validate it; the
    # header documents that an index outside [0, E) is clamped into the bank.  Checked here: the result
    # equals the call with the clamped indices, bit for bit, and nothing outside the bank is read
    say("index clamp")
    shp = synth.LayerShape(256, 6, 96, 3, 32, act="bf16")
    pair = LayerPair(ctx, shp, seed=7)
    x = dev(synth.activations(7, 1, 256, "bf16")[0])
    w = dev(np.array([0.5, 0.3, 0.2], np.float32))
    mask = dev(np.array([3, 1, 3, 1, 3, 1], np.uint8))
    p1 = torch.empty(3, dtype=torch.uint8, device="cuda:0")
    p2 = torch.empty(3, dtype=torch.uint8, device="cuda:0")
    y_bad = B.smoe_expert_ffn(ctx, pair.routed, None, x, dev(np.array([-7, 2, 1 << 20], np.int32)), w, mask, prec_out=p1)
    y_ok = B.smoe_expert_ffn(ctx, pair.routed, None, x, dev(np.array([0, 2, 5], np.int32)), w, mask, prec_out=p2)
    assert torch.equal(y_bad, y_ok) and torch.equal(p1, p2)
    yref = O.moe_layer(t2np(x).astype(np.float64), pair.oracle_routed(), [0, 2, 5], [0.5, 0.3, 0.2], [1, 1, 0], [])
    assert O.max_abs_rel(t2np(y_ok), yref) <= TOL["bf16"]


def test_stream_read_measurement_aid(ctx):
    # the streaming-read kernel bench.py uses as a practical roof: runs, and rejects bad arguments
    say("stream read aid")
    lib = B.lib()
    buf = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda:0")
    sink = torch.zeros(64, dtype=torch.uint8, device="cuda:0")
    p = lambda t: C.c_void_p(t.data_ptr())
    assert lib.smoe_stream_read(ctx.h, p(buf), C.c_size_t(1 << 20), 16, p(sink)) == 0
    assert lib.smoe_stream_read(ctx.h, p(buf), C.c_size_t(1000), 3, p(sink)) == 0      # ragged size: whole 16-byte units only
    torch.cuda.synchronize()
    assert int(sink.sum()) == 0
    assert lib.smoe_stream_read(ctx.h, None, C.c_size_t(1 << 20), 16, p(sink)) == -1
    assert lib.smoe_stream_read(ctx.h, C.c_void_p(buf.data_ptr() + 4), C.c_size_t(1 << 10), 16, p(sink)) == -3
    assert lib.smoe_stream_read(ctx.h, p(buf), C.c_size_t(1 << 20), 0, p(sink)) == -2
