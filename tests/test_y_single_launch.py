"""GPU parity of the single-launch decode mode: one kernel launch per token instead of two must give
bit-identical outputs (and the same oracle agreement) wherever it is taken, and must fall back to the
two launches where the case does not fit."""
import numpy as np
import pytest
import torch

from oracle import slicemoe_oracle as O
from paper_2512_12990_amd import binding as B
from paper_2512_12990_amd import synth
from helpers import LayerPair, t2np
from test_gpu_decode import TOL, _run_layer_steps, ctx, dev, say      # noqa: F401  (ctx is a fixture)

pytestmark = pytest.mark.gpu


def _both(ctx2, ctx1, pair, shp, x, z, mask, **kw):
    k = shp.top_k
    outs = []
    for c in (ctx2, ctx1):
        idx = torch.full((4,) if k <= 4 else (k,), -1, dtype=torch.int32, device="cuda:0")
        w = torch.zeros(k, dtype=torch.float32, device="cuda:0")
        p = torch.zeros(k, dtype=torch.uint8, device="cuda:0")
        y = B.smoe_decode_layer(c, pair.routed, pair.shared, x, k, logits=z, slice_mask=mask, idx_out=idx, w_out=w, prec_out=p, **kw)
        torch.cuda.synchronize()
        outs.append((y.clone(), idx.clone(), w.clone(), p.clone()))
    for a, b in zip(outs[0], outs[1]):
        assert torch.equal(a, b)
    return outs[0][0]


@pytest.mark.parametrize("shape", [
    synth.LayerShape(512, 12, 352, 3, 128, n_shared=1, shared_d_ff=608, act="bf16"),
    synth.LayerShape(256, 8, 512, 2, 64, n_shared=0, act="f32"),
    synth.LayerShape(1024, 16, 704, 4, 32, n_shared=2, shared_d_ff=704, act="bf16"),
    synth.LayerShape(2048, 8, 1408, 6, 128, n_shared=0, act="bf16"),
])
def test_single_launch_small_layers(ctx, shape):
    say("single launch", shape)
    one = B.Ctx(0)
    one.single_launch(True)
    pair = LayerPair(ctx, shape, seed=91)
    n = 6
    x = synth.activations(91, n, shape.d_model, shape.act).cuda()
    z = synth.normal_logits(91, n, shape.n_experts).cuda()
    masks = synth.bernoulli_masks(91, n, shape.n_experts)
    for rep in range(3):
        for i in range(n):
            _both(ctx, one, pair, shape, x[i], z[i], dev(masks[i]), add_residual=bool(i & 1), tau_head=0.1 * (i % 3))
    calls, timeouts = one.single_launch_status()
    say("  single-launch calls", calls, "timeouts", timeouts)
    assert calls == 3 * n and timeouts == 0
    # and against the oracle, through the same harness as the two-launch tests
    wl = synth.Workload("one", shape, steps=n, seed=91)
    worst = _run_layer_steps(one, wl, pair, range(n), masks, None, synth.normal_logits(91, n, shape.n_experts),
                             synth.activations(91, n, shape.d_model, shape.act), True)
    say("  oracle worst", worst)
    one.close()


def test_single_launch_headline_layer_graph_replays(ctx):
    """The benchmark layer: 64 steps eagerly in both modes (bit-identical), then the single-launch steps
    recorded in a graph and replayed with eager work in between."""
    wl = synth.DSV2_LAYER
    shp = wl.layer
    say("single launch, dsv2-lite layer")
    side = torch.cuda.Stream()
    one = B.Ctx(0, stream=side)
    one.single_launch(True)
    two = B.Ctx(0, stream=side)
    pair = LayerPair(ctx, shp, seed=wl.seed, gen_device="cuda:0", keep_dense=False)
    n, k, d = 64, shp.top_k, shp.d_model
    x = synth.activations(wl.seed, n, d, shp.act).cuda()
    z = synth.normal_logits(wl.seed, n, shp.n_experts).cuda()
    mask, bias = synth.cached_set_mask(wl.seed, shp.n_experts, 32, 16, 1.0)
    mask_d, bias_d = dev(mask), dev(torch.from_numpy(bias))
    side.wait_stream(torch.cuda.current_stream())

    def steps(c, y, idx):
        for i in range(n):
            B.smoe_decode_layer(c, pair.routed, pair.shared, x[i], k, logits=z[i], bias=bias_d, slice_mask=mask_d, add_residual=True,
                                y=y[i], idx_out=idx[i])

    y2 = torch.zeros((n, d), dtype=torch.bfloat16, device="cuda:0")
    i2 = torch.zeros((n, 8), dtype=torch.int32, device="cuda:0")
    y1, i1 = torch.zeros_like(y2), torch.zeros_like(i2)
    with torch.cuda.stream(side):
        steps(two, y2, i2)
        steps(one, y1, i1)
    side.synchronize()
    assert torch.equal(y1, y2) and torch.equal(i1, i2)
    assert float(y2.float().abs().max()) > 0
    graph = torch.cuda.CUDAGraph()
    yg, ig = torch.zeros_like(y2), torch.zeros_like(i2)
    with torch.cuda.graph(graph, stream=side):
        steps(one, yg, ig)
    for rep in range(4):
        yg.fill_(0)
        ig.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(yg, y2) and torch.equal(ig[:, :k], i2[:, :k]), rep
        with torch.cuda.stream(side):
            steps(one, y1, i1)
        side.synchronize()
        assert torch.equal(y1, y2)
    calls, timeouts = one.single_launch_status()
    say("  calls", calls, "timeouts", timeouts)
    assert calls == 6 * n and timeouts == 0
    one.close()
    two.close()


def test_single_launch_falls_back_where_it_does_not_fit(ctx):
    # d_model / 8 above the number of gate/up work-groups, wide rows, several tokens: two launches, same results
    one = B.Ctx(0)
    one.single_launch(True)
    for shape in (synth.LayerShape(1024, 8, 64, 2, 32, n_shared=0, act="bf16"),        # 16 gate/up work-groups, 128 down work-groups
                  synth.LayerShape(4096, 8, 128, 2, 128, n_shared=0, act="bf16")):     # wide rows
        pair = LayerPair(ctx, shape, seed=5)
        x = synth.activations(5, 2, shape.d_model, shape.act).cuda()
        z = synth.normal_logits(5, 2, shape.n_experts).cuda()
        m = dev(synth.bernoulli_masks(5, 1, shape.n_experts)[0])
        for i in range(2):
            _both(ctx, one, pair, shape, x[i], z[i], m)
    calls, timeouts = one.single_launch_status()
    assert calls == 0 and timeouts == 0
    one.close()


def test_single_launch_wait_is_bounded(ctx):
    # a spin limit of one poll: work-groups give up at once, the launch ends, the give-ups are counted;
    # switching the mode on again clears the words and the next calls are right again
    shape = synth.LayerShape(1024, 16, 704, 4, 32, n_shared=2, shared_d_ff=704, act="bf16")
    one = B.Ctx(0)
    one.single_launch(True, spin_limit=1)
    pair = LayerPair(ctx, shape, seed=17)
    x = synth.activations(17, 4, shape.d_model, shape.act).cuda()
    z = synth.normal_logits(17, 4, shape.n_experts).cuda()
    m = dev(synth.bernoulli_masks(17, 1, shape.n_experts)[0])
    for i in range(4):
        B.smoe_decode_layer(one, pair.routed, pair.shared, x[i], shape.top_k, logits=z[i], slice_mask=m)
    calls, timeouts = one.single_launch_status()
    say("  spin limit 1: calls", calls, "work-groups that gave up", timeouts)
    assert calls == 4
    one.single_launch(True)
    for i in range(4):
        _both(ctx, one, pair, shape, x[i], z[i], m)
    calls, timeouts2 = one.single_launch_status()
    assert calls == 8 and timeouts2 == 0
    one.close()
