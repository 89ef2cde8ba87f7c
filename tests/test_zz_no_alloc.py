"""The no-allocation decode entry point (smoe_decode_layer_static: workspace in a file-scope device
array of the library) against smoe_decode_layer, through the C ABI: two calls in a row, the second
on a smaller layer, every output compared bit for bit (same kernels, same order of operations), plus
the oracle on the first; the size limit is refused with a clear status."""
import ctypes as C
import sys

import numpy as np
import pytest
import torch

from oracle import slicemoe_oracle as O
from paper_2512_12990_amd import binding as B
from paper_2512_12990_amd import synth
from helpers import LayerPair, t2np

pytestmark = pytest.mark.gpu


def _outputs(k, d, dtype):
    return (torch.zeros(d, dtype=dtype, device="cuda:0"), torch.full((k,), -1, dtype=torch.int32, device="cuda:0"),
            torch.zeros(k, dtype=torch.float32, device="cuda:0"), torch.full((k,), 9, dtype=torch.uint8, device="cuda:0"))


def test_static_scratch_entry_matches_the_workspace_entry():
    assert torch.cuda.is_available(), "this test needs the MI355X"
    print("no-alloc entry point", flush=True)
    sys.stdout.flush()
    assert B.smoe_static_scratch_bytes() == 512 << 10
    ref_ctx = B.Ctx(0)                              # the existing entry point: caller-owned workspace
    bare_ctx = B.Ctx(0, workspace_bytes=0)          # a context that owns no device memory at all
    big = synth.LayerShape(2048, 16, 1408, 6, 128, n_shared=2, shared_d_ff=1408, act="bf16")
    small = synth.LayerShape(256, 8, 96, 2, 32, n_shared=1, shared_d_ff=160, shared_gate=True, act="f32")
    for shp, seed in ((big, 61), (small, 62)):      # the second call is the smaller one
        pair = LayerPair(ref_ctx, shp, seed=seed, gen_device="cuda:0" if shp is big else "cpu")
        k, E, d = shp.top_k, shp.n_experts, shp.d_model
        x = synth.activations(seed, 1, d, shp.act)[0].cuda()
        z = synth.normal_logits(seed, 1, E)[0].cuda()
        mask_np = synth.bernoulli_masks(seed, 1, E)[0]
        mask = torch.from_numpy(mask_np).cuda()
        bias = torch.from_numpy(np.where(mask_np == 3, np.float32(0.5), np.float32(0)).astype(np.float32)).cuda()
        wsg = synth.shared_gate_weight(seed, 0, d, shp.act).cuda() if shp.shared_gate else None
        wr = synth.router_weight(seed, 0, E, d).cuda()
        for logits, w_router in ((z, None), (None, wr)):      # supplied logits; router mat-vec into the scratch
            y0, i0, w0, p0 = _outputs(k, d, x.dtype)
            y1, i1, w1, p1 = _outputs(k, d, x.dtype)
            B.smoe_decode_layer(ref_ctx, pair.routed, pair.shared, x, k, logits=logits, w_router=w_router, bias=bias,
                                norm_topk=True, routed_scale=1.5, slice_mask=mask, tau_head=0.1, shared_gate_w=wsg,
                                add_residual=True, y=y0, idx_out=i0, w_out=w0, prec_out=p0)
            B.smoe_decode_layer_static(bare_ctx, pair.routed, pair.shared, x, k, y1, logits=logits, w_router=w_router,
                                       bias=bias, norm_topk=True, routed_scale=1.5, slice_mask=mask, tau_head=0.1,
                                       shared_gate_w=wsg, add_residual=True, idx_out=i1, w_out=w1, prec_out=p1)
            torch.cuda.synchronize()
            assert torch.equal(i0, i1) and torch.equal(w0, w1) and torch.equal(p0, p1)
            assert torch.equal(y0, y1)
            assert float(y1.float().abs().max()) > 0
        # and against the oracle (supplied logits)
        y1, i1, w1, p1 = _outputs(k, d, x.dtype)
        B.smoe_decode_layer_static(bare_ctx, pair.routed, pair.shared, x, k, y1, logits=z, bias=bias, slice_mask=mask,
                                   shared_gate_w=wsg, idx_out=i1, w_out=w1, prec_out=p1)
        torch.cuda.synchronize()
        ridx, rw = O.route(z.cpu().numpy()[None], bias.cpu().numpy(), k)
        assert np.array_equal(i1.cpu().numpy(), ridx[0])
        w_used = w1.cpu().numpy().astype(np.float64)
        rprec = O.precision_select(ridx[0], w_used, mask_np)
        assert np.array_equal(p1.cpu().numpy(), rprec)
        yref = O.moe_layer(t2np(x).astype(np.float64), pair.oracle_routed(), ridx[0], w_used, rprec, pair.oracle_shared(),
                           None if wsg is None else t2np(wsg))
        assert O.max_abs_rel(t2np(y1), yref) <= (2e-2 if shp.act == "bf16" else 1e-4)
    # the context without a workspace serves only the static entry point
    with pytest.raises(B.SmoeError):
        B.smoe_decode_layer(bare_ctx, pair.routed, pair.shared, x, k, logits=z)
    # beyond the array: 64 KiB + 4 * (k * d_ff + n_shared * shared_d_ff) bytes must fit 512 KiB
    wide = B.Bank(ref_ctx, 2, 64, 57376, 32, "f32", "f32")      # 2 * 57376 floats + 64 KiB: 256 bytes over 512 KiB
    xw = torch.zeros(64, dtype=torch.float32, device="cuda:0")
    yw = torch.zeros_like(xw)
    zw = torch.zeros(2, dtype=torch.float32, device="cuda:0")
    rc = B.lib().smoe_decode_layer_static(bare_ctx.h, wide.h, None, C.c_void_p(xw.data_ptr()), 0, 2, C.c_void_p(zw.data_ptr()),
                                          None, None, 0, C.c_float(1.0), None, C.c_float(0.0), None, 0,
                                          C.c_void_p(yw.data_ptr()), None, None, None)
    assert rc == -4
    torch.cuda.synchronize()
    bare_ctx.close()
    ref_ctx.close()
