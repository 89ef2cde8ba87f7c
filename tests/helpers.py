"""Shared test plumbing: builds a HIP-side bank and the oracle's quantised experts from the SAME
seeded dense weights.  No method arithmetic lives here."""
from __future__ import annotations

import numpy as np
import torch

from oracle import slicemoe_oracle as O
from paper_2512_12990_amd import binding as B
from paper_2512_12990_amd import synth


def t2np(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu", torch.float32).numpy()


class LayerPair:
    """One MoE layer on both sides.  Dense weights are drawn per expert (on `gen_device`), handed
    to the HIP quantiser, and kept only for the experts the oracle is asked about."""

    def __init__(self, ctx, shape: synth.LayerShape, seed=0, layer=0, gen_device="cpu", keep_dense=True,
                 routed=True, shared_d_ff=None):
        self.ctx, self.shape, self.seed, self.layer, self.gen_device = ctx, shape, seed, layer, gen_device
        self.dt = shape.act
        self._oracle_cache = {}
        self._dense = {}
        self.keep_dense = keep_dense
        self.routed = self.shared = None
        if routed and shape.n_experts > 0:
            self.routed = B.Bank(ctx, shape.n_experts, shape.d_model, shape.d_ff, shape.group, self.dt, self.dt,
                                 shape.b_high, shape.b_low, shape.symmetric)
            for e in range(shape.n_experts):
                self._quantise_into(self.routed, e, e, shape.d_ff)
        if shape.n_shared > 0:
            sf = shape.shared_d_ff
            self.shared = B.Bank(ctx, shape.n_shared, shape.d_model, sf, shape.group, self.dt, self.dt, shape.b_high,
                                 shape.b_low, shape.symmetric)
            for i in range(shape.n_shared):
                self._quantise_into(self.shared, i, 1000 + i, sf)
        torch.cuda.synchronize()

    def _weights(self, tag, d_ff):
        return synth.expert_weights(self.seed, self.layer, tag, self.shape.d_model, d_ff, self.dt, self.gen_device)

    def _quantise_into(self, bank, slot, tag, d_ff):
        wg, wu, wd = self._weights(tag, d_ff)
        if self.keep_dense:
            self._dense[tag] = tuple(w.cpu() for w in (wg, wu, wd))
        dev = "cuda:%d" % self.ctx.device
        B.smoe_quantize_slice(self.ctx, bank, slot, wg.to(dev)[None].contiguous(), wu.to(dev)[None].contiguous(),
                              wd.to(dev)[None].contiguous())

    def dense(self, tag, d_ff):
        if tag not in self._dense:
            self._dense[tag] = tuple(w.cpu() for w in self._weights(tag, d_ff))
        return self._dense[tag]

    def oracle_expert(self, tag) -> O.QExpert:
        if tag not in self._oracle_cache:
            d_ff = self.shape.shared_d_ff if tag >= 1000 else self.shape.d_ff
            wg, wu, wd = (t2np(w) for w in self.dense(tag, d_ff))
            self._oracle_cache[tag] = O.quantize_expert(wg, wu, wd, self.shape.group, self.shape.b_high, self.shape.b_low,
                                                        scale_dtype=self.dt, symmetric=self.shape.symmetric)
        return self._oracle_cache[tag]

    def oracle_routed(self):
        pair = self

        class _Lazy:
            def __getitem__(self, e):
                return pair.oracle_expert(int(e))
        return _Lazy()

    def oracle_shared(self):
        return [self.oracle_expert(1000 + i) for i in range(self.shape.n_shared)]
