"""CPU oracle for the SliceMoE expert-FFN hot path.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition of what the
hot path computes.  Only the tests, the smoke check and the bench's CPU-baseline
leg may import it; the product (the HIP library and its Python binding) never
does, and this module imports nothing from the product.

Every function is a direct statement of one step of the method, in numpy, with
fp64 for all floating-point accumulation.  The only fp32 arithmetic is the
quantiser (its integer results must be reproducible bit for bit, so the paper's
FP16/FP32 storage precision is part of its definition).

Paper passages followed (SliceMoE, arXiv 2512.12990):
  * Section 4.2 and its display equation: shift = b_high - b_low,
    q_low = floor(q_high / 2^shift), zp_low = floor(zp_high / 2^shift)  (AMAT).
  * Table 1, note 1: experts are group-wise asymmetric integer quantised.
  * Section 2.1: cache-aware routing boosts the gating scores of cached experts
    before top-k selection.
  * Section 4.1: each expert has an MSB and an LSB slice with separate hit/miss
    state; full precision only when both are present, MSB-only otherwise; MSB
    slices are LRU managed, LSB slices have the lowest priority.
  * Section 4.3: prefill accumulates per-expert access frequency; LSB slices go
    first, then MSB slices with low prefill frequency; the cache order at the
    start of decode follows accumulated frequency.
  * Section 6.1 item 3: one LRU cache shared by all layers.

Parity status: every function below is pinned by tests/test_oracle_*.py against
closed forms, exhaustive integer identities, brute force on tiny inputs or a
library routine.  Nothing here is "parity unpinned"; the paper's accuracy,
perplexity and energy results are outside this oracle altogether.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

F32 = np.float32
HIGH = 1
LOW = 0


# --------------------------------------------------------------------------
# storage-precision helper
# --------------------------------------------------------------------------
def round_to_bf16(a) -> np.ndarray:
    """Round fp32 values to the nearest bfloat16 (ties to even); result is fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    r = (u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))) & np.uint64(0xFFFF0000)
    return r.astype(np.uint32).view(np.float32).reshape(a.shape)


def _round_scale(s32: np.ndarray, scale_dtype: str) -> np.ndarray:
    if scale_dtype == "f32":
        return s32.astype(np.float32)
    if scale_dtype == "bf16":
        return round_to_bf16(s32)
    raise ValueError("scale_dtype must be 'f32' or 'bf16'")


# --------------------------------------------------------------------------
# AMAT quantised matrix
# --------------------------------------------------------------------------
@dataclass
class QMat:
    """One group-wise asymmetric quantised matrix W[N, K] (groups run along K).

    q      uint8 [N, K]        b_high-bit codes
    zp     uint8 [N, n_groups] integer zero-points (b_high-bit)
    scale  fp32  [N, n_groups] stored scales (already rounded to the scale dtype)
    """
    q: np.ndarray
    zp: np.ndarray
    scale: np.ndarray
    group: int
    b_high: int = 8
    b_low: int = 4

    @property
    def shift(self) -> int:
        return self.b_high - self.b_low

    def msb(self) -> np.ndarray:
        """Low-bit codes = MSB slice: floor(q / 2^shift)  (Section 4.2 equation)."""
        return (self.q >> self.shift).astype(np.uint8)

    def lsb(self) -> np.ndarray:
        """LSB slice: the bits the truncation drops."""
        return (self.q & ((1 << self.shift) - 1)).astype(np.uint8)

    def zp_low(self) -> np.ndarray:
        """Truncated zero-point: floor(zp / 2^shift)  (Section 4.2 equation)."""
        return (self.zp >> self.shift).astype(np.uint8)

    def _expand(self, per_group: np.ndarray) -> np.ndarray:
        K = self.q.shape[1]
        return np.repeat(per_group, self.group, axis=1)[:, :K]

    def dequant(self, prec: int) -> np.ndarray:
        """fp64 weights at HIGH (MSB and LSB recombined) or LOW (MSB slice only).

        HIGH: s * ((msb << shift | lsb) - zp)
        LOW : (2^shift * s) * (msb - zp_low)   -- code and zero-point truncated
              together; the scale grows by the dropped factor so both forms
              approximate the same real weight.
        """
        s = self._expand(self.scale.astype(np.float64))
        if prec == HIGH:
            code = (self.msb().astype(np.int64) << self.shift) | self.lsb().astype(np.int64)
            return s * (code - self._expand(self.zp.astype(np.int64)))
        code = self.msb().astype(np.int64)
        return (s * float(1 << self.shift)) * (code - self._expand(self.zp_low().astype(np.int64)))


def _quant_groups_symmetric(Wg: np.ndarray, qmax: int, scale_dtype: str):
    """Symmetric variant (Section 6.1 item 1: the non-expert weights are symmetric INT8): the
    signed code c = rint(w / s) with s = max|w| / (2^(b-1) - 1), kept in the same unsigned
    store as c + 2^(b-1), i.e. with the zero-point fixed at mid-range."""
    Wg = Wg.astype(np.float32)
    half = (qmax + 1) // 2
    amax = np.abs(Wg).max(axis=2).astype(np.float32)
    s = _round_scale((amax / F32(half - 1)).astype(np.float32), scale_dtype)
    s = np.where(s > F32(0.0), s, F32(1.0)).astype(np.float32)
    r = np.rint(Wg / s[:, :, None]).astype(np.float32)
    q = np.clip(r.astype(np.int64) + half, 0, qmax)
    zp = np.full(s.shape, half, dtype=np.uint8)
    return q.astype(np.uint8), zp, s


def _quant_groups(Wg: np.ndarray, qmax: int, scale_dtype: str, symmetric: bool = False):
    """Quantise W[N, g, Gsz]: every [n, j, :] is one group.  fp32 throughout."""
    if symmetric:
        return _quant_groups_symmetric(Wg, qmax, scale_dtype)
    Wg = Wg.astype(np.float32)
    lo = np.minimum(Wg.min(axis=2), F32(0.0)).astype(np.float32)
    hi = np.maximum(Wg.max(axis=2), F32(0.0)).astype(np.float32)
    s32 = ((hi - lo).astype(np.float32) / F32(qmax)).astype(np.float32)
    s = _round_scale(s32, scale_dtype)
    s = np.where(s > F32(0.0), s, F32(1.0)).astype(np.float32)       # flat (or vanishing) group
    zp = np.clip(np.rint((-lo) / s), F32(0.0), F32(qmax)).astype(np.int32)
    r = np.rint(Wg / s[:, :, None]).astype(np.float32)               # round half to even
    q = np.clip(r.astype(np.int64) + zp[:, :, None].astype(np.int64), 0, qmax)
    return q.astype(np.uint8), zp.astype(np.uint8), s


def quantize(W, group: int, b_high: int = 8, b_low: int = 4, scale_dtype: str = "f32",
             symmetric: bool = False) -> QMat:
    """Group-wise asymmetric min-max quantisation of W[N, K] to b_high-bit codes.

    The paper names the format (Table 1 note 1; Section 4.2 needs an integer
    zero-point that can be shifted) but prints no formula.  Reading used:
    per group, the range [lo, hi] is widened to contain 0; s = (hi - lo)/qmax in
    fp32, then rounded to the storage dtype and used in that rounded form;
    zp = clamp(rint(-lo / s)); q = clamp(rint(w / s) + zp).  A last group
    shorter than `group` (K not a multiple) has its own range.
    symmetric=True selects the mid-range zero-point variant instead (see
    _quant_groups_symmetric); slicing and both dequantisation rules are unchanged.
    """
    W = np.asarray(W, dtype=np.float32)
    N, K = W.shape
    if group <= 0 or not (1 <= b_low < b_high <= 8):
        raise ValueError("bad group / bit widths")
    qmax = (1 << b_high) - 1
    nfull = K // group
    qs, zps, ss = [], [], []
    if nfull:
        q, zp, s = _quant_groups(W[:, : nfull * group].reshape(N, nfull, group), qmax, scale_dtype, symmetric)
        qs.append(q.reshape(N, nfull * group)); zps.append(zp); ss.append(s)
    if K % group:
        q, zp, s = _quant_groups(W[:, nfull * group:].reshape(N, 1, K - nfull * group), qmax, scale_dtype, symmetric)
        qs.append(q.reshape(N, -1)); zps.append(zp); ss.append(s)
    return QMat(np.concatenate(qs, axis=1), np.concatenate(zps, axis=1),
                np.concatenate(ss, axis=1), group, b_high, b_low)


@dataclass
class QExpert:
    """SwiGLU expert: gate, up are [d_ff, d_model]; down is [d_model, d_ff]."""
    gate: QMat
    up: QMat
    down: QMat


def quantize_expert(w_gate, w_up, w_down, group, b_high=8, b_low=4, scale_dtype="f32", symmetric=False) -> QExpert:
    return QExpert(quantize(w_gate, group, b_high, b_low, scale_dtype, symmetric),
                   quantize(w_up, group, b_high, b_low, scale_dtype, symmetric),
                   quantize(w_down, group, b_high, b_low, scale_dtype, symmetric))


# --------------------------------------------------------------------------
# routing
# --------------------------------------------------------------------------
def router_logits(x, w_router) -> np.ndarray:
    """z[t, e] = sum_i W_r[e, i] x[t, i], accumulated in fp64, returned as fp32."""
    x = np.atleast_2d(np.asarray(x, dtype=np.float64))
    return (x @ np.asarray(w_router, dtype=np.float64).T).astype(np.float32)


def route(logits, bias, k: int, norm_topk: bool = False, routed_scale: float = 1.0):
    """Cache-aware top-k (Section 2.1).

    score = logits + bias (one fp32 add) decides WHICH experts run: the k largest
    scores, equal scores resolved towards the lower expert index, listed from
    the highest score down.  The mixing weights come from the softmax of the
    unbiased logits (fp64), so the boost changes locality only, not the mixture
    given the selection.
    Returns idx int32 [T, k], w fp64 [T, k].
    """
    z = np.atleast_2d(np.asarray(logits, dtype=np.float32))
    T, E = z.shape
    if not (1 <= k <= E):
        raise ValueError("k out of range")
    b = np.zeros(E, np.float32) if bias is None else np.asarray(bias, dtype=np.float32)
    score = (z + b[None, :]).astype(np.float32)
    idx = np.argsort(-score, axis=1, kind="stable")[:, :k].astype(np.int32)
    z64 = z.astype(np.float64)
    p = np.exp(z64 - z64.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    w = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    if norm_topk:
        w = w / w.sum(axis=1, keepdims=True)
    return idx, w * float(routed_scale)


def precision_select(idx, w, slice_mask, tau_head: float = 0.0) -> np.ndarray:
    """Per selected expert: HIGH iff it asks for both slices AND both are resident.

    slice_mask[e] bit0 = MSB slice resident, bit1 = LSB slice resident
    (Section 4.1: separate hit/miss per slice; full precision needs both).
    An expert asks for the LSB slice when its gate weight reaches tau_head
    (the paper's criticality test; its threshold is not printed, so 0 = always).
    """
    idx = np.asarray(idx)
    m = np.asarray(slice_mask, dtype=np.uint8)[idx]
    want = np.ones(idx.shape, bool) if tau_head <= 0.0 else (np.asarray(w) >= tau_head)
    return (((m & 3) == 3) & want).astype(np.uint8)


# --------------------------------------------------------------------------
# expert FFN
# --------------------------------------------------------------------------
def silu(a):
    return a / (1.0 + np.exp(-a))


def expert_ffn(x, ex: QExpert, prec: int) -> np.ndarray:
    """o = Wd (silu(Wg x) * (Wu x)) with all three matrices at precision `prec`.

    x may be [d] or [n, d]; fp64 throughout, h is never rounded.
    """
    x = np.asarray(x, dtype=np.float64)
    a = x @ ex.gate.dequant(prec).T
    u = x @ ex.up.dequant(prec).T
    return (silu(a) * u) @ ex.down.dequant(prec).T


def moe_layer(x, routed: Sequence[QExpert], idx, w, prec,
              shared: Sequence[QExpert] = (), shared_gate_w=None,
              add_residual: bool = False) -> np.ndarray:
    """One token through one MoE layer.

    y = sum_j w[j] * FFN_{idx[j]}^{prec[j]}(x)  (slot order)
        + sum_shared gamma * FFN_shared^HIGH(x),   gamma = 1 or sigmoid(w_sg . x)
        (+ x).
    """
    x = np.asarray(x, dtype=np.float64)
    y = np.zeros_like(x)
    for j in range(len(idx)):
        y = y + float(w[j]) * expert_ffn(x, routed[int(idx[j])], int(prec[j]))
    gamma = 1.0
    if shared_gate_w is not None:
        gamma = 1.0 / (1.0 + np.exp(-float(np.asarray(shared_gate_w, np.float64) @ x)))
    for ex in shared:
        y = y + gamma * expert_ffn(x, ex, HIGH)
    if add_residual:
        y = y + x
    return y


# --------------------------------------------------------------------------
# prefill: route all tokens, histogram, grouped high-bit FFN
# --------------------------------------------------------------------------
def histogram(idx, n_experts: int) -> np.ndarray:
    """hist[e] = number of (token, slot) pairs routed to expert e."""
    h = np.zeros(n_experts, np.uint32)
    for e in np.asarray(idx).reshape(-1):
        h[int(e)] += 1
    return h


def prefill_layer(X, routed: Sequence[QExpert], idx, w,
                  shared: Sequence[QExpert] = (), shared_gate_w=None,
                  add_residual: bool = False) -> np.ndarray:
    """Y[t] of moe_layer for every token, all experts HIGH (prefill is high-bit)."""
    X = np.asarray(X, dtype=np.float64)
    T, k = np.asarray(idx).shape
    Y = np.zeros_like(X)
    for j in range(k):                                   # slot order
        for e in np.unique(idx[:, j]):
            rows = np.nonzero(idx[:, j] == e)[0]
            Y[rows] += np.asarray(w)[rows, j][:, None] * expert_ffn(X[rows], routed[int(e)], HIGH)
    if shared:
        gamma = np.ones((T, 1))
        if shared_gate_w is not None:
            gamma = 1.0 / (1.0 + np.exp(-(X @ np.asarray(shared_gate_w, np.float64))))[:, None]
        for ex in shared:
            Y += gamma * expert_ffn(X, ex, HIGH)
    if add_residual:
        Y += X
    return Y


def topn_slices(hist, n: int) -> np.ndarray:
    """Warm-up retention order (Section 4.3), hottest first.

    Slice id = ((layer * E + expert) << 1) | is_lsb.  LSB slices are the first
    to go, so every MSB slice outranks every LSB slice; within a plane higher
    prefill frequency first; equal counts by layer, then expert.
    """
    hist = np.asarray(hist)
    L, E = hist.shape
    keys = []
    for is_lsb in (0, 1):
        for l in range(L):
            for e in range(E):
                keys.append((is_lsb, -int(hist[l, e]), l, e))
    keys.sort()
    ids = [(((l * E + e) << 1) | p) for (p, _, l, e) in keys]
    return np.asarray(ids[: max(0, min(n, len(ids)))], dtype=np.uint32)


# --------------------------------------------------------------------------
# slice cache (host bookkeeping that produces the mask)
# --------------------------------------------------------------------------
class SliceLRU:
    """Unified slice-level cache over all layers (Section 4.1; Section 6.1 item 3).

    `order` lists resident slice ids from most- to least-recently used.
    MSB request: hit -> move to front; miss -> fetch, insert at front.
    LSB request: hit -> position unchanged; miss -> fetch, insert at the BACK
    (first eviction candidate).  A fetch into a full cache first drops the back.
    """

    def __init__(self, n_layers: int, n_experts: int, capacity: int):
        if capacity < 2:
            raise ValueError("capacity must hold at least two slices")
        self.L, self.E, self.cap = n_layers, n_experts, capacity
        self.order: List[int] = []
        self.stats = dict(msb_hit=0, msb_miss=0, lsb_hit=0, lsb_miss=0)

    def sid(self, layer, expert, is_lsb):
        return ((layer * self.E + expert) << 1) | is_lsb

    def init_order(self, slice_ids):
        ids = [int(s) for s in slice_ids][: self.cap]
        assert len(set(ids)) == len(ids)
        self.order = ids

    def snapshot(self, layer: int, beta: float):
        res = set(self.order)
        mask = np.zeros(self.E, np.uint8)
        for e in range(self.E):
            mask[e] = (1 if self.sid(layer, e, 0) in res else 0) | (2 if self.sid(layer, e, 1) in res else 0)
        bias = np.where(mask & 1, np.float32(beta), np.float32(0.0)).astype(np.float32)
        return mask, bias

    def access(self, layer: int, idx, want_high):
        for e, wh in zip(idx, want_high):
            s = self.sid(layer, int(e), 0)
            if s in self.order:
                self.stats["msb_hit"] += 1
                self.order.remove(s)
            else:
                self.stats["msb_miss"] += 1
                if len(self.order) >= self.cap:
                    self.order.pop()
            self.order.insert(0, s)
            if wh:
                s = self.sid(layer, int(e), 1)
                if s in self.order:
                    self.stats["lsb_hit"] += 1
                else:
                    self.stats["lsb_miss"] += 1
                    if len(self.order) >= self.cap:
                        self.order.pop()
                    self.order.append(s)


# --------------------------------------------------------------------------
# modeled cost on the paper's target system (Section 5)
# --------------------------------------------------------------------------
PAPER_SYSTEM = dict(flash_gbit_s=10.0, dram_gbit_s=104.0, xpu_tops=16.4,      # bandwidths, throughput
                    flash_pj_bit=103.0, dram_pj_bit=1.5, xpu_tops_w=3.18)     # energies, efficiency


def cost_model(stats, msb_slice_bytes: int, lsb_slice_bytes: int, ops: float, system=None) -> dict:
    """Energy and latency of the slice accesses counted in `stats` (Section 5's device).

    A missed slice is read from Flash and written to DRAM; every requested slice (hit or miss) is
    then read from DRAM by the PE array.  Energy adds the three terms; latency serves Flash, DRAM
    and compute one after the other.  The high-bit-normalised miss rate relates the Flash bytes
    to what a cache of whole high-bit experts would fetch if every request missed.
    """
    sy = PAPER_SYSTEM if system is None else system
    miss = stats["msb_miss"] * msb_slice_bytes + stats["lsb_miss"] * lsb_slice_bytes
    used = ((stats["msb_hit"] + stats["msb_miss"]) * msb_slice_bytes +
            (stats["lsb_hit"] + stats["lsb_miss"]) * lsb_slice_bytes)
    flash_bits = 8.0 * miss
    dram_bits = 8.0 * (used + miss)
    energy = flash_bits * sy["flash_pj_bit"] * 1e-12 + dram_bits * sy["dram_pj_bit"] * 1e-12 + ops / (sy["xpu_tops_w"] * 1e12)
    latency = flash_bits / (sy["flash_gbit_s"] * 1e9) + dram_bits / (sy["dram_gbit_s"] * 1e9) + ops / (sy["xpu_tops"] * 1e12)
    req = stats["msb_hit"] + stats["msb_miss"]
    rate = miss / (req * (msb_slice_bytes + lsb_slice_bytes)) if req else 0.0
    return dict(flash_bits=flash_bits, dram_bits=dram_bits, ops=float(ops), energy_j=energy, latency_s=latency,
                miss_rate_high=rate)


# --------------------------------------------------------------------------
# comparison metric
# --------------------------------------------------------------------------
def max_abs_rel(y, y_ref) -> float:
    """max_i |y_i - ref_i| / max_i |ref_i| over one output vector or matrix."""
    y = np.asarray(y, dtype=np.float64); y_ref = np.asarray(y_ref, dtype=np.float64)
    den = float(np.max(np.abs(y_ref)))
    return float(np.max(np.abs(y - y_ref)) / (den if den > 0 else 1.0))
