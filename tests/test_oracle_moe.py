"""Pins for the oracle's routing, precision select, expert FFN, prefill, top-N and slice LRU.

CPU only.  Checks are brute force on tiny inputs, library routines (torch fp64 ops) on
special cases where the answer does not depend on the oracle's own formulas, invariants and
hand-traced sequences.
"""
import itertools
from collections import OrderedDict

import numpy as np
import pytest
import torch

from oracle import slicemoe_oracle as O


# ------------------------------------------------------------------ routing
def test_zero_bias_is_plain_softmax_topk():
    rng = np.random.default_rng(0)
    z = rng.standard_normal((50, 16)).astype(np.float32)
    idx, w = O.route(z, None, 4)
    p = torch.softmax(torch.from_numpy(z).double(), dim=1)
    tv, ti = torch.topk(p, 4, dim=1)                      # sorted descending
    assert np.array_equal(idx, ti.numpy().astype(np.int32))
    np.testing.assert_allclose(w, tv.numpy(), rtol=1e-12)
    assert np.all(w.sum(1) <= 1.0 + 1e-12)
    _, wn = O.route(z, None, 4, norm_topk=True, routed_scale=2.5)
    np.testing.assert_allclose(wn.sum(1), 2.5, rtol=1e-12)


def test_topk_brute_force_all_subsets():
    rng = np.random.default_rng(1)
    for E, k in [(4, 1), (5, 2), (6, 3), (6, 6)]:
        for _ in range(20):
            z = rng.standard_normal(E).astype(np.float32)
            b = rng.choice([0.0, 1.0], size=E).astype(np.float32)
            idx, _ = O.route(z[None], b, k)
            score = (z + b).astype(np.float32)
            best = max(itertools.combinations(range(E), k), key=lambda S: sum(float(score[i]) for i in S))
            assert set(idx[0].tolist()) == set(best)
            assert all(score[idx[0, i]] >= score[idx[0, i + 1]] for i in range(k - 1))


def test_bias_confines_selection_but_not_weights():
    rng = np.random.default_rng(2)
    z = rng.standard_normal((30, 12)).astype(np.float32)
    S = [1, 4, 7, 9, 10]
    b = np.zeros(12, np.float32)
    b[S] = float(z.max() - z.min()) + 1.0
    idx, w = O.route(z, b, 3)
    assert all(set(r.tolist()) <= set(S) for r in idx)
    p = torch.softmax(torch.from_numpy(z).double(), dim=1).numpy()       # unbiased mixture weights
    np.testing.assert_allclose(w, np.take_along_axis(p, idx.astype(np.int64), 1), rtol=1e-12)


def test_ties_go_to_lower_index_and_permutation_equivariance():
    z = np.array([[0.5, 2.0, 2.0, -1.0, 2.0, 0.5]], np.float32)
    idx, _ = O.route(z, None, 4)
    assert idx[0].tolist() == [1, 2, 4, 0]
    rng = np.random.default_rng(3)
    z = rng.standard_normal((8, 10)).astype(np.float32)
    b = rng.standard_normal(10).astype(np.float32)
    perm = rng.permutation(10)
    i0, w0 = O.route(z, b, 3)
    i1, w1 = O.route(z[:, perm], b[perm], 3)
    assert np.array_equal(perm[i1], i0)
    np.testing.assert_allclose(w1, w0, rtol=1e-12)


def test_router_logits_match_library_matvec():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((3, 40)).astype(np.float32)
    Wr = rng.standard_normal((7, 40)).astype(np.float32)              # [E, d]: not square
    ref = (torch.from_numpy(x).double() @ torch.from_numpy(Wr).double().T).float().numpy()
    assert np.array_equal(O.router_logits(x, Wr), ref)


def test_precision_select_truth_table():
    mask = np.array([0, 1, 2, 3, 3], np.uint8)
    idx = np.array([0, 1, 2, 3, 4])
    w = np.array([0.5, 0.5, 0.5, 0.5, 0.05])
    assert O.precision_select(idx, w, mask).tolist() == [0, 0, 0, 1, 1]
    assert O.precision_select(idx, w, mask, tau_head=0.1).tolist() == [0, 0, 0, 1, 0]


# ------------------------------------------------------------------ expert FFN
def _grid_expert(rng, d, f, G):
    """Weights lying exactly on an 8-bit grid with power-of-two scales: quantisation is lossless,
    so HIGH-precision results must equal those of the dense fp64 model."""
    def grid(N, K):
        ng = K // G
        j = rng.integers(0, 256, size=(N, K))
        j[:, ::G] = 0
        j[:, G - 1::G] = 255
        z0 = rng.integers(96, 160, size=(N, ng))
        s0 = 2.0 ** rng.integers(-10, -7, size=(N, ng))
        return ((j - np.repeat(z0, G, 1)) * np.repeat(s0, G, 1)).astype(np.float32)
    return grid(f, d), grid(f, d), grid(d, f)


def _dense_swiglu(x, wg, wu, wd):
    x = torch.as_tensor(x, dtype=torch.float64)
    a = torch.as_tensor(wg, dtype=torch.float64) @ x
    u = torch.as_tensor(wu, dtype=torch.float64) @ x
    return (torch.as_tensor(wd, dtype=torch.float64) @ (torch.nn.functional.silu(a) * u)).numpy()


def test_high_precision_ffn_equals_dense_model_on_grid_weights():
    rng = np.random.default_rng(5)
    d, f, G = 96, 64, 32                                   # non-square on purpose
    wg, wu, wd = _grid_expert(rng, d, f, G)
    ex = O.quantize_expert(wg, wu, wd, G)
    x = rng.standard_normal(d)
    np.testing.assert_allclose(O.expert_ffn(x, ex, O.HIGH), _dense_swiglu(x, wg, wu, wd), rtol=1e-11, atol=1e-13)


def test_low_precision_ffn_equals_dense_model_with_amat_shifted_weights():
    # Dense matrices for the low-bit model are built from the exhaustive identity
    # low = high + s*((zp&15)-(q&15)) (pinned in test_oracle_quant), not from the oracle's dequant.
    rng = np.random.default_rng(6)
    d, f, G = 64, 96, 32
    wg, wu, wd = [(rng.standard_normal(s) * 0.02).astype(np.float32) for s in ((f, d), (f, d), (d, f))]
    ex = O.quantize_expert(wg, wu, wd, G, scale_dtype="bf16")

    def dense(m, low):
        s = np.repeat(m.scale.astype(np.float64), G, 1)
        zp = np.repeat(m.zp.astype(np.int64), G, 1)
        q = m.q.astype(np.int64)
        w = s * (q - zp)
        return w + s * ((zp % 16) - (q % 16)) if low else w
    x = rng.standard_normal(d)
    for prec in (O.HIGH, O.LOW):
        ref = _dense_swiglu(x, dense(ex.gate, prec == O.LOW), dense(ex.up, prec == O.LOW), dense(ex.down, prec == O.LOW))
        np.testing.assert_allclose(O.expert_ffn(x, ex, prec), ref, rtol=1e-10, atol=1e-14)


def _tiny_layer(rng, E=5, d=64, f=32, G=32, n_shared=1):
    mk = lambda: [(rng.standard_normal(s) * 0.05).astype(np.float32) for s in ((f, d), (f, d), (d, f))]
    routed = [O.quantize_expert(*mk(), G) for _ in range(E)]
    shared = [O.quantize_expert(*mk(), G) for _ in range(n_shared)]
    return routed, shared


def test_layer_is_the_weighted_sum_of_its_experts():
    rng = np.random.default_rng(7)
    routed, shared = _tiny_layer(rng)
    x = rng.standard_normal(64)
    z = rng.standard_normal((1, 5)).astype(np.float32)
    # k = E with renormalisation is the full soft mixture
    idx, w = O.route(z, None, 5, norm_topk=True)
    prec = np.ones(5, np.uint8)
    y = O.moe_layer(x, routed, idx[0], w[0], prec)
    p = torch.softmax(torch.from_numpy(z[0]).double(), 0).numpy()
    ref = sum(p[e] * O.expert_ffn(x, routed[e], O.HIGH) for e in range(5))
    np.testing.assert_allclose(y, ref, rtol=1e-10, atol=1e-14)
    # mixed precision, shared expert with a sigmoid gate, residual
    idx, w = O.route(z, None, 2)
    wsg = rng.standard_normal(64) * 0.1
    y = O.moe_layer(x, routed, idx[0], w[0], [1, 0], shared, wsg, add_residual=True)
    gamma = float(torch.sigmoid(torch.tensor(float(wsg @ x), dtype=torch.float64)))
    ref = (w[0, 0] * O.expert_ffn(x, routed[idx[0, 0]], O.HIGH) + w[0, 1] * O.expert_ffn(x, routed[idx[0, 1]], O.LOW)
           + gamma * O.expert_ffn(x, shared[0], O.HIGH) + x)
    np.testing.assert_allclose(y, ref, rtol=1e-10, atol=1e-14)
    # linear in the gate weights
    y1 = O.moe_layer(x, routed, idx[0], w[0], [1, 0])
    y2 = O.moe_layer(x, routed, idx[0], 3.0 * w[0], [1, 0])
    np.testing.assert_allclose(y2, 3.0 * y1, rtol=1e-10, atol=1e-14)
    # HIGH and LOW really differ (a precision flag that is ignored would pass everything above)
    assert O.max_abs_rel(O.expert_ffn(x, routed[0], O.LOW), O.expert_ffn(x, routed[0], O.HIGH)) > 1e-3


# ------------------------------------------------------------------ prefill
def test_prefill_matches_token_by_token_and_histogram_is_bincount():
    rng = np.random.default_rng(8)
    routed, shared = _tiny_layer(rng, E=6)
    T, k = 37, 2
    X = rng.standard_normal((T, 64))
    z = rng.standard_normal((T, 6)).astype(np.float32)
    idx, w = O.route(z, None, k)
    wsg = rng.standard_normal(64) * 0.1
    Y = O.prefill_layer(X, routed, idx, w, shared, wsg, add_residual=True)
    for t in range(T):
        yt = O.moe_layer(X[t], routed, idx[t], w[t], np.ones(k, np.uint8), shared, wsg, add_residual=True)
        np.testing.assert_allclose(Y[t], yt, rtol=1e-9, atol=1e-13)
    h = O.histogram(idx, 6)
    assert h.sum() == T * k and h.dtype == np.uint32
    assert np.array_equal(h, np.bincount(idx.reshape(-1), minlength=6))


def test_topn_order_properties():
    rng = np.random.default_rng(9)
    L, E = 3, 5
    hist = rng.integers(0, 4, size=(L, E)).astype(np.uint32)          # many ties
    full = O.topn_slices(hist, 2 * L * E)
    assert sorted(full.tolist()) == list(range(2 * L * E))            # a permutation of every slice id
    planes = full & 1
    assert np.all(planes[: L * E] == 0) and np.all(planes[L * E:] == 1)   # every MSB before any LSB
    for part in (full[: L * E], full[L * E:]):
        cnt = np.array([hist[(s >> 1) // E, (s >> 1) % E] for s in part])
        assert np.all(cnt[:-1] >= cnt[1:])
        for a, b, ca, cb in zip(part[:-1], part[1:], cnt[:-1], cnt[1:]):
            if ca == cb:
                assert a < b                                              # layer, then expert ascending
    assert np.array_equal(O.topn_slices(hist, 7), full[:7])
    assert O.topn_slices(hist, 10 ** 6).size == 2 * L * E and O.topn_slices(hist, 0).size == 0


# ------------------------------------------------------------------ slice LRU
def test_slice_lru_hand_trace():
    c = O.SliceLRU(1, 8, 4)
    M = lambda e: e << 1
    Ls = lambda e: (e << 1) | 1
    c.access(0, [0, 1], [0, 0]);            assert c.order == [M(1), M(0)]
    c.access(0, [2], [1]);                  assert c.order == [M(2), M(1), M(0), Ls(2)]      # LSB enters at the back
    c.access(0, [0], [0]);                  assert c.order == [M(0), M(2), M(1), Ls(2)]      # MSB hit -> front
    c.access(0, [2], [1]);                  assert c.order == [M(2), M(0), M(1), Ls(2)]      # LSB hit: not promoted
    assert c.stats == dict(msb_hit=2, msb_miss=3, lsb_hit=1, lsb_miss=1)
    c.access(0, [3], [0]);                  assert c.order == [M(3), M(2), M(0), M(1)]       # LSB is the first victim
    c.access(0, [4], [1]);                  assert c.order == [M(4), M(3), M(2), Ls(4)]      # two fetches, two evictions
    mask, bias = c.snapshot(0, 1.0)
    assert mask.tolist() == [0, 0, 1, 1, 3, 0, 0, 0]
    assert bias.tolist() == [0, 0, 1, 1, 1, 0, 0, 0]


def test_slice_lru_without_lsb_requests_is_textbook_lru():
    rng = np.random.default_rng(10)
    L, E, cap = 3, 7, 6
    c = O.SliceLRU(L, E, cap)
    ref = OrderedDict()
    for _ in range(400):
        l, e = int(rng.integers(L)), int(rng.integers(E))
        c.access(l, [e], [0])
        key = (l * E + e) << 1
        if key in ref:
            ref.move_to_end(key)
        else:
            if len(ref) >= cap:
                ref.popitem(last=False)
            ref[key] = True
        assert len(c.order) <= cap
        assert c.order == list(reversed(ref.keys()))


def test_slice_lru_init_order_and_capacity():
    c = O.SliceLRU(2, 4, 5)
    c.init_order(O.topn_slices(np.array([[5, 1, 0, 2], [3, 3, 0, 9]], np.uint32), 5))
    # MSB slices by count: (1,3)=9, (0,0)=5, (1,0)=3, (1,1)=3, (0,3)=2
    assert c.order == [(7 << 1), (0 << 1), (4 << 1), (5 << 1), (3 << 1)]
    rng = np.random.default_rng(11)
    for _ in range(200):
        c.access(int(rng.integers(2)), rng.integers(4, size=2).tolist(), rng.integers(2, size=2).tolist())
        assert len(c.order) <= 5 and len(set(c.order)) == len(c.order)
