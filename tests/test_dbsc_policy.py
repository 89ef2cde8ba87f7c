"""CPU-only tests of the host policy layer around the hot path: the modeled cost of a slice-access
trace on the paper's device (Section 5), the criticality threshold of Dynamic Bit-Sliced Caching
(Section 4.1) and Predictive Cache Warmup (Section 4.3) on synthetic routing traces.  The library's
C++ bookkeeping runs in lockstep with the oracle's; the oracle's cost model is pinned to closed
forms first."""
import numpy as np
import pytest

from oracle import slicemoe_oracle as O
from paper_2512_12990_amd import binding as B, synth


# ------------------------------------------------------------------ cost model: pins of the oracle
def test_cost_model_closed_forms():
    # Section 5: 8,192 8-bit PEs at 1 GHz, one multiply-accumulate (2 operations) each per cycle
    assert abs(O.PAPER_SYSTEM["xpu_tops"] - 2 * 8192 * 1e9 / 1e12) < 0.05
    # one missed MSB slice of 1.25e9 bytes = 1e10 bits: 1 s of Flash at 10 Gbit/s and 1.03 J at 103 pJ/bit;
    # it is written to DRAM and read back: 2e10 bits = 2e10/104e9 s and 2e10 * 1.5 pJ
    c = O.cost_model(dict(msb_hit=0, msb_miss=1, lsb_hit=0, lsb_miss=0), 1_250_000_000, 7, 0.0)
    assert c["flash_bits"] == 1e10 and c["dram_bits"] == 2e10
    assert c["latency_s"] == pytest.approx(1.0 + 2e10 / 104e9, rel=1e-12)
    assert c["energy_j"] == pytest.approx(1.03 + 0.03, rel=1e-12)
    # every request missing both slices = the traffic of a whole-expert high-bit cache that always misses
    assert c["miss_rate_high"] == pytest.approx(1_250_000_000 / (1_250_000_000 + 7))
    c = O.cost_model(dict(msb_hit=0, msb_miss=5, lsb_hit=0, lsb_miss=5), 1000, 600, 0.0)
    assert c["miss_rate_high"] == pytest.approx(1.0)
    # hits only: no Flash term; compute only: ops / 16.4 TOPS and ops / 3.18 TOPS/W
    c = O.cost_model(dict(msb_hit=3, msb_miss=0, lsb_hit=2, lsb_miss=0), 1000, 600, 16.4e12)
    assert c["flash_bits"] == 0 and c["miss_rate_high"] == 0
    assert c["dram_bits"] == 8 * (3 * 1000 + 2 * 600)
    assert c["latency_s"] == pytest.approx(1.0 + c["dram_bits"] / 104e9)
    assert c["energy_j"] == pytest.approx(16.4 / 3.18 + c["dram_bits"] * 1.5e-12)
    # energy and latency are additive over traces
    a = dict(msb_hit=7, msb_miss=2, lsb_hit=1, lsb_miss=3)
    b = dict(msb_hit=1, msb_miss=9, lsb_hit=0, lsb_miss=4)
    ab = {k: a[k] + b[k] for k in a}
    ca, cb, cab = (O.cost_model(s, 4096, 4000, 1e9) for s in (a, b, ab))
    assert cab["energy_j"] == pytest.approx(ca["energy_j"] + cb["energy_j"] - 1e9 / 3.18e12)
    assert cab["flash_bits"] == ca["flash_bits"] + cb["flash_bits"]


def test_cost_model_library_matches_oracle():
    spec = B.smoe_system_spec_paper()
    for n, v in O.PAPER_SYSTEM.items():
        assert getattr(spec, n) == v
    rng = np.random.default_rng(5)
    for _ in range(50):
        st = {k: int(rng.integers(0, 10_000)) for k in ("msb_hit", "msb_miss", "lsb_hit", "lsb_miss")}
        bm, bl, ops = int(rng.integers(1, 1 << 24)), int(rng.integers(1, 1 << 24)), float(rng.integers(0, 1 << 40))
        got, ref = B.smoe_cost_model(spec, st, bm, bl, ops), O.cost_model(st, bm, bl, ops)
        for k in ref:
            assert got[k] == pytest.approx(ref[k], rel=1e-12, abs=0.0), k
    zero = dict(msb_hit=0, msb_miss=0, lsb_hit=0, lsb_miss=0)
    assert B.smoe_cost_model(spec, zero, 10, 10, 0.0)["miss_rate_high"] == 0.0
    bad = B.SystemSpec(0.0, 104.0, 16.4, 103.0, 1.5, 3.18)
    with pytest.raises(B.SmoeError):
        B.smoe_cost_model(bad, zero, 10, 10, 0.0)


# ------------------------------------------------------------------ traces
def _trace(seed, L, E, k, steps, period):
    """Routing decisions of `steps` tokens through L layers on popularity-skewed logits (the oracle's
    router, no cache bias): idx [steps, L, k], w [steps, L, k]."""
    idx = np.empty((steps, L, k), np.int32)
    w = np.empty((steps, L, k), np.float64)
    for l in range(L):
        z = synth.zipf_logits(seed, l, steps, E, period=period).numpy()
        i, ww = O.route(z, None, k)
        idx[:, l], w[:, l] = i, ww
    return idx, w


def _run(cache_pair, idx, w, tau, first=None):
    """Feeds a trace to the library's cache and the oracle's in lockstep; returns the library's
    stats after `first` steps (all if None)."""
    c, o = cache_pair
    n = idx.shape[0] if first is None else first
    for t in range(n):
        for l in range(idx.shape[1]):
            want = (w[t, l] >= tau).astype(np.uint8)
            c.access(l, idx[t, l], want)
            o.access(l, idx[t, l], want)
    assert c.stats() == o.stats and c.order() == o.order
    return c.stats()


def test_predictive_warmup_cuts_cold_misses():
    """Section 4.3: a cache re-ordered by prefill access frequency misses less in early decode than
    an empty one.  The prefill prompt and the first decode steps share one popularity permutation."""
    L, E, k = 4, 32, 4
    idx, w = _trace(11, L, E, k, 192, period=256)
    pre, dec = idx[:128], idx[128:]
    hist = np.stack([O.histogram(pre[:, l].reshape(-1), E) for l in range(L)]).astype(np.uint32)
    cap = (2 * L * E) // 4
    ids = B.smoe_topn_slices(hist, cap)
    assert np.array_equal(ids, O.topn_slices(hist, cap))
    warm = (B.Cache(L, E, cap), O.SliceLRU(L, E, cap))
    warm[0].init_order(ids)
    warm[1].init_order(ids)
    cold = (B.Cache(L, E, cap), O.SliceLRU(L, E, cap))
    tau = 0.0
    sw = _run(warm, dec, w[128:], tau, first=10)
    sc = _run(cold, dec, w[128:], tau, first=10)
    assert sw["msb_miss"] < sc["msb_miss"] // 2, (sw, sc)
    # every MSB slice is retained before any LSB slice: with capacity <= L*E the warm cache holds no LSB slice
    assert all((s & 1) == 0 for s in ids)


def test_criticality_threshold_trades_lsb_traffic():
    """Section 4.1: only experts whose gate weight reaches the threshold ask for their LSB slice.
    Raising it lowers the LSB requests monotonically down to none, and with them the Flash traffic
    of the trace's first steps (no eviction yet: every request of a new slice is a miss)."""
    L, E, k = 2, 32, 4
    idx, w = _trace(13, L, E, k, 64, period=64)
    spec = B.smoe_system_spec_paper()
    bm, bl = 4_528_128, 4_325_376          # MSB slice (planes + metadata) and LSB slice of a 2048 x 1408 expert, group 128
    prev_req, prev_flash = None, None
    for tau in [0.0, 0.2, 0.4, 0.6, 2.0]:
        pair = (B.Cache(L, E, 2 * L * E), O.SliceLRU(L, E, 2 * L * E))
        st = _run(pair, idx, w, tau)
        req = st["lsb_hit"] + st["lsb_miss"]
        cost = B.smoe_cost_model(spec, st, bm, bl, 0.0)
        assert cost == pytest.approx(O.cost_model(st, bm, bl, 0.0))
        if prev_req is not None:
            assert req <= prev_req and cost["flash_bits"] <= prev_flash
        prev_req, prev_flash = req, cost["flash_bits"]
    assert prev_req == 0
    # at tau = 0 every request asks for both slices
    pair = (B.Cache(L, E, 2 * L * E), O.SliceLRU(L, E, 2 * L * E))
    st = _run(pair, idx, w, 0.0)
    assert st["lsb_hit"] + st["lsb_miss"] == st["msb_hit"] + st["msb_miss"] == 64 * L * k


def test_warmup_beats_the_naive_initial_states():
    """Section 4.3 names three naive cache states at the start of decode -- empty, only what the
    layer-wise prefill touched last, a random retention -- and says each does poorly in early decode.
    All four are just different retention orders handed to the same LRU: on a popularity-skewed trace
    the frequency-ordered state misses least, and no filled state misses more than the empty one."""
    L, E, k = 4, 32, 4
    idx, w = _trace(17, L, E, k, 192, period=256)
    pre, dec, wdec = idx[:128], idx[128:], w[128:]
    hist = np.stack([O.histogram(pre[:, l].reshape(-1), E) for l in range(L)]).astype(np.uint32)
    cap = (2 * L * E) // 4
    sid = lambda l, e, lsb: ((l * E + e) << 1) | lsb
    # prefill runs layer by layer at high precision and loads every expert: the cache ends up holding
    # both slices of the layers processed last
    last = [sid(l, e, b) for l in range(L - 1, -1, -1) for e in range(E) for b in (0, 1)][:cap]
    rnd = np.random.default_rng(17).permutation(2 * L * E)[:cap].tolist()
    states = {"empty": None, "last": last, "random": rnd, "pcw": B.smoe_topn_slices(hist, cap).tolist()}
    miss = {}
    for name, ids in states.items():
        pair = (B.Cache(L, E, cap), O.SliceLRU(L, E, cap))
        if ids is not None:
            pair[0].init_order(np.asarray(ids, np.int32))
            pair[1].init_order(np.asarray(ids, np.int32))
        miss[name] = _run(pair, dec, wdec, 0.0, first=10)["msb_miss"]
    assert miss["pcw"] < miss["last"] and miss["pcw"] < miss["random"] and miss["pcw"] < miss["empty"], miss
    assert miss["last"] <= miss["empty"] and miss["random"] <= miss["empty"], miss
    assert 2 * miss["pcw"] < min(miss["last"], miss["random"]), miss
