"""CPU-only tests of the library's host side: the C ABI loads and exports every declared symbol,
argument validation that needs no GPU, and the host bookkeeping against the oracle."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import slicemoe_oracle as O
from paper_2512_12990_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "slicemoe.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(smoe_[a-z_0-9]+)\s*\(", hdr))
    assert len(declared) >= 20
    lib = B.lib()
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(B.EXPORTS)


def test_strerror_and_bank_bytes_validation():
    lib = B.lib()
    assert lib.smoe_strerror(0) == b"ok"
    assert b"aligned" in lib.smoe_strerror(-3)
    d = B.BankDesc(64, 2048, 1408, 128, 8, 4, B.BF16, B.BF16)
    n = B.smoe_bank_bytes(d)
    # two nibble planes (= one 8-bit copy, no duplication) + 3 bytes of metadata per group; a row of
    # scales is padded to an even count (the down rows have 11 groups -> 12 stored)
    weights = 64 * 3 * 2048 * 1408
    groups = 64 * (2 * 1408 * 16 + 2048 * 11)
    pad = 64 * 2048 * 2
    assert weights + 3 * groups + pad <= n <= weights + 3 * groups + pad + 8 * 256 + 64 * 64
    nbytes = C.c_size_t()
    for bad, rc in [(B.BankDesc(0, 2048, 1408, 128, 8, 4, 0, 0), -2), (B.BankDesc(4, 2040, 1408, 128, 8, 4, 0, 0), -2),
                    (B.BankDesc(4, 2048, 1408, 100, 8, 4, 0, 0), -2), (B.BankDesc(4, 2048, 1408, 128, 8, 2, 0, 0), -6),
                    (B.BankDesc(4, 2048, 1408, 128, 4, 4, 0, 0), -2), (B.BankDesc(4, 2048, 1408, 128, 8, 4, 7, 0), -1),
                    (B.BankDesc(4, 2048, 1408, 128, 8, 4, 0, 0, 2), -1)]:
        assert lib.smoe_bank_bytes(C.byref(bad), C.byref(nbytes)) == rc
    # the lower nests store b_low bits per plane value: 3/4 and 1/2 of the plane bytes of the 8/4 nest
    for bh, bl in [(6, 3), (4, 2)]:
        nl = B.smoe_bank_bytes(B.BankDesc(64, 2048, 1408, 128, bh, bl, B.BF16, B.BF16))
        assert weights * bl // 4 + 3 * groups + pad <= nl <= weights * bl // 4 + 3 * groups + pad + 8 * 256 + 64 * 64
    assert lib.smoe_bank_bytes(None, C.byref(nbytes)) == -1
    assert lib.smoe_bank_bytes(C.byref(d), None) == -1


def test_topn_matches_oracle():
    rng = np.random.default_rng(0)
    for L, E in [(1, 4), (3, 5), (24, 60)]:
        hist = rng.integers(0, 6, size=(L, E)).astype(np.uint32)
        for n in [0, 1, L * E, L * E + 3, 2 * L * E, 2 * L * E + 10]:
            assert np.array_equal(B.smoe_topn_slices(hist, n), O.topn_slices(hist, n))


def test_cache_matches_oracle_in_lockstep():
    rng = np.random.default_rng(1)
    L, E, cap, k = 3, 16, 24, 4
    c, o = B.Cache(L, E, cap), O.SliceLRU(L, E, cap)
    hist = rng.integers(0, 9, size=(L, E)).astype(np.uint32)
    ids = O.topn_slices(hist, cap // 2)
    c.init_order(ids)
    o.init_order(ids)
    for step in range(300):
        l = int(rng.integers(L))
        idx = rng.choice(E, size=k, replace=False).astype(np.int32)
        wh = rng.integers(0, 2, size=k).astype(np.uint8)
        m1, b1 = c.snapshot(l, 1.0)
        m2, b2 = o.snapshot(l, 1.0)
        assert np.array_equal(m1, m2) and np.array_equal(b1, b2)
        c.access(l, idx, wh)
        o.access(l, idx, wh)
        assert c.order() == o.order
    assert c.stats() == o.stats
    assert len(c.order()) <= cap


def test_cache_argument_errors():
    lib = B.lib()
    h = C.c_void_p()
    assert lib.smoe_cache_create(1, 4, 1, C.byref(h)) == -2
    assert lib.smoe_cache_create(1, 4, 4, None) == -1
    c = B.Cache(2, 4, 4)
    bad = np.array([0, 9], np.int32)
    assert lib.smoe_cache_access(c.h, 0, 2, bad.ctypes.data_as(C.c_void_p), None) == -2
    assert lib.smoe_cache_access(c.h, 5, 1, bad.ctypes.data_as(C.c_void_p), None) == -2
    dup = np.array([1, 1], np.uint32)
    assert lib.smoe_cache_init_order(c.h, dup.ctypes.data_as(C.c_void_p), 2) == -1
    assert c.order() == []


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2512_12990_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".cpp", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.replace("the CPU oracle's tests", ""), f


def test_cache_all_layer_calls_match_per_layer_calls():
    """smoe_cache_snapshot_all / smoe_cache_access_all = the per-layer calls in layer order (and the oracle's LRU)."""
    rng = np.random.default_rng(3)
    L, E, cap, k = 5, 12, 30, 3
    a, b, o = B.Cache(L, E, cap), B.Cache(L, E, cap), O.SliceLRU(L, E, cap)
    masks, bias = np.empty((L, E), np.uint8), np.empty((L, E), np.float32)
    for t in range(60):
        idx = np.zeros((L, 16), np.int32)                         # padded rows, as a device buffer would have
        for l in range(L):
            idx[l, :k] = rng.choice(E, size=k, replace=False)
        want = (rng.random((L, k)) < 0.6).astype(np.uint8)
        a.snapshot_all(0.75, masks, bias)
        for l in range(L):
            m, bb = b.snapshot(l, 0.75)
            om, ob = o.snapshot(l, 0.75)
            assert np.array_equal(masks[l], m) and np.array_equal(bias[l], bb)
            assert np.array_equal(m, om) and np.array_equal(bb, ob)
        a.access_all(idx, k, want)
        for l in range(L):
            b.access(l, idx[l, :k], want[l])
            o.access(l, idx[l, :k], want[l])
        assert a.order() == b.order() == o.order and a.stats() == b.stats() == o.stats
    # an invalid index anywhere leaves the cache untouched
    bad = np.zeros((L, 16), np.int32)
    bad[L - 1, 1] = E
    before = a.order()
    with pytest.raises(B.SmoeError):
        a.access_all(bad, k, None)
    assert a.order() == before



def test_workspace_bytes_and_ctx_create_validation():
    lib = B.lib()
    # one token of the DeepSeek-V2-Lite-shaped layer: 64 KiB of records + (6 + 2) * 1408 floats
    assert B.smoe_workspace_bytes(1, 6, 1408, 2, 1408) == (64 << 10) + 8 * 1408 * 4
    # several tokens: vectors a fixed stride apart with room for the largest top-k (16)
    assert B.smoe_workspace_bytes(4, 6, 1408, 2, 1408) == (64 << 10) + 4 * (2 + 16) * 1408 * 4
    n = C.c_size_t()
    for args in [(0, 6, 1408, 2, 1408), (17, 6, 1408, 2, 1408), (1, 17, 1408, 0, 0), (1, 6, -1, 0, 0), (1, 6, 32, 9, 32)]:
        assert lib.smoe_workspace_bytes(*[C.c_int(a) for a in args], C.byref(n)) == -2
    assert lib.smoe_workspace_bytes(C.c_int(1), C.c_int(1), C.c_int(32), C.c_int(0), C.c_int(0), None) == -1
    # the context borrows its workspace: a null, misaligned or too small one is refused before any device call
    h = C.c_void_p()
    create = lib.smoe_ctx_create
    assert create(C.c_int(0), None, None, C.c_size_t(1 << 20), C.byref(h)) == -1
    assert create(C.c_int(0), None, C.c_void_p(0x1000 + 16), C.c_size_t(1 << 20), C.byref(h)) == -3
    assert create(C.c_int(0), None, C.c_void_p(0x1000), C.c_size_t(1024), C.byref(h)) == -4
    assert create(C.c_int(-1), None, C.c_void_p(0x1000), C.c_size_t(1 << 20), C.byref(h)) == -1


def test_single_launch_calls_reject_null_arguments():
    # (argument checks only: they return before any device call)
    lib = B.lib()
    n, t = C.c_longlong(), C.c_uint()
    assert lib.smoe_ctx_single_launch(None, C.c_int(1), C.c_int(0)) == -1
    assert lib.smoe_ctx_single_launch_status(None, C.byref(n), C.byref(t)) == -1


def test_no_device_allocation_in_the_library_sources():
    # the boundary's rule: device memory belongs to the caller
    csrc = os.path.join(ROOT, "paper_2512_12990_amd", "csrc")
    for name in os.listdir(csrc):
        text = open(os.path.join(csrc, name)).read()
        for call in ("hipMalloc", "hipFree", "hipMallocAsync", "hipExtMallocWithFlags", "hipHostMalloc"):
            assert not re.search(r"\b%s\s*\(" % call, text), (name, call)


def test_entry_division_is_exact_for_every_accepted_split(tmp_path):
    # The decode kernels turn an entry index into (slot, position) with a multiply-high by a launch
    # constant (csrc/fastdiv.hpp).  Checked here against integer division for EVERY row-pair count per
    # slot (cap) and every entry index the host lets through (slots * cap below the stated limit).
    src = tmp_path / "fastdiv_check.cpp"
    src.write_text(r'''
#include "fastdiv.hpp"
#include <stdio.h>
int main() {
  long long n = 0;
  for (int cap = 1; cap < SMOE_FASTDIV_LIMIT; cap++) {
    const uint32_t m = fastdiv_magic(cap);
    for (int e = 0; e < SMOE_FASTDIV_LIMIT; e++) {
      const int s = fastdiv(e, m);
      if (s != e / cap || e - s * cap != e % cap) { printf("FAIL cap=%d e=%d got %d want %d\n", cap, e, s, e / cap); return 1; }
      n++;
    }
  }
  printf("ok %lld\n", n);
  return 0;
}
''')
    exe = tmp_path / "fastdiv_check"
    import subprocess
    subprocess.run(["g++", "-O2", "-I", os.path.join(ROOT, "paper_2512_12990_amd", "csrc"), str(src), "-o", str(exe)], check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0 and r.stdout.startswith("ok"), r.stdout
