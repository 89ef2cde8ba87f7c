"""Thin ctypes binding of libslicemoe.so: argument marshalling only.

Every function has the name and meaning of the C entry point in include/slicemoe.h; torch
tensors are used for device memory and the current stream only.  There is no CPU fallback:
if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libslicemoe.so")

F32, BF16 = 0, 1
_DT = {torch.float32: F32, torch.bfloat16: BF16, "f32": F32, "bf16": BF16}


class SmoeError(RuntimeError):
    pass


class BankDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_experts", "d_model", "d_ff", "group", "b_high", "b_low", "w_dtype", "scale_dtype", "symmetric")]


class CacheStats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("msb_hit", "msb_miss", "lsb_hit", "lsb_miss")]


class SystemSpec(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("flash_gbit_s", "dram_gbit_s", "xpu_tops", "flash_pj_bit", "dram_pj_bit",
                                          "xpu_tops_w")]


class Cost(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("flash_bits", "dram_bits", "ops", "energy_j", "latency_s", "miss_rate_high")]


_lib = None

EXPORTS = [
    "smoe_workspace_bytes", "smoe_ctx_create", "smoe_ctx_destroy", "smoe_strerror", "smoe_last_hip_error", "smoe_ctx_timing",
    "smoe_ctx_timing_read", "smoe_stream_read", "smoe_ctx_single_launch", "smoe_ctx_single_launch_status",
    "smoe_bank_bytes", "smoe_bank_create", "smoe_bank_destroy", "smoe_quantize_slice", "smoe_export_codes",
    "smoe_route", "smoe_expert_ffn", "smoe_decode_layer", "smoe_decode_layer_multi", "smoe_static_scratch_bytes", "smoe_decode_layer_static",
    "smoe_prefill_bytes", "smoe_prefill_histogram", "smoe_topn_slices",
    "smoe_cache_create", "smoe_cache_destroy", "smoe_cache_init_order", "smoe_cache_snapshot",
    "smoe_cache_access", "smoe_cache_snapshot_all", "smoe_cache_access_all", "smoe_cache_stats_get", "smoe_cache_order",
    "smoe_system_spec_paper", "smoe_cost_model",
]


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise SmoeError("libslicemoe.so is not built: run `python -m paper_2512_12990_amd.build` "
                            "(there is no CPU fallback)")
        _lib = C.CDLL(LIB_PATH)
        _lib.smoe_strerror.restype = C.c_char_p
        _lib.smoe_strerror.argtypes = [C.c_int]
        for name in EXPORTS:
            getattr(_lib, name)            # fail loudly on a missing symbol
    return _lib


def _chk(rc: int, what: str, ctx=None):
    if rc != 0:
        msg = lib().smoe_strerror(rc).decode()
        if ctx is not None and rc == -5:
            msg += " (hipError %d)" % lib().smoe_last_hip_error(ctx)
        raise SmoeError("%s failed: %s [%d]" % (what, msg, rc))


def _p(t: Optional[torch.Tensor]):
    if t is None:
        return C.c_void_p(0)
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA/HIP tensors"
    return C.c_void_p(t.data_ptr())


def smoe_workspace_bytes(tokens: int, k: int, d_ff: int, n_shared: int = 0, shared_d_ff: int = 0) -> int:
    n = C.c_size_t()
    _chk(lib().smoe_workspace_bytes(C.c_int(tokens), C.c_int(k), C.c_int(d_ff), C.c_int(n_shared), C.c_int(shared_d_ff),
                                    C.byref(n)), "smoe_workspace_bytes")
    return n.value


class Ctx:
    """A library context; the torch tensor `workspace` owns the device workspace it borrows."""

    def __init__(self, device: int = 0, stream: Optional[torch.cuda.Stream] = None, workspace_bytes: int = 4 << 20):
        self.device = device
        s = stream if stream is not None else torch.cuda.current_stream(device)
        self._stream = s
        self.workspace, base = None, 0
        if workspace_bytes:                       # 0: a context for the calls that need no workspace
            self.workspace = torch.empty(workspace_bytes + 256, dtype=torch.uint8, device="cuda:%d" % device)
            base = self.workspace.data_ptr() + (-self.workspace.data_ptr()) % 256
        self.h = C.c_void_p()
        _chk(lib().smoe_ctx_create(C.c_int(device), C.c_void_p(s.cuda_stream), C.c_void_p(base),
                                   C.c_size_t(workspace_bytes), C.byref(self.h)), "smoe_ctx_create")

    def timing(self, enable: bool):
        _chk(lib().smoe_ctx_timing(self.h, C.c_int(int(enable))), "smoe_ctx_timing")

    def timing_read(self):
        """(gateup_us_sum, down_us_sum, n_calls) since the last read; synchronises."""
        g, d, n = C.c_double(), C.c_double(), C.c_int()
        _chk(lib().smoe_ctx_timing_read(self.h, C.byref(g), C.byref(d), C.byref(n)), "smoe_ctx_timing_read", self.h)
        return g.value, d.value, n.value

    def single_launch(self, enable: bool, spin_limit: int = 0):
        """One kernel launch per decode call where the case fits (see smoe_ctx_single_launch)."""
        _chk(lib().smoe_ctx_single_launch(self.h, C.c_int(int(enable)), C.c_int(spin_limit)), "smoe_ctx_single_launch", self.h)

    def single_launch_status(self):
        """(decode calls that took the single launch, work-groups that gave up waiting); synchronises."""
        n, t = C.c_longlong(), C.c_uint()
        _chk(lib().smoe_ctx_single_launch_status(self.h, C.byref(n), C.byref(t)), "smoe_ctx_single_launch_status", self.h)
        return n.value, t.value

    def close(self):
        if self.h:
            lib().smoe_ctx_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def smoe_bank_bytes(desc: BankDesc) -> int:
    n = C.c_size_t()
    _chk(lib().smoe_bank_bytes(C.byref(desc), C.byref(n)), "smoe_bank_bytes")
    return n.value


class Bank:
    """A sliced expert store; the torch tensor `store` owns the device memory."""

    def __init__(self, ctx: Ctx, n_experts, d_model, d_ff, group, w_dtype="f32", scale_dtype="f32", b_high=8, b_low=4,
                 symmetric=False):
        self.ctx = ctx
        self.desc = BankDesc(n_experts, d_model, d_ff, group, b_high, b_low, _DT[w_dtype], _DT[scale_dtype], int(symmetric))
        self.nbytes = smoe_bank_bytes(self.desc)
        self.store = torch.empty(self.nbytes + 256, dtype=torch.uint8, device="cuda:%d" % ctx.device)
        off = (-self.store.data_ptr()) % 256
        self._base = self.store.data_ptr() + off
        self.h = C.c_void_p()
        _chk(lib().smoe_bank_create(ctx.h, C.byref(self.desc), C.c_void_p(self._base), C.c_size_t(self.nbytes),
                                    C.byref(self.h)), "smoe_bank_create", ctx.h)

    def close(self):
        if self.h:
            lib().smoe_bank_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def smoe_quantize_slice(ctx: Ctx, bank: Bank, e0: int, w_gate: torch.Tensor, w_up: torch.Tensor, w_down: torch.Tensor):
    """w_gate/w_up [n, d_ff, d_model], w_down [n, d_model, d_ff] on the device, dtype = bank w_dtype."""
    n = w_gate.shape[0]
    d, f = bank.desc.d_model, bank.desc.d_ff
    assert tuple(w_gate.shape) == (n, f, d) and tuple(w_up.shape) == (n, f, d) and tuple(w_down.shape) == (n, d, f)
    want = torch.float32 if bank.desc.w_dtype == F32 else torch.bfloat16
    assert w_gate.dtype == want and w_up.dtype == want and w_down.dtype == want
    _chk(lib().smoe_quantize_slice(ctx.h, bank.h, C.c_int(e0), C.c_int(n), _p(w_gate), _p(w_up), _p(w_down)),
         "smoe_quantize_slice", ctx.h)


def smoe_export_codes(ctx: Ctx, bank: Bank, expert: int, matrix: int):
    """Returns dict(q, msb, lsb [N,K] uint8; zp [N,ng] uint8; scale [N,ng] fp32) as numpy arrays."""
    d, f, G = bank.desc.d_model, bank.desc.d_ff, bank.desc.group
    N, K = (d, f) if matrix == 2 else (f, d)
    ng = -(-K // G)
    out = dict(q=np.empty((N, K), np.uint8), msb=np.empty((N, K), np.uint8), lsb=np.empty((N, K), np.uint8),
               zp=np.empty((N, ng), np.uint8), scale=np.empty((N, ng), np.float32))
    ptr = lambda a: a.ctypes.data_as(C.c_void_p)
    _chk(lib().smoe_export_codes(ctx.h, bank.h, C.c_int(expert), C.c_int(matrix), ptr(out["q"]), ptr(out["msb"]),
                                 ptr(out["lsb"]), ptr(out["zp"]), ptr(out["scale"])), "smoe_export_codes", ctx.h)
    return out


def smoe_route(ctx: Ctx, k: int, logits: Optional[torch.Tensor] = None, x: Optional[torch.Tensor] = None,
               w_router: Optional[torch.Tensor] = None, bias: Optional[torch.Tensor] = None, norm_topk: bool = False,
               routed_scale: float = 1.0, want_logits: bool = False):
    dev = "cuda:%d" % ctx.device
    if logits is not None:
        T, E = logits.shape
        d = 0
        act = F32
    else:
        T, d = x.shape
        E = w_router.shape[0]
        act = _DT[x.dtype]
    idx = torch.empty((T, k), dtype=torch.int32, device=dev)
    w = torch.empty((T, k), dtype=torch.float32, device=dev)
    zout = torch.empty((T, E), dtype=torch.float32, device=dev) if want_logits else None
    _chk(lib().smoe_route(ctx.h, C.c_int(T), C.c_int(E), C.c_int(k), C.c_int(d), _p(logits), _p(x), C.c_int(act),
                          _p(w_router), _p(bias), C.c_int(int(norm_topk)), C.c_float(routed_scale), _p(zout),
                          _p(idx), _p(w)), "smoe_route", ctx.h)
    return (idx, w, zout) if want_logits else (idx, w)


def smoe_expert_ffn(ctx: Ctx, routed: Optional[Bank], shared: Optional[Bank], x: torch.Tensor, idx, w, slice_mask,
                    tau_head: float = 0.0, shared_gate_w=None, add_residual: bool = False, y=None, prec_out=None):
    k = 0 if idx is None else idx.numel()
    if y is None:
        y = torch.empty_like(x)
    _chk(lib().smoe_expert_ffn(ctx.h, routed.h if routed else None, shared.h if shared else None, _p(x),
                               C.c_int(_DT[x.dtype]), C.c_int(k), _p(idx), _p(w), _p(slice_mask),
                               C.c_float(tau_head), _p(shared_gate_w), C.c_int(int(add_residual)), _p(y),
                               _p(prec_out)), "smoe_expert_ffn", ctx.h)
    return y


def smoe_decode_layer(ctx: Ctx, routed: Bank, shared: Optional[Bank], x: torch.Tensor, k: int, logits=None,
                      w_router=None, bias=None, norm_topk: bool = False, routed_scale: float = 1.0, slice_mask=None,
                      tau_head: float = 0.0, shared_gate_w=None, add_residual: bool = False, y=None, idx_out=None,
                      w_out=None, prec_out=None):
    if y is None:
        y = torch.empty_like(x)
    _chk(lib().smoe_decode_layer(ctx.h, routed.h, shared.h if shared else None, _p(x), C.c_int(_DT[x.dtype]),
                                 C.c_int(k), _p(logits), _p(w_router), _p(bias), C.c_int(int(norm_topk)),
                                 C.c_float(routed_scale), _p(slice_mask), C.c_float(tau_head), _p(shared_gate_w),
                                 C.c_int(int(add_residual)), _p(y), _p(idx_out), _p(w_out), _p(prec_out)),
         "smoe_decode_layer", ctx.h)
    return y


def smoe_static_scratch_bytes() -> int:
    n = C.c_size_t()
    _chk(lib().smoe_static_scratch_bytes(C.byref(n)), "smoe_static_scratch_bytes")
    return n.value


def smoe_decode_layer_static(ctx: Ctx, routed: Bank, shared: Optional[Bank], x: torch.Tensor, k: int, y: torch.Tensor,
                             logits=None, w_router=None, bias=None, norm_topk: bool = False, routed_scale: float = 1.0,
                             slice_mask=None, tau_head: float = 0.0, shared_gate_w=None, add_residual: bool = False,
                             idx_out=None, w_out=None, prec_out=None):
    """smoe_decode_layer over the library's static workspace; the caller passes every buffer (y included)."""
    _chk(lib().smoe_decode_layer_static(ctx.h, routed.h, shared.h if shared else None, _p(x), C.c_int(_DT[x.dtype]),
                                        C.c_int(k), _p(logits), _p(w_router), _p(bias), C.c_int(int(norm_topk)),
                                        C.c_float(routed_scale), _p(slice_mask), C.c_float(tau_head), _p(shared_gate_w),
                                        C.c_int(int(add_residual)), _p(y), _p(idx_out), _p(w_out), _p(prec_out)),
         "smoe_decode_layer_static", ctx.h)
    return y


def smoe_decode_layer_multi(ctx: Ctx, routed: Bank, shared: Optional[Bank], x: torch.Tensor, k: int, logits: torch.Tensor,
                            bias=None, norm_topk: bool = False, routed_scale: float = 1.0, slice_mask=None,
                            tau_head: float = 0.0, shared_gate_w=None, add_residual: bool = False, y=None, idx_out=None,
                            w_out=None, prec_out=None):
    T = x.shape[0]
    if y is None:
        y = torch.empty_like(x)
    _chk(lib().smoe_decode_layer_multi(ctx.h, routed.h, shared.h if shared else None, C.c_int(T), _p(x),
                                       C.c_int(_DT[x.dtype]), C.c_int(k), _p(logits), _p(bias), C.c_int(int(norm_topk)),
                                       C.c_float(routed_scale), _p(slice_mask), C.c_float(tau_head), _p(shared_gate_w),
                                       C.c_int(int(add_residual)), _p(y), _p(idx_out), _p(w_out), _p(prec_out)),
         "smoe_decode_layer_multi", ctx.h)
    return y


def smoe_prefill_bytes(T, E, k, d_model, d_ff, shared_d_ff=0) -> int:
    n = C.c_size_t()
    _chk(lib().smoe_prefill_bytes(C.c_int(T), C.c_int(E), C.c_int(k), C.c_int(d_model), C.c_int(d_ff),
                                  C.c_int(shared_d_ff), C.byref(n)), "smoe_prefill_bytes")
    return n.value


def smoe_prefill_histogram(ctx: Ctx, routed: Bank, shared: Optional[Bank], x: torch.Tensor, k: int, logits=None,
                           w_router=None, norm_topk=False, routed_scale=1.0, shared_gate_w=None, add_residual=False,
                           scratch: Optional[torch.Tensor] = None):
    T, d = x.shape
    E = routed.desc.n_experts
    dev = x.device
    need = smoe_prefill_bytes(T, E, k, d, routed.desc.d_ff, shared.desc.d_ff if shared else 0)
    if scratch is None:
        scratch = torch.empty(need, dtype=torch.uint8, device=dev)
    y = torch.empty_like(x)
    idx = torch.empty((T, k), dtype=torch.int32, device=dev)
    w = torch.empty((T, k), dtype=torch.float32, device=dev)
    hist = torch.empty((E,), dtype=torch.int32, device=dev)     # bit pattern of uint32 counts
    _chk(lib().smoe_prefill_histogram(ctx.h, routed.h, shared.h if shared else None, C.c_int(T), _p(x),
                                      C.c_int(_DT[x.dtype]), C.c_int(k), _p(logits), _p(w_router),
                                      C.c_int(int(norm_topk)), C.c_float(routed_scale), _p(shared_gate_w),
                                      C.c_int(int(add_residual)), _p(scratch), C.c_size_t(scratch.numel()), _p(y),
                                      _p(idx), _p(w), _p(hist)), "smoe_prefill_histogram", ctx.h)
    return y, idx, w, hist


# ---- host-only calls ----------------------------------------------------------------------------
def smoe_topn_slices(hist: np.ndarray, n: int) -> np.ndarray:
    hist = np.ascontiguousarray(hist, dtype=np.uint32)
    L, E = hist.shape
    out = np.empty(max(1, min(n, 2 * L * E)), np.uint32)
    cnt = C.c_int()
    _chk(lib().smoe_topn_slices(hist.ctypes.data_as(C.c_void_p), C.c_int(L), C.c_int(E), C.c_int(n),
                                out.ctypes.data_as(C.c_void_p), C.byref(cnt)), "smoe_topn_slices")
    return out[: cnt.value].copy()


def smoe_system_spec_paper() -> SystemSpec:
    spec = SystemSpec()
    _chk(lib().smoe_system_spec_paper(C.byref(spec)), "smoe_system_spec_paper")
    return spec


def smoe_cost_model(spec: SystemSpec, stats: dict, msb_slice_bytes: int, lsb_slice_bytes: int, ops: float) -> dict:
    st = CacheStats(stats["msb_hit"], stats["msb_miss"], stats["lsb_hit"], stats["lsb_miss"])
    out = Cost()
    _chk(lib().smoe_cost_model(C.byref(spec), C.byref(st), C.c_uint64(msb_slice_bytes), C.c_uint64(lsb_slice_bytes),
                               C.c_double(ops), C.byref(out)), "smoe_cost_model")
    return {n: getattr(out, n) for n, _ in Cost._fields_}


class Cache:
    def __init__(self, L: int, E: int, capacity: int):
        self.L, self.E, self.cap = L, E, capacity
        self.h = C.c_void_p()
        _chk(lib().smoe_cache_create(C.c_int(L), C.c_int(E), C.c_int(capacity), C.byref(self.h)), "smoe_cache_create")

    def init_order(self, slice_ids):
        a = np.ascontiguousarray(slice_ids, dtype=np.uint32)
        _chk(lib().smoe_cache_init_order(self.h, a.ctypes.data_as(C.c_void_p), C.c_int(a.size)), "smoe_cache_init_order")

    def snapshot(self, layer: int, beta: float):
        mask = np.empty(self.E, np.uint8)
        bias = np.empty(self.E, np.float32)
        _chk(lib().smoe_cache_snapshot(self.h, C.c_int(layer), C.c_float(beta), mask.ctypes.data_as(C.c_void_p),
                                       bias.ctypes.data_as(C.c_void_p)), "smoe_cache_snapshot")
        return mask, bias

    def access(self, layer: int, idx, want_high):
        i = np.ascontiguousarray(idx, dtype=np.int32)
        wh = np.ascontiguousarray(want_high, dtype=np.uint8)
        _chk(lib().smoe_cache_access(self.h, C.c_int(layer), C.c_int(i.size), i.ctypes.data_as(C.c_void_p),
                                     wh.ctypes.data_as(C.c_void_p)), "smoe_cache_access")

    def snapshot_all(self, beta: float, mask_out: np.ndarray, bias_out: Optional[np.ndarray] = None):
        """Masks (uint8 [L, E]) and routing bias (float32 [L, E]) of all layers into the caller's arrays."""
        assert mask_out.dtype == np.uint8 and mask_out.flags.c_contiguous and mask_out.size == self.L * self.E
        bp = None
        if bias_out is not None:
            assert bias_out.dtype == np.float32 and bias_out.flags.c_contiguous and bias_out.size == self.L * self.E
            bp = bias_out.ctypes.data_as(C.c_void_p)
        _chk(lib().smoe_cache_snapshot_all(self.h, C.c_float(beta), mask_out.ctypes.data_as(C.c_void_p), bp),
             "smoe_cache_snapshot_all")

    def access_all(self, idx: np.ndarray, k: int, want_high: Optional[np.ndarray] = None):
        """One token's selections in all layers: idx int32 [L, stride >= k] (C-contiguous), want_high uint8 [L, k]."""
        assert idx.dtype == np.int32 and idx.flags.c_contiguous and idx.shape[0] == self.L and idx.shape[1] >= k
        wp = None
        if want_high is not None:
            wh = np.ascontiguousarray(want_high, dtype=np.uint8)
            assert wh.size == self.L * k
            wp = wh.ctypes.data_as(C.c_void_p)
        _chk(lib().smoe_cache_access_all(self.h, C.c_int(k), idx.ctypes.data_as(C.c_void_p), C.c_int(idx.shape[1]), wp),
             "smoe_cache_access_all")

    def stats(self) -> dict:
        s = CacheStats()
        _chk(lib().smoe_cache_stats_get(self.h, C.byref(s)), "smoe_cache_stats_get")
        return dict(msb_hit=s.msb_hit, msb_miss=s.msb_miss, lsb_hit=s.lsb_hit, lsb_miss=s.lsb_miss)

    def order(self) -> list:
        out = np.empty(max(1, self.cap), np.uint32)
        n = C.c_int()
        _chk(lib().smoe_cache_order(self.h, out.ctypes.data_as(C.c_void_p), C.c_int(self.cap), C.byref(n)),
             "smoe_cache_order")
        return out[: n.value].tolist()

    def close(self):
        if self.h:
            lib().smoe_cache_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
