"""ctypes binding of libmadakv.so: argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI (include/madakv.h).
torch is used for device memory and streams.  There is no CPU fallback: if the library
has not been built, loading fails.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmadakv.so")

FP32, BF16 = 0, 1
OK = 0
STATUS = {0: "OK", -1: "INVALID_ARG", -2: "BAD_SHAPE", -3: "BAD_BUDGET", -4: "WORKSPACE_TOO_SMALL",
          -5: "UNSUPPORTED_DTYPE", -6: "HIP_ERROR", -7: "UNIMPLEMENTED"}


class Config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("batch", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("ctx_len", C.c_int32),
                ("window", C.c_int32), ("budget", C.c_int32), ("dtype", C.c_int32),
                ("pool_k", C.c_int32), ("mpa_mode", C.c_int32), ("hcc_mode", C.c_int32),
                ("hcc_rho", C.c_int32), ("theta", C.c_float), ("softmax_scale", C.c_float),
                ("max_new_tokens", C.c_int32), ("out_fp32", C.c_int32), ("pool_mode", C.c_int32),
                ("share_mode", C.c_int32), ("select_mode", C.c_int32), ("sink_tokens", C.c_int32),
                ("cache_fp8", C.c_int32), ("n_modalities", C.c_int32), ("page_rows", C.c_int32)]


class MadaKVError(RuntimeError):
    def __init__(self, call: str, status: int):
        super().__init__(f"{call} -> {status} ({STATUS.get(status, '?')})")
        self.status = status


_lib = None


def lib() -> C.CDLL:
    """The loaded library.  Raises if it was never built (python -m paper_2506_15724_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -m paper_2506_15724_amd.build` first")
        L = C.CDLL(LIB_PATH)
        vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
        L.madakv_create.argtypes = [C.POINTER(Config), C.POINTER(vp)]
        L.madakv_destroy.argtypes = [vp]
        L.madakv_last_hip_error.argtypes = [vp]
        L.madakv_workspace_bytes.argtypes = [vp, i32, C.POINTER(sz), C.POINTER(sz), C.POINTER(sz)]
        L.madakv_compact_capacity_tokens.argtypes = [vp, C.POINTER(C.c_int64)]
        L.madakv_score.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.madakv_score_lse.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.madakv_allocate.argtypes = [vp, i32, i32, vp, vp, vp, vp]
        L.madakv_select_gather.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.madakv_evict.argtypes = [vp, i32, i32] + [vp] * 14 + [vp, sz, vp, sz, vp]
        L.madakv_decode_attn.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.madakv_decode_attn_static.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.madakv_page_table.argtypes = [vp, C.POINTER(vp), C.POINTER(i32)]
        L.madakv_window_attn_workspace_bytes.argtypes = [vp, i32, C.POINTER(sz)]
        L.madakv_window_attn_score.argtypes = [vp, i32, i32] + [vp] * 10 + [vp, sz, vp]
        L.madakv_reevict_workspace_bytes.argtypes = [vp, i32, C.POINTER(sz)]
        L.madakv_reevict.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        for name in EXPORTS:
            getattr(L, name).restype = i32
        _lib = L
    return _lib


EXPORTS = ["madakv_create", "madakv_destroy", "madakv_last_hip_error", "madakv_workspace_bytes",
           "madakv_compact_capacity_tokens", "madakv_score", "madakv_score_lse", "madakv_allocate", "madakv_select_gather", "madakv_evict",
           "madakv_decode_attn", "madakv_decode_attn_static", "madakv_page_table",
           "madakv_reevict_workspace_bytes", "madakv_reevict", "madakv_window_attn_workspace_bytes", "madakv_window_attn_score"]


def _ptr(t):
    if t is None:
        return None
    assert t.is_contiguous(), "tensors passed to the library must be contiguous"
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(call, rc):
    if rc != OK:
        raise MadaKVError(call, rc)


# ---- the C calls, name for name ------------------------------------------------------
def madakv_create(cfg: Config):
    h = C.c_void_p()
    _check("madakv_create", lib().madakv_create(C.byref(cfg), C.byref(h)))
    return h


def madakv_destroy(h):
    _check("madakv_destroy", lib().madakv_destroy(h))


def madakv_workspace_bytes(h, n_layers_per_call: int):
    a, b, c = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check("madakv_workspace_bytes", lib().madakv_workspace_bytes(h, n_layers_per_call, C.byref(a), C.byref(b), C.byref(c)))
    return a.value, b.value, c.value


def madakv_compact_capacity_tokens(h) -> int:
    t = C.c_int64()
    _check("madakv_compact_capacity_tokens", lib().madakv_compact_capacity_tokens(h, C.byref(t)))
    return t.value


def madakv_score(h, layer0, n, q_win, k, mask, psi, psi_pool, stats, n_mod, ws):
    _check("madakv_score", lib().madakv_score(h, layer0, n, _ptr(q_win), _ptr(k), _ptr(mask), _ptr(psi), _ptr(psi_pool),
                                              _ptr(stats), _ptr(n_mod), _ptr(ws), ws.numel() * ws.element_size(), _stream()))


def madakv_score_lse(h, layer0, n, q_win, k, mask, row_lse, psi, psi_pool, stats, n_mod, ws):
    _check("madakv_score_lse", lib().madakv_score_lse(h, layer0, n, _ptr(q_win), _ptr(k), _ptr(mask), _ptr(row_lse), _ptr(psi),
                                                      _ptr(psi_pool), _ptr(stats), _ptr(n_mod), _ptr(ws),
                                                      ws.numel() * ws.element_size(), _stream()))


def madakv_allocate(h, layer0, n, stats, n_mod, budgets):
    _check("madakv_allocate", lib().madakv_allocate(h, layer0, n, _ptr(stats), _ptr(n_mod), _ptr(budgets), _stream()))


def madakv_select_gather(h, layer0, n, psi_pool, mask, budgets, k, v, kept_idx, kv_off, kv_len, k_c, v_c, ws):
    _check("madakv_select_gather", lib().madakv_select_gather(
        h, layer0, n, _ptr(psi_pool), _ptr(mask), _ptr(budgets), _ptr(k), _ptr(v), _ptr(kept_idx), _ptr(kv_off),
        _ptr(kv_len), _ptr(k_c), _ptr(v_c), _ptr(ws), ws.numel() * ws.element_size(), _stream()))


def madakv_evict(h, layer0, n, q_win, k, v, mask, psi, psi_pool, stats, n_mod, budgets, kept_idx, kv_off, kv_len, k_c, v_c,
                 score_ws, select_ws):
    _check("madakv_evict", lib().madakv_evict(
        h, layer0, n, _ptr(q_win), _ptr(k), _ptr(v), _ptr(mask), _ptr(psi), _ptr(psi_pool), _ptr(stats), _ptr(n_mod),
        _ptr(budgets), _ptr(kept_idx), _ptr(kv_off), _ptr(kv_len), _ptr(k_c), _ptr(v_c),
        _ptr(score_ws), score_ws.numel() * score_ws.element_size(), _ptr(select_ws),
        select_ws.numel() * select_ws.element_size(), _stream()))


def madakv_decode_attn(h, layer0, n, q, k_new, v_new, k_c, v_c, kv_off, kv_len, out, ws):
    _check("madakv_decode_attn", lib().madakv_decode_attn(
        h, layer0, n, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_c), _ptr(v_c), _ptr(kv_off), _ptr(kv_len),
        _ptr(out), _ptr(ws), ws.numel() * ws.element_size(), _stream()))


def madakv_decode_attn_static(h, layer0, n, q, k_new, v_new, k_c, v_c, kv_off, kv_len, out):
    _check("madakv_decode_attn_static", lib().madakv_decode_attn_static(
        h, layer0, n, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_c), _ptr(v_c), _ptr(kv_off), _ptr(kv_len), _ptr(out), _stream()))


def madakv_window_attn_workspace_bytes(h, n_layers_per_call: int) -> int:
    b = C.c_size_t()
    _check("madakv_window_attn_workspace_bytes", lib().madakv_window_attn_workspace_bytes(h, n_layers_per_call, C.byref(b)))
    return b.value


def madakv_window_attn_score(h, layer0, n, q_win, k, v, mask, out, row_lse, psi, psi_pool, stats, n_mod, ws):
    _check("madakv_window_attn_score", lib().madakv_window_attn_score(
        h, layer0, n, _ptr(q_win), _ptr(k), _ptr(v), _ptr(mask), _ptr(out), _ptr(row_lse), _ptr(psi), _ptr(psi_pool),
        _ptr(stats), _ptr(n_mod), _ptr(ws), ws.numel() * ws.element_size(), _stream()))


def madakv_reevict_workspace_bytes(h, n_layers_per_call: int) -> int:
    b = C.c_size_t()
    _check("madakv_reevict_workspace_bytes", lib().madakv_reevict_workspace_bytes(h, n_layers_per_call, C.byref(b)))
    return b.value


def madakv_reevict(h, layer0, n, q_recent, mask, k_c, v_c, kept_idx, kv_off, kv_len, budgets, ws):
    _check("madakv_reevict", lib().madakv_reevict(
        h, layer0, n, _ptr(q_recent), _ptr(mask), _ptr(k_c), _ptr(v_c), _ptr(kept_idx), _ptr(kv_off), _ptr(kv_len),
        _ptr(budgets), _ptr(ws), ws.numel() * ws.element_size(), _stream()))


def madakv_page_table(h):
    """(device address of the page table or None, entries per head)"""
    ptr, n = C.c_void_p(), C.c_int32()
    _check("madakv_page_table", lib().madakv_page_table(h, C.byref(ptr), C.byref(n)))
    return ptr.value, n.value


# ---- a thin holder for the handle and the buffers a full run needs -------------------
class MadaKV:
    """Owns one library handle plus the device buffers of the interface (allocated with
    torch).  Methods forward to the C calls; nothing is computed here."""

    def __init__(self, *, n_layers, batch, n_q_heads, n_kv_heads, head_dim, ctx_len, window, budget,
                 dtype="bf16", pool_k=7, mpa_mode=1, hcc_mode=1, hcc_rho=2, theta=0.9, softmax_scale=0.0,
                 max_new_tokens=0, out_fp32=1, pool_mode=0, share_mode=0, select_mode=0, sink_tokens=4,
                 n_modalities=2, cache_fp8=0, page_rows=0, layers_per_call=None, device="cuda:0"):
        self.cfg = Config(n_layers, batch, n_q_heads, n_kv_heads, head_dim, ctx_len, window, budget,
                          BF16 if dtype == "bf16" else FP32, pool_k, mpa_mode, hcc_mode, hcc_rho, theta,
                          softmax_scale, max_new_tokens, out_fp32, pool_mode, share_mode, select_mode, sink_tokens, cache_fp8, n_modalities, page_rows)
        self.device = torch.device(device)
        self.tdtype = torch.bfloat16 if dtype == "bf16" else torch.float32
        with torch.cuda.device(self.device):
            self.h = madakv_create(self.cfg)
        self.n_call = layers_per_call or n_layers
        s_ws, sel_ws, d_ws = madakv_workspace_bytes(self.h, self.n_call)
        d1 = madakv_workspace_bytes(self.h, 1)[2]
        dev = self.device
        self.score_ws = torch.empty(max(s_ws, 16), dtype=torch.uint8, device=dev)
        self.select_ws = torch.empty(max(sel_ws, 16), dtype=torch.uint8, device=dev)
        self.decode_ws = torch.empty(max(d_ws, d1, 16), dtype=torch.uint8, device=dev)
        NL, B, H, L, W = n_layers, batch, n_kv_heads, ctx_len, window
        M = self.M = n_modalities
        self.psi = torch.empty(NL, B, H, L, dtype=torch.float32, device=dev)
        self.psi_pool = torch.empty(NL, B, H, L - W, dtype=torch.float32, device=dev)
        self.stats = torch.empty(NL, B, H, 2 * M, dtype=torch.int32, device=dev)  # {f32 w[M]; i32 k[M]}
        self.n_mod = torch.empty(B, M, dtype=torch.int32, device=dev)
        self.budgets = torch.empty(NL, B, H, M, dtype=torch.int32, device=dev)
        self.capacity = madakv_compact_capacity_tokens(self.h)
        self.kept_idx = torch.empty(self.capacity, dtype=torch.int32, device=dev)
        self.kv_off = torch.empty(NL, B, H, dtype=torch.int64, device=dev)
        self.kv_len = torch.empty(NL, B, H, dtype=torch.int32, device=dev)
        cdt = torch.uint8 if cache_fp8 else self.tdtype
        self.k_c = torch.empty(self.capacity, head_dim, dtype=cdt, device=dev)
        self.v_c = torch.empty(self.capacity, head_dim, dtype=cdt, device=dev)

    def close(self):
        if self.h is not None:
            madakv_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # layer-range views of the interface buffers
    def _sl(self, t, l0, n):
        return t[l0:l0 + n]

    def score(self, l0, n, q_win, k, mask):
        madakv_score(self.h, l0, n, q_win, k, mask, self._sl(self.psi, l0, n), self._sl(self.psi_pool, l0, n),
                     self._sl(self.stats, l0, n), self.n_mod, self.score_ws)

    def score_lse(self, l0, n, q_win, k, mask, row_lse):
        madakv_score_lse(self.h, l0, n, q_win, k, mask, row_lse, self._sl(self.psi, l0, n), self._sl(self.psi_pool, l0, n),
                         self._sl(self.stats, l0, n), self.n_mod, self.score_ws)

    def allocate(self, l0, n, stats=None, n_mod=None, budgets=None):
        madakv_allocate(self.h, l0, n, self._sl(self.stats, l0, n) if stats is None else stats,
                        self.n_mod if n_mod is None else n_mod,
                        self._sl(self.budgets, l0, n) if budgets is None else budgets)

    def select_gather(self, l0, n, k, v, mask, psi_pool=None, budgets=None):
        madakv_select_gather(self.h, l0, n, self._sl(self.psi_pool, l0, n) if psi_pool is None else psi_pool, mask,
                             self._sl(self.budgets, l0, n) if budgets is None else budgets, k, v, self.kept_idx,
                             self._sl(self.kv_off, l0, n), self._sl(self.kv_len, l0, n), self.k_c, self.v_c,
                             self.select_ws)

    def evict(self, l0, n, q_win, k, v, mask):
        madakv_evict(self.h, l0, n, q_win, k, v, mask, self._sl(self.psi, l0, n), self._sl(self.psi_pool, l0, n),
                     self._sl(self.stats, l0, n), self.n_mod, self._sl(self.budgets, l0, n), self.kept_idx,
                     self._sl(self.kv_off, l0, n), self._sl(self.kv_len, l0, n), self.k_c, self.v_c,
                     self.score_ws, self.select_ws)

    def _check_out(self, out, numel):
        """`out` is written in the handle's output type: a buffer of another type or size would be overrun."""
        want = torch.float32 if self.cfg.out_fp32 else self.tdtype
        if out.dtype != want or out.numel() < numel:
            raise ValueError(f"out must hold {numel} elements of {want} (out_fp32={self.cfg.out_fp32}); got {out.numel()} of {out.dtype}")

    def decode_attn(self, l0, n, q, k_new, v_new, out):
        self._check_out(out, n * self.cfg.batch * self.cfg.n_q_heads * self.cfg.head_dim)
        madakv_decode_attn(self.h, l0, n, q, k_new, v_new, self.k_c, self.v_c, self._sl(self.kv_off, l0, n),
                           self._sl(self.kv_len, l0, n), out, self.decode_ws)

    def decode_attn_static(self, l0, n, q, k_new, v_new, out):
        self._check_out(out, n * self.cfg.batch * self.cfg.n_q_heads * self.cfg.head_dim)
        madakv_decode_attn_static(self.h, l0, n, q, k_new, v_new, self.k_c, self.v_c, self._sl(self.kv_off, l0, n),
                                  self._sl(self.kv_len, l0, n), out)

    def window_attn_score(self, l0, n, q_win, k, v, mask, out, row_lse=None):
        self._check_out(out, n * self.cfg.batch * self.cfg.n_q_heads * self.cfg.window * self.cfg.head_dim)
        if getattr(self, "window_ws", None) is None:
            self.window_ws = torch.empty(max(16, madakv_window_attn_workspace_bytes(self.h, self.n_call)), dtype=torch.uint8, device=self.device)
        madakv_window_attn_score(self.h, l0, n, q_win, k, v, mask, out, row_lse, self._sl(self.psi, l0, n),
                                 self._sl(self.psi_pool, l0, n), self._sl(self.stats, l0, n), self.n_mod, self.window_ws)

    def reevict(self, l0, n, q_recent, mask):
        if getattr(self, "reevict_ws", None) is None:
            self.reevict_ws = torch.empty(madakv_reevict_workspace_bytes(self.h, self.n_call), dtype=torch.uint8, device=self.device)
        madakv_reevict(self.h, l0, n, q_recent, mask, self.k_c, self.v_c, self.kept_idx, self._sl(self.kv_off, l0, n),
                       self._sl(self.kv_len, l0, n), self._sl(self.budgets, l0, n), self.reevict_ws)

    def page_table_host(self):
        """Host copy of the page table as int32 [n_layers, B, H, entries] (paged cache only)."""
        ptr, n = madakv_page_table(self.h)
        c = self.cfg
        import numpy as np
        out = np.empty((c.n_layers, c.batch, c.n_kv_heads, n), dtype=np.int32)
        torch.cuda.synchronize()
        hip = C.CDLL("libamdhip64.so")                       # the runtime torch has already loaded
        hip.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
        rc = hip.hipMemcpy(out.ctypes.data, ptr, out.nbytes, 2)      # device to host
        assert rc == 0, f"hipMemcpy -> {rc}"
        return out

    # host copies of the statistics in their declared types
    def stats_host(self):
        s = self.stats.cpu()
        w = s[..., :self.M].contiguous().view(torch.float32).numpy()
        k = s[..., self.M:].contiguous().numpy()
        return w, k
