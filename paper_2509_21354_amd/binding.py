"""Thin Python binding of the kvev C ABI (``include/kvev.h``).

Argument marshalling only: every step of the path runs in the HIP kernels of
``libkvev.so``.  Tensors are torch device tensors (torch is used for device
memory and streams, nothing else); work is enqueued on torch's current stream.
There is no CPU fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Tuple

import torch

from . import synth

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkvev.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP, ERR_STATIC_SCRATCH = range(6)
STATIC_SCRATCH_BYTES = 4 << 20
F32, BF16 = 0, 1
POOL_MEAN, POOL_MLP, POOL_MAX, POOL_TOKEN_MLP = 0, 1, 2, 3
SELECT_TOPK, SELECT_THRESHOLD = 0, 1
OP_CHUNK_POOL, OP_LSTM_GATE, OP_SELECT, OP_GATED_ATTENTION, OP_DENSE_ATTENTION, OP_COMPACT_ATTENTION = range(6)
OP_LSTM_PREPARE, OP_LSTM_GATE_PREPARED = 6, 7

EXPORTS = ("kvev_chunk_pool", "kvev_lstm_gate", "kvev_lstm_prepare", "kvev_lstm_gate_prepared", "kvev_select", "kvev_gated_attention",
           "kvev_gated_attention_static", "kvev_dense_attention", "kvev_retain", "kvev_compact_attention", "kvev_workspace_bytes",
           "kvev_status_string", "kvev_last_hip_error", "kvev_version")
TEST_HOOKS = ("kvev_debug_pair_wait", "kvev_debug_lstm_fused_min_groups", "kvev_debug_lstm_quad_groups", "kvev_debug_stream_probe",
              "kvev_debug_attn_stream_bytes")      # include/kvev_test_hooks.h


class Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("L", "B", "H", "d", "T", "T_cap", "C", "N_cap", "W", "d_sum", "d_g", "dtype", "H_kv")]


class MlpW(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("W1", "b1", "W2", "b2")]


class LstmW(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("W_ih", "W_hh", "b_ih", "b_hh", "w_s", "b_s")]


class KvevError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(what)


_lib = None


def lib() -> ctypes.CDLL:
    """Loads libkvev.so (built by ``python -m paper_2509_21354_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2509_21354_amd.build`; "
                "there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        shp = ctypes.POINTER(Shape)
        L.kvev_chunk_pool.argtypes = [shp, vp, vp, ci, ctypes.POINTER(MlpW), ctypes.POINTER(MlpW), ci, ci,
                                      vp, vp, vp, sz, vp]
        L.kvev_lstm_gate.argtypes = [shp, vp, vp, ctypes.POINTER(LstmW), ci, ci, vp, vp, vp, vp, vp, sz, vp]
        L.kvev_lstm_prepare.argtypes = [shp, ctypes.POINTER(LstmW), vp, sz, vp]
        L.kvev_lstm_gate_prepared.argtypes = [shp, vp, vp, ctypes.POINTER(LstmW), vp, sz, ci, ci, vp, vp, vp, vp, vp, sz, vp]
        L.kvev_select.argtypes = [shp, vp, vp, ci, ci, ctypes.c_float, ci, vp, vp, vp]
        L.kvev_gated_attention.argtypes = [shp, vp, ci, vp, vp, vp, vp, vp, vp, ci, ci, vp, vp, sz, vp]
        L.kvev_gated_attention_static.argtypes = [shp, vp, ci, vp, vp, vp, vp, vp, vp, ci, ci, vp, vp]
        L.kvev_dense_attention.argtypes = [shp, vp, ci, vp, vp, ci, vp, vp, sz, vp]
        L.kvev_retain.argtypes = [shp, ci, ci, vp, vp, vp, ci, ci, ci, vp, vp, vp, vp, vp, vp]
        L.kvev_compact_attention.argtypes = [shp, vp, ci, vp, vp, ci, vp, vp, vp, ci, ci, vp, vp, sz, vp]
        L.kvev_workspace_bytes.argtypes = [ci, shp, ci, ci]
        L.kvev_workspace_bytes.restype = sz
        L.kvev_debug_pair_wait.argtypes = [ci, ci]
        L.kvev_debug_pair_wait.restype = ci
        L.kvev_debug_attn_stream_bytes.argtypes = [sz]
        L.kvev_debug_attn_stream_bytes.restype = ci
        L.kvev_debug_lstm_fused_min_groups.argtypes = [ci]
        L.kvev_debug_lstm_fused_min_groups.restype = ci
        L.kvev_debug_lstm_quad_groups.argtypes = [ci]
        L.kvev_debug_lstm_quad_groups.restype = ci
        L.kvev_debug_stream_probe.argtypes = [vp, sz, ci, vp, sz, ci, ci, vp]
        L.kvev_debug_stream_probe.restype = ci
        L.kvev_status_string.argtypes = [ci]
        L.kvev_status_string.restype = ctypes.c_char_p
        L.kvev_last_hip_error.restype = ctypes.c_char_p
        for n in ("kvev_chunk_pool", "kvev_lstm_gate", "kvev_lstm_prepare", "kvev_lstm_gate_prepared", "kvev_select", "kvev_gated_attention",
                  "kvev_gated_attention_static", "kvev_dense_attention", "kvev_retain", "kvev_compact_attention", "kvev_version"):
            getattr(L, n).restype = ci
        _lib = L
    return _lib


def _check(status: int, what: str):
    if status != OK:
        msg = lib().kvev_status_string(status).decode()
        if status == ERR_HIP:
            msg += ": " + lib().kvev_last_hip_error().decode()
        raise KvevError(status, f"{what}: {msg}")


class RowsFrom:
    """Rows r0 .. of the second-to-last (or, for a score array, last) axis of a contiguous tensor, passed as a
    bare pointer: for entry points that take a row capacity of their own (kvev_retain's n_new_cap is then the
    tensor's full row count), so that a range of rows needs no copy."""

    def __init__(self, t: torch.Tensor, r0: int, row_elems: int):
        assert t.is_contiguous(), "kvev takes contiguous tensors"
        self.ptr = t.data_ptr() + r0 * row_elems * t.element_size()


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, RowsFrom):
        return ctypes.c_void_p(t.ptr)
    assert t.is_contiguous(), "kvev takes contiguous tensors"
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_shape(cfg=None, **kw) -> Shape:
    """Shape from a synth.Config (plus overrides) or from keywords."""
    v: Dict[str, int] = {}
    if cfg is not None:
        v.update(L=cfg.L, B=cfg.B, H=cfg.H, d=cfg.d, T=cfg.T, T_cap=cfg.T, C=cfg.C, N_cap=cfg.T // cfg.C,
                 W=cfg.W, d_sum=cfg.d_sum, d_g=cfg.d_g, dtype=F32 if cfg.dtype == "f32" else BF16,
                 H_kv=getattr(cfg, "H_kv", 0))
    v.update(kw)
    return Shape(**v)


def kvev_debug_pair_wait(spin_limit: int = 1 << 22, mute_member: int = -1) -> None:
    _check(lib().kvev_debug_pair_wait(spin_limit, mute_member), "kvev_debug_pair_wait")


def kvev_debug_attn_stream_bytes(nbytes: int = 0) -> None:
    _check(lib().kvev_debug_attn_stream_bytes(nbytes), "kvev_debug_attn_stream_bytes")


def kvev_debug_lstm_quad_groups(groups: int = 0) -> None:
    _check(lib().kvev_debug_lstm_quad_groups(groups), "kvev_debug_lstm_quad_groups")


def kvev_debug_lstm_fused_min_groups(min_groups: int = 0) -> None:
    _check(lib().kvev_debug_lstm_fused_min_groups(min_groups), "kvev_debug_lstm_fused_min_groups")


def kvev_debug_stream_probe(src: torch.Tensor, tile_bytes: int, dst: torch.Tensor, write_bytes_per_tile: int,
                            hints: int = 0) -> None:
    st = lib().kvev_debug_stream_probe(_ptr(src), src.numel() * src.element_size(), tile_bytes, _ptr(dst),
                                       dst.numel() * dst.element_size(), write_bytes_per_tile, hints, _stream())
    _check(st, "kvev_debug_stream_probe")


def workspace_bytes(op: int, shape: Shape, n: int, k_cap: int = 0) -> int:
    return int(lib().kvev_workspace_bytes(op, ctypes.byref(shape), n, k_cap))


def alloc_workspace(nbytes: int, device="cuda") -> Optional[torch.Tensor]:
    """Scratch for one op, zero-filled: the attention calls keep their split tickets in it, which start at zero."""
    return torch.zeros(max(nbytes, 16), dtype=torch.uint8, device=device)


def _mlp(w: Optional[Tuple[torch.Tensor, ...]]):
    if w is None:
        return None
    return ctypes.byref(MlpW(*[t.data_ptr() for t in w]))


def kvev_chunk_pool(shape: Shape, K, V, pool_mode, wK, wV, chunk_begin, chunk_end, Kbar, Vbar, ws=None):
    st = lib().kvev_chunk_pool(ctypes.byref(shape), _ptr(K), _ptr(V), pool_mode, _mlp(wK), _mlp(wV),
                               chunk_begin, chunk_end, _ptr(Kbar), _ptr(Vbar), _ptr(ws),
                               ws.numel() if ws is not None else 0, _stream())
    _check(st, "kvev_chunk_pool")


def kvev_lstm_gate(shape: Shape, Kbar, Vbar, w, chunk_begin, chunk_end, h, c, util, gate, ws=None):
    lw = LstmW(*[t.data_ptr() for t in w])
    st = lib().kvev_lstm_gate(ctypes.byref(shape), _ptr(Kbar), _ptr(Vbar), ctypes.byref(lw), chunk_begin,
                              chunk_end, _ptr(h), _ptr(c), _ptr(util), _ptr(gate), _ptr(ws),
                              ws.numel() if ws is not None else 0, _stream())
    _check(st, "kvev_lstm_gate")


def kvev_lstm_prepare(shape: Shape, w, packed):
    lw = LstmW(*[t.data_ptr() for t in w])
    st = lib().kvev_lstm_prepare(ctypes.byref(shape), ctypes.byref(lw), _ptr(packed),
                                 packed.numel() if packed is not None else 0, _stream())
    _check(st, "kvev_lstm_prepare")


def kvev_lstm_gate_prepared(shape: Shape, Kbar, Vbar, w, packed, chunk_begin, chunk_end, h, c, util, gate, ws=None):
    lw = LstmW(*[t.data_ptr() for t in w])
    st = lib().kvev_lstm_gate_prepared(ctypes.byref(shape), _ptr(Kbar), _ptr(Vbar), ctypes.byref(lw), _ptr(packed),
                                       packed.numel() if packed is not None else 0, chunk_begin, chunk_end, _ptr(h),
                                       _ptr(c), _ptr(util), _ptr(gate), _ptr(ws), ws.numel() if ws is not None else 0,
                                       _stream())
    _check(st, "kvev_lstm_gate_prepared")


def kvev_select(shape: Shape, util, gate, mode, k, tau, k_cap, idx, count):
    st = lib().kvev_select(ctypes.byref(shape), _ptr(util), _ptr(gate), mode, k, float(tau), k_cap,
                           _ptr(idx), _ptr(count), _stream())
    _check(st, "kvev_select")


def kvev_gated_attention(shape: Shape, Q, Tq, K, V, Kbar, Vbar, idx, count, k_cap, O, ws=None, causal=0):
    st = lib().kvev_gated_attention(ctypes.byref(shape), _ptr(Q), Tq, _ptr(K), _ptr(V), _ptr(Kbar),
                                    _ptr(Vbar), _ptr(idx), _ptr(count), k_cap, causal, _ptr(O), _ptr(ws),
                                    ws.numel() if ws is not None else 0, _stream())
    _check(st, "kvev_gated_attention")


def kvev_gated_attention_static(shape: Shape, Q, Tq, K, V, Kbar, Vbar, idx, count, k_cap, O, causal=0):
    st = lib().kvev_gated_attention_static(ctypes.byref(shape), _ptr(Q), Tq, _ptr(K), _ptr(V), _ptr(Kbar),
                                           _ptr(Vbar), _ptr(idx), _ptr(count), k_cap, causal, _ptr(O), _stream())
    _check(st, "kvev_gated_attention_static")


def kvev_dense_attention(shape: Shape, Q, Tq, K, V, O, ws=None, causal=0):
    st = lib().kvev_dense_attention(ctypes.byref(shape), _ptr(Q), Tq, _ptr(K), _ptr(V), causal, _ptr(O),
                                    _ptr(ws), ws.numel() if ws is not None else 0, _stream())
    _check(st, "kvev_dense_attention")


def kvev_retain(shape: Shape, k, k_cap, Kbar_new, Vbar_new, util_new, n_new_cap, first_chunk, n_new, Kc, Vc,
                chunk_id, util_c, count):
    st = lib().kvev_retain(ctypes.byref(shape), k, k_cap, _ptr(Kbar_new), _ptr(Vbar_new), _ptr(util_new),
                           n_new_cap, first_chunk, n_new, _ptr(Kc), _ptr(Vc), _ptr(chunk_id), _ptr(util_c),
                           _ptr(count), _stream())
    _check(st, "kvev_retain")


def kvev_compact_attention(shape: Shape, Q, Tq, Kw, Vw, Kc, Vc, count, k_cap, O, ws=None, causal=0, win_first=0):
    st = lib().kvev_compact_attention(ctypes.byref(shape), _ptr(Q), Tq, _ptr(Kw), _ptr(Vw), win_first, _ptr(Kc), _ptr(Vc),
                                      _ptr(count), k_cap, causal, _ptr(O), _ptr(ws),
                                      ws.numel() if ws is not None else 0, _stream())
    _check(st, "kvev_compact_attention")


class DecodeState:
    """Caller-owned buffers of one gated cache (summaries, gate state, scores,
    kept indices, scratch).  Allocation only; no arithmetic."""

    def __init__(self, cfg: synth.Config, k_cap: Optional[int] = None, device="cuda",
                 T_cap: Optional[int] = None, Tq: Optional[int] = None):
        self.cfg = cfg
        T_cap = cfg.T if T_cap is None else T_cap
        self.N_cap = T_cap // cfg.C
        self.k_cap = cfg.k if k_cap is None else k_cap
        dt, dev = cfg.torch_dtype, device
        lead = (cfg.L, cfg.B, cfg.kv_heads)       # summaries, gate state and kept sets exist per key-value head
        self.Kbar = torch.zeros(lead + (self.N_cap, cfg.d), dtype=dt, device=dev)
        self.Vbar = torch.zeros_like(self.Kbar)
        self.hc = torch.zeros((2,) + lead + (cfg.d_g,), dtype=torch.float32, device=dev)    # one buffer: one fill resets both
        self.h, self.c = self.hc[0], self.hc[1]
        self.util = torch.zeros(lead + (self.N_cap,), dtype=torch.float32, device=dev)
        self.gate = torch.zeros_like(self.util)
        self.idx = torch.full(lead + (max(self.k_cap, 1),), -1, dtype=torch.int32, device=dev)
        self.count = torch.zeros(lead, dtype=torch.int32, device=dev)
        self.shape = make_shape(cfg, T_cap=T_cap, N_cap=self.N_cap)
        Tq = cfg.Tq if Tq is None else Tq
        full = make_shape(cfg, T=T_cap, T_cap=T_cap, N_cap=self.N_cap)
        # the gate's scratch, and the attention calls' own (their tickets must stay zero between calls, so it is
        # never lent to the gate)
        self.ws = alloc_workspace(workspace_bytes(OP_LSTM_GATE, full, self.N_cap), dev)
        self.packed = alloc_workspace(workspace_bytes(OP_LSTM_PREPARE, full, 0), dev)    # for kvev_lstm_prepare
        self.ws_pool = alloc_workspace(workspace_bytes(OP_CHUNK_POOL, full, self.N_cap), dev)   # optional: the MLP weights re-laid
        nbytes = max(workspace_bytes(OP_GATED_ATTENTION, full, Tq, self.k_cap),
                     workspace_bytes(OP_DENSE_ATTENTION, full, Tq),
                     max(workspace_bytes(OP_GATED_ATTENTION, make_shape(cfg, T=t, T_cap=T_cap, N_cap=self.N_cap),
                                         Tq, self.k_cap) for t in {cfg.T, min(T_cap, cfg.W + cfg.C)}))
        self.ws_attn = alloc_workspace(nbytes, dev)


def mlp_weights(w: Dict[str, torch.Tensor], kv: str):
    return tuple(w[n + kv] for n in ("W1", "b1", "W2", "b2"))


def lstm_weights(w: Dict[str, torch.Tensor]):
    return tuple(w[n] for n in ("W_ih", "W_hh", "b_ih", "b_hh", "w_s", "b_s"))


def cold_step(st: DecodeState, t: Dict[str, torch.Tensor], O: torch.Tensor, T: Optional[int] = None,
              pool_mode: int = POOL_MLP):
    """One whole decode step from scratch: pool every completed chunk, run the
    gate from a zero state, select, attend (section 3.3).  Ordering only."""
    cfg = st.cfg
    sh = st.shape
    if T is not None:
        sh.T = T
    N = sh.T // cfg.C
    kvev_chunk_pool(sh, t["K"], t["V"], pool_mode, mlp_weights(t, "K"), mlp_weights(t, "V"), 0, N,
                    st.Kbar, st.Vbar, st.ws_pool)
    kvev_lstm_gate(sh, st.Kbar, st.Vbar, lstm_weights(t), 0, N, st.h, st.c, st.util, st.gate, st.ws)
    kvev_select(sh, st.util, st.gate, SELECT_TOPK, cfg.k, 0.0, st.k_cap, st.idx, st.count)
    kvev_gated_attention(sh, t["Q"], t["Q"].shape[3], t["K"], t["V"], st.Kbar, st.Vbar, st.idx, st.count,
                         st.k_cap, O, st.ws_attn)
