"""ctypes front end of the CPU oracle (``kvev_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
bench's CPU-baseline leg.  It imports nothing from the GPU package.  Arrays are
numpy: float32 for fp32 storage, uint16 (raw bits) for bfloat16 storage; torch
CPU tensors are accepted and converted without changing a bit.

The chain functions at the bottom (``cold_step``, ``stream``) only order the
stage calls the way section 3.3 of the paper describes a decode step; they add
no arithmetic.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kvev_oracle.c")
_LIB = os.path.join(_HERE, "libkvev_oracle.so")

F32, BF16 = 0, 1
POOL_MEAN, POOL_MLP, POOL_MAX, POOL_TOKEN_MLP = 0, 1, 2, 3


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C11, -O2, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.kvo_gelu.restype = ctypes.c_double
        _lib.kvo_gelu.argtypes = [ctypes.c_double]
        _lib.kvo_bf16_round.restype = ctypes.c_uint16
        _lib.kvo_bf16_round.argtypes = [ctypes.c_double]
        vp, ci = ctypes.c_void_p, ctypes.c_int
        _lib.kvo_select_threshold.argtypes = [ci, ci, ci, ci, ci, vp, ctypes.c_float, ci, vp, vp]
    return _lib


def to_np(x):
    """numpy view of a numpy array or torch CPU tensor (bf16 -> uint16 bits)."""
    if x is None:
        return None
    if isinstance(x, np.ndarray):
        return np.ascontiguousarray(x)
    import torch  # conversion only
    x = x.detach().cpu().contiguous()
    if x.dtype == torch.bfloat16:
        return x.view(torch.int16).numpy().view(np.uint16)
    return x.numpy()


def from_bits(a: np.ndarray) -> np.ndarray:
    """float64 values of an array in either storage form."""
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"unsupported storage dtype {a.dtype}")


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what}: bad argument (status {rc})")


def gelu(x: float) -> float:
    return lib().kvo_gelu(float(x))


def bf16_round(x: float) -> int:
    return int(lib().kvo_bf16_round(float(x)))


def chunk_pool(K, V, T, C, N_cap, d_sum, mode, wK, wV, c0, c1, Kbar=None, Vbar=None):
    """Eq. 2.  K, V [L,B,H,T_cap,d]; wK / wV = (W1, b1, W2, b2) per layer or
    None in MEAN mode.  Returns (Kbar, Vbar) [L,B,H,N_cap,d], rows [c0,c1) written."""
    K, V = to_np(K), to_np(V)
    L, B, H, T_cap, d = K.shape
    if Kbar is None:
        Kbar = np.zeros((L, B, H, N_cap, d), dtype=K.dtype)
        Vbar = np.zeros((L, B, H, N_cap, d), dtype=K.dtype)
    wK = [to_np(w) for w in wK] if wK is not None else [None] * 4
    wV = [to_np(w) for w in wV] if wV is not None else [None] * 4
    rc = lib().kvo_chunk_pool(dtype_code(K), L, B, H, d, T, T_cap, C, N_cap, d_sum, mode,
                              _p(K), _p(V), *[_p(w) for w in wK], *[_p(w) for w in wV],
                              c0, c1, _p(Kbar), _p(Vbar))
    _check(rc, "chunk_pool")
    return Kbar, Vbar


def lstm_gate(Kbar, Vbar, lstm_w, c0, c1, h=None, c=None, util=None, gate=None):
    """Eq. 3.  lstm_w = (W_ih, W_hh, b_ih, b_hh, w_s, b_s).  h, c [L,B,H,d_g]
    fp32 are updated in place (zeros when omitted); util / gate [L,B,H,N_cap]."""
    Kbar, Vbar = to_np(Kbar), to_np(Vbar)
    L, B, H, N_cap, d = Kbar.shape
    w = [to_np(x) for x in lstm_w]
    d_g = w[1].shape[-1]
    if h is None:
        h = np.zeros((L, B, H, d_g), np.float32)
    if c is None:
        c = np.zeros((L, B, H, d_g), np.float32)
    if util is None:
        util = np.zeros((L, B, H, N_cap), np.float32)
    if gate is None:
        gate = np.zeros((L, B, H, N_cap), np.float32)
    for a in (h, c, util, gate):
        assert a.dtype == np.float32 and a.flags.c_contiguous
    rc = lib().kvo_lstm_gate(dtype_code(Kbar), L, B, H, d, N_cap, d_g, _p(Kbar), _p(Vbar),
                             *[_p(x) for x in w], c0, c1, _p(h), _p(c), _p(util), _p(gate))
    _check(rc, "lstm_gate")
    return h, c, util, gate


def select_topk(util, T, C, W, k, k_cap):
    """Keep the min(k, N_cand) candidates of largest utility (ties: lower
    index), ascending.  util [..., N_cap].  Returns (idx [...,k_cap], count [...])."""
    util = np.ascontiguousarray(to_np(util), dtype=np.float32)
    lead, N_cap = util.shape[:-1], util.shape[-1]
    S = int(np.prod(lead)) if lead else 1
    idx = np.full(lead + (k_cap,), -1, np.int32)
    count = np.zeros(lead, np.int32)
    rc = lib().kvo_select_topk(S, T, C, W, N_cap, _p(util), k, k_cap, _p(idx), _p(count))
    _check(rc, "select_topk")
    return idx, count


def select_threshold(gate, T, C, W, tau, k_cap):
    """Section 3.2's literal rule: keep candidate c iff gate[c] >= tau."""
    gate = np.ascontiguousarray(to_np(gate), dtype=np.float32)
    lead, N_cap = gate.shape[:-1], gate.shape[-1]
    S = int(np.prod(lead)) if lead else 1
    idx = np.full(lead + (k_cap,), -1, np.int32)
    count = np.zeros(lead, np.int32)
    rc = lib().kvo_select_threshold(S, T, C, W, N_cap, _p(gate), float(tau), k_cap,
                                    _p(idx), _p(count))
    _check(rc, "select_threshold")
    return idx, count


def gated_attention(Q, K, V, Kbar, Vbar, idx, count, T, C, W, want_probs=False):
    """Eq. 1 over kept summaries + raw window.  Q [L,B,H,Tq,d] -> O same shape."""
    Q, K, V, Kbar, Vbar = (to_np(x) for x in (Q, K, V, Kbar, Vbar))
    idx = np.ascontiguousarray(to_np(idx), dtype=np.int32)
    count = np.ascontiguousarray(to_np(count), dtype=np.int32)
    L, B, H, Tq, d = Q.shape
    T_cap, N_cap, k_cap = K.shape[3], Kbar.shape[3], idx.shape[-1]
    O = np.zeros_like(Q)
    probs, stride = None, 0
    if want_probs:
        n_cand = max(0, T - W) // C
        stride = k_cap + T - n_cand * C
        probs = np.zeros((L, B, H, Tq, stride), np.float64)
    rc = lib().kvo_gated_attention(dtype_code(Q), L, B, H, d, T, T_cap, C, N_cap, W, _p(Q), Tq,
                                   _p(K), _p(V), _p(Kbar), _p(Vbar), _p(idx), _p(count), k_cap,
                                   _p(O), _p(probs), stride)
    _check(rc, "gated_attention")
    return (O, probs) if want_probs else O


def attention_ext(Q, K, V, T, C=1, W=0, Kbar=None, Vbar=None, idx=None, count=None, causal=0):
    """Eq. 1 with grouped-query heads (K, V and the kept set have H_kv <= H heads) and, optionally,
    a causal frame of queries (the Tq queries are the last Tq cached tokens).  Gated when Kbar is given."""
    Q, K, V = (to_np(x) for x in (Q, K, V))
    L, B, H, Tq, d = Q.shape
    H_kv, T_cap = K.shape[2], K.shape[3]
    gated = Kbar is not None
    O = np.zeros_like(Q)
    if gated:
        Kbar, Vbar = to_np(Kbar), to_np(Vbar)
        idx = np.ascontiguousarray(to_np(idx), dtype=np.int32)
        count = np.ascontiguousarray(to_np(count), dtype=np.int32)
        N_cap, k_cap = Kbar.shape[3], idx.shape[-1]
    else:
        N_cap, k_cap = 0, 0
    rc = lib().kvo_attention_ext(dtype_code(Q), L, B, H, H_kv, d, T, T_cap, C, N_cap, W, int(gated), int(causal),
                                 _p(Q), Tq, _p(K), _p(V), _p(Kbar) if gated else None, _p(Vbar) if gated else None,
                                 _p(idx) if gated else None, _p(count) if gated else None, k_cap, _p(O))
    _check(rc, "attention_ext")
    return O


def retain(Kbar_new, Vbar_new, util_new, first_chunk, n_new, k, Kc, Vc, chunk_id, util_c, count):
    """Physical eviction (sections 3.2-3.3): merge n_new freshly scored chunks into the compact
    store (Kc, Vc [...,k_cap,d], chunk_id, util_c [...,k_cap], count [...]), in place."""
    Kn, Vn = to_np(Kbar_new), to_np(Vbar_new)
    un = np.ascontiguousarray(to_np(util_new), dtype=np.float32)
    assert Kc.flags.c_contiguous and Vc.flags.c_contiguous and chunk_id.dtype == np.int32
    assert util_c.dtype == np.float32 and count.dtype == np.int32
    lead, k_cap, d = Kc.shape[:-2], Kc.shape[-2], Kc.shape[-1]
    S = int(np.prod(lead)) if lead else 1
    rc = lib().kvo_retain(dtype_code(Kc), S, d, k, k_cap, _p(Kn), _p(Vn), _p(un), Kn.shape[-2], first_chunk,
                          n_new, _p(Kc), _p(Vc), _p(chunk_id), _p(util_c), _p(count))
    _check(rc, "retain")


def compact_attention(Q, Kw, Vw, win_len, Kc, Vc, count, causal=0, win_first=0):
    """Eq. 1 over kept summaries (compact store) + resident raw window; causal: the queries are the
    window's last Tq tokens; win_first: the window buffer is a ring that starts at this row."""
    Q, Kw, Vw, Kc, Vc = (to_np(x) for x in (Q, Kw, Vw, Kc, Vc))
    count = np.ascontiguousarray(to_np(count), dtype=np.int32)
    L, B, H, Tq, d = Q.shape
    O = np.zeros_like(Q)
    rc = lib().kvo_compact_attention(dtype_code(Q), L, B, H, Kw.shape[2], d, win_len, Kw.shape[3], int(win_first), _p(Q), Tq, _p(Kw), _p(Vw),
                                     _p(Kc), _p(Vc), _p(count), Kc.shape[3], int(causal), _p(O))
    _check(rc, "compact_attention")
    return O


def dense_attention(Q, K, V, T, want_probs=False):
    """Eq. 1 over the whole cache."""
    Q, K, V = (to_np(x) for x in (Q, K, V))
    L, B, H, Tq, d = Q.shape
    T_cap = K.shape[3]
    O = np.zeros_like(Q)
    probs = np.zeros((L, B, H, Tq, T), np.float64) if want_probs else None
    rc = lib().kvo_dense_attention(dtype_code(Q), L, B, H, d, T, T_cap, _p(Q), Tq, _p(K), _p(V),
                                   _p(O), _p(probs), T)
    _check(rc, "dense_attention")
    return (O, probs) if want_probs else O


# --------------------------------------------------------------------------
# The chain: one decode step (section 3.3) and the streaming loop.
# --------------------------------------------------------------------------

def _weights(w: Dict[str, object]):
    wK = (w["W1K"], w["b1K"], w["W2K"], w["b2K"])
    wV = (w["W1V"], w["b1V"], w["W2V"], w["b2V"])
    lw = (w["W_ih"], w["W_hh"], w["b_ih"], w["b_hh"], w["w_s"], w["b_s"])
    return wK, wV, lw


def cold_step(Q, K, V, w, T, C, W, k, d_sum, pool_mode=POOL_MLP, k_cap: Optional[int] = None):
    """pool all completed chunks -> gate from zero state -> top-k -> attend."""
    K_, V_ = to_np(K), to_np(V)
    N_cap = K_.shape[3] // C
    N = T // C
    wK, wV, lw = _weights(w)
    Kbar, Vbar = chunk_pool(K_, V_, T, C, N_cap, d_sum, pool_mode, wK, wV, 0, N)
    h, c, util, gate = lstm_gate(Kbar, Vbar, lw, 0, N)
    k_cap = k if k_cap is None else k_cap
    idx, count = select_topk(util, T, C, W, k, k_cap)
    O = gated_attention(Q, K_, V_, Kbar, Vbar, idx, count, T, C, W)
    return dict(Kbar=Kbar, Vbar=Vbar, h=h, c=c, util=util, gate=gate, idx=idx, count=count, O=O)


def stream(Qs, K, V, w, frame, steps, C, W, k, d_sum, pool_mode=POOL_MLP):
    """Streaming trigger (section 3.3, last sentence of its second paragraph):
    after every appended frame, pool only the newly completed chunks, advance
    the carried LSTM state over them, re-select, then decode.  Qs is
    [steps, n_dec, L,B,H,1,d]; the decoded tokens' own K/V are not appended.
    Returns the per-step state snapshots and outputs."""
    K_, V_, Qs = to_np(K), to_np(V), to_np(Qs)
    L, B, H, T_cap, d = K_.shape
    N_cap = T_cap // C
    wK, wV, lw = _weights(w)
    d_g = to_np(lw[1]).shape[-1]
    Kbar = np.zeros((L, B, H, N_cap, d), K_.dtype)
    Vbar = np.zeros_like(Kbar)
    h = np.zeros((L, B, H, d_g), np.float32)
    c = np.zeros_like(h)
    util = np.zeros((L, B, H, N_cap), np.float32)
    gate = np.zeros_like(util)
    done = 0
    out = []
    for s in range(steps):
        T = (s + 1) * frame
        N = T // C
        chunk_pool(K_, V_, T, C, N_cap, d_sum, pool_mode, wK, wV, done, N, Kbar, Vbar)
        lstm_gate(Kbar, Vbar, lw, done, N, h, c, util, gate)
        done = N
        idx, count = select_topk(util, T, C, W, k, k)
        Os = [gated_attention(Qs[s, i], K_, V_, Kbar, Vbar, idx, count, T, C, W)
              for i in range(Qs.shape[1])]
        out.append(dict(T=T, idx=idx, count=count, O=Os, h=h.copy(), c=c.copy(),
                        util=util.copy()))
    return out
