"""Boundary checks that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad arguments before touching HIP."""
import ctypes
import os
import re

import pytest

from paper_2509_21354_amd import binding as kb
from paper_2509_21354_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(header="kvev.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvev_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert set(kb.EXPORTS) == set(names)
    hooks = _declared("kvev_test_hooks.h")
    assert set(kb.TEST_HOOKS) == set(hooks)
    assert not any("debug" in n for n in names)          # test hooks stay out of the public header
    L = kb.lib()
    for n in names + hooks:
        assert getattr(L, n) is not None
    assert L.kvev_version() >= 100
    assert L.kvev_status_string(0) == b"ok"
    assert b"workspace" in L.kvev_status_string(kb.ERR_WORKSPACE)


def test_debug_pair_wait_validation():
    L = kb.lib()
    assert L.kvev_debug_pair_wait(0, -1) == kb.ERR_INVALID_ARG
    assert L.kvev_debug_pair_wait(16, 2) == kb.ERR_INVALID_ARG
    assert L.kvev_debug_pair_wait(16, -2) == kb.ERR_INVALID_ARG
    assert L.kvev_debug_pair_wait(1 << 22, -1) == kb.OK      # the defaults
    assert L.kvev_debug_lstm_fused_min_groups(-1) == kb.ERR_INVALID_ARG
    assert L.kvev_debug_lstm_quad_groups(-1) == kb.ERR_INVALID_ARG
    big = kb.make_shape(synth.CONFIGS[3])
    small = kb.make_shape(synth.CONFIGS[2])
    w_small = kb.workspace_bytes(kb.OP_LSTM_GATE, small, 128)
    assert L.kvev_debug_lstm_fused_min_groups(1) == kb.OK
    try:       # the single-kernel form keeps no projections in scratch
        assert 0 < kb.workspace_bytes(kb.OP_LSTM_GATE, small, 128) < w_small
    finally:
        assert L.kvev_debug_lstm_fused_min_groups(0) == kb.OK
    assert kb.workspace_bytes(kb.OP_LSTM_GATE, small, 128) == w_small
    assert kb.workspace_bytes(kb.OP_LSTM_GATE, big, 256) < (64 << 20)          # config 3: packed weights only


FAKE = ctypes.c_void_p(0x1000)       # aligned, never dereferenced: validation fails first


def test_stream_probe_validation():
    """The calibration hook checks its arguments on the host before any launch."""
    L = kb.lib()
    f = L.kvev_debug_stream_probe
    ok_args = dict(src=FAKE, src_bytes=1 << 20, tile=4096, dst=FAKE, dst_bytes=1 << 20, wb=16, hints=0)

    def call(**kw):
        a = dict(ok_args, **kw)
        return f(a["src"], a["src_bytes"], a["tile"], a["dst"], a["dst_bytes"], a["wb"], a["hints"], None)
    assert call(src=None) == kb.ERR_INVALID_ARG
    assert call(dst=ctypes.c_void_p(0x1008)) == kb.ERR_INVALID_ARG              # not 16-byte aligned
    assert call(tile=4000) == kb.ERR_INVALID_ARG                                # not a multiple of 4096
    assert call(src_bytes=(1 << 20) + 4096, tile=8192) == kb.ERR_INVALID_ARG    # the tile does not divide the source
    assert call(wb=24) == kb.ERR_INVALID_ARG                                    # not a multiple of 16
    assert call(wb=8192, dst_bytes=4096) == kb.ERR_INVALID_ARG                  # 256 tiles x 8 KiB do not fit
    assert call(hints=8) == kb.ERR_INVALID_ARG and call(hints=-1) == kb.ERR_INVALID_ARG
    assert call(hints=4, wb=64 * 1024, dst_bytes=1 << 30) == kb.ERR_INVALID_ARG  # bursts hold at most 48 KiB per tile


def _shape(**kw):
    return kb.make_shape(synth.CONFIGS[2], **kw)


def test_shape_validation():
    L = kb.lib()
    for bad in (dict(L=0), dict(d=-1), dict(C=0), dict(T=5000), dict(N_cap=3), dict(W=-1), dict(d_g=0)):
        sh = _shape(**bad)
        assert L.kvev_dense_attention(ctypes.byref(sh), FAKE, 1, FAKE, FAKE, 0, FAKE, None, 0, None) == kb.ERR_INVALID_ARG
    for bad in (dict(d=96), dict(dtype=7)):
        sh = _shape(**bad)
        assert L.kvev_dense_attention(ctypes.byref(sh), FAKE, 1, FAKE, FAKE, 0, FAKE, None, 0, None) == kb.ERR_UNSUPPORTED
    assert L.kvev_dense_attention(None, FAKE, 1, FAKE, FAKE, 0, FAKE, None, 0, None) == kb.ERR_INVALID_ARG


def test_pointer_range_and_mode_validation():
    L = kb.lib()
    sh = _shape()
    r = ctypes.byref(sh)
    odd = ctypes.c_void_p(0x1004)
    w = kb.MlpW(0x1000, 0x1000, 0x1000, 0x1000)
    wr = ctypes.byref(w)
    # attention
    assert L.kvev_dense_attention(r, None, 1, FAKE, FAKE, 0, FAKE, None, 0, None) == kb.ERR_INVALID_ARG
    assert L.kvev_dense_attention(r, odd, 1, FAKE, FAKE, 0, FAKE, None, 0, None) == kb.ERR_INVALID_ARG
    assert L.kvev_dense_attention(r, FAKE, -1, FAKE, FAKE, 0, FAKE, None, 0, None) == kb.ERR_INVALID_ARG
    assert L.kvev_dense_attention(r, FAKE, 1, FAKE, FAKE, 2, FAKE, None, 0, None) == kb.ERR_INVALID_ARG      # causal is 0 or 1
    assert L.kvev_dense_attention(r, FAKE, 5000, FAKE, FAKE, 1, FAKE, None, 0, None) == kb.ERR_INVALID_ARG   # frame longer than the cache
    assert L.kvev_gated_attention(r, FAKE, 400, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 32, 1, FAKE, None, 0, None) == kb.ERR_INVALID_ARG  # frame outside the raw window
    bad_kv = _shape(H_kv=5)
    assert L.kvev_dense_attention(ctypes.byref(bad_kv), FAKE, 1, FAKE, FAKE, 0, FAKE, None, 0, None) == kb.ERR_INVALID_ARG
    assert L.kvev_dense_attention(r, FAKE, 1, FAKE, FAKE, 0, FAKE, None, 0, None) == kb.ERR_WORKSPACE
    assert L.kvev_dense_attention(r, FAKE, 1, FAKE, FAKE, 0, FAKE, FAKE, 64, None) == kb.ERR_WORKSPACE
    assert L.kvev_dense_attention(r, FAKE, 0, FAKE, FAKE, 0, FAKE, None, 0, None) == kb.OK   # Tq = 0: nothing to do
    assert L.kvev_gated_attention(r, FAKE, 1, FAKE, FAKE, FAKE, FAKE, None, FAKE, 32, 0, FAKE, None, 0, None) == kb.ERR_INVALID_ARG
    assert L.kvev_gated_attention(r, FAKE, 1, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, -1, 0, FAKE, None, 0, None) == kb.ERR_INVALID_ARG
    # pool
    assert L.kvev_chunk_pool(r, FAKE, FAKE, 5, wr, wr, 0, 1, FAKE, FAKE, None, 0, None) == kb.ERR_UNSUPPORTED
    assert L.kvev_chunk_pool(r, FAKE, FAKE, kb.POOL_MLP, None, wr, 0, 1, FAKE, FAKE, None, 0, None) == kb.ERR_INVALID_ARG
    assert L.kvev_chunk_pool(r, FAKE, FAKE, kb.POOL_MLP, wr, wr, 3, 2, FAKE, FAKE, None, 0, None) == kb.ERR_INVALID_ARG
    assert L.kvev_chunk_pool(r, FAKE, FAKE, kb.POOL_MLP, wr, wr, 0, 129, FAKE, FAKE, None, 0, None) == kb.ERR_INVALID_ARG
    assert L.kvev_chunk_pool(r, FAKE, FAKE, kb.POOL_MLP, wr, wr, -1, 4, FAKE, FAKE, None, 0, None) == kb.ERR_INVALID_ARG
    assert L.kvev_chunk_pool(r, FAKE, FAKE, kb.POOL_MEAN, None, None, 7, 7, FAKE, FAKE, None, 0, None) == kb.OK  # empty range
    assert L.kvev_chunk_pool(r, FAKE, FAKE, kb.POOL_TOKEN_MLP, wr, None, 0, 1, FAKE, FAKE, None, 0, None) == kb.ERR_INVALID_ARG  # needs both weight sets
    assert L.kvev_chunk_pool(r, FAKE, FAKE, kb.POOL_TOKEN_MLP, wr, wr, 7, 7, FAKE, FAKE, None, 0, None) == kb.OK
    assert L.kvev_chunk_pool(r, FAKE, FAKE, -1, wr, wr, 0, 1, FAKE, FAKE, None, 0, None) == kb.ERR_UNSUPPORTED
    # a trailing partial chunk is not poolable
    sh2 = _shape(T=4095)
    assert L.kvev_chunk_pool(ctypes.byref(sh2), FAKE, FAKE, kb.POOL_MEAN, None, None, 0, 128, FAKE, FAKE, None, 0, None) == kb.ERR_INVALID_ARG
    # gate
    lw = kb.LstmW(*([0x1000] * 6))
    assert L.kvev_lstm_gate(r, FAKE, FAKE, None, 0, 1, FAKE, FAKE, FAKE, FAKE, None, 0, None) == kb.ERR_INVALID_ARG
    assert L.kvev_lstm_gate(r, FAKE, FAKE, ctypes.byref(lw), 0, 129, FAKE, FAKE, FAKE, FAKE, None, 0, None) == kb.ERR_INVALID_ARG
    assert L.kvev_lstm_gate(r, FAKE, FAKE, ctypes.byref(lw), 2, 1, FAKE, FAKE, FAKE, FAKE, None, 0, None) == kb.ERR_INVALID_ARG
    assert L.kvev_lstm_gate(r, FAKE, FAKE, ctypes.byref(lw), 4, 4, FAKE, FAKE, FAKE, FAKE, None, 0, None) == kb.OK
    lw0 = kb.LstmW(0x1000, 0, 0x1000, 0x1000, 0x1000, 0x1000)
    assert L.kvev_lstm_gate(r, FAKE, FAKE, ctypes.byref(lw0), 0, 1, FAKE, FAKE, FAKE, FAKE, None, 0, None) == kb.ERR_INVALID_ARG
    assert L.kvev_lstm_gate(r, FAKE, FAKE, ctypes.byref(lw), 0, 1, odd, FAKE, FAKE, FAKE, None, 0, None) == kb.ERR_INVALID_ARG   # h misaligned
    assert L.kvev_lstm_gate(r, FAKE, FAKE, ctypes.byref(lw), 0, 1, FAKE, FAKE, FAKE, FAKE, None, 0, None) == kb.ERR_WORKSPACE
    # weights prepared once
    need = kb.workspace_bytes(kb.OP_LSTM_PREPARE, sh, 0)
    assert need == 4 * 256 * (256 + 256) * 2 + 256                      # packed W_hh + W_ih, one layer, and the maxima
    assert L.kvev_lstm_prepare(r, None, FAKE, need, None) == kb.ERR_INVALID_ARG
    assert L.kvev_lstm_prepare(r, ctypes.byref(lw0), FAKE, need, None) == kb.ERR_INVALID_ARG
    assert L.kvev_lstm_prepare(r, ctypes.byref(lw), None, need, None) == kb.ERR_WORKSPACE
    assert L.kvev_lstm_prepare(r, ctypes.byref(lw), FAKE, need - 1, None) == kb.ERR_WORKSPACE
    f32 = _shape(dtype=kb.F32)
    assert kb.workspace_bytes(kb.OP_LSTM_PREPARE, f32, 0) == 0
    assert L.kvev_lstm_prepare(ctypes.byref(f32), ctypes.byref(lw), None, 0, None) == kb.OK      # nothing to prepare
    assert L.kvev_lstm_gate_prepared(r, FAKE, FAKE, ctypes.byref(lw), None, 0, 0, 1, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == kb.ERR_WORKSPACE
    assert L.kvev_lstm_gate_prepared(r, FAKE, FAKE, ctypes.byref(lw), FAKE, need, 0, 1, FAKE, FAKE, FAKE, FAKE, None, 0, None) == kb.ERR_WORKSPACE
    assert L.kvev_lstm_gate_prepared(r, FAKE, FAKE, ctypes.byref(lw), FAKE, need, 3, 3, FAKE, FAKE, FAKE, FAKE, None, 0, None) == kb.OK
    assert (kb.workspace_bytes(kb.OP_LSTM_GATE, sh, 128) - kb.workspace_bytes(kb.OP_LSTM_GATE_PREPARED, sh, 128)) == need
    # select
    assert L.kvev_select(r, FAKE, None, 9, 4, 0.0, 4, FAKE, FAKE, None) == kb.ERR_UNSUPPORTED
    assert L.kvev_select(r, None, None, kb.SELECT_TOPK, 4, 0.0, 4, FAKE, FAKE, None) == kb.ERR_INVALID_ARG
    assert L.kvev_select(r, FAKE, None, kb.SELECT_TOPK, -1, 0.0, 4, FAKE, FAKE, None) == kb.ERR_INVALID_ARG
    assert L.kvev_select(r, FAKE, None, kb.SELECT_TOPK, 32, 0.0, 31, FAKE, FAKE, None) == kb.ERR_INVALID_ARG
    assert L.kvev_select(r, None, FAKE, kb.SELECT_THRESHOLD, 0, 0.5, 119, FAKE, FAKE, None) == kb.ERR_INVALID_ARG
    assert L.kvev_select(r, None, FAKE, kb.SELECT_THRESHOLD, 0, float("nan"), 120, FAKE, FAKE, None) == kb.ERR_INVALID_ARG


def test_workspace_query():
    L_ = kb.lib()
    sh = _shape()
    dense = kb.workspace_bytes(kb.OP_DENSE_ATTENTION, sh, 1)
    gated = kb.workspace_bytes(kb.OP_GATED_ATTENTION, sh, 1, 32)
    assert dense > 0 and gated >= 0 and dense % 8 == 0
    assert kb.workspace_bytes(kb.OP_SELECT, sh, 1) == 0
    # pooling: optional room for the MLP weights re-laid (a 256-byte head + 8 d_sum d + 8 (d_sum + d) bytes per layer)
    assert kb.workspace_bytes(kb.OP_CHUNK_POOL, sh, 128) == (256 + sh.L * (8 * sh.d_sum * sh.d + 8 * (sh.d_sum + sh.d))
                                                             if sh.dtype == kb.BF16 and sh.d_sum % 32 == 0 else 0)
    assert kb.workspace_bytes(kb.OP_CHUNK_POOL, kb.make_shape(synth.CONFIGS[1]), 4) == 0      # fp32 storage: nothing to re-lay
    assert kb.workspace_bytes(kb.OP_DENSE_ATTENTION, _shape(L=0), 1) == 0
    big = kb.make_shape(synth.CONFIGS[3])
    assert kb.workspace_bytes(kb.OP_GATED_ATTENTION, big, 1, 64) == 0    # 8192 sequences: no split needed
    # the gate's scratch: forms that run as one kernel keep no projections, so the block length does not matter
    # (config 3: d_g = 256, a group of 32 sequences per compute unit; config 5: d_g = 512, four workgroups per 32
    # sequences, whose exchange slots take 128 KiB per group), the two-kernel form grows with it (config 2)
    for cfg, groups32 in ((synth.CONFIGS[3], 0), (synth.CONFIGS[5], 32 * 2)):
        g = kb.make_shape(cfg)
        one, many = kb.workspace_bytes(kb.OP_LSTM_GATE_PREPARED, g, 1), kb.workspace_bytes(kb.OP_LSTM_GATE_PREPARED, g, 128)
        assert one == many == 256 + groups32 * 131072
    # a d_g = 512 call with more groups than fit at once runs as several launches that share the slots of one
    huge = kb.make_shape(synth.CONFIGS[5], B=256)        # 256 groups of 32 sequences
    assert kb.workspace_bytes(kb.OP_LSTM_GATE_PREPARED, huge, 512) == 256 + 64 * 131072
    assert L_.kvev_debug_lstm_quad_groups(3) == kb.OK
    try:
        assert kb.workspace_bytes(kb.OP_LSTM_GATE_PREPARED, huge, 512) == 256 + 3 * 131072
    finally:
        assert L_.kvev_debug_lstm_quad_groups(0) == kb.OK
    small = kb.make_shape(synth.CONFIGS[2])
    assert kb.workspace_bytes(kb.OP_LSTM_GATE_PREPARED, small, 8) > kb.workspace_bytes(kb.OP_LSTM_GATE_PREPARED, small, 1) > 0


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(kb, "_lib", None)
    monkeypatch.setattr(kb, "LIB_PATH", str(tmp_path / "libkvev.so"))
    with pytest.raises(FileNotFoundError):
        kb.lib()


def test_retain_and_compact_attention_validation():
    L = kb.lib()
    sh = _shape()
    r = ctypes.byref(sh)
    ok = (FAKE, FAKE, FAKE, 8, 0, 4, FAKE, FAKE, FAKE, FAKE, FAKE, None)
    assert L.kvev_retain(r, 33, 32, *ok) == kb.ERR_INVALID_ARG               # k > k_cap
    assert L.kvev_retain(r, -1, 32, *ok) == kb.ERR_INVALID_ARG
    assert L.kvev_retain(r, 4, 32, FAKE, FAKE, FAKE, 8, 0, 9, FAKE, FAKE, FAKE, FAKE, FAKE, None) == kb.ERR_INVALID_ARG   # n_new > cap
    assert L.kvev_retain(r, 4, 3990, FAKE, FAKE, FAKE, 16, 0, 16, FAKE, FAKE, FAKE, FAKE, FAKE, None) == kb.ERR_INVALID_ARG
    assert L.kvev_retain(r, 4, 32, None, FAKE, FAKE, 8, 0, 4, FAKE, FAKE, FAKE, FAKE, FAKE, None) == kb.ERR_INVALID_ARG
    assert L.kvev_retain(r, 4, 32, FAKE, FAKE, FAKE, 8, 0, 4, None, FAKE, FAKE, FAKE, FAKE, None) == kb.ERR_INVALID_ARG
    assert L.kvev_retain(r, 4, 32, FAKE, FAKE, FAKE, 8, -1, 4, FAKE, FAKE, FAKE, FAKE, FAKE, None) == kb.ERR_INVALID_ARG
    assert L.kvev_compact_attention(r, FAKE, 1, FAKE, FAKE, 0, None, FAKE, FAKE, 32, 0, FAKE, None, 0, None) == kb.ERR_INVALID_ARG
    assert L.kvev_compact_attention(r, FAKE, 1, FAKE, FAKE, 0, FAKE, FAKE, None, 32, 0, FAKE, None, 0, None) == kb.ERR_INVALID_ARG
    assert L.kvev_compact_attention(r, FAKE, 1, FAKE, FAKE, 0, FAKE, FAKE, FAKE, -1, 0, FAKE, None, 0, None) == kb.ERR_INVALID_ARG
    big = _shape()                                                            # T = 4096 raw rows: split, needs scratch
    assert kb.workspace_bytes(kb.OP_COMPACT_ATTENTION, big, 1, 32) > 0
    assert L.kvev_compact_attention(ctypes.byref(big), FAKE, 1, FAKE, FAKE, 0, FAKE, FAKE, FAKE, 32, 0, FAKE, None, 0, None) == kb.ERR_WORKSPACE
    assert L.kvev_compact_attention(r, FAKE, 1, FAKE, FAKE, 0, FAKE, FAKE, FAKE, 32, 2, FAKE, None, 0, None) == kb.ERR_INVALID_ARG   # causal is 0 or 1
    assert L.kvev_compact_attention(r, FAKE, 1, FAKE, FAKE, -1, FAKE, FAKE, FAKE, 32, 0, FAKE, None, 0, None) == kb.ERR_INVALID_ARG  # ring start outside the buffer
    assert L.kvev_compact_attention(r, FAKE, 1, FAKE, FAKE, sh.T_cap, FAKE, FAKE, FAKE, 32, 0, FAKE, None, 0, None) == kb.ERR_INVALID_ARG
    assert L.kvev_compact_attention(r, FAKE, 5000, FAKE, FAKE, 0, FAKE, FAKE, FAKE, 32, 1, FAKE, None, 0, None) == kb.ERR_INVALID_ARG   # frame longer than the window



def test_static_scratch_entry_validates_and_rejects_oversized_shapes():
    """kvev_gated_attention_static: the usual validation, and a shape whose split scratch would not fit the
    library's array is refused before any GPU call.  With the default planning no shape needs more than the array
    holds, so the refusal is provoked in a child process that asks for far more workgroups per launch."""
    import subprocess
    import sys
    L = kb.lib()
    sh = _shape()
    r = ctypes.byref(sh)
    assert L.kvev_gated_attention_static(r, None, 1, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 32, 0, FAKE, None) == kb.ERR_INVALID_ARG
    assert L.kvev_gated_attention_static(r, FAKE, 1, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, -1, 0, FAKE, None) == kb.ERR_INVALID_ARG
    assert L.kvev_gated_attention_static(r, FAKE, 0, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 32, 0, FAKE, None) == kb.OK
    assert b"static" in L.kvev_status_string(kb.ERR_STATIC_SCRATCH)
    code = (
        "import ctypes\n"
        "from paper_2509_21354_amd import binding as kb, synth\n"
        "L = kb.lib()\n"
        "sh = kb.make_shape(synth.CONFIGS[2], T=131072, T_cap=131072, N_cap=4096, W=131072)\n"
        "F = ctypes.c_void_p(0x1000)\n"
        "need = kb.workspace_bytes(kb.OP_GATED_ATTENTION, sh, 1, 32)\n"
        "assert need > kb.STATIC_SCRATCH_BYTES, need\n"
        "rc = L.kvev_gated_attention_static(ctypes.byref(sh), F, 1, F, F, F, F, F, F, 32, 0, F, None)\n"
        "assert rc == kb.ERR_STATIC_SCRATCH, rc\n")
    env = dict(os.environ, KVEV_ATTN_TARGET_BLOCKS="65536", KVEV_ATTN_MIN_ROWS="64", PYTHONPATH=ROOT)
    res = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, cwd=ROOT)
    assert res.returncode == 0, res.stderr
