"""Host-side checks that need no GPU: the library loads, exports what the header declares, and
rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest
import torch

import paper_2407_11550_amd as adakv
from paper_2407_11550_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "adakv.h")).read()
    names = set(re.findall(r"\b(adakv_[a-z_]+)\s*\(", header))
    assert {"adakv_score", "adakv_allocate", "adakv_select", "adakv_compact",
            "adakv_workspace_bytes", "adakv_strerror"} <= names
    for name in names:
        assert hasattr(lib, name), name


def test_strerror(lib):
    assert lib.adakv_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4, 17):
        assert len(lib.adakv_strerror(code)) > 0


def _layer(**kw):
    args = dict(dtype=torch.bfloat16, h_q=32, h_kv=8, d=128, w=32, pool_k=7, alpha=0.2,
                n=[4096], B=[8 * 160])
    args.update(kw)
    return adakv.Layer(**args)


def test_workspace_bytes(lib):
    small, big = _layer(), _layer(n=[65536], B=[8 * 1024])
    assert 0 < adakv.workspace_bytes(small) < adakv.workspace_bytes(big)


@pytest.mark.parametrize("kw", [
    dict(h_q=30), dict(w=0), dict(pool_k=4), dict(alpha=1.5), dict(alpha=-0.1),
    dict(B=[8 * 32 - 1]), dict(B=[8 * 32 + 8 * 4096 + 1]), dict(n=[0]),
    dict(n=[100, 100], B=[300, 300], tok_off=[0, 100, 264]),       # second sequence overlaps
])
def test_invalid_layers_are_rejected(lib, kw):
    L = _layer(**kw)
    assert adakv.workspace_bytes(L) == 0
    one = ctypes.c_void_p(16)      # never dereferenced: validation comes first
    st = lib.adakv_score(ctypes.byref(L.c), one, one, None, one, one, 1 << 30, None)
    assert st == -1
    assert lib.adakv_allocate(ctypes.byref(L.c), one, one, one, one, 1 << 30, None) == -1
    assert lib.adakv_select(ctypes.byref(L.c), one, one, one, one, one, 1 << 30, None) == -1
    assert lib.adakv_compact(ctypes.byref(L.c), one, one, one, one, one, one, None) == -1


@pytest.mark.parametrize("kw", [dict(d=96), dict(dtype=torch.float64), dict(k_strides=(8 * 128 + 4, 128))])
def test_unsupported_layers(lib, kw):
    L = _layer(**kw)
    one = ctypes.c_void_p(16)
    assert lib.adakv_score(ctypes.byref(L.c), one, one, None, one, one, 1 << 30, None) == -2


def test_null_pointers_and_small_workspace(lib):
    L = _layer()
    one = ctypes.c_void_p(16)
    assert lib.adakv_score(ctypes.byref(L.c), None, one, None, one, one, 1 << 30, None) == -1
    assert lib.adakv_score(ctypes.byref(L.c), one, one, None, one, one, 8, None) == -3
    assert lib.adakv_score(ctypes.byref(L.c), one, one, None, one, None, 1 << 30, None) == -3
    assert lib.adakv_allocate(ctypes.byref(L.c), one, None, one, one, 1 << 30, None) == -1
    assert lib.adakv_score(None, one, one, None, one, one, 1 << 30, None) == -1


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", "/nonexistent/libadakv.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        binding.load_library()


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)


def test_trace_arm_rejects_bad_arguments(lib):
    assert lib.adakv_trace_arm(None, 4) == -1
    arr = (ctypes.c_void_p * 2)()
    assert lib.adakv_trace_arm(arr, 1) == -1 and lib.adakv_trace_arm(arr, 100000) == -1
    assert lib.adakv_trace_disarm() == 0


def test_probe_read_rejects_bad_arguments(lib):
    lib.adakv_probe_read.restype = ctypes.c_int
    lib.adakv_probe_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
    assert lib.adakv_probe_read(None, 16, 4096, None) == -1
    assert lib.adakv_probe_read(4096, 16, None, None) == -1
    assert lib.adakv_probe_read(4096, 24, 8192, None) == -1
    assert lib.adakv_probe_read(4100, 16, 8192, None) == -2
    assert lib.adakv_probe_read(4096, 16, 8200, None) == -2


def test_generator_is_deterministic_and_shaped():
    from paper_2407_11550_amd import synth
    wl = synth.small_workload(8, 2, 128, 16, 7, [300, 77], [2 * 40, 2 * 20], seed=5)
    a = synth.generate(wl)
    b = synth.generate(wl)
    for x, y in zip(a, b):
        assert torch.equal(x, y)
    q, K, V = a
    assert q.shape == (2, 8, 16, 128) and K.shape == (300 + 16 + 77 + 16, 2, 128) and V.shape == K.shape
    assert wl.tok_off == [0, 316, 409]
    c = synth.generate(wl, layer=1)
    assert not torch.equal(c[1], K)                      # another layer, other values
    names = ["tiny", "llama8b_32k", "llama8b_128k", "llama8b_ragged", "llama70b_128k"]
    for nm in names:
        w = synth.workload(nm)
        for nb, Bb in zip(w.n, w.B):
            assert w.w * w.h_kv <= Bb <= w.w * w.h_kv + w.h_kv * nb


def test_decode_side_argument_checks(lib):
    L = _layer()
    one = ctypes.c_void_p(16)
    by = ctypes.byref(L.c)
    assert adakv.decode_workspace_bytes(L, 0) > 0
    assert adakv.decode_workspace_bytes(L, 64) >= adakv.decode_workspace_bytes(L, 0)
    assert adakv.decode_workspace_bytes(L, -1) == 0
    assert adakv.decode_workspace_bytes(_layer(h_q=24), 4) == 0          # g = 3 has no kernel
    assert adakv.decode_workspace_bytes(_layer(w=0), 4) == 0
    # invalid head-room, NULL pointers, unsupported group size, workspace too small
    assert lib.adakv_cache_build(by, one, one, one, one, -1, one, one, one, None) == -1
    assert lib.adakv_cache_build(by, one, one, one, one, 4, None, one, one, None) == -1
    assert lib.adakv_cache_build(by, one, one, one, one, 1 << 30, one, one, one, None) == -2   # rows >= 2^31
    assert lib.adakv_append(by, one, None, one, 4, one, one, one, None, None) == -1
    assert lib.adakv_append(by, one, one, one, -5, one, one, one, None, None) == -1
    assert lib.adakv_decode_attn(by, one, one, 4, one, one, one, None, None, one, 1 << 30, None) == -1
    assert lib.adakv_decode_attn(by, one, one, 4, one, one, one, one, None, one, 8, None) == -3
    assert lib.adakv_decode_attn(by, one, one, 4, one, one, one, one, None, None, 1 << 30, None) == -3
    L3 = _layer(h_q=24)
    assert lib.adakv_decode_attn(ctypes.byref(L3.c), one, one, 4, one, one, one, one, None, one, 1 << 30, None) == -2
    assert adakv.cache_rows(L, 5) == L.num_rows_out + L.num_segments * 5


def test_generated_prefill_lse_is_the_prefix_plus_window_normaliser():
    """synth.prefill_row_lse must be the log of the denominator the oracle's
    norm="prefix+window" uses: scores from the one equal scores from the other."""
    import numpy as np
    from oracle import adakv_oracle as O
    from paper_2407_11550_amd import synth
    wl = synth.small_workload(4, 2, 64, 5, 3, [70, 33], [2 * 12, 2 * 9], dtype=torch.float32, seed=4)
    q, K, V = synth.generate(wl)
    lse = synth.prefill_row_lse(wl, q, K)
    assert lse.shape == (2, 4, 5)
    off = wl.tok_off
    for b in range(2):
        qd, Kd = q[b].double().numpy(), K[off[b]:off[b + 1]].double().numpy()
        a = O.attention_rows(qd, Kd, wl.n[b], wl.w, norm="prefix+window")
        c = O.attention_rows(qd, Kd, wl.n[b], wl.w, row_lse=lse[b].double().numpy())
        assert np.allclose(a, c, rtol=2e-5, atol=1e-12)


def test_compress_checks_everything_before_launching(lib):
    L = _layer()
    one = ctypes.c_void_p(16)
    by = ctypes.byref(L.c)
    big = 1 << 30
    assert lib.adakv_compress(by, one, one, one, None, one, one, one, one, one, None, one, big, None) == -1
    assert lib.adakv_compress(by, one, one, one, None, one, one, one, one, one, one, one, 8, None) == -3
    assert lib.adakv_compress(by, one, one, one, None, one, one, one, one, one, one, None, big, None) == -3
    assert lib.adakv_compress(by, one, one, ctypes.c_void_p(24), None, one, one, one, one, one, one, one, big, None) == -2
    bad = _layer(alpha=2.0)
    assert lib.adakv_compress(ctypes.byref(bad.c), one, one, one, None, one, one, one, one, one, one, one, big, None) == -1


def test_binding_rejects_buffers_that_do_not_fit_the_layer(lib):
    """The kernels index every buffer by the layer's sizes; the binding compares them with the
    tensors before any pointer reaches the library.  CPU tensors suffice: the size checks come
    before the device check."""
    L = _layer(n=[100], B=[8 * 40])
    bf = torch.bfloat16
    q = torch.zeros(1, 32, 32, 128, dtype=bf)
    K = torch.zeros(132, 8, 128, dtype=bf)
    sc = torch.zeros(800)
    with pytest.raises(ValueError, match="K reaches"):
        adakv.score(L, q, K[:131])                                   # one row short of n + w
    with pytest.raises(ValueError, match="contiguous"):
        adakv.score(L, q, torch.zeros(132, 8, 144, dtype=bf)[:, :, :128])   # padded rows, strides not declared
    with pytest.raises(ValueError, match="q_window"):
        adakv.score(L, q[:, :31], K)
    with pytest.raises(ValueError, match="q_window must be contiguous"):
        adakv.score(L, q.transpose(1, 2), K)
    with pytest.raises(ValueError, match="scores holds 799"):
        adakv.score(L, q, K, out=torch.zeros(799))
    with pytest.raises(ValueError, match="row_lse"):
        adakv.score(L, q, K, row_lse=torch.zeros(32 * 31))
    with pytest.raises(ValueError, match="budgets"):
        adakv.allocate(L, sc, budgets=torch.zeros(7, dtype=torch.int32))
    with pytest.raises(ValueError, match="cu_seqlens"):
        adakv.allocate(L, sc, cu_seqlens=torch.zeros(8, dtype=torch.int32))
    with pytest.raises(ValueError, match="scores"):
        adakv.allocate(L, sc[:-1])
    i32 = lambda k: torch.zeros(k, dtype=torch.int32)
    with pytest.raises(ValueError, match="indices"):
        adakv.select(L, sc, i32(8), i32(9), indices=i32(319))
    with pytest.raises(ValueError, match="V reaches"):
        adakv.compact(L, K, K[:100], i32(320), i32(9))
    with pytest.raises(ValueError, match="K_out"):
        adakv.compact(L, K, K, i32(320), i32(9), K_out=torch.zeros(319, 128, dtype=bf))
    with pytest.raises(ValueError, match="ws must be a uint8"):
        adakv.compress(L, q, K, K, ws=torch.zeros(1 << 20, dtype=torch.float32))
    with pytest.raises(ValueError, match="indices"):
        adakv.compress(L, q, K, K, ws=torch.zeros(adakv.workspace_bytes(L), dtype=torch.uint8),
                       bufs=dict(indices=i32(10)))
    # declared strides: a view into a fused [token][2][head][d] buffer is accepted up to the device check
    kv = torch.zeros(132, 2, 8, 128, dtype=bf)
    Ls = _layer(n=[100], B=[8 * 40], k_strides=(2 * 8 * 128, 128), v_strides=(2 * 8 * 128, 128))
    with pytest.raises(ValueError, match="device tensor"):
        adakv.compact(Ls, kv[:, 0], kv[:, 1], i32(320), i32(9))
    with pytest.raises(ValueError, match="K reaches"):
        adakv.compact(Ls, kv[:131, 0], kv[:, 1], i32(320), i32(9))
    # a ragged batch: the last sequence's rows count
    Lb = _layer(n=[50, 60], B=[8 * 40, 8 * 40])
    with pytest.raises(ValueError, match="K reaches"):
        adakv.score(Lb, torch.zeros(2, 32, 32, 128, dtype=bf), torch.zeros(50 + 32 + 60 + 31, 8, 128, dtype=bf))
    # decode side
    with pytest.raises(ValueError, match="seg_len"):
        adakv.decode_attn(L, torch.zeros(1, 32, 128, dtype=bf), i32(9), 0, torch.zeros(320, 128, dtype=bf),
                          torch.zeros(320, 128, dtype=bf), i32(7), ws=torch.zeros(1 << 20, dtype=torch.uint8))
    with pytest.raises(ValueError, match="ws must be"):
        adakv.decode_attn(L, torch.zeros(1, 32, 128, dtype=bf), i32(9), 0, torch.zeros(320, 128, dtype=bf),
                          torch.zeros(320, 128, dtype=bf), i32(8), ws=torch.zeros(1 << 18, dtype=torch.int32))
