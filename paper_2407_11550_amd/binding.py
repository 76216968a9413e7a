"""ctypes binding of libadakv.so: argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI (include/adakv.h).
PyTorch is used for device memory and for the stream handle, nothing else.  There is
no fallback: if the library is missing, calls raise.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "lib", "libadakv.so")
_lib = None

ADAKV_BF16, ADAKV_FP32, ADAKV_FP16 = 0, 1, 2
ADAKV_FLAG_PIPELINE = 2
ADAKV_FLAG_POOL_THEN_MEAN = 4
MAX_BATCH = 64


class AdaKVError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = load_library().adakv_strerror(status).decode()
        super().__init__(f"{where}: {msg} (status {status})")


class _CLayer(ctypes.Structure):
    _fields_ = [
        ("dtype", ctypes.c_int32), ("h_q", ctypes.c_int32), ("h_kv", ctypes.c_int32),
        ("d", ctypes.c_int32), ("w", ctypes.c_int32), ("pool_k", ctypes.c_int32),
        ("alpha", ctypes.c_float), ("scale", ctypes.c_float), ("batch", ctypes.c_int32),
        ("n", ctypes.POINTER(ctypes.c_int32)), ("B", ctypes.POINTER(ctypes.c_int32)),
        ("tok_off", ctypes.POINTER(ctypes.c_int64)),
        ("k_stride_tok", ctypes.c_int64), ("k_stride_head", ctypes.c_int64),
        ("v_stride_tok", ctypes.c_int64), ("v_stride_head", ctypes.c_int64),
        ("flags", ctypes.c_uint32),
    ]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libadakv.so (built by __graft_entry__.build()).  Raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it first "
                           "(python -c 'import __graft_entry__ as g; g.build()'); "
                           "there is no fallback path")
    lib = ctypes.CDLL(_LIB_PATH)
    P, V, Z = ctypes.POINTER(_CLayer), ctypes.c_void_p, ctypes.c_size_t
    lib.adakv_workspace_bytes.restype = Z
    lib.adakv_workspace_bytes.argtypes = [P]
    lib.adakv_strerror.restype = ctypes.c_char_p
    lib.adakv_strerror.argtypes = [ctypes.c_int]
    for name, args in (("adakv_score", [P, V, V, V, V, V, Z, V]),
                       ("adakv_allocate", [P, V, V, V, V, Z, V]),
                       ("adakv_select", [P, V, V, V, V, V, Z, V]),
                       ("adakv_compact", [P, V, V, V, V, V, V, V])):
        fn = getattr(lib, name)
        fn.restype = ctypes.c_int
        fn.argtypes = args
    lib.adakv_compress.restype = ctypes.c_int
    lib.adakv_compress.argtypes = [P, V, V, V, V, V, V, V, V, V, V, V, Z, V]
    lib.adakv_compress_static.restype = ctypes.c_int
    lib.adakv_compress_static.argtypes = [P, V, V, V, V, V, V, V, V, V, V, V]
    I = ctypes.c_int32
    for name, args in (("adakv_cache_build", [P, V, V, V, V, I, V, V, V, V]),
                       ("adakv_append", [P, V, V, V, I, V, V, V, V, V]),
                       ("adakv_decode_attn", [P, V, V, I, V, V, V, V, V, V, Z, V]),
                       ("adakv_decode_step", [P, V, V, V, V, I, V, V, V, V, V, V, V, Z, V])):
        fn = getattr(lib, name)
        fn.restype = ctypes.c_int
        fn.argtypes = args
    lib.adakv_decode_workspace_bytes.restype = Z
    lib.adakv_decode_workspace_bytes.argtypes = [P, I]
    lib.adakv_pyramid_budgets.restype = ctypes.c_int
    lib.adakv_pyramid_budgets.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_double,
                                          ctypes.POINTER(ctypes.c_int64)]
    lib.adakv_trace_arm.restype = ctypes.c_int
    lib.adakv_trace_arm.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int]
    lib.adakv_trace_disarm.restype = ctypes.c_int
    lib.adakv_trace_disarm.argtypes = []
    lib.adakv_trace_name.restype = ctypes.c_char_p
    lib.adakv_trace_name.argtypes = [ctypes.c_int]
    lib.adakv_describe.restype = ctypes.c_int
    lib.adakv_describe.argtypes = [P, ctypes.c_int, ctypes.c_char_p, Z]
    lib.adakv_probe_read.restype = ctypes.c_int
    lib.adakv_probe_read.argtypes = [V, Z, V, V]
    _lib = lib
    return lib


class Layer:
    """Host-side description of one layer's compression problem (adakv_layer)."""

    def __init__(self, dtype, h_q, h_kv, d, w, pool_k, alpha, n, B, tok_off=None, scale=0.0,
                 k_strides=None, v_strides=None, flags=0):
        self.torch_dtype = dtype
        self.h_q, self.h_kv, self.d, self.w, self.pool_k = h_q, h_kv, d, w, pool_k
        self.alpha, self.scale = float(alpha), float(scale)
        self.n = [int(v) for v in (n if isinstance(n, (list, tuple)) else [n])]
        self.B = [int(v) for v in (B if isinstance(B, (list, tuple)) else [B])]
        self.batch = len(self.n)
        if tok_off is None:
            tok_off = [0]
            for nb in self.n:
                tok_off.append(tok_off[-1] + nb + w)
        self.tok_off = [int(v) for v in tok_off]
        self._n = (ctypes.c_int32 * self.batch)(*self.n)
        self._B = (ctypes.c_int32 * len(self.B))(*self.B)
        self._off = (ctypes.c_int64 * len(self.tok_off))(*self.tok_off)
        ks = k_strides or (h_kv * d, d)
        vs = v_strides or (h_kv * d, d)
        self.k_strides, self.v_strides = tuple(int(v) for v in ks), tuple(int(v) for v in vs)
        self.strides_given = (k_strides is not None, v_strides is not None)
        code = {torch.bfloat16: ADAKV_BF16, torch.float32: ADAKV_FP32, torch.float16: ADAKV_FP16}.get(dtype, 99)
        self.c = _CLayer(code, h_q, h_kv, d, w, pool_k, self.alpha, self.scale, self.batch,
                         self._n, self._B, self._off, ks[0], ks[1], vs[0], vs[1], flags)

    @classmethod
    def from_workload(cls, wl, **kw):
        return cls(wl.dtype, wl.h_q, wl.h_kv, wl.d, wl.w, wl.pool_k, wl.alpha, wl.n, wl.B,
                   tok_off=wl.tok_off, **kw)

    @property
    def last_token_row(self):
        """One past the last K/V row any sequence of the layer owns."""
        return max(self.tok_off[b] + self.n[b] + self.w for b in range(self.batch))

    @property
    def num_scores(self):
        return self.h_kv * sum(self.n)

    @property
    def num_rows_out(self):
        return sum(self.B)

    @property
    def num_segments(self):
        return self.batch * self.h_kv


def workspace_bytes(layer: Layer) -> int:
    return int(load_library().adakv_workspace_bytes(ctypes.byref(layer.c)))


def _ptr(t, name, dtype=None):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _need(t, numel, name):
    """A caller-supplied buffer must hold at least `numel` elements (the kernels index it by the
    layer's sizes and never look at the tensor)."""
    if t is not None and t.numel() < numel:
        raise ValueError(f"{name} holds {t.numel()} elements, the layer needs {numel}")


def _check_kv(layer, t, name, strides, given):
    """K or V must cover every row the layer addresses: element offset of the last one read is
    (tok_off[-1] - 1) * stride_tok + (h_kv - 1) * stride_head + d - 1.  When the layer was built
    without explicit strides it assumes a contiguous [tokens, h_kv, d] tensor."""
    if t is None:
        return
    if not given:
        want = (layer.h_kv * layer.d, layer.d, 1)
        if t.dim() != 3 or tuple(t.stride()) != want or t.shape[1] != layer.h_kv or t.shape[2] != layer.d:
            raise ValueError(f"{name} must be a contiguous [tokens, {layer.h_kv}, {layer.d}] tensor "
                             "(or give the Layer its strides)")
    rows = layer.last_token_row
    last = (rows - 1) * strides[0] + (layer.h_kv - 1) * strides[1] + layer.d
    # a view's reachable extent, from its own shape and strides
    extent = 1 + sum((sz - 1) * st for sz, st in zip(t.shape, t.stride())) if t.numel() else 0
    if extent < last:
        raise ValueError(f"{name} reaches {extent} elements from its first one, the layer addresses {last}")


def _check_q(layer, q):
    if not q.is_contiguous():
        raise ValueError("q_window must be contiguous")
    _need(q, layer.batch * layer.h_q * layer.w * layer.d, "q_window")


def _stream(stream):
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _workspace(layer, ws):
    if ws is None:
        ws = torch.empty(max(workspace_bytes(layer), 16), dtype=torch.uint8, device="cuda")
    if ws.dtype != torch.uint8:
        raise ValueError("ws must be a uint8 tensor (its size is taken in bytes)")
    return ws, ctypes.c_void_p(ws.data_ptr()), ctypes.c_size_t(ws.numel())


def score(layer: Layer, q_window, K, row_lse=None, out=None, ws=None, stream=None):
    """adakv_score: eviction scores [sum_b h_kv*n_b] fp32 (sequence-major, then head)."""
    lib = load_library()
    _check_q(layer, q_window)
    _check_kv(layer, K, "K", layer.k_strides, layer.strides_given[0])
    _need(row_lse, layer.batch * layer.h_q * layer.w, "row_lse")
    if out is None:
        out = torch.empty(layer.num_scores, dtype=torch.float32, device=K.device)
    _need(out, layer.num_scores, "scores")
    ws, wp, wn = _workspace(layer, ws)
    st = lib.adakv_score(ctypes.byref(layer.c), _ptr(q_window, "q_window", layer.torch_dtype),
                         _ptr(K, "K", layer.torch_dtype), _ptr(row_lse, "row_lse", torch.float32),
                         _ptr(out, "scores", torch.float32), wp, wn, _stream(stream))
    if st != 0:
        raise AdaKVError(st, "adakv_score")
    return out


def allocate(layer: Layer, scores, budgets=None, cu_seqlens=None, ws=None, stream=None):
    """adakv_allocate: budgets [batch*h_kv] and cu_seqlens [batch*h_kv+1], int32."""
    lib = load_library()
    if budgets is None:
        budgets = torch.empty(layer.num_segments, dtype=torch.int32, device=scores.device)
    if cu_seqlens is None:
        cu_seqlens = torch.empty(layer.num_segments + 1, dtype=torch.int32, device=scores.device)
    _need(scores, layer.num_scores, "scores")
    _need(budgets, layer.num_segments, "budgets")
    _need(cu_seqlens, layer.num_segments + 1, "cu_seqlens")
    ws, wp, wn = _workspace(layer, ws)
    st = lib.adakv_allocate(ctypes.byref(layer.c), _ptr(scores, "scores", torch.float32),
                            _ptr(budgets, "budgets", torch.int32),
                            _ptr(cu_seqlens, "cu_seqlens", torch.int32), wp, wn, _stream(stream))
    if st != 0:
        raise AdaKVError(st, "adakv_allocate")
    return budgets, cu_seqlens


def select(layer: Layer, scores, budgets, cu_seqlens, indices=None, ws=None, stream=None):
    """adakv_select: retained positions [sum_b B_b] int32, flattened by (sequence, head)."""
    lib = load_library()
    if indices is None:
        indices = torch.empty(layer.num_rows_out, dtype=torch.int32, device=scores.device)
    _need(scores, layer.num_scores, "scores")
    _need(budgets, layer.num_segments, "budgets")
    _need(cu_seqlens, layer.num_segments + 1, "cu_seqlens")
    _need(indices, layer.num_rows_out, "indices")
    ws, wp, wn = _workspace(layer, ws)
    st = lib.adakv_select(ctypes.byref(layer.c), _ptr(scores, "scores", torch.float32),
                          _ptr(budgets, "budgets", torch.int32),
                          _ptr(cu_seqlens, "cu_seqlens", torch.int32),
                          _ptr(indices, "indices", torch.int32), wp, wn, _stream(stream))
    if st != 0:
        raise AdaKVError(st, "adakv_select")
    return indices


def compact(layer: Layer, K, V, indices, cu_seqlens, K_out=None, V_out=None, stream=None):
    """adakv_compact: K_out, V_out [sum_b B_b, d] in the layer's dtype."""
    lib = load_library()
    if K_out is None:
        K_out = torch.empty((layer.num_rows_out, layer.d), dtype=layer.torch_dtype, device=K.device)
    if V_out is None:
        V_out = torch.empty((layer.num_rows_out, layer.d), dtype=layer.torch_dtype, device=K.device)
    _check_kv(layer, K, "K", layer.k_strides, layer.strides_given[0])
    _check_kv(layer, V, "V", layer.v_strides, layer.strides_given[1])
    _need(indices, layer.num_rows_out, "indices")
    _need(cu_seqlens, layer.num_segments + 1, "cu_seqlens")
    _need(K_out, layer.num_rows_out * layer.d, "K_out")
    _need(V_out, layer.num_rows_out * layer.d, "V_out")
    st = lib.adakv_compact(ctypes.byref(layer.c), _ptr(K, "K", layer.torch_dtype),
                           _ptr(V, "V", layer.torch_dtype), _ptr(indices, "indices", torch.int32),
                           _ptr(cu_seqlens, "cu_seqlens", torch.int32),
                           _ptr(K_out, "K_out", layer.torch_dtype),
                           _ptr(V_out, "V_out", layer.torch_dtype), _stream(stream))
    if st != 0:
        raise AdaKVError(st, "adakv_compact")
    return K_out, V_out


def compress(layer: Layer, q_window, K, V, row_lse=None, ws=None, stream=None, bufs=None,
             pipeline=True):
    """The whole step on one stream, no host synchronisation: adakv_compress (one ABI call, pipeline
    mode), or with pipeline=False the four self-contained calls one after the other.
    `bufs` may carry pre-allocated outputs (scores, budgets, cu_seqlens, indices, K_out, V_out)."""
    b = bufs or {}
    dev = K.device
    if ws is None:
        ws = torch.empty(max(workspace_bytes(layer), 16), dtype=torch.uint8, device=dev)
    if not pipeline:
        sc = score(layer, q_window, K, row_lse=row_lse, out=b.get("scores"), ws=ws, stream=stream)
        bud, cu = allocate(layer, sc, b.get("budgets"), b.get("cu_seqlens"), ws=ws, stream=stream)
        idx = select(layer, sc, bud, cu, b.get("indices"), ws=ws, stream=stream)
        K_out, V_out = compact(layer, K, V, idx, cu, b.get("K_out"), b.get("V_out"), stream=stream)
        return dict(scores=sc, budgets=bud, cu_seqlens=cu, indices=idx, K_out=K_out, V_out=V_out)
    lib = load_library()
    _check_q(layer, q_window)
    _check_kv(layer, K, "K", layer.k_strides, layer.strides_given[0])
    _check_kv(layer, V, "V", layer.v_strides, layer.strides_given[1])
    _need(row_lse, layer.batch * layer.h_q * layer.w, "row_lse")

    def buf(name, shape, dtype):
        t = b.get(name)
        return t if t is not None else torch.empty(shape, dtype=dtype, device=dev)

    sc = buf("scores", layer.num_scores, torch.float32)
    bud = buf("budgets", layer.num_segments, torch.int32)
    cu = buf("cu_seqlens", layer.num_segments + 1, torch.int32)
    idx = buf("indices", layer.num_rows_out, torch.int32)
    K_out = buf("K_out", (layer.num_rows_out, layer.d), layer.torch_dtype)
    V_out = buf("V_out", (layer.num_rows_out, layer.d), layer.torch_dtype)
    for t, numel, name in ((sc, layer.num_scores, "scores"), (bud, layer.num_segments, "budgets"),
                           (cu, layer.num_segments + 1, "cu_seqlens"), (idx, layer.num_rows_out, "indices"),
                           (K_out, layer.num_rows_out * layer.d, "K_out"), (V_out, layer.num_rows_out * layer.d, "V_out")):
        _need(t, numel, name)
    if ws.dtype != torch.uint8:                    # its size travels to the library, which checks it
        raise ValueError("ws must be a uint8 tensor (its size is taken in bytes)")
    st = lib.adakv_compress(ctypes.byref(layer.c), _ptr(q_window, "q_window", layer.torch_dtype),
                            _ptr(K, "K", layer.torch_dtype), _ptr(V, "V", layer.torch_dtype),
                            _ptr(row_lse, "row_lse", torch.float32), _ptr(sc, "scores", torch.float32),
                            _ptr(bud, "budgets", torch.int32), _ptr(cu, "cu_seqlens", torch.int32),
                            _ptr(idx, "indices", torch.int32), _ptr(K_out, "K_out", layer.torch_dtype),
                            _ptr(V_out, "V_out", layer.torch_dtype), ctypes.c_void_p(ws.data_ptr()),
                            ctypes.c_size_t(ws.numel()), _stream(stream))
    if st != 0:
        raise AdaKVError(st, "adakv_compress")
    return dict(scores=sc, budgets=bud, cu_seqlens=cu, indices=idx, K_out=K_out, V_out=V_out)


STATIC_SCRATCH_BYTES = 24 << 20        # ADAKV_STATIC_SCRATCH_BYTES


def compress_static(layer: Layer, q_window, K, V, row_lse=None, stream=None, bufs=None):
    """adakv_compress_static: the whole step with the library's built-in scratch array instead
    of a workspace; the C call allocates nothing (outputs not found in `bufs` are made here)."""
    lib = load_library()
    b = bufs or {}
    dev = K.device
    _check_q(layer, q_window)
    _check_kv(layer, K, "K", layer.k_strides, layer.strides_given[0])
    _check_kv(layer, V, "V", layer.v_strides, layer.strides_given[1])
    _need(row_lse, layer.batch * layer.h_q * layer.w, "row_lse")
    want = (("scores", layer.num_scores, (layer.num_scores,), torch.float32),
            ("budgets", layer.num_segments, (layer.num_segments,), torch.int32),
            ("cu_seqlens", layer.num_segments + 1, (layer.num_segments + 1,), torch.int32),
            ("indices", layer.num_rows_out, (layer.num_rows_out,), torch.int32),
            ("K_out", layer.num_rows_out * layer.d, (layer.num_rows_out, layer.d), layer.torch_dtype),
            ("V_out", layer.num_rows_out * layer.d, (layer.num_rows_out, layer.d), layer.torch_dtype))
    out = {}
    for name, numel, shape, dtype in want:
        t = b.get(name)
        out[name] = t if t is not None else torch.empty(shape, dtype=dtype, device=dev)
        _need(out[name], numel, name)
    st = lib.adakv_compress_static(
        ctypes.byref(layer.c), _ptr(q_window, "q_window", layer.torch_dtype),
        _ptr(K, "K", layer.torch_dtype), _ptr(V, "V", layer.torch_dtype),
        _ptr(row_lse, "row_lse", torch.float32), _ptr(out["scores"], "scores", torch.float32),
        _ptr(out["budgets"], "budgets", torch.int32), _ptr(out["cu_seqlens"], "cu_seqlens", torch.int32),
        _ptr(out["indices"], "indices", torch.int32), _ptr(out["K_out"], "K_out", layer.torch_dtype),
        _ptr(out["V_out"], "V_out", layer.torch_dtype), _stream(stream))
    if st != 0:
        raise AdaKVError(st, "adakv_compress_static")
    return out


def pyramid_budgets(n_layers: int, avg_budget: int, ratio: float):
    """adakv_pyramid_budgets: per-layer budgets of the pyramidal variant, largest first."""
    out = (ctypes.c_int64 * max(int(n_layers), 1))()
    st = load_library().adakv_pyramid_budgets(int(n_layers), int(avg_budget), float(ratio), out)
    if st != 0:
        raise AdaKVError(st, "adakv_pyramid_budgets")
    return [int(v) for v in out]


def describe(layer: Layer, row_lse: bool = False) -> dict:
    """adakv_describe: the kernel variant a layer of this shape gets, as a dict of its words."""
    buf = ctypes.create_string_buffer(512)
    st = load_library().adakv_describe(ctypes.byref(layer.c), int(bool(row_lse)), buf, 512)
    if st != 0:
        raise AdaKVError(st, "adakv_describe")
    return dict(word.split("=", 1) for word in buf.value.decode().split())


PROBE_SINK_BYTES = 2048 * 4 * 16      # ADAKV_PROBE_SINK_BYTES


def probe_read(src, sink=None, stream=None):
    """adakv_probe_read: one plain streaming read of `src` (a contiguous device tensor whose
    size in bytes is a multiple of 16); returns the sink, one 16-byte XOR word per wave."""
    if not src.is_contiguous():
        raise ValueError("src must be contiguous")
    if sink is None:
        sink = torch.empty(PROBE_SINK_BYTES, dtype=torch.uint8, device=src.device)
    if sink.numel() * sink.element_size() < PROBE_SINK_BYTES:
        raise ValueError("sink too small")
    st = load_library().adakv_probe_read(_ptr(src, "src"), ctypes.c_size_t(src.numel() * src.element_size()),
                                         _ptr(sink, "sink"), _stream(stream))
    if st != 0:
        raise AdaKVError(st, "adakv_probe_read")
    return sink


# ---- decode side of the flattened layout ---------------------------------------------------------
def cache_rows(layer: Layer, headroom: int) -> int:
    """Rows of K_cache / V_cache: every segment's retained rows plus `headroom` spare rows each."""
    return layer.num_rows_out + layer.num_segments * int(headroom)


def _check_cache(layer, K_cache, V_cache):
    """The cache tensors are addressed as contiguous rows of d elements."""
    for t, name in ((K_cache, "K_cache"), (V_cache, "V_cache")):
        if not t.is_contiguous() or t.shape[-1] != layer.d:
            raise ValueError(f"{name} must be a contiguous [rows, {layer.d}] tensor")


def _check_decode_bufs(layer, headroom, K_cache, V_cache, cu_seqlens, seg_len, out, lse, ws):
    _check_cache(layer, K_cache, V_cache)
    _need(cu_seqlens, layer.num_segments + 1, "cu_seqlens")
    _need(seg_len, layer.num_segments, "seg_len")
    _need(out, layer.batch * layer.h_q * layer.d, "out")
    _need(lse, layer.batch * layer.h_q, "lse")
    if ws.dtype != torch.uint8:                    # its size travels to the library, which checks it
        raise ValueError("ws must be a uint8 tensor (its size is taken in bytes)")


def decode_workspace_bytes(layer: Layer, headroom: int) -> int:
    return int(load_library().adakv_decode_workspace_bytes(ctypes.byref(layer.c), int(headroom)))


def cache_build(layer: Layer, K, V, indices, cu_seqlens, headroom, K_cache=None, V_cache=None,
                seg_len=None, stream=None):
    """adakv_cache_build: the gather of adakv_compact into the layout with head-room; returns
    (K_cache, V_cache, seg_len)."""
    lib = load_library()
    rows = cache_rows(layer, headroom)
    if K_cache is None:
        K_cache = torch.empty((rows, layer.d), dtype=layer.torch_dtype, device=K.device)
    if V_cache is None:
        V_cache = torch.empty((rows, layer.d), dtype=layer.torch_dtype, device=K.device)
    if seg_len is None:
        seg_len = torch.empty(layer.num_segments, dtype=torch.int32, device=K.device)
    if K_cache.shape[0] < rows or V_cache.shape[0] < rows or seg_len.numel() < layer.num_segments:
        raise ValueError("cache or seg_len too small for this layer and head-room")
    _check_kv(layer, K, "K", layer.k_strides, layer.strides_given[0])
    _check_kv(layer, V, "V", layer.v_strides, layer.strides_given[1])
    _need(indices, layer.num_rows_out, "indices")
    _need(cu_seqlens, layer.num_segments + 1, "cu_seqlens")
    _check_cache(layer, K_cache, V_cache)
    st = lib.adakv_cache_build(ctypes.byref(layer.c), _ptr(K, "K", layer.torch_dtype),
                               _ptr(V, "V", layer.torch_dtype), _ptr(indices, "indices", torch.int32),
                               _ptr(cu_seqlens, "cu_seqlens", torch.int32), int(headroom),
                               _ptr(K_cache, "K_cache", layer.torch_dtype),
                               _ptr(V_cache, "V_cache", layer.torch_dtype),
                               _ptr(seg_len, "seg_len", torch.int32), _stream(stream))
    if st != 0:
        raise AdaKVError(st, "adakv_cache_build")
    return K_cache, V_cache, seg_len


def append(layer: Layer, k_new, v_new, cu_seqlens, headroom, K_cache, V_cache, seg_len,
           overflow=None, stream=None):
    """adakv_append: one new K/V row per (sequence, KV head) behind each segment; seg_len grows."""
    lib = load_library()
    want = (layer.batch, layer.h_kv, layer.d)
    if tuple(k_new.shape) != want or tuple(v_new.shape) != want:
        raise ValueError(f"k_new and v_new must be {want}")
    if not (k_new.is_contiguous() and v_new.is_contiguous()):
        raise ValueError("k_new and v_new must be contiguous")
    if K_cache.shape[0] < cache_rows(layer, headroom) or V_cache.shape[0] < cache_rows(layer, headroom):
        raise ValueError("cache too small for this layer and head-room")
    _check_cache(layer, K_cache, V_cache)
    _need(cu_seqlens, layer.num_segments + 1, "cu_seqlens")
    _need(seg_len, layer.num_segments, "seg_len")
    _need(overflow, 1, "overflow")
    st = lib.adakv_append(ctypes.byref(layer.c), _ptr(k_new, "k_new", layer.torch_dtype),
                          _ptr(v_new, "v_new", layer.torch_dtype),
                          _ptr(cu_seqlens, "cu_seqlens", torch.int32), int(headroom),
                          _ptr(K_cache, "K_cache", layer.torch_dtype),
                          _ptr(V_cache, "V_cache", layer.torch_dtype),
                          _ptr(seg_len, "seg_len", torch.int32),
                          _ptr(overflow, "overflow", torch.int32), _stream(stream))
    if st != 0:
        raise AdaKVError(st, "adakv_append")
    return seg_len


def decode_attn(layer: Layer, q_new, cu_seqlens, headroom, K_cache, V_cache, seg_len, out=None,
                lse=None, ws=None, stream=None, want_lse=False):
    """adakv_decode_attn: out [batch, h_q, d] fp32 (and lse [batch, h_q] if asked for)."""
    lib = load_library()
    want = (layer.batch, layer.h_q, layer.d)
    if tuple(q_new.shape) != want or not q_new.is_contiguous():
        raise ValueError(f"q_new must be contiguous {want}")
    if K_cache.shape[0] < cache_rows(layer, headroom) or V_cache.shape[0] < cache_rows(layer, headroom):
        raise ValueError("cache too small for this layer and head-room")
    if out is None:
        out = torch.empty(want, dtype=torch.float32, device=q_new.device)
    if lse is None and want_lse:
        lse = torch.empty(want[:2], dtype=torch.float32, device=q_new.device)
    if ws is None:
        ws = torch.empty(max(decode_workspace_bytes(layer, headroom), 16), dtype=torch.uint8,
                         device=q_new.device)
    _check_decode_bufs(layer, headroom, K_cache, V_cache, cu_seqlens, seg_len, out, lse, ws)
    st = lib.adakv_decode_attn(ctypes.byref(layer.c), _ptr(q_new, "q_new", layer.torch_dtype),
                               _ptr(cu_seqlens, "cu_seqlens", torch.int32), int(headroom),
                               _ptr(K_cache, "K_cache", layer.torch_dtype),
                               _ptr(V_cache, "V_cache", layer.torch_dtype),
                               _ptr(seg_len, "seg_len", torch.int32),
                               _ptr(out, "out", torch.float32), _ptr(lse, "lse", torch.float32),
                               ctypes.c_void_p(ws.data_ptr()), ctypes.c_size_t(ws.numel()),
                               _stream(stream))
    if st != 0:
        raise AdaKVError(st, "adakv_decode_attn")
    return (out, lse) if (want_lse or lse is not None) else out


def decode_step(layer: Layer, q_new, k_new, v_new, cu_seqlens, headroom, K_cache, V_cache, seg_len,
                overflow=None, out=None, lse=None, ws=None, stream=None, want_lse=False):
    """adakv_decode_step: append k_new/v_new to every segment and attend, in one call."""
    lib = load_library()
    want = (layer.batch, layer.h_q, layer.d)
    wkv = (layer.batch, layer.h_kv, layer.d)
    if tuple(q_new.shape) != want or not q_new.is_contiguous():
        raise ValueError(f"q_new must be contiguous {want}")
    if tuple(k_new.shape) != wkv or tuple(v_new.shape) != wkv or not (k_new.is_contiguous() and v_new.is_contiguous()):
        raise ValueError(f"k_new and v_new must be contiguous {wkv}")
    if K_cache.shape[0] < cache_rows(layer, headroom) or V_cache.shape[0] < cache_rows(layer, headroom):
        raise ValueError("cache too small for this layer and head-room")
    if out is None:
        out = torch.empty(want, dtype=torch.float32, device=q_new.device)
    if lse is None and want_lse:
        lse = torch.empty(want[:2], dtype=torch.float32, device=q_new.device)
    if ws is None:
        ws = torch.empty(max(decode_workspace_bytes(layer, headroom), 16), dtype=torch.uint8,
                         device=q_new.device)
    _check_decode_bufs(layer, headroom, K_cache, V_cache, cu_seqlens, seg_len, out, lse, ws)
    _need(overflow, 1, "overflow")
    st = lib.adakv_decode_step(ctypes.byref(layer.c), _ptr(q_new, "q_new", layer.torch_dtype),
                               _ptr(k_new, "k_new", layer.torch_dtype),
                               _ptr(v_new, "v_new", layer.torch_dtype),
                               _ptr(cu_seqlens, "cu_seqlens", torch.int32), int(headroom),
                               _ptr(K_cache, "K_cache", layer.torch_dtype),
                               _ptr(V_cache, "V_cache", layer.torch_dtype),
                               _ptr(seg_len, "seg_len", torch.int32),
                               _ptr(overflow, "overflow", torch.int32),
                               _ptr(out, "out", torch.float32), _ptr(lse, "lse", torch.float32),
                               ctypes.c_void_p(ws.data_ptr()), ctypes.c_size_t(ws.numel()),
                               _stream(stream))
    if st != 0:
        raise AdaKVError(st, "adakv_decode_step")
    return (out, lse) if (want_lse or lse is not None) else out


class KernelTrace:
    """Per-kernel timing through adakv_trace_arm: inside the `with` block every kernel the
    library launches carries a pair of events that receive its own start and end time."""

    def __init__(self, capacity=128):
        self.events = [torch.cuda.Event(enable_timing=True) for _ in range(capacity)]
        for ev in self.events:                      # the first record creates the HIP event
            ev.record()
        self._arr = (ctypes.c_void_p * capacity)(*[ev.cuda_event for ev in self.events])
        self.used = 0
        self.names = []

    def __enter__(self):
        st = load_library().adakv_trace_arm(self._arr, len(self.events))
        if st != 0:
            raise AdaKVError(st, "adakv_trace_arm")
        return self

    def __exit__(self, *exc):
        lib = load_library()
        self.names = [lib.adakv_trace_name(i).decode() for i in range(len(self.events))]
        self.used = lib.adakv_trace_disarm()
        self.names = self.names[:self.used]
        return False

    def durations_us(self):
        """[(kernel name, microseconds)] for every traced kernel; call after a synchronize."""
        return [(self.names[i], 1000.0 * self.events[i].elapsed_time(self.events[i + 1]))
                for i in range(0, self.used - 1, 2)]
