"""Plain fp64 CPU oracle for the decode side of the flattened per-head cache.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the tests, the smoke check and
the benchmark's cpu_baseline leg may import it.  It shares no code with the HIP
path and never imports the package that wraps the HIP library.

What it covers (Section 3.5, "Variable-length Attention with Variable-sized Cache
Elements", on top of Section 3.1):
    * the flattened storage layout: the retained rows of all heads of a layer in one
      [rows, d] tensor, head after head, each head's segment with its own length;
    * the cache update of Eq. (1), K_i = Cat[K_i : k_i], V_i likewise, for every head;
    * one decoding step of Eq. (2) per head on that layout: A_i = softmax(q_i K_i^T),
      o_i = A_i V_i (the projection by W^O and the sum over heads are a dense matmul
      outside this path).

Notation:
    segment s = b*h + c    the cache of KV head c of sequence b
    cu_seqlens [S+1]       as written at compression time: segment s then held
                           cu[s+1]-cu[s] rows (its budget plus the w window rows)
    headroom               spare rows left behind every segment for appended tokens
    start_s                cu[s] + s*headroom, first row of segment s
    cap_s                  cu[s+1]-cu[s] + headroom, rows the segment can hold
    lens [S]               rows currently held
    g                      query heads per KV head; query head i reads KV head i // g

Readings (the paper fixes none of these; Section 3.5 names the layout and the two
operations and nothing else):
    D1  a segment's spare rows follow it directly, the same number for every segment.
    D2  an append into a full segment changes nothing and is reported.
    D3  logits are scaled by 1/sqrt(d) unless a scale is given (Section 3.1's footnote:
        the factor is only left out of the formulas).
    D4  a segment of length 0 yields a zero output row and lse = -inf.
"""
from __future__ import annotations

import math

import numpy as np


def segment_starts(cu_seqlens, headroom: int) -> np.ndarray:
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    S = len(cu) - 1
    return cu[:-1] + headroom * np.arange(S, dtype=np.int64)


def segment_caps(cu_seqlens, headroom: int) -> np.ndarray:
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    return cu[1:] - cu[:-1] + headroom


def build_cache(K_rows, V_rows, cu_seqlens, headroom: int):
    """Spread the tightly packed retained rows ([cu[-1], d], segment s at cu[s]) into
    the layout with head-room.  Returns (K_cache, V_cache, lens); spare rows are zero."""
    K_rows = np.asarray(K_rows); V_rows = np.asarray(V_rows)
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    S = len(cu) - 1
    start = segment_starts(cu, headroom)
    total = int(cu[-1]) + S * headroom
    Kc = np.zeros((total, K_rows.shape[1]), dtype=K_rows.dtype)
    Vc = np.zeros((total, V_rows.shape[1]), dtype=V_rows.dtype)
    lens = (cu[1:] - cu[:-1]).astype(np.int64)
    for s in range(S):
        Kc[start[s]:start[s] + lens[s]] = K_rows[cu[s]:cu[s + 1]]
        Vc[start[s]:start[s] + lens[s]] = V_rows[cu[s]:cu[s + 1]]
    return Kc, Vc, lens


def append(K_cache, V_cache, cu_seqlens, headroom: int, lens, k_new, v_new):
    """Eq. (1) for every segment, in place: row k_new[s] goes behind the lens[s] rows of
    segment s.  k_new, v_new [S, d].  Returns True if some segment was full (reading D2:
    that segment is left as it was)."""
    start = segment_starts(cu_seqlens, headroom)
    cap = segment_caps(cu_seqlens, headroom)
    overflow = False
    for s in range(len(lens)):
        if lens[s] >= cap[s]:
            overflow = True
            continue
        K_cache[start[s] + lens[s]] = k_new[s]
        V_cache[start[s] + lens[s]] = v_new[s]
        lens[s] += 1
    return overflow


def decode_attention(q_new, K_cache, V_cache, cu_seqlens, headroom: int, lens, g: int,
                     scale=None):
    """Eq. (2) head by head.  q_new [batch, h_q, d]; segment (b, c) serves the query heads
    c*g .. c*g+g-1 of sequence b.  Returns (out [batch, h_q, d], lse [batch, h_q]) in
    float64, lse = natural log of the sum of exp(scaled logit) over the segment's rows."""
    q_new = np.asarray(q_new, dtype=np.float64)
    batch, h_q, d = q_new.shape
    h = h_q // g
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    start = segment_starts(cu_seqlens, headroom)
    out = np.zeros((batch, h_q, d), dtype=np.float64)
    lse = np.full((batch, h_q), -np.inf, dtype=np.float64)
    for b in range(batch):
        for i in range(h_q):
            s = b * h + i // g
            L = int(lens[s])
            if L == 0:
                continue
            Ki = np.asarray(K_cache[start[s]:start[s] + L], dtype=np.float64)
            Vi = np.asarray(V_cache[start[s]:start[s] + L], dtype=np.float64)
            logit = scale * (Ki @ q_new[b, i])
            mx = logit.max()
            e = np.exp(logit - mx)
            A = e / e.sum()
            out[b, i] = A @ Vi
            lse[b, i] = mx + math.log(e.sum())
    return out, lse
