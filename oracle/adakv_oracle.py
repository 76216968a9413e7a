"""Plain fp64 CPU oracle for the Ada-KV per-layer cache compression step.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the tests, the smoke check and
the benchmark's cpu_baseline leg may import it.  It shares no code with the HIP
path and never imports the package that wraps the HIP library.

What it computes is Algorithm 2 of the paper ("Ada-SnapKV/Ada-Pyramid in One
Layer") with Algorithm 1 ("Adaptive Budget Allocation") inside it, written out as
the plain definition, in numpy float64, with sort-based Top-k.  A matmul, an exp
and a stable sort are the only library steps.  No blocking, fusion or reordering.

Notation (kept from the paper where it has one):
    n        number of cache elements OUTSIDE the observation window (the eviction
             candidates, Alg. 2 input "cache outside observation window")
    w        observation window size ("winsize"); the cache holds N = n + w rows
    h        number of KV heads; g = h_q / h query heads share one KV head
             (Section 3.5: the group-mean attention weight is the criterion)
    B        layer budget including the w window rows of every head (Alg. 2 l.6)
    B'       B - w*h, the budget that Algorithm 1 distributes
    alpha    safeguard hyper-parameter (Alg. 2 l.8, Section 3.4)
    k        max-pool kernel size (Section 4.1: 7)

Readings taken where the paper is silent, garbled or at odds with itself
(each one is pinned or declared unpinned in the tests):
    R1  softmax is normalised over the n prefix keys only (Alg. 2 l.3 as
        printed).  norm="prefix+window" gives the other reading, where each
        window query also sees the window keys up to itself (causal).
        Which one the authors ran: parity unpinned.
    R2  logits are scaled by 1/sqrt(d) (the paper's footnote says it only
        omits the factor from the formulas).
    R3  the g*w rows of a KV head are averaged first and the pool is applied
        once to the averaged row (Section 3.4 prose).  order="pool_then_mean"
        is Alg. 2 l.4 as printed (pool every row, then mean).  For k = 1 the
        two agree.  The order itself: parity unpinned.
    R4  pooling is stride 1, same length, window clipped to [0, n).
    R5  alpha is the share given to the uniform allocation:
        x_i = (1-alpha)*f_i + alpha*B'/h.  Alg. 2 l.8 prints the two factors the
        other way round, which contradicts Section 3.4 (alpha prevents very
        small budgets), the robustness appendix (smaller alpha = more aggressive)
        and the alpha = 0 row of its table.
    R6  x_i is made integer with fixed-point alpha (16 fractional bits) and
        largest-remainder rounding, remainder ties to the lower head index, so
        that sum_i B_i = B' exactly.  Rounding rule: parity unpinned.
    R7  Top-k ties: larger score first, then smaller flat index (head-major,
        then position).  This makes every result unique.
    R8  retained rows of a head are in ascending position, window rows last.
"""
from __future__ import annotations

import math

import numpy as np

ALPHA_FRACTION_BITS = 16


# --------------------------------------------------------------------------- #
# Step 1 -- observation-window attention scores (Alg. 2 lines 1-5)
# --------------------------------------------------------------------------- #
def max_pool_same(x: np.ndarray, k: int) -> np.ndarray:
    """1-D max-pool along the last axis: stride 1, output length = input length,
    window [j - k//2, j + k//2] clipped to the array (Section 4.1, reading R4)."""
    if k < 1 or k % 2 == 0:
        raise ValueError("pool kernel must be odd and >= 1")
    n = x.shape[-1]
    r = k // 2
    out = np.empty_like(x)
    for j in range(n):
        lo, hi = max(0, j - r), min(n - 1, j + r)
        out[..., j] = x[..., lo:hi + 1].max(axis=-1)
    return out


def attention_rows(q_window, K, n, w, scale=None, norm="prefix", row_lse=None):
    """Softmax attention weights of every window query over the n prefix keys.

    q_window [h_q, w, d], K [n + w, h, d] (rows n.. are the window's own keys).
    Returns A [h_q, w, n] float64 (Alg. 2 l.3: A_i = softmax(Q_i^win K_i^T)).

    norm="prefix": the denominator runs over the n prefix keys (R1).
    norm="prefix+window": window query r also sees window keys 0..r (causal) and
        the denominator includes them; the returned weights are still only the
        prefix part, so each row sums to 1 - (its window mass).
    row_lse [h_q, w]: if given, it IS the log of the denominator (natural log of
        the sum of exp(scaled logit)) and `norm` is ignored.
    """
    q = np.asarray(q_window, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    h_q, w_, d = q.shape
    N, h, d2 = K.shape
    if w_ != w or d2 != d or N < n + (w if norm == "prefix+window" and row_lse is None else 0):
        raise ValueError("shape mismatch")
    if h_q % h != 0:
        raise ValueError("h_q must be a multiple of h")
    g = h_q // h
    if scale is None:
        scale = 1.0 / math.sqrt(d)                      # R2
    A = np.empty((h_q, w, n), dtype=np.float64)
    for hq in range(h_q):
        c = hq // g                                     # KV head of this query head
        s = scale * (q[hq] @ K[:n, c, :].T)             # [w, n] logits
        if row_lse is not None:
            A[hq] = np.exp(s - np.asarray(row_lse, dtype=np.float64)[hq][:, None])
            continue
        if norm == "prefix":
            m = s.max(axis=1, keepdims=True)
            e = np.exp(s - m)
            A[hq] = e / e.sum(axis=1, keepdims=True)
        elif norm == "prefix+window":
            sw = scale * (q[hq] @ K[n:n + w, c, :].T)   # [w, w] logits on window keys
            sw = np.where(np.tri(w, dtype=bool), sw, -np.inf)   # query r sees keys <= r
            m = np.maximum(s.max(axis=1, keepdims=True), sw.max(axis=1, keepdims=True))
            e = np.exp(s - m)
            den = e.sum(axis=1, keepdims=True) + np.exp(sw - m).sum(axis=1, keepdims=True)
            A[hq] = e / den
        else:
            raise ValueError("unknown norm")
    return A


def score(q_window, K, n, w, pool_k, scale=None, norm="prefix", row_lse=None,
          order="mean_then_pool"):
    """Per-KV-head eviction scores [h, n], float32 (the interchange format that every
    later step reads).

    Alg. 2 lines 2-4 plus Section 3.5: attention weights of the window queries,
    mean over the w window rows and over the g query heads of the group, max-pool.
    """
    A = attention_rows(q_window, K, n, w, scale=scale, norm=norm, row_lse=row_lse)
    h_q = A.shape[0]
    h = np.asarray(K).shape[1]
    g = h_q // h
    A = A.reshape(h, g * w, n)                          # rows of KV head c: its g heads x w
    if order == "mean_then_pool":                       # R3
        raw = A.mean(axis=1)
        pooled = max_pool_same(raw, pool_k)
    elif order == "pool_then_mean":                     # Alg. 2 l.4 as printed
        pooled = max_pool_same(A, pool_k).mean(axis=1)
    else:
        raise ValueError("unknown order")
    return pooled.astype(np.float32)


# --------------------------------------------------------------------------- #
# Step 2 -- adaptive budget allocation (Alg. 1, Alg. 2 lines 6-8)
# --------------------------------------------------------------------------- #
def topk_flat(values: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest entries of a 1-D array under the total order
    (value descending, index ascending) (R7), in that order."""
    v = np.asarray(values)
    if not 0 <= k <= v.size:
        raise ValueError("k out of range")
    order = np.argsort(-v.astype(np.float64), kind="stable")   # stable: equal values keep index order
    return order[:k]


def adaptive_counts(scores: np.ndarray, Bp: int) -> np.ndarray:
    """Algorithm 1: concatenate all heads' scores, take the Top-B', count per head."""
    h, n = scores.shape
    top = topk_flat(scores.reshape(-1), Bp)
    return np.bincount(top // n, minlength=h).astype(np.int64)


def safeguard(f: np.ndarray, Bp: int, alpha: float) -> np.ndarray:
    """Alg. 2 l.8 under readings R5/R6: integer budgets with sum = B'.

    x_i = (1-alpha) f_i + alpha B'/h, with alpha = a/65536, equals num_i/den for
    num_i = (65536-a) h f_i + a B' and den = 65536 h.  Floor, then hand the R
    missing units to the heads with the largest remainders (ties: lower index).
    """
    if not 0.0 <= alpha <= 1.0:
        raise ValueError("alpha must be in [0, 1]")
    f = [int(v) for v in f]
    h = len(f)
    one = 1 << ALPHA_FRACTION_BITS
    a = int(math.floor(alpha * one + 0.5))
    den = one * h
    num = [(one - a) * h * fi + a * Bp for fi in f]     # Python ints: exact
    base = [v // den for v in num]
    rem = [v % den for v in num]
    R = Bp - sum(base)
    assert 0 <= R < max(h, 1) or (h == 0 and R == 0)
    by_rem = sorted(range(h), key=lambda i: (-rem[i], i))
    for i in by_rem[:R]:
        base[i] += 1
    return np.asarray(base, dtype=np.int32)


def allocate(scores, B: int, w: int, alpha: float):
    """Budgets [h] (prefix rows only) and cu_seqlens [h+1] (each head's segment holds
    its budget plus the w window rows).  Alg. 2 lines 6-8."""
    scores = np.asarray(scores, dtype=np.float32)
    h, n = scores.shape
    Bp = B - w * h                                      # Alg. 2 l.6
    if Bp < 0 or Bp > h * n:
        raise ValueError("budget out of range")
    f = adaptive_counts(scores, Bp)                     # Alg. 2 l.7 / Alg. 1
    budgets = safeguard(f, Bp, alpha)                   # Alg. 2 l.8
    cu = np.zeros(h + 1, dtype=np.int32)
    cu[1:] = np.cumsum(budgets.astype(np.int64) + w)
    return budgets, cu


# --------------------------------------------------------------------------- #
# Step 3 -- per-head Top-k eviction decision (Alg. 2 line 9)
# --------------------------------------------------------------------------- #
def select(scores, budgets, w: int) -> np.ndarray:
    """Retained positions, flattened by head: for head i the B_i prefix positions with
    the largest scores (ties R7) in ascending order, then the window positions
    n .. n+w-1 (Alg. 2 lines 9-11, R8)."""
    scores = np.asarray(scores, dtype=np.float32)
    h, n = scores.shape
    out = []
    for i in range(h):
        keep = np.sort(topk_flat(scores[i], int(budgets[i])))
        out.append(keep.astype(np.int32))
        out.append(np.arange(n, n + w, dtype=np.int32))
    return np.concatenate(out) if out else np.zeros(0, np.int32)


# --------------------------------------------------------------------------- #
# Step 4 -- gather into the flattened per-head cache (Alg. 2 lines 10-11, Sec. 3.5)
# --------------------------------------------------------------------------- #
def compact(K, V, indices, cu_seqlens):
    """K_out, V_out [cu[-1], d]: row cu[i]+t of the output is row indices[cu[i]+t] of
    head i of the input."""
    K = np.asarray(K)
    V = np.asarray(V)
    h = len(cu_seqlens) - 1
    d = K.shape[2]
    K_out = np.empty((int(cu_seqlens[-1]), d), dtype=K.dtype)
    V_out = np.empty((int(cu_seqlens[-1]), d), dtype=V.dtype)
    for i in range(h):
        for t in range(int(cu_seqlens[i]), int(cu_seqlens[i + 1])):
            K_out[t] = K[indices[t], i]
            V_out[t] = V[indices[t], i]
    return K_out, V_out


# --------------------------------------------------------------------------- #
# Whole step, and the ragged batch (sequences are independent: Alg. 1 acts within
# one layer of one sequence)
# --------------------------------------------------------------------------- #
def compress_layer(q_window, K, V, n, w, pool_k, B, alpha, scale=None, norm="prefix",
                   row_lse=None, order="mean_then_pool"):
    """Algorithm 2 top to bottom for one sequence."""
    sc = score(q_window, K, n, w, pool_k, scale=scale, norm=norm, row_lse=row_lse, order=order)
    budgets, cu = allocate(sc, B, w, alpha)
    idx = select(sc, budgets, w)
    K_out, V_out = compact(K, V, idx, cu)
    return dict(scores=sc, budgets=budgets, cu_seqlens=cu, indices=idx, K_out=K_out, V_out=V_out)


def compress_batch(q_window, K, V, n_list, B_list, tok_off, w, pool_k, alpha, scale=None):
    """Ragged batch in the packed layout: sequence b owns rows tok_off[b] ..
    tok_off[b] + n_b + w - 1 of K/V and q_window[b].  Outputs are concatenated
    sequence-major; cu_seqlens has batch*h + 1 entries and runs on across sequences."""
    outs = [compress_layer(q_window[b], K[tok_off[b]:tok_off[b] + n_list[b] + w],
                           V[tok_off[b]:tok_off[b] + n_list[b] + w], n_list[b], w, pool_k,
                           B_list[b], alpha, scale=scale) for b in range(len(n_list))]
    cu = [np.zeros(1, np.int32)]
    base = 0
    for o in outs:
        cu.append(o["cu_seqlens"][1:] + base)
        base += int(o["cu_seqlens"][-1])
    return dict(scores=np.concatenate([o["scores"].reshape(-1) for o in outs]),
                budgets=np.concatenate([o["budgets"] for o in outs]),
                cu_seqlens=np.concatenate(cu).astype(np.int32),
                indices=np.concatenate([o["indices"] for o in outs]),
                K_out=np.concatenate([o["K_out"] for o in outs]),
                V_out=np.concatenate([o["V_out"] for o in outs]))


# --------------------------------------------------------------------------- #
# The quantity the theory optimises (Theorems 3.1-3.3): epsilon = 2hC - 2C * (retained
# attention weight), so minimising epsilon is maximising the retained weight.
# --------------------------------------------------------------------------- #
def retained_weight(scores, indices, cu_seqlens, n) -> float:
    """Sum over heads of the scores of the retained prefix positions, in float64."""
    scores = np.asarray(scores, dtype=np.float64)
    tot = 0.0
    for i in range(len(cu_seqlens) - 1):
        seg = np.asarray(indices[int(cu_seqlens[i]):int(cu_seqlens[i + 1])])
        seg = seg[seg < n]
        tot += float(scores[i, seg].sum())
    return tot


def eviction_loss_and_bound(q, K, V, WO, keep):
    """Window-1 setting of Section 3.2.  q [h, d_h], K, V [n, h, d_h], WO [h, d_h, d_model],
    keep [h, n] in {0,1}.  Returns (||y - y_hat||_1, epsilon) of eqs. (4)-(6):
    y = sum_i A_i V_i W_i^O with A_i = softmax(q_i K_i^T) (no scale, as in Section 3.1),
    y_hat with evicted logits at -inf, epsilon = 2hC - 2C sum_i sum_j I_i^j A_i^j,
    C = max_i ||V_i W_i^O||_inf (max absolute row sum)."""
    q = np.asarray(q, np.float64); K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64); WO = np.asarray(WO, np.float64)
    keep = np.asarray(keep, bool)
    h = q.shape[0]
    y = 0.0; y_hat = 0.0; C = 0.0; kept_mass = 0.0
    for i in range(h):
        s = K[:, i, :] @ q[i]
        e = np.exp(s - s.max())
        A = e / e.sum()
        s_hat = np.where(keep[i], s, -np.inf)
        e_hat = np.exp(s_hat - s_hat.max())
        A_hat = e_hat / e_hat.sum()
        VW = V[:, i, :] @ WO[i]
        y = y + A @ VW
        y_hat = y_hat + A_hat @ VW
        C = max(C, float(np.abs(VW).sum(axis=1).max()))
        kept_mass += float(A[keep[i]].sum())
    return float(np.abs(y - y_hat).sum()), 2 * h * C - 2 * C * kept_mass


# --------------------------------------------------------------------------- #
# Layer budgets of the pyramidal variant (Section 3.4).  The paper leaves the schedule's
# hyper-parameters open; reading taken: linear in depth, largest first, mean = avg, the
# first-to-last ratio given.  Exact rational arithmetic.  Parity unpinned (the choice
# of schedule); the properties below it are pinned in the tests.
# --------------------------------------------------------------------------- #
def pyramid_budgets(n_layers: int, avg_budget: int, ratio) -> list:
    from fractions import Fraction
    r = Fraction(ratio)
    if n_layers == 1:
        return [avg_budget]
    b_min = Fraction(2 * avg_budget) / (1 + r)
    b_max = r * b_min
    real = [b_max - (b_max - b_min) * Fraction(l, n_layers - 1) for l in range(n_layers)]
    out = [math.floor(x) for x in real]
    left = n_layers * avg_budget - sum(out)
    for l in range(left):
        out[l % n_layers] += 1
    return out
