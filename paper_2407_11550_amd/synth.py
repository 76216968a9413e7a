"""Seeded synthetic layers shaped like the paper's workloads.

The paper measures on Ruler-16K and LongBench prompts run through Llama-3.1-8B/70B
and Mistral-7B (Section 4.1); neither the datasets nor the weights are available, so
these inputs stand in for them: the tensor shapes are those models' attention layers
(32 or 64 query heads over 8 KV heads, head dimension 128), the hyper-parameters are
the paper's (window 32, pool kernel 7, alpha 0.2, Section 4.1), and the value
structure imitates what Figure 1 describes: heads range from dispersed to sharply
concentrated, a few "critical" keys per head carry most of the weight, and the first
token is an attention sink.

This module holds no arithmetic of the method itself.  It serves the oracle-side
tests, the GPU parity tests and the benchmark alike; the oracle and the HIP binding
do not import each other.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np
import torch


@dataclasses.dataclass
class Workload:
    name: str
    dtype: torch.dtype
    h_q: int
    h_kv: int
    d: int
    w: int
    pool_k: int
    alpha: float
    n: list            # prefix length per sequence
    B: list            # layer budget per sequence (window rows included)
    temps: object      # list of per-q-head temperatures, or (lo, hi) for log-uniform
    planted: object    # int, or (lo, hi) for a log-uniform count per KV head
    seed: int
    layers: int = 1

    @property
    def batch(self):
        return len(self.n)

    @property
    def g(self):
        return self.h_q // self.h_kv

    @property
    def tok_off(self):
        off = [0]
        for nb in self.n:
            off.append(off[-1] + nb + self.w)
        return off

    @property
    def total_prefix_tokens(self):
        return int(sum(self.n))


def _ragged_lengths(seed, batch, lo, hi):
    rng = np.random.Generator(np.random.PCG64(seed))
    return [int(v) for v in rng.integers(lo, hi + 1, size=batch)]


def workload(name: str, alpha: float | None = None) -> Workload:
    """The five configurations the build is measured and tested on."""
    if name == "tiny":          # 4 heads, no GQA, fp32
        wl = Workload("tiny", torch.float32, 4, 4, 64, 8, 7, 0.2, [1024], [512],
                      [0.5, 1.0, 2.0, 4.0], 16, seed=0)
    elif name == "llama8b_32k":
        wl = Workload("llama8b_32k", torch.bfloat16, 32, 8, 128, 32, 7, 0.2, [32768], [8192],
                      (0.25, 4.0), (8, 4096), seed=1000)
    elif name == "llama8b_128k":
        wl = Workload("llama8b_128k", torch.bfloat16, 32, 8, 128, 32, 7, 0.2, [131072],
                      [8 * 2048], (0.25, 4.0), (8, 4096), seed=2000)
    elif name == "llama8b_ragged":
        n = _ragged_lengths(3000, 8, 4096, 65536)
        B = [8 * max(32, int(round(0.05 * nb))) for nb in n]
        wl = Workload("llama8b_ragged", torch.bfloat16, 32, 8, 128, 32, 7, 0.2, n, B,
                      (0.25, 4.0), (8, 4096), seed=3000, layers=32)
    elif name == "llama70b_128k":
        wl = Workload("llama70b_128k", torch.bfloat16, 64, 8, 128, 64, 7, 0.2, [131072],
                      [8 * 4096], (0.25, 4.0), (8, 4096), seed=4000)
    else:
        raise KeyError(name)
    if alpha is not None:
        wl.alpha = alpha
    return wl


def small_workload(h_q, h_kv, d, w, pool_k, n, B, alpha=0.2, dtype=torch.bfloat16, seed=7,
                   temps=(0.25, 4.0), planted=(2, 64)) -> Workload:
    """Free-form shape for parity tests (same generator as the named workloads)."""
    n = list(n) if isinstance(n, (list, tuple)) else [n]
    B = list(B) if isinstance(B, (list, tuple)) else [B]
    return Workload("custom", dtype, h_q, h_kv, d, w, pool_k, alpha, n, B, temps, planted, seed)


def _log_uniform(rng, lo, hi, size):
    return np.exp(rng.uniform(math.log(lo), math.log(hi), size=size))


def generate(wl: Workload, layer: int = 0, device="cpu"):
    """q_window [batch, h_q, w, d], K, V [sum_b (n_b + w), h_kv, d] in wl.dtype, packed
    sequence after sequence (sequence b owns rows tok_off[b] .. tok_off[b+1]-1, its window
    being the last w of them).

    Recipe, per sequence:
      1. K, V ~ N(0,1) i.i.d.
      2. q_window[hq] = t_hq * N(0,1): t_hq is the head's temperature (a larger t gives a
         more concentrated head).
      3. every KV head gets planted critical prefix positions (never position 0); the key
         there is 3 * qbar, qbar = mean of the group's g*w window queries.
      4. attention sink: K[0, c] += 2*sqrt(d) * qbar / |qbar|^2, which adds exactly +2 to
         the scaled logit of the mean query on token 0.
      5. everything is rounded to wl.dtype once, at the end.
    """
    dev = torch.device(device)
    seed = wl.seed + layer
    tg = torch.Generator(device=dev)
    tg.manual_seed(seed)
    rng = np.random.Generator(np.random.PCG64(seed))
    h_q, h, d, w, g = wl.h_q, wl.h_kv, wl.d, wl.w, wl.g
    off = wl.tok_off
    K = torch.empty((off[-1], h, d), dtype=wl.dtype, device=dev)
    V = torch.empty((off[-1], h, d), dtype=wl.dtype, device=dev)
    q = torch.empty((wl.batch, h_q, w, d), dtype=wl.dtype, device=dev)
    for b, nb in enumerate(wl.n):
        if isinstance(wl.temps, tuple):
            t = _log_uniform(rng, wl.temps[0], wl.temps[1], h_q)
        else:
            t = np.asarray(wl.temps, dtype=np.float64)
        tt = torch.tensor(t, dtype=torch.float32, device=dev).view(h_q, 1, 1)
        qb = torch.randn((h_q, w, d), generator=tg, dtype=torch.float32, device=dev) * tt
        Kb = torch.randn((nb + w, h, d), generator=tg, dtype=torch.float32, device=dev)
        Vb = torch.randn((nb + w, h, d), generator=tg, dtype=torch.float32, device=dev)
        qbar = qb.view(h, g * w, d).mean(dim=1)                       # [h, d]
        for c in range(h):
            if isinstance(wl.planted, tuple):
                cnt = int(round(float(_log_uniform(rng, wl.planted[0], wl.planted[1], 1)[0])))
            else:
                cnt = int(wl.planted)
            cnt = max(0, min(cnt, nb // 2, nb - 1))
            if cnt > 0:
                pos = rng.choice(nb - 1, size=cnt, replace=False) + 1
                Kb[torch.as_tensor(pos, device=dev), c, :] = 3.0 * qbar[c]
            Kb[0, c, :] += 2.0 * math.sqrt(d) * qbar[c] / (qbar[c] * qbar[c]).sum()
        K[off[b]:off[b + 1]] = Kb.to(wl.dtype)
        V[off[b]:off[b + 1]] = Vb.to(wl.dtype)
        q[b] = qb.to(wl.dtype)
    return q, K, V


def concentration(scores_head: np.ndarray, top_fraction: float = 0.05) -> float:
    """Share of a head's total score held by its largest `top_fraction` of positions
    (the statistic Figure 1a plots); a description of the generated inputs only."""
    v = np.sort(np.asarray(scores_head, dtype=np.float64))[::-1]
    k = max(1, int(round(top_fraction * v.size)))
    return float(v[:k].sum() / v.sum())


# ---- decode side: compressed caches of uneven per-head length, and per-step inputs -------------
def skewed_budgets(wl: Workload, seed: int = 0, skew: float = 1.5):
    """Per-segment prefix budgets [batch*h_kv] with sum over the heads of sequence b equal to
    B_b - w*h_kv, spread unevenly (weights exp(skew * N(0,1)), capped at n_b): the kind of
    length mix adaptive allocation produces (a few long heads, some holding little more than
    the window).  A description of inputs only; no part of the allocation rule."""
    rng = np.random.Generator(np.random.PCG64(10_000 + seed))
    out = []
    for nb, Bb in zip(wl.n, wl.B):
        Bp = Bb - wl.w * wl.h_kv
        if not 0 <= Bp <= nb * wl.h_kv:
            raise ValueError(f"budget {Bb} does not fit {wl.h_kv} heads of {nb} prefix tokens plus the window")
        wgt = np.exp(skew * rng.standard_normal(wl.h_kv))
        raw = np.minimum(np.floor(Bp * wgt / wgt.sum()).astype(np.int64), nb)
        left = Bp - int(raw.sum())
        c = 0
        while left > 0:                       # hand the remainder out wherever there is room
            room = nb - int(raw[c % wl.h_kv])
            take = min(room, left)
            raw[c % wl.h_kv] += take
            left -= take
            c += 1
        out.extend(int(v) for v in raw)
    return out


def ragged_cache(wl: Workload, budgets, headroom: int, seed: int = 0, device="cpu"):
    """A compressed cache in the flattened layout without running the compression: segment
    s = b*h_kv + c holds budgets[s] + w rows of N(0,1) keys and values (in wl.dtype) at row
    cu[s] + s*headroom; spare rows are zero.  Returns (K_cache, V_cache, cu_seqlens, seg_len),
    the last two int32."""
    dev = torch.device(device)
    tg = torch.Generator(device=dev)
    tg.manual_seed(20_000 + seed)
    lens = [int(b) + wl.w for b in budgets]
    cu = [0]
    for v in lens:
        cu.append(cu[-1] + v)
    rows = cu[-1] + len(lens) * headroom
    Kc = torch.zeros((rows, wl.d), dtype=wl.dtype, device=dev)
    Vc = torch.zeros((rows, wl.d), dtype=wl.dtype, device=dev)
    for s, L in enumerate(lens):
        a = cu[s] + s * headroom
        Kc[a:a + L] = torch.randn((L, wl.d), generator=tg, dtype=torch.float32, device=dev).to(wl.dtype)
        Vc[a:a + L] = torch.randn((L, wl.d), generator=tg, dtype=torch.float32, device=dev).to(wl.dtype)
    return (Kc, Vc, torch.tensor(cu, dtype=torch.int32, device=dev),
            torch.tensor(lens, dtype=torch.int32, device=dev))


def decode_inputs(wl: Workload, steps: int, seed: int = 0, device="cpu", temp: float = 2.0):
    """Per-step decode inputs in wl.dtype: q_new [steps, batch, h_q, d] (N(0,1) times `temp`,
    so that the softmax is neither flat nor one-hot), k_new, v_new [steps, batch, h_kv, d]."""
    dev = torch.device(device)
    tg = torch.Generator(device=dev)
    tg.manual_seed(30_000 + seed)
    q = temp * torch.randn((steps, wl.batch, wl.h_q, wl.d), generator=tg, dtype=torch.float32, device=dev)
    k = torch.randn((steps, wl.batch, wl.h_kv, wl.d), generator=tg, dtype=torch.float32, device=dev)
    v = torch.randn((steps, wl.batch, wl.h_kv, wl.d), generator=tg, dtype=torch.float32, device=dev)
    return q.to(wl.dtype), k.to(wl.dtype), v.to(wl.dtype)


def prefill_row_lse(wl: Workload, q, K):
    """What a prefill attention kernel would hand over for the window rows: the natural
    log-sum-exp of the scaled logits of window row r over every key it sees, i.e. the n prefix
    keys and the window keys up to and including itself (causal).  [batch, h_q, w] float32 on
    q's device.  Input preparation only (the scoring call takes it as `row_lse`)."""
    scale = 1.0 / math.sqrt(wl.d)
    off = wl.tok_off
    out = torch.empty((wl.batch, wl.h_q, wl.w), dtype=torch.float32, device=q.device)
    causal = torch.tril(torch.ones((wl.w, wl.w), dtype=torch.bool, device=q.device))
    for b, nb in enumerate(wl.n):
        for c in range(wl.h_kv):
            Kc = K[off[b]:off[b + 1], c, :].float()                         # [n + w, d]
            qg = q[b, c * wl.g:(c + 1) * wl.g].float()                      # [g, w, d]
            logit = torch.matmul(qg, Kc.t()) * scale                        # [g, w, n + w]
            logit[:, :, nb:] = logit[:, :, nb:].masked_fill(~causal, float("-inf"))
            out[b, c * wl.g:(c + 1) * wl.g] = torch.logsumexp(logit, dim=-1)
    return out
