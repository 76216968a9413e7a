"""Comparison helpers for the GPU parity tests (HIP path vs CPU oracle on the same inputs)."""
import numpy as np

from oracle import adakv_oracle as O

SCORE_RTOL = 2e-3          # bf16 inputs, fp32 accumulation: the tolerance the target states
SCORE_ATOL = 1e-37         # fp32 flush-to-zero of sub-normal scores is not a failure
BAND = 4e-3                # element and threshold may both move by SCORE_RTOL


def to_f64(t):
    return t.detach().double().cpu().numpy()


def oracle_layer(wl, q, K, V, b=0, **kw):
    off = wl.tok_off
    Kb, Vb = K[off[b]:off[b + 1]], V[off[b]:off[b + 1]]
    return O.compress_layer(to_f64(q[b]), to_f64(Kb), Vb.float().cpu().numpy(), wl.n[b], wl.w,
                            wl.pool_k, wl.B[b], wl.alpha, **kw)


def oracle_batch(wl, q, K, V, **kw):
    """The oracle on the whole packed batch (O.compress_batch), plus, per sequence, the same
    outputs cut back out with offsets made relative to the sequence."""
    ref = O.compress_batch(to_f64(q), to_f64(K), V.float().cpu().numpy(), wl.n, wl.B, wl.tok_off[:-1],
                           wl.w, wl.pool_k, wl.alpha, **kw)
    h, per_seq, s0, row0 = wl.h_kv, [], 0, 0
    for b in range(wl.batch):
        per_seq.append(dict(scores=ref["scores"][s0:s0 + h * wl.n[b]].reshape(h, wl.n[b]),
                            budgets=ref["budgets"][b * h:(b + 1) * h],
                            cu_seqlens=ref["cu_seqlens"][b * h:(b + 1) * h + 1] - row0,
                            indices=ref["indices"][row0:row0 + wl.B[b]]))
        s0 += h * wl.n[b]
        row0 += wl.B[b]
    return ref, per_seq


def assert_scores_close(gpu, ref, what=""):
    gpu = np.asarray(gpu, np.float64).reshape(-1)
    ref = np.asarray(ref, np.float64).reshape(-1)
    assert gpu.shape == ref.shape
    assert np.all(np.isfinite(gpu)), f"{what}: non-finite scores"
    bad = np.abs(gpu - ref) > SCORE_RTOL * np.abs(ref) + SCORE_ATOL
    if bad.any():
        i = int(np.flatnonzero(bad)[0])
        worst = float((np.abs(gpu - ref) / (np.abs(ref) + SCORE_ATOL)).max())
        raise AssertionError(f"{what}: {int(bad.sum())} of {gpu.size} scores outside tolerance; first at {i}: "
                             f"gpu {gpu[i]!r} oracle {ref[i]!r}; worst rel {worst:.3e}")


def assert_exact_on_scores(out, scores, wl, K, V, b=0, seg0=0, row0=0):
    """allocate / select / compact are exact functions of the fp32 scores: replay them with the
    oracle on the scores the GPU used and demand bit-equality."""
    h, n, w = wl.h_kv, wl.n[b], wl.w
    sc = np.asarray(scores, np.float32).reshape(h, n)
    bud, cu = O.allocate(sc, wl.B[b], w, wl.alpha)
    idx = O.select(sc, bud, w)
    got_bud = out["budgets"].cpu().numpy()[seg0:seg0 + h]
    got_cu = out["cu_seqlens"].cpu().numpy()[seg0:seg0 + h + 1]
    got_idx = out["indices"].cpu().numpy()[row0:row0 + wl.B[b]]
    assert np.array_equal(got_bud, bud), (got_bud, bud)
    assert np.array_equal(got_cu, cu + row0), (got_cu, cu + row0)
    assert np.array_equal(got_idx, idx), f"{int((got_idx != idx).sum())} indices differ"
    if "K_out" in out and K is not None:
        off = wl.tok_off
        Kb = K[off[b]:off[b + 1]].float().cpu().numpy()
        Vb = V[off[b]:off[b + 1]].float().cpu().numpy()
        Kr, Vr = O.compact(Kb, Vb, idx, cu)
        assert np.array_equal(out["K_out"][row0:row0 + wl.B[b]].float().cpu().numpy(), Kr)
        assert np.array_equal(out["V_out"][row0:row0 + wl.B[b]].float().cpu().numpy(), Vr)


def assert_end_to_end_close(out, ref, wl, b=0, seg0=0, row0=0):
    """GPU pipeline on its own scores vs the oracle pipeline on oracle scores: equal except
    where an oracle score lies within BAND of a Top-k threshold."""
    h, n, w = wl.h_kv, wl.n[b], wl.w
    osc = ref["scores"].astype(np.float64)
    Bp = wl.B[b] - w * h
    g_bud = out["budgets"].cpu().numpy()[seg0:seg0 + h].astype(np.int64)
    o_bud = ref["budgets"].astype(np.int64)
    assert g_bud.sum() == Bp
    flat = np.sort(osc.reshape(-1))[::-1]
    if 0 < Bp < flat.size:
        tau = flat[Bp - 1]
        # sub-normal scores are flushed to zero on the GPU: the band gets the same absolute slack
        # as the score comparison
        near = int(((osc >= tau * (1 - BAND) - SCORE_ATOL) & (osc <= tau * (1 + BAND) + SCORE_ATOL)).sum())
    else:
        near = 0
    assert np.abs(g_bud - o_bud).sum() <= 2 * near + h, (g_bud, o_bud, near)
    g_cu = out["cu_seqlens"].cpu().numpy()[seg0:seg0 + h + 1] - row0
    g_idx = out["indices"].cpu().numpy()[row0:row0 + wl.B[b]]
    for c in range(h):
        gs = g_idx[g_cu[c]:g_cu[c + 1]]
        os_ = ref["indices"][ref["cu_seqlens"][c]:ref["cu_seqlens"][c + 1]]
        assert list(gs[-w:]) == list(range(n, n + w))
        gs, os_ = set(gs[:-w].tolist()), set(os_[:-w].tolist())
        diff = gs ^ os_
        if not diff:
            continue
        v = np.sort(osc[c])[::-1]
        lo, hi = min(g_bud[c], o_bud[c]), max(g_bud[c], o_bud[c])
        top = v[max(lo - 1, 0)] * (1 + BAND) + SCORE_ATOL
        bot = v[min(hi, n - 1)] * (1 - BAND) - SCORE_ATOL
        for j in diff:
            assert bot <= osc[c, j] <= top, (c, j, osc[c, j], bot, top)
