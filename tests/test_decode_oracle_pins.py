"""Pins of the decode-side oracle (flattened layout, cache update, one decoding step) to
things other than itself: closed forms, special cases, a library softmax on the dense masked
form of Eqs. (4)-(5), and brute force with scalar loops."""
import math

import numpy as np
import pytest
import scipy.special

from oracle import adakv_oracle as O
from oracle import decode_oracle as D


def _ragged(rng, S, d, lo=1, hi=40):
    lens = rng.integers(lo, hi, size=S)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    K = rng.standard_normal((int(cu[-1]), d))
    V = rng.standard_normal((int(cu[-1]), d))
    return K, V, cu


def test_layout_starts_caps_and_spare_rows():
    cu = np.array([0, 3, 4, 9])
    assert D.segment_starts(cu, 0).tolist() == [0, 3, 4]
    assert D.segment_starts(cu, 5).tolist() == [0, 8, 14]
    assert D.segment_caps(cu, 5).tolist() == [8, 6, 10]
    K = np.arange(9 * 2, dtype=np.float64).reshape(9, 2) + 1
    Kc, Vc, lens = D.build_cache(K, -K, cu, 5)
    assert Kc.shape == (9 + 3 * 5, 2) and lens.tolist() == [3, 1, 5]
    assert np.array_equal(Kc[0:3], K[0:3]) and np.array_equal(Kc[8:9], K[3:4]) and np.array_equal(Kc[14:19], K[4:9])
    assert not Kc[3:8].any() and not Kc[9:14].any() and not Kc[19:].any()
    assert np.array_equal(Vc, -Kc)


def test_one_row_segment_returns_its_value_row():
    rng = np.random.default_rng(0)
    K, V, cu = _ragged(rng, 4, 8, 1, 2)           # every segment has exactly one row
    Kc, Vc, lens = D.build_cache(K, V, cu, 2)
    q = rng.standard_normal((2, 4, 8))            # batch 2, h_q 4, g 2 -> h 2, S 4
    out, lse = D.decode_attention(q, Kc, Vc, cu, 2, lens, g=2)
    for b in range(2):
        for i in range(4):
            s = b * 2 + i // 2
            assert np.allclose(out[b, i], V[s], rtol=0, atol=1e-15)
            assert lse[b, i] == pytest.approx(float(K[s] @ q[b, i]) / math.sqrt(8), abs=1e-14)


def test_identical_keys_give_the_mean_value_and_lse_plus_log_length():
    rng = np.random.default_rng(1)
    L, d = 37, 16
    k = rng.standard_normal(d)
    K = np.tile(k, (L, 1)); V = rng.standard_normal((L, d))
    cu = np.array([0, L])
    q = rng.standard_normal((1, 3, d))
    out, lse = D.decode_attention(q, K, V, cu, 0, [L], g=3)
    for i in range(3):
        assert np.allclose(out[0, i], V.mean(axis=0), atol=1e-14)
        assert lse[0, i] == pytest.approx(float(k @ q[0, i]) / math.sqrt(d) + math.log(L), abs=1e-13)


def test_scale_zero_is_the_plain_average_and_default_scale_is_inverse_sqrt_d():
    rng = np.random.default_rng(2)
    K, V, cu = _ragged(rng, 3, 4)
    lens = np.diff(cu)
    q = rng.standard_normal((1, 3, 4))
    out, lse = D.decode_attention(q, K, V, cu, 0, lens, g=1, scale=0.0)
    for s in range(3):
        assert np.allclose(out[0, s], V[cu[s]:cu[s + 1]].mean(axis=0), atol=1e-14)
        assert lse[0, s] == pytest.approx(math.log(lens[s]), abs=1e-14)
    a, _ = D.decode_attention(q, K, V, cu, 0, lens, g=1)
    b, _ = D.decode_attention(2.0 * q, K, V, cu, 0, lens, g=1, scale=0.25)   # 2 * 0.25 = 1/sqrt(4)
    assert np.allclose(a, b, atol=1e-14)


def test_brute_force_scalar_loops():
    rng = np.random.default_rng(3)
    batch, h, g, d, hr = 2, 2, 2, 4, 3
    K, V, cu = _ragged(rng, batch * h, d, 1, 6)
    Kc, Vc, lens = D.build_cache(K, V, cu, hr)
    q = rng.standard_normal((batch, h * g, d))
    out, lse = D.decode_attention(q, Kc, Vc, cu, hr, lens, g=g, scale=0.7)
    for b in range(batch):
        for i in range(h * g):
            s = b * h + i // g
            first = int(cu[s]) + s * hr
            w = []
            for t in range(int(lens[s])):
                acc = 0.0
                for e in range(d):
                    acc += q[b, i, e] * Kc[first + t, e]
                w.append(math.exp(0.7 * acc))
            tot = sum(w)
            for e in range(d):
                val = sum(w[t] * Vc[first + t, e] for t in range(len(w))) / tot
                assert out[b, i, e] == pytest.approx(val, rel=1e-12, abs=1e-14)
            assert lse[b, i] == pytest.approx(math.log(tot), rel=1e-12, abs=1e-13)


def test_rows_of_a_segment_may_be_permuted_and_groups_share_a_segment():
    rng = np.random.default_rng(4)
    K, V, cu = _ragged(rng, 2, 8, 5, 9)
    lens = np.diff(cu)
    q = rng.standard_normal((1, 4, 8))
    a, la = D.decode_attention(q, K, V, cu, 0, lens, g=2)
    K2, V2 = K.copy(), V.copy()
    for s in range(2):
        p = rng.permutation(int(lens[s])) + int(cu[s])
        K2[cu[s]:cu[s + 1]] = K[p]; V2[cu[s]:cu[s + 1]] = V[p]
    b, lb = D.decode_attention(q, K2, V2, cu, 0, lens, g=2)
    assert np.allclose(a, b, atol=1e-13) and np.allclose(la, lb, atol=1e-13)
    # query heads 0,1 read segment 0 and 2,3 read segment 1: same query -> same output inside a group
    q[0, 1] = q[0, 0]; q[0, 3] = q[0, 2]
    c, _ = D.decode_attention(q, K, V, cu, 0, lens, g=2)
    assert np.array_equal(c[0, 0], c[0, 1]) and np.array_equal(c[0, 2], c[0, 3])
    assert not np.allclose(c[0, 0], c[0, 2])


def test_gather_route_equals_the_masked_dense_route_of_eqs_4_and_5():
    """Compress one layer with the main oracle, attend over the compacted cache, and compare
    with a library softmax over ALL rows where the evicted logits are set to -inf."""
    rng = np.random.default_rng(5)
    h, g, d, n, w = 2, 2, 8, 50, 4
    qw = rng.standard_normal((h * g, w, d))
    K = rng.standard_normal((n + w, h, d)); V = rng.standard_normal((n + w, h, d))
    res = O.compress_layer(qw, K, V, n, w, 3, h * (w + 6), 0.2)
    cu, idx = res["cu_seqlens"], res["indices"]
    Kc, Vc, lens = D.build_cache(res["K_out"], res["V_out"], cu, 0)
    q = rng.standard_normal((1, h * g, d))
    out, _ = D.decode_attention(q, Kc, Vc, cu, 0, lens, g=g)
    for i in range(h * g):
        c = i // g
        keep = np.zeros(n + w, bool); keep[idx[cu[c]:cu[c + 1]]] = True
        logit = (K[:, c, :] @ q[0, i]) / math.sqrt(d)
        A_hat = scipy.special.softmax(np.where(keep, logit, -np.inf))
        assert np.allclose(out[0, i], A_hat @ V[:, c, :], atol=1e-13)


def test_full_budget_equals_dense_attention_over_all_rows():
    rng = np.random.default_rng(6)
    h, g, d, n, w = 3, 1, 4, 20, 2
    qw = rng.standard_normal((h, w, d))
    K = rng.standard_normal((n + w, h, d)); V = rng.standard_normal((n + w, h, d))
    res = O.compress_layer(qw, K, V, n, w, 1, h * (n + w), 0.0)
    Kc, Vc, lens = D.build_cache(res["K_out"], res["V_out"], res["cu_seqlens"], 0)
    assert lens.tolist() == [n + w] * h
    q = rng.standard_normal((1, h, d))
    out, lse = D.decode_attention(q, Kc, Vc, res["cu_seqlens"], 0, lens, g=1)
    for i in range(h):
        logit = (K[:, i, :] @ q[0, i]) / math.sqrt(d)
        assert np.allclose(out[0, i], scipy.special.softmax(logit) @ V[:, i, :], atol=1e-13)
        assert lse[0, i] == pytest.approx(scipy.special.logsumexp(logit), abs=1e-13)


def test_append_is_concatenation_and_full_segments_are_left_alone():
    rng = np.random.default_rng(7)
    S, d, hr = 3, 4, 2
    K, V, cu = _ragged(rng, S, d, 1, 5)
    Kc, Vc, lens = D.build_cache(K, V, cu, hr)
    lens0 = lens.copy()
    news = [(rng.standard_normal((S, d)), rng.standard_normal((S, d))) for _ in range(3)]
    flags = [D.append(Kc, Vc, cu, hr, lens, kn, vn) for kn, vn in news]
    assert flags == [False, False, True]                  # the third append finds every segment full
    assert (lens == lens0 + hr).all()
    start = D.segment_starts(cu, hr)
    for s in range(S):
        want_K = np.concatenate([K[cu[s]:cu[s + 1]], news[0][0][s:s + 1], news[1][0][s:s + 1]])
        want_V = np.concatenate([V[cu[s]:cu[s + 1]], news[0][1][s:s + 1], news[1][1][s:s + 1]])
        assert np.array_equal(Kc[start[s]:start[s] + lens[s]], want_K)
        assert np.array_equal(Vc[start[s]:start[s] + lens[s]], want_V)
    assert Kc.shape[0] == int(cu[-1]) + S * hr            # nothing grew
    # attention after the appends = attention over the concatenated rows, tightly packed
    q = rng.standard_normal((1, S, d))
    a, _ = D.decode_attention(q, Kc, Vc, cu, hr, lens, g=1)
    cu2 = np.concatenate([[0], np.cumsum(lens)])
    K2 = np.concatenate([Kc[start[s]:start[s] + lens[s]] for s in range(S)])
    V2 = np.concatenate([Vc[start[s]:start[s] + lens[s]] for s in range(S)])
    b, _ = D.decode_attention(q, K2, V2, cu2, 0, lens, g=1)
    assert np.array_equal(a, b)


def test_empty_segment_gives_zero_row_and_minus_infinity():
    K = np.ones((2, 4)); V = np.ones((2, 4))
    cu = np.array([0, 2, 2])
    out, lse = D.decode_attention(np.ones((1, 2, 4)), K, V, cu, 0, [2, 0], g=1)
    assert np.allclose(out[0, 0], 1.0) and not out[0, 1].any() and lse[0, 1] == -np.inf


def test_output_is_a_convex_combination_of_value_rows():
    rng = np.random.default_rng(8)
    K, V, cu = _ragged(rng, 4, 8, 2, 30)
    lens = np.diff(cu)
    q = 3.0 * rng.standard_normal((2, 2, 8))
    out, _ = D.decode_attention(q, K, V, cu, 0, lens, g=1)
    for b in range(2):
        for c in range(2):
            s = b * 2 + c
            seg = V[cu[s]:cu[s + 1]]
            assert (out[b, c] <= seg.max(axis=0) + 1e-12).all() and (out[b, c] >= seg.min(axis=0) - 1e-12).all()
