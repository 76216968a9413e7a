"""GPU parity: every C-ABI call against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

import paper_2407_11550_amd as adakv
from oracle import adakv_oracle as O
from paper_2407_11550_amd import synth

from parity_util import (assert_end_to_end_close, assert_exact_on_scores, assert_scores_close,
                         oracle_batch, oracle_layer, to_f64)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _say(msg):
    print(msg, flush=True)


def _run(wl, q, K, V, **kw):
    layer = adakv.Layer.from_workload(wl, **kw)
    out = adakv.compress(layer, q, K, V)
    torch.cuda.synchronize()
    return layer, out


def _check_all(wl, q, K, V, out):
    row0 = 0
    soff = 0
    whole, per_seq = oracle_batch(wl, q, K, V)
    assert out["scores"].numel() == whole["scores"].size and out["indices"].numel() == whole["indices"].size
    assert out["cu_seqlens"].numel() == whole["cu_seqlens"].size
    assert int(out["cu_seqlens"][-1]) == int(whole["cu_seqlens"][-1]) == sum(wl.B)
    for b in range(wl.batch):
        ref = per_seq[b]
        ns = wl.h_kv * wl.n[b]
        sc = out["scores"][soff:soff + ns].cpu().numpy()
        assert_scores_close(sc, ref["scores"], f"{wl.name} seq {b}")
        assert_exact_on_scores(out, sc, wl, K, V, b, seg0=b * wl.h_kv, row0=row0)
        assert_end_to_end_close(out, ref, wl, b, seg0=b * wl.h_kv, row0=row0)
        row0 += wl.B[b]
        soff += ns


# ------------------------------------------------------------------ whole step, small shapes
SHAPES = [
    # h_q h_kv  d   w  k   n     B(per kv head incl. window)   dtype
    (4, 4, 64, 8, 7, 1024, 128, torch.float32),       # the tiny config's shape
    (8, 2, 128, 32, 7, 3000, 300, torch.bfloat16),    # GQA 4, ragged tail
    (32, 8, 128, 32, 7, 4099, 250, torch.bfloat16),   # Llama-3.1-8B heads, prime-ish length
    (8, 8, 64, 16, 5, 777, 100, torch.bfloat16),      # d = 64, no GQA
    (16, 2, 128, 64, 7, 2500, 400, torch.bfloat16),   # 70B-like group: g*w = 512 rows
    (6, 2, 128, 8, 3, 513, 64, torch.float32),        # g = 3: rows not a multiple of 16
    (4, 2, 64, 4, 1, 300, 50, torch.bfloat16),        # no pooling
    (2, 1, 128, 1, 7, 5, 3, torch.bfloat16),          # n smaller than the pool kernel
    (8, 8, 128, 1, 1, 6000, 151, torch.bfloat16),     # no pooling over several chunks, one window row
    (4, 2, 64, 4, 1, 5000, 90, torch.bfloat16),       # the same with d = 64
    (4, 4, 64, 8, 1, 3000, 100, torch.float32),       # no pooling on the fp32 path
    (8, 2, 128, 16, 3, 4500, 200, torch.bfloat16),    # pool radius 1 over several chunks
    (32, 8, 128, 32, 7, 4099, 250, torch.float16),    # IEEE half on the matrix cores
    (8, 8, 64, 16, 5, 2777, 100, torch.float16),      # half, d = 64
    (6, 2, 128, 8, 3, 513, 64, torch.float16),        # half, g = 3
    (64, 8, 128, 16, 7, 1500, 120, torch.float16),    # half, 128 window rows per head
    (16, 16, 64, 4, 7, 900, 30, torch.bfloat16),      # 16 KV heads: two rounds of heads in the finishing kernel
    (64, 64, 64, 2, 3, 5000, 12, torch.bfloat16),     # the most KV heads the library takes, several chunks
    (48, 24, 128, 3, 5, 700, 25, torch.float32),      # 24 KV heads on the fp32 path
    (16, 2, 64, 64, 7, 2500, 400, torch.bfloat16),    # d = 64 with 512 window rows per head: more rows than threads
    (10, 2, 64, 64, 5, 1800, 90, torch.float16),      # d = 64, 320 rows (padded to 512)
    (16, 2, 64, 64, 7, 17500, 300, torch.bfloat16),   # the same with so many chunks that the statistics get their own kernel
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "hq%d_h%d_d%d_w%d_k%d_n%d_B%d_%s" % (s[:7] + (str(s[7])[6:],)))
def test_whole_step_matches_oracle(shape):
    h_q, h, d, w, k, n, Bh, dt = shape
    _say(f"whole step {shape}")
    wl = synth.small_workload(h_q, h, d, w, k, n, h * Bh, dtype=dt, seed=11)
    q, K, V = synth.generate(wl, device=DEV)
    _, out = _run(wl, q, K, V)
    _check_all(wl, q, K, V, out)


def variant_shapes():
    """One shape per instantiation of the MFMA scoring kernels (both 16-bit types, both head
    dimensions, every rows-per-head class and chunk length), plus the two forms that are not
    fused (the statistics combined and the pool applied by kernels of their own).  Same tuple
    layout as SHAPES.  tests/test_variant_coverage.py checks on the CPU that the list does
    reach every variant."""
    out = []
    for dt in (torch.bfloat16, torch.float16):
        for d in (64, 128):
            out += [
                (4, 2, d, 8, 7, 700, 60, dt),            # 16 rows per head
                (4, 2, d, 24, 5, 900, 70, dt),           # 48 rows
                (8, 2, d, 32, 7, 3000, 150, dt),         # 128 rows, few workgroups: 512-key chunks
                (64, 64, d, 100, 7, 7000, 130, dt),      # 100 rows, 64 heads: 1024-key chunks
                (64, 64, d, 100, 3, 15000, 120, dt),     # enough workgroups for 2048-key chunks
                (4, 2, d, 100, 7, 2500, 200, dt),        # 200 rows
                (8, 2, d, 96, 9, 2100, 180, dt),         # 384 rows (padded to 512)
            ]
    out += [
        (18, 2, 128, 64, 7, 1500, 100, torch.bfloat16),   # 576 rows per head: beyond the matrix-core
        (18, 2, 64, 64, 5, 900, 80, torch.float16),       # kernels, the plain-FMA path on 16-bit inputs
        (18, 2, 64, 64, 5, 700, 80, torch.bfloat16),
        (18, 2, 128, 64, 3, 800, 90, torch.float16),
        (8, 2, 128, 32, 71, 3000, 150, torch.bfloat16),   # pool radius beyond the fused halo
        (8, 2, 64, 32, 67, 2600, 150, torch.float16),
        (16, 2, 128, 64, 7, 35100, 300, torch.float16),   # 512 rows x 18 chunks: statistics kernel
    ]
    return out


@pytest.mark.parametrize("shape", variant_shapes(), ids=lambda s: "hq%d_h%d_d%d_w%d_k%d_n%d_B%d_%s" % (s[:7] + (str(s[7])[6:],)))
def test_every_scoring_variant_matches_oracle(shape):
    h_q, h, d, w, k, n, Bh, dt = shape
    _say(f"variant {shape}")
    wl = synth.small_workload(h_q, h, d, w, k, n, h * Bh, dtype=dt, seed=13)
    q, K, V = synth.generate(wl, device=DEV)
    layer, out = _run(wl, q, K, V)
    _say("  " + " ".join(f"{k_}={v}" for k_, v in adakv.describe(layer).items()))
    _check_all(wl, q, K, V, out)


SHAPE_512_ROWS_4096_KEYS = (256, 32, 128, 64, 7, [4200, 33, 64, 31, 50, 40, 35, 47])   # 8 sequences x 32 KV heads
SHAPES_128_ROWS_4096_KEYS = [(64, 64, d, 100, 7, [4200, 33, 64, 31, 50, 40, 35]) for d in (64, 128)]   # 7 x 64 KV heads


SHAPES_256_ROWS_2048_KEYS = [(128, 64, d, 100, 7, [2300, 33, 64, 31, 50, 40, 35]) for d in (64, 128)]   # 200 rows per head


@pytest.mark.parametrize("dt", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("shape", SHAPES_256_ROWS_2048_KEYS, ids=lambda s_: "d%d" % s_[2])
def test_256_rows_with_2048_key_chunks(shape, dt):
    """The 256-row kernels take 2048-key chunks under the same rule (448 workgroups or more)."""
    _say(f"256 rows, 2048-key chunks, {shape} {dt}")
    h_q, h, d, w, k, n = shape
    wl = synth.small_workload(h_q, h, d, w, k, n, [h * (w + max(1, nb // 10)) for nb in n], dtype=dt, seed=45)
    q, K, V = synth.generate(wl, device=DEV)
    layer, out = _run(wl, q, K, V)
    desc = adakv.describe(layer)
    assert desc["chunk"] == "2048" and (desc["mb"], desc["rs"], desc["kg"]) == ("2", "4", "1")
    _check_all(wl, q, K, V, out)


@pytest.mark.parametrize("dt", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("shape", SHAPES_128_ROWS_4096_KEYS, ids=lambda s_: "d%d" % s_[2])
def test_128_rows_with_4096_key_chunks(shape, dt):
    """The 128-row kernels take 4096-key chunks when those nearly fill the chip by themselves
    (448 workgroups or more); seven sequences x 64 KV heads do, one of them longer than a chunk."""
    _say(f"128 rows, 4096-key chunks, {shape} {dt}")
    h_q, h, d, w, k, n = shape
    wl = synth.small_workload(h_q, h, d, w, k, n, [h * (w + max(1, nb // 10)) for nb in n], dtype=dt, seed=43)
    q, K, V = synth.generate(wl, device=DEV)
    layer, out = _run(wl, q, K, V)
    desc = adakv.describe(layer)
    assert desc["chunk"] == "4096" and (desc["mb"], desc["rs"], desc["kg"]) == ("2", "2", "2")
    _check_all(wl, q, K, V, out)


@pytest.mark.parametrize("dt", [torch.bfloat16, torch.float16])
def test_512_rows_with_4096_key_chunks(dt):
    """The 512-row shape takes 4096-key chunks as soon as that still gives 256 workgroups; here
    eight sequences x 32 KV heads do, one sequence being longer than a chunk and ragged."""
    _say(f"512 rows, 4096-key chunks, {dt}")
    h_q, h, d, w, k, n = SHAPE_512_ROWS_4096_KEYS
    wl = synth.small_workload(h_q, h, d, w, k, n, [h * (w + max(1, nb // 10)) for nb in n], dtype=dt, seed=41)
    q, K, V = synth.generate(wl, device=DEV)
    layer, out = _run(wl, q, K, V)
    assert adakv.describe(layer)["chunk"] == "4096" and adakv.describe(layer)["rs"] == "8"
    _check_all(wl, q, K, V, out)


@pytest.mark.parametrize("h_q, rs", [(8, "4"), (16, "8")])      # 256 and 512 rows per KV head
def test_statistics_sweep_survives_logits_far_above_its_first_tile(h_q, rs):
    """The statistics sweep of the many-row shapes keeps the reference its first tile gave a row
    and only looks for a new maximum when a sum overflows.  Here the first 64 keys are tiny and
    later keys give logits more than 128 powers of two above them, so that path is taken (in the
    512-row shape from inside the loop of tile pairs)."""
    _say(f"statistics sweep: overflow of the kept reference, {h_q} query heads")
    wl = synth.small_workload(h_q, 2, 128, 64, 7, 3000, 2 * 300, dtype=torch.bfloat16, seed=77)
    q, K, V = synth.generate(wl, device=DEV)
    q = (q.float() * 4).to(torch.bfloat16)
    K = K.float()
    K[:64] *= 0.01
    K[64:] *= 6
    K = K.to(torch.bfloat16)
    logits = torch.einsum("hwd,nd->hwn", q[0, :4].float(), K[:3000, 0].float()) / 128 ** 0.5
    assert float((logits[:, :, 64:].amax(-1) - logits[:, :, :64].amax(-1)).max()) * 1.4427 > 128
    _, out = _run(wl, q, K, V)
    assert adakv.describe(adakv.Layer.from_workload(wl))["rs"] == rs
    _check_all(wl, q, K, V, out)


def test_tiny_config():
    _say("tiny config")
    wl = synth.workload("tiny")
    q, K, V = synth.generate(wl, device=DEV)
    _, out = _run(wl, q, K, V)
    _check_all(wl, q, K, V, out)


@pytest.mark.parametrize("alpha", [0.0, 0.2, 0.5, 1.0])
def test_alpha_sweep(alpha):
    _say(f"alpha {alpha}")
    wl = synth.small_workload(8, 4, 128, 16, 7, 2048, 4 * 116, alpha=alpha, seed=5)
    q, K, V = synth.generate(wl, device=DEV)
    _, out = _run(wl, q, K, V)
    _check_all(wl, q, K, V, out)
    if alpha == 1.0:
        assert out["budgets"].cpu().tolist() == [100] * 4


def test_ragged_batch():
    _say("ragged batch")
    wl = synth.small_workload(8, 2, 128, 32, 7, [1500, 37, 4096, 600], [2 * 150, 2 * 40, 2 * 500, 2 * 32], seed=21)
    q, K, V = synth.generate(wl, device=DEV)
    _, out = _run(wl, q, K, V)
    _check_all(wl, q, K, V, out)
    assert int(out["cu_seqlens"][-1]) == sum(wl.B)


def test_row_lse_input_gives_prefix_plus_window_normalisation():
    _say("row_lse")
    wl = synth.small_workload(8, 2, 128, 16, 7, 1200, 2 * 100, seed=31)
    q, K, V = synth.generate(wl, device=DEV)
    qd, Kd = to_f64(q[0]), to_f64(K)
    n, w, d = wl.n[0], wl.w, wl.d
    lse = np.empty((wl.h_q, w))
    for hq in range(wl.h_q):
        c = hq // wl.g
        s = (qd[hq] @ Kd[:, c].T) / np.sqrt(d)
        for r in range(w):
            vis = np.concatenate([s[r, :n], s[r, n:n + r + 1]])
            lse[hq, r] = vis.max() + np.log(np.exp(vis - vis.max()).sum())
    layer = adakv.Layer.from_workload(wl, flags=1)
    lse_t = torch.tensor(lse, dtype=torch.float32, device=DEV).reshape(1, wl.h_q, w)
    sc = adakv.score(layer, q, K, row_lse=lse_t)
    torch.cuda.synchronize()
    ref = O.score(qd, Kd, n, w, wl.pool_k, norm="prefix+window")
    # the fp32 rounding of lse itself moves every score of a row by up to |lse| * 2^-24
    assert_scores_close(sc.cpu().numpy(), O.score(qd, Kd, n, w, wl.pool_k, row_lse=lse_t[0].double().cpu().numpy()), "row_lse")
    np.testing.assert_allclose(sc.cpu().numpy().reshape(wl.h_kv, n), ref, rtol=2e-3)


# ------------------------------------------------------- allocate / select on given scores
def _alloc_select(scores_np, w, B, alpha):
    h, n = scores_np.shape
    layer = adakv.Layer(torch.bfloat16, h, h, 128, w, 7, alpha, [n], [B])
    sc = torch.tensor(scores_np, device=DEV).reshape(-1)
    bud, cu = adakv.allocate(layer, sc)
    idx = adakv.select(layer, sc, bud, cu)
    torch.cuda.synchronize()
    return bud.cpu().numpy(), cu.cpu().numpy(), idx.cpu().numpy()


@pytest.mark.parametrize("case", ["random", "quantised", "all_equal", "zeros_and_spikes", "plateaus",
                                  "one_narrow_band", "long_bucket_in_one_block", "runs_in_one_band"])
@pytest.mark.parametrize("alpha", [0.0, 0.2, 1.0])
def test_allocate_select_bit_exact_on_oracle_scores(case, alpha):
    _say(f"allocate/select {case} alpha {alpha}")
    rng = np.random.default_rng(3)
    h, n, w = 4, 10007, 8
    extra = ()
    if case == "random":
        s = rng.random((h, n)) ** np.array([1, 4, 16, 64])[:, None]
    elif case == "quantised":
        s = np.round(rng.random((h, n)) * 50) / 50
    elif case == "all_equal":
        s = np.full((h, n), 0.25)
    elif case == "zeros_and_spikes":
        s = np.zeros((h, n)); s[rng.integers(0, h, 300), rng.integers(0, n, 300)] = rng.random(300)
    elif case == "one_narrow_band":
        # every score inside one 22-bit key prefix (1024 consecutive floats), all last digits in use:
        # far more prefix-sharing elements than a finishing block holds at once
        base = np.array([0.3], np.float32).view(np.uint32)[0] & ~np.uint32(1023)
        s = (base + rng.integers(0, 1024, (h, n)).astype(np.uint32)).view(np.float32)
    elif case == "runs_in_one_band":
        # the same band, but in runs of one value, 1 to 700 positions long: stretches where whole
        # wavefronts read one last digit call after call, stretches where only some lanes' eight
        # entries agree, and value changes in between
        base = np.array([0.3], np.float32).view(np.uint32)[0] & ~np.uint32(1023)
        lens = rng.integers(1, 700, h * n) ** rng.integers(0, 2, h * n)
        vals = np.repeat(rng.integers(0, 1024, h * n), lens)[:h * n].reshape(h, n)
        s = (base + vals.astype(np.uint32)).view(np.float32)
    elif case == "long_bucket_in_one_block":
        # few prefix-sharing elements overall, but 1500 of them inside one block of 4096 positions
        s = (rng.random((h, n)) ** 8).astype(np.float32)
        base = np.array([0.3], np.float32).view(np.uint32)[0] & ~np.uint32(1023)
        s[1, 100:1600] = (base + rng.integers(0, 1024, 1500).astype(np.uint32)).view(np.float32)
        extra = (w * h + int((s > 0.31).sum()) + 700,)
    else:
        s = O.max_pool_same(rng.random((h, n)) ** 8, 7)
    s = s.astype(np.float32)
    for B in (w * h, w * h + 1, w * h + 1000, w * h + h * n // 2, w * h + h * n - 1, w * h + h * n) + extra:
        bud, cu, idx = _alloc_select(s, w, B, alpha)
        rb, rcu = O.allocate(s, B, w, alpha)
        assert np.array_equal(bud, rb), (case, B, bud, rb)
        assert np.array_equal(cu, rcu)
        assert np.array_equal(idx, O.select(s, rb, w)), (case, B)


@pytest.mark.parametrize("case", ["runs_in_one_band", "band_beside_random"])
def test_allocate_select_plateaus_across_many_blocks(case):
    """Plateaus over 37 blocks of 4096 positions per head: the finishing kernels stream more
    blocks than they have wavefronts, so every wavefront looks a block ahead while it streams one
    (with the 10007-position heads above no wavefront ever has a second block)."""
    _say(f"allocate/select many blocks {case}")
    rng = np.random.default_rng(5)
    h, n, w = 3, 150001, 8
    base = np.array([0.3], np.float32).view(np.uint32)[0] & ~np.uint32(1023)
    if case == "runs_in_one_band":
        lens = rng.integers(1, 5000, h * n) ** rng.integers(0, 2, h * n)
        vals = np.repeat(rng.integers(0, 1024, h * n), lens)[:h * n].reshape(h, n)
        s = (base + vals.astype(np.uint32)).view(np.float32)
    else:
        band = (base + rng.integers(0, 4, (h, n)).astype(np.uint32)).view(np.float32)
        s = np.where(rng.random((h, n)) < 0.5, band, (rng.random((h, n)) ** 6).astype(np.float32))
    for alpha, B in ((0.2, w * h + 5000), (0.0, w * h + h * n // 3), (1.0, w * h + h * n - 7)):
        bud, cu, idx = _alloc_select(s, w, B, alpha)
        rb, rcu = O.allocate(s, B, w, alpha)
        assert np.array_equal(bud, rb), (case, alpha, B, bud, rb)
        assert np.array_equal(cu, rcu)
        assert np.array_equal(idx, O.select(s, rb, w)), (case, alpha, B)


def test_select_with_zero_budget_heads_and_full_heads():
    _say("select zero/full budgets")
    rng = np.random.default_rng(4)
    h, n, w = 3, 5000, 4
    s = rng.random((h, n)).astype(np.float32)
    budgets = np.array([0, n, 123], np.int32)
    cu = np.concatenate([[0], np.cumsum(budgets + w)]).astype(np.int32)
    layer = adakv.Layer(torch.bfloat16, h, h, 128, w, 7, 0.2, [n], [int(cu[-1])])
    idx = adakv.select(layer, torch.tensor(s, device=DEV).reshape(-1), torch.tensor(budgets, device=DEV),
                       torch.tensor(cu, device=DEV))
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), O.select(s, budgets, w))


def test_select_long_heads_take_the_chunk_parallel_emit():
    # heads longer than 262144 positions are emitted by the two chunk-parallel kernels instead of
    # by the block that finishes the last radix pass
    _say("select long heads")
    rng = np.random.default_rng(8)
    h, n, w = 2, 300001, 4
    s = O.max_pool_same((rng.random((h, n)) ** 12).astype(np.float32), 7)
    for alpha, B in ((0.2, w * h + 20000), (0.0, w * h + 3)):
        bud, cu, idx = _alloc_select(s, w, B, alpha)
        rb, rcu = O.allocate(s, B, w, alpha)
        assert np.array_equal(bud, rb) and np.array_equal(cu, rcu)
        assert np.array_equal(idx, O.select(s, rb, w))


@pytest.mark.parametrize("dt,d,layout", [(torch.bfloat16, 128, "fused_kv"), (torch.float16, 64, "padded_head"),
                                          (torch.float32, 64, "fused_kv"), (torch.bfloat16, 128, "padded_head")])
def test_whole_step_on_strided_k_and_v(dt, d, layout):
    """K and V as views into larger tensors: K and V of a token side by side in one row
    ([token][2][head][d], token stride 2*h*d), or a head dimension padded to d + 16 elements.  The
    whole step must give what it gives on contiguous copies of the same values."""
    _say(f"strided K/V {dt} {d} {layout}")
    h_q, h, w, n = 8, 2, 16, [2300, 700]
    wl = synth.small_workload(h_q, h, d, w, 7, n, [h * (w + 150), h * (w + 60)], dtype=dt, seed=44)
    q, K, V = synth.generate(wl, device=DEV)
    rows = K.shape[0]
    if layout == "fused_kv":
        both = torch.empty((rows, 2, h, d), dtype=dt, device=DEV)
        both[:, 0], both[:, 1] = K, V
        Ks, Vs = both[:, 0], both[:, 1]
        strides = dict(k_strides=(2 * h * d, d), v_strides=(2 * h * d, d))
    else:
        Kp = torch.full((rows, h, d + 16), 3.0, dtype=dt, device=DEV)
        Vp = torch.full((rows, h, d + 16), -3.0, dtype=dt, device=DEV)
        Kp[:, :, :d], Vp[:, :, :d] = K, V
        Ks, Vs = Kp[:, :, :d], Vp[:, :, :d]
        strides = dict(k_strides=(h * (d + 16), d + 16), v_strides=(h * (d + 16), d + 16))
    plain = adakv.compress(adakv.Layer.from_workload(wl), q, K, V)
    out = adakv.compress(adakv.Layer.from_workload(wl, **strides), q, Ks, Vs)
    torch.cuda.synchronize()
    for key in plain:
        assert torch.equal(plain[key], out[key]), key
    _check_all(wl, q, K, V, out)


@pytest.mark.parametrize("dt", [torch.bfloat16, torch.float32], ids=["bf16", "fp32"])
def test_loose_packing_and_a_caller_scale(dt):
    """Sequences need not be packed tightly (tok_off may leave rows between them, here 37 and 5 rows
    of NaN that must never be read) and the logit scale may be the caller's (Section 3.1's footnote
    only says that 1/sqrt(d) is left out of the formulas)."""
    _say(f"loose packing, scale {dt}")
    h_q, h, d, w = 8, 2, 128 if dt == torch.bfloat16 else 64, 8
    n, B = [1900, 640, 33], [h * (w + 120), h * (w + 50), h * (w + 9)]
    wl = synth.small_workload(h_q, h, d, w, 5, n, B, dtype=dt, seed=61)
    q, K, V = synth.generate(wl, device=DEV)
    gaps = [37, 5, 0]
    off = [0]
    for nb, gp in zip(n, gaps):
        off.append(off[-1] + nb + w + gp)
    Kl = torch.full((off[-1], h, d), float("nan"), dtype=dt, device=DEV)
    Vl = torch.full((off[-1], h, d), float("nan"), dtype=dt, device=DEV)
    for b in range(len(n)):
        rows = n[b] + w
        Kl[off[b]:off[b] + rows] = K[wl.tok_off[b]:wl.tok_off[b] + rows]
        Vl[off[b]:off[b] + rows] = V[wl.tok_off[b]:wl.tok_off[b] + rows]
    scale = 0.11
    layer = adakv.Layer.from_workload(wl, scale=scale)
    layer_loose = adakv.Layer(dt, h_q, h, d, w, 5, wl.alpha, n, B, tok_off=off, scale=scale)
    tight = adakv.compress(layer, q, K, V)
    loose = adakv.compress(layer_loose, q, Kl, Vl)
    torch.cuda.synchronize()
    for key in tight:
        assert torch.equal(tight[key], loose[key]), key
    assert torch.isfinite(loose["scores"]).all() and torch.isfinite(loose["K_out"].float()).all()
    soff = 0
    for b in range(len(n)):
        ref = oracle_layer(wl, q, K, V, b, scale=scale)
        ns = h * n[b]
        assert_scores_close(tight["scores"][soff:soff + ns].cpu().numpy(), ref["scores"], f"scaled seq {b}")
        soff += ns
    other = adakv.score(adakv.Layer.from_workload(wl), q, K)
    assert not torch.equal(other, tight["scores"])                # the scale is really applied


# ------------------------------------------------------------------------------ compaction
@pytest.mark.parametrize("dt,d", [(torch.bfloat16, 128), (torch.bfloat16, 64), (torch.float32, 64), (torch.float32, 128)])
def test_compact_bit_exact_with_strides_and_canaries(dt, d):
    _say(f"compact {dt} {d}")
    g = torch.Generator(device=DEV); g.manual_seed(9)
    h, n, w = 3, 700, 5
    pad = 16
    Kfull = torch.randn((n + w, h, d + pad), generator=g, device=DEV).to(dt)
    Vfull = torch.randn((n + w, h + 1, d), generator=g, device=DEV).to(dt)
    K, V = Kfull[:, :, :d], Vfull[:, :h, :]
    rng = np.random.default_rng(9)
    budgets = np.array([10, 0, 333], np.int32)
    cu = np.concatenate([[0], np.cumsum(budgets + w)]).astype(np.int32)
    s = rng.random((h, n)).astype(np.float32)
    idx = O.select(s, budgets, w)
    layer = adakv.Layer(dt, h, h, d, w, 7, 0.2, [n], [int(cu[-1])],
                        k_strides=(h * (d + pad), d + pad), v_strides=((h + 1) * d, d))
    rows = int(cu[-1])
    Kbuf = torch.full((rows + 2, d), 7.0, device=DEV).to(dt)
    Vbuf = torch.full((rows + 2, d), 7.0, device=DEV).to(dt)
    adakv.compact(layer, K, V, torch.tensor(idx, device=DEV), torch.tensor(cu, device=DEV), Kbuf[1:-1], Vbuf[1:-1])
    torch.cuda.synchronize()
    Kr, Vr = O.compact(K.float().cpu().numpy(), V.float().cpu().numpy(), idx, cu)
    assert np.array_equal(Kbuf[1:-1].float().cpu().numpy(), Kr)
    assert np.array_equal(Vbuf[1:-1].float().cpu().numpy(), Vr)
    for buf in (Kbuf, Vbuf):
        assert torch.all(buf[0] == 7.0) and torch.all(buf[-1] == 7.0)      # canaries untouched


# ------------------------------------------------------------------------------ determinism
def test_two_runs_are_bit_identical():
    _say("determinism")
    wl = synth.small_workload(32, 8, 128, 32, 7, 9000, 8 * 300, seed=77)
    q, K, V = synth.generate(wl, device=DEV)
    _, a = _run(wl, q, K, V)
    _, b = _run(wl, q, K, V)
    for key in a:
        assert torch.equal(a[key], b[key]), key


# ------------------------------------------------------------------------------ full sizes
@pytest.mark.parametrize("name,alpha", [("llama8b_32k", None), ("llama8b_128k", None),
                                        ("llama70b_128k", 0.2), ("llama70b_128k", 1.0)])
def test_full_size_layer(name, alpha):
    _say(f"full size {name} alpha {alpha}")
    wl = synth.workload(name, alpha=alpha)
    q, K, V = synth.generate(wl, device=DEV)
    _, out = _run(wl, q, K, V)
    _say("  gpu done, oracle running")
    _check_all(wl, q, K, V, out)
    bud = out["budgets"].cpu().numpy()
    _say(f"  budgets min {bud.min()} max {bud.max()}")


def test_pyramid_schedule_feeds_the_layer_budgets():
    """The pyramidal variant (Section 3.4) only changes the budget each layer gets: six layers of
    one shape, budgets from adakv_pyramid_budgets (largest first, mean = the average budget),
    every layer compressed with its own B and compared with the oracle."""
    _say("pyramid schedule")
    h, w, n, layers, per_head = 4, 8, 2600, 6, 150
    prefix = adakv.pyramid_budgets(layers, h * per_head, 3.0)       # B' of each layer
    assert prefix == O.pyramid_budgets(layers, h * per_head, 3.0)
    assert sum(prefix) == layers * h * per_head and all(a >= b for a, b in zip(prefix, prefix[1:]))
    assert prefix[0] > 2 * prefix[-1]
    kept = []
    for l, bp in enumerate(prefix):
        wl = synth.small_workload(8, h, 128, w, 7, n, h * w + bp, seed=70)
        q, K, V = synth.generate(wl, layer=l, device=DEV)
        _, out = _run(wl, q, K, V)
        _check_all(wl, q, K, V, out)
        assert int(out["budgets"].sum()) == bp
        kept.append(int(out["cu_seqlens"][-1]))
    assert kept == [bp + h * w for bp in prefix]


def test_very_long_sequence_folds_the_partial_statistics_in_several_rounds():
    """600 000 prefix tokens with 4 window rows per head: 293 chunks of statistics per head, more
    than one round (256) of the fused combination in the weights sweep, and 147 emit blocks per
    head.  Whole output compared."""
    _say("very long sequence")
    wl = synth.small_workload(2, 2, 128, 4, 7, 600_000, 2 * (4 + 9000), seed=91)
    q, K, V = synth.generate(wl, device=DEV)
    layer, out = _run(wl, q, K, V)
    v = adakv.describe(layer)
    assert v["lse"] == "fused" and v["chunk"] == "2048"
    _say("  gpu done, oracle running")
    _check_all(wl, q, K, V, out)


@pytest.mark.parametrize("layer_no", [3, 17, 31])
def test_full_size_ragged_batch_one_layer(layer_no):
    # batch 8, prefix lengths drawn from [4096, 65536], budgets 5 % of n per head, packed layout:
    # three of the 32 layers of the ragged workload, every sequence compared in full
    _say(f"full size ragged batch, layer {layer_no}")
    wl = synth.workload("llama8b_ragged")
    q, K, V = synth.generate(wl, layer=layer_no, device=DEV)
    _, out = _run(wl, q, K, V)
    _say(f"  gpu done, n = {wl.n}")
    _check_all(wl, q, K, V, out)
    assert int(out["cu_seqlens"][-1]) == sum(wl.B)


def test_kernel_trace_names_every_kernel_and_costs_nothing_when_disarmed():
    _say("kernel trace")
    wl = synth.small_workload(8, 2, 128, 32, 7, 5000, 2 * 300, seed=3)
    q, K, V = synth.generate(wl, device=DEV)
    layer = adakv.Layer.from_workload(wl)
    ref = adakv.compress(layer, q, K, V)
    with adakv.KernelTrace(64) as tr:
        out = adakv.compress(layer, q, K, V)
    torch.cuda.synchronize()
    names = [n for n, _ in tr.durations_us()]
    assert names[0].startswith("score_") and names[-1] == "compact"
    assert sum(n.startswith("alloc_") for n in names) >= 2 and sum(n.startswith("select_") for n in names) >= 2
    assert all(0 < us < 1e5 for _, us in tr.durations_us()) and tr.used == 2 * len(names)
    for key in ref:
        assert torch.equal(ref[key], out[key]), key


def test_sixty_four_sequences_in_one_call():
    """The largest batch the ABI takes: 64 short sequences of different lengths and budgets."""
    _say("batch 64")
    n = [130 + 53 * i for i in range(64)]
    B = [2 * (8 + 5 + (7 * i) % 90) for i in range(64)]
    wl = synth.small_workload(8, 2, 128, 8, 7, n, B, seed=64)
    q, K, V = synth.generate(wl, device=DEV)
    _, out = _run(wl, q, K, V)
    _check_all(wl, q, K, V, out)


@pytest.mark.parametrize("case", [
    (32, 8, 128, 32, 7, [4099], [8 * 250], None),              # two sweeps clear and count
    (32, 8, 128, 32, 7, [9000, 700, 2048], [8 * 300, 8 * 40, 8 * 2080], None),   # ragged, one full budget
    (8, 2, 128, 32, 7, [3000], [2 * 300], "lse"),              # row_lse given: clearing kernel instead
    (16, 2, 128, 64, 7, [2500], [2 * 400], None),              # 512 window rows per head
    (4, 4, 64, 8, 7, [1024], [4 * 128], None),                 # fp32: the flag is accepted and ignored
    (8, 2, 128, 32, 7, [1500, 900], [2 * 32, 2 * 33], None),   # nothing / one position to select
], ids=["one_seq", "ragged", "row_lse", "rows512", "fp32", "empty_budget"])
def test_pipeline_flag_changes_nothing(case):
    """ADAKV_FLAG_PIPELINE (scoring clears the histograms and counts first digits itself) must
    give bit-identical scores, budgets, offsets, indices and rows."""
    h_q, h, d, w, k, n, B, mode = case
    _say(f"pipeline flag {case}")
    dt = torch.float32 if d == 64 else torch.bfloat16
    wl = synth.small_workload(h_q, h, d, w, k, n, B, dtype=dt, seed=23)
    q, K, V = synth.generate(wl, device=DEV)
    layer = adakv.Layer.from_workload(wl)
    lse = synth.prefill_row_lse(wl, q, K) if mode == "lse" else None
    ws = torch.empty(adakv.workspace_bytes(layer), dtype=torch.uint8, device=DEV)
    ws.fill_(0xAB)                                           # stale bytes in the workspace
    a = adakv.compress(layer, q, K, V, row_lse=lse, ws=ws, pipeline=False)
    ws.fill_(0xCD)
    b = adakv.compress(layer, q, K, V, row_lse=lse, ws=ws, pipeline=True)
    c = adakv.compress(layer, q, K, V, row_lse=lse, ws=ws, pipeline=True)      # on its own leftovers
    torch.cuda.synchronize()
    for key in a:
        assert torch.equal(a[key], b[key]), key
        assert torch.equal(a[key], c[key]), key
    assert int(a["budgets"].sum()) == sum(B) - w * h * len(n)


def _fuzz_shapes():
    """Forty seeded shapes across every dispatch branch of the scoring path (window rows per head
    from 1 to 512, both head dimensions and dtypes, pool kernels 1 to 15, one to four ragged
    sequences from a handful of tokens to several chunks, budgets from nothing to everything)."""
    rng = np.random.default_rng(424242)
    shapes = []
    for i in range(40):
        d = int(rng.choice([64, 128]))
        g = int(rng.choice([1, 2, 3, 4, 8]))
        h = int(rng.choice([1, 2, 4, 8]))
        w = int(rng.choice([1, 2, 5, 8, 16, 32, 64]))
        if g * w > 512:
            w = 512 // g
        k = int(rng.choice([1, 3, 5, 7, 9, 15]))
        batch = int(rng.integers(1, 5))
        top = int(rng.choice([40, 700, 2500, 7000, 20000]))
        n = [int(rng.integers(1, top + 1)) for _ in range(batch)]
        frac = float(rng.choice([0.0, 0.02, 0.1, 0.5, 1.0]))
        B = [h * w + int(round(frac * h * nb)) for nb in n]
        alpha = float(rng.choice([0.0, 0.2, 0.5, 1.0]))
        dt = torch.float32 if (i % 5 == 4) else torch.bfloat16
        shapes.append((g * h, h, d, w, k, n, B, alpha, dt, 500 + i))
    return shapes


def test_seeded_shape_sweep_matches_oracle():
    for shape in _fuzz_shapes():
        h_q, h, d, w, k, n, B, alpha, dt, seed = shape
        _say(f"shape sweep {shape}")
        wl = synth.small_workload(h_q, h, d, w, k, n, B, alpha=alpha, dtype=dt, seed=seed)
        q, K, V = synth.generate(wl, device=DEV)
        _, out = _run(wl, q, K, V)
        _check_all(wl, q, K, V, out)


def test_whole_step_replays_from_a_hip_graph():
    """The four calls only enqueue kernels (no memset nodes, no allocation when the outputs and the
    workspace are handed in), so a caller can capture them into a HIP graph.  Three replays with
    eager work and synchronisations in between, on changing inputs, each checked against the
    eager result."""
    _say("graph replay")
    wl = synth.small_workload(32, 8, 128, 32, 7, [5000, 1200], [8 * 200, 8 * 90], seed=31)
    layer = adakv.Layer.from_workload(wl)
    sets = [synth.generate(wl, layer=i, device=DEV) for i in range(3)]
    q, K, V = [t.clone() for t in sets[0]]
    ws = torch.empty(adakv.workspace_bytes(layer), dtype=torch.uint8, device=DEV)
    bufs = dict(scores=torch.empty(layer.num_scores, dtype=torch.float32, device=DEV),
                budgets=torch.empty(layer.num_segments, dtype=torch.int32, device=DEV),
                cu_seqlens=torch.empty(layer.num_segments + 1, dtype=torch.int32, device=DEV),
                indices=torch.empty(layer.num_rows_out, dtype=torch.int32, device=DEV),
                K_out=torch.empty((layer.num_rows_out, wl.d), dtype=wl.dtype, device=DEV),
                V_out=torch.empty((layer.num_rows_out, wl.d), dtype=wl.dtype, device=DEV))
    adakv.compress(layer, q, K, V, ws=ws, bufs=bufs)             # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        adakv.compress(layer, q, K, V, ws=ws, bufs=bufs)
    for i in (1, 2, 0):
        for dst, src in zip((q, K, V), sets[i]):
            dst.copy_(src)
        eager = adakv.compress(layer, q, K, V)                   # fresh outputs, eager launches
        torch.cuda.synchronize()
        for t in bufs.values():
            t.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for key in eager:
            assert torch.equal(eager[key], bufs[key]), (i, key)


POOL_FIRST_CASES = [
    (8, 2, 128, 8, 7, [3000, 41], torch.bfloat16, False),
    (4, 4, 64, 8, 5, [1024], torch.float32, False),
    (6, 2, 128, 5, 15, [700, 9, 260], torch.bfloat16, True),
    (8, 8, 64, 2, 1, [500], torch.bfloat16, False),
    (2, 1, 128, 3, 201, [333], torch.float32, False),      # the largest pool radius this order takes
    (8, 2, 128, 8, 7, [900], torch.float16, False),
    (4, 2, 64, 16, 3, [1300, 70], torch.float16, False),
    # pool radius beyond what the matrix-core kernels take in this order (7): the plain-FMA kernels
    (8, 2, 128, 8, 17, [1100], torch.bfloat16, False),
    (8, 2, 64, 8, 21, [900, 300], torch.bfloat16, False),
    (8, 2, 128, 8, 19, [700], torch.float16, True),
    (4, 2, 64, 16, 17, [1300], torch.float16, False),
]
# ... and every instantiation of the matrix-core kernels in this order: the shapes of
# variant_shapes() that are scored on the matrix cores, with their own pool kernels (3 to 9)
POOL_FIRST_CASES += [(h_q, h, d, w, k, [n], dt, False) for h_q, h, d, w, k, n, _, dt in variant_shapes()
                     if h_q // h * w <= 512 and k // 2 <= 7]
# ... and the 512-row shape in 4096-key chunks
POOL_FIRST_CASES += [SHAPE_512_ROWS_4096_KEYS + (dt, False) for dt in (torch.bfloat16, torch.float16)]
POOL_FIRST_CASES += [shape + (dt, False) for shape in SHAPES_128_ROWS_4096_KEYS + SHAPES_256_ROWS_2048_KEYS
                     for dt in (torch.bfloat16, torch.float16)]


@pytest.mark.parametrize("case", POOL_FIRST_CASES,
                         ids=lambda c: "hq%d_h%d_d%d_w%d_k%d_n%d_%s%s" % (c[:5] + (c[5][0], str(c[6])[6:], "_lse" if c[7] else "")))
def test_pool_then_mean_flag_matches_oracle_order(case):
    """ADAKV_FLAG_POOL_THEN_MEAN: scores follow the oracle's order="pool_then_mean"; the later
    steps are exact functions of the scores as always."""
    from paper_2407_11550_amd.binding import ADAKV_FLAG_POOL_THEN_MEAN
    h_q, h, d, w, k, n, dt, with_lse = case
    _say(f"pool then mean {case}")
    B = [h * (w + max(1, nb // 10)) for nb in n]
    wl = synth.small_workload(h_q, h, d, w, k, n, B, dtype=dt, seed=41)
    q, K, V = synth.generate(wl, device=DEV)
    layer = adakv.Layer.from_workload(wl, flags=ADAKV_FLAG_POOL_THEN_MEAN)
    lse = synth.prefill_row_lse(wl, q, K) if with_lse else None
    out = adakv.compress(layer, q, K, V, row_lse=lse)
    torch.cuda.synchronize()
    off, soff, row0 = wl.tok_off, 0, 0
    for b in range(wl.batch):
        qd, Kd = to_f64(q[b]), to_f64(K[off[b]:off[b + 1]])
        ref = O.score(qd, Kd, wl.n[b], w, k, order="pool_then_mean",
                      row_lse=None if lse is None else to_f64(lse[b]))
        ns = h * wl.n[b]
        sc = out["scores"][soff:soff + ns].cpu().numpy()
        assert_scores_close(sc, ref, f"pool then mean seq {b}")
        assert_exact_on_scores(out, sc, wl, K, V, b, seg0=b * h, row0=row0)
        soff += ns
        row0 += wl.B[b]
    plain = adakv.score(adakv.Layer.from_workload(wl), q, K, row_lse=lse)
    if 1 < k <= 15:                                                     # (a pool window that always holds
        assert not torch.equal(plain, out["scores"])                      # the head's peak hides the order)
    elif k == 1:
        assert_scores_close(plain.cpu().numpy(), out["scores"].cpu().numpy(), "orders agree without pooling")


def test_pool_then_mean_flag_at_full_size():
    """The printed order of Alg. 2 l.4 on a complete llama8b_32k layer (matrix-core kernels,
    pipeline mode): every score against the oracle's order="pool_then_mean", the rest exact."""
    from paper_2407_11550_amd.binding import ADAKV_FLAG_POOL_THEN_MEAN
    _say("pool then mean, llama8b_32k")
    wl = synth.workload("llama8b_32k")
    q, K, V = synth.generate(wl, device=DEV)
    layer = adakv.Layer.from_workload(wl, flags=ADAKV_FLAG_POOL_THEN_MEAN)
    assert adakv.describe(layer)["score"] == "mfma-pool-first"
    out = adakv.compress(layer, q, K, V)
    torch.cuda.synchronize()
    ref = O.score(to_f64(q[0]), to_f64(K), wl.n[0], wl.w, wl.pool_k, order="pool_then_mean")
    sc = out["scores"].cpu().numpy()
    assert_scores_close(sc, ref, "pool then mean, llama8b_32k")
    assert_exact_on_scores(out, sc, wl, K, V)
    plain = adakv.score(adakv.Layer.from_workload(wl), q, K)
    assert not torch.equal(plain, out["scores"])


@pytest.mark.parametrize("dt", [torch.bfloat16, torch.float32, torch.float16], ids=["bf16", "fp32", "fp16"])
def test_c_abi_from_a_plain_cpp_program(dt, tmp_path):
    """The library needs neither Python nor PyTorch: tests/abi_driver.bin (hipMalloc, default
    stream) runs the four calls on files and its outputs are checked like the binding's."""
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "abi_driver.bin")
    if not os.path.exists(exe):
        pytest.fail("tests/abi_driver.bin is missing: run __graft_entry__.build()")
    _say(f"abi_driver {dt}")
    wl = synth.small_workload(8, 2, 64 if dt == torch.float32 else 128, 16, 7, [2500, 310], [2 * 150, 2 * 40],
                              dtype=dt, seed=71)
    q, K, V = synth.generate(wl)                                    # on the host
    raw = (lambda t: t.numpy()) if dt == torch.float32 else (lambda t: t.view(torch.int16).numpy())
    for name, t in (("q", q), ("K", K), ("V", V)):
        raw(t.contiguous()).tofile(str(tmp_path / f"{name}.bin"))
    code = {torch.bfloat16: 0, torch.float32: 1, torch.float16: 2}[dt]
    meta = [code, wl.h_q, wl.h_kv, wl.d, wl.w, wl.pool_k, wl.alpha, 0, wl.batch] + wl.n + wl.B
    (tmp_path / "meta.txt").write_text(" ".join(str(v) for v in meta) + "\n")
    r = subprocess.run([exe, str(tmp_path)], capture_output=True, text=True, timeout=100)
    assert r.returncode == 0, r.stdout + r.stderr
    rows = sum(wl.B)
    out = dict(scores=torch.from_numpy(np.fromfile(str(tmp_path / "scores.bin"), dtype=np.float32)),
               budgets=torch.from_numpy(np.fromfile(str(tmp_path / "budgets.bin"), dtype=np.int32)),
               cu_seqlens=torch.from_numpy(np.fromfile(str(tmp_path / "cu_seqlens.bin"), dtype=np.int32)),
               indices=torch.from_numpy(np.fromfile(str(tmp_path / "indices.bin"), dtype=np.int32)))
    for name in ("K_out", "V_out"):
        if dt != torch.float32:
            t = torch.from_numpy(np.fromfile(str(tmp_path / f"{name}.bin"), dtype=np.int16)).view(dt)
        else:
            t = torch.from_numpy(np.fromfile(str(tmp_path / f"{name}.bin"), dtype=np.float32))
        out[name] = t.view(rows, wl.d)
    _check_all(wl, q, K, V, out)


def test_side_stream_and_unaligned_workspace_give_the_same_result():
    """Calls only enqueue on the stream they are given, and the workspace may start anywhere."""
    _say("side stream, unaligned workspace")
    wl = synth.small_workload(16, 4, 128, 16, 7, [2600, 900], [4 * 100, 4 * 60], seed=55)
    q, K, V = synth.generate(wl, device=DEV)
    layer = adakv.Layer.from_workload(wl)
    ref = adakv.compress(layer, q, K, V)
    torch.cuda.synchronize()
    big = torch.empty(adakv.workspace_bytes(layer) + 64, dtype=torch.uint8, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    out = adakv.compress(layer, q, K, V, ws=big[24:], stream=side)
    side.synchronize()
    for key in ref:
        assert torch.equal(ref[key], out[key]), key
    # a workspace that is too small is refused before anything is launched
    with pytest.raises(adakv.AdaKVError) as e:
        adakv.score(layer, q, K, ws=big[:1000])
    assert e.value.status == -3


@pytest.mark.parametrize("nbytes", [0, 16, 16 * 1000, 16 * (2048 * 256 * 4 + 12345), 16 * (5 * 2048 * 256 * 4)])
def test_streaming_read_probe_reads_every_word_once(nbytes):
    """The read-rate reference of the benchmark: the XOR of its per-wave words must be the XOR of
    the buffer's 16-byte words (every word read, none twice), for sizes below one pass of the
    grid, with a ragged tail, and of several passes."""
    _say(f"probe_read {nbytes} bytes")
    rng = np.random.Generator(np.random.PCG64(nbytes % 9973))
    host = rng.integers(0, 2 ** 32, size=max(nbytes // 4, 4), dtype=np.uint32)
    src = torch.from_numpy(host.view(np.int32)).to(DEV)[: nbytes // 4]
    sink = torch.full((adakv.PROBE_SINK_BYTES // 4,), -1, dtype=torch.int32, device=DEV)
    adakv.probe_read(src, sink)
    torch.cuda.synchronize()
    got = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32).reshape(-1, 4), axis=0)
    want = np.bitwise_xor.reduce(host[: nbytes // 4].reshape(-1, 4), axis=0) if nbytes else np.zeros(4, np.uint32)
    assert np.array_equal(got, want)
    with pytest.raises(adakv.AdaKVError):
        adakv.probe_read(torch.zeros(6, dtype=torch.int32, device=DEV), sink)      # 24 bytes


# ------------------------------------------------------------------ out-of-contract data
def test_compact_clamps_indices_that_leave_the_sequence():
    """A corrupt index must not take the gather outside the sequence's own rows: it is clamped to
    [0, n + w - 1] (the rows around K and V hold NaN and must not show up in the outputs)."""
    _say("compact with corrupt indices")
    h, n, w, d = 2, 300, 4, 128
    g = torch.Generator(device=DEV); g.manual_seed(5)
    pad = 50
    Kbig = torch.full((pad + n + w + pad, h, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    Vbig = torch.full_like(Kbig, float("nan"))
    Kbig[pad:pad + n + w] = torch.randn((n + w, h, d), generator=g, device=DEV).to(torch.bfloat16)
    Vbig[pad:pad + n + w] = torch.randn((n + w, h, d), generator=g, device=DEV).to(torch.bfloat16)
    K, V = Kbig[pad:pad + n + w], Vbig[pad:pad + n + w]
    budgets = np.array([6, 3], np.int32)
    cu = np.concatenate([[0], np.cumsum(budgets + w)]).astype(np.int32)
    idx = np.array([0, -5, 10 ** 9, n + w + 100, 17, -(2 ** 31), n, n + 1, n + 2, n + 3,
                    5, 2 ** 31 - 1, -1, n, n + 1, n + 2, n + 3], np.int32)
    assert len(idx) == cu[-1]
    layer = adakv.Layer(torch.bfloat16, h, h, d, w, 7, 0.2, [n], [int(cu[-1])])
    Ko, Vo = adakv.compact(layer, K, V, torch.tensor(idx, device=DEV), torch.tensor(cu, device=DEV))
    torch.cuda.synchronize()
    clamped = np.clip(idx.astype(np.int64), 0, n + w - 1)
    Kr, Vr = O.compact(K.float().cpu().numpy(), V.float().cpu().numpy(), clamped, cu)
    assert np.array_equal(Ko.float().cpu().numpy(), Kr) and np.array_equal(Vo.float().cpu().numpy(), Vr)


def test_select_with_inconsistent_budgets_stays_inside_its_output():
    """Budgets that ask for more than a head holds, or for less than nothing, and offsets that do
    not match them: the result is unspecified, but nothing outside indices[0 .. sum B) is written."""
    _say("select with corrupt budgets")
    rng = np.random.default_rng(12)
    h, n, w = 3, 6000, 4
    s = rng.random((h, n)).astype(np.float32)
    good = np.array([40, 50, 60], np.int32)
    cu = np.concatenate([[0], np.cumsum(good + w)]).astype(np.int32)
    rows = int(cu[-1])
    layer = adakv.Layer(torch.bfloat16, h, h, 128, w, 7, 0.2, [n], [rows])
    for budgets, offsets in (([n + 500, -3, 50], cu), ([40, 50, 60], [0, 10 ** 6, -7, 5]), ([2 ** 30, 2 ** 30, 2 ** 30], cu)):
        big = torch.full((rows + 16,), -77, dtype=torch.int32, device=DEV)
        adakv.select(layer, torch.tensor(s, device=DEV).reshape(-1), torch.tensor(budgets, dtype=torch.int32, device=DEV),
                     torch.tensor(np.asarray(offsets, np.int32), device=DEV), indices=big[8:8 + rows])
        torch.cuda.synchronize()
        assert (big[:8] == -77).all() and (big[8 + rows:] == -77).all(), budgets
        inside = big[8:8 + rows]
        assert ((inside == -77) | ((inside >= 0) & (inside < n + w))).all(), budgets
