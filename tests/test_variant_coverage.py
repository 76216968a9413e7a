"""CPU-side check that the GPU parity shapes reach every instantiation of the scoring kernels.

adakv_describe reports, on the host, which variant a layer shape is scored with; the shapes are
the ones the GPU tests run (imported from them, nothing is launched here)."""
import itertools

import torch

import paper_2407_11550_amd as adakv
from paper_2407_11550_amd import synth

import test_gpu_decode as GD
import test_gpu_parity as G


def _variants_reached():
    seen = set()
    shapes = list(G.SHAPES) + list(G.variant_shapes())
    layers = [synth.small_workload(h_q, h, d, w, k, n, h * Bh, dtype=dt) for h_q, h, d, w, k, n, Bh, dt in shapes]
    layers += [synth.small_workload(h_q, h, d, w, k, n, B, alpha=a, dtype=dt) for h_q, h, d, w, k, n, B, a, dt, _ in G._fuzz_shapes()]
    layers += [synth.workload(nm) for nm in ("tiny", "llama8b_32k", "llama8b_128k", "llama8b_ragged", "llama70b_128k")]
    h_q, h, d, w, k, n = G.SHAPE_512_ROWS_4096_KEYS
    layers += [synth.small_workload(h_q, h, d, w, k, n, [h * (w + 1)] * len(n), dtype=dt) for dt in (torch.bfloat16, torch.float16)]
    layers += [synth.small_workload(h_q, h, d, w, k, n, [h * (w + 1)] * len(n), dtype=dt)
               for h_q, h, d, w, k, n in G.SHAPES_128_ROWS_4096_KEYS + G.SHAPES_256_ROWS_2048_KEYS
               for dt in (torch.bfloat16, torch.float16)]
    described = [adakv.describe(adakv.Layer.from_workload(wl)) for wl in layers]
    for h_q, h, d, w, k, n, dt, _ in G.POOL_FIRST_CASES:
        wl = synth.small_workload(h_q, h, d, w, k, n, [h * (w + max(1, nb // 10)) for nb in n], dtype=dt)
        described.append(adakv.describe(adakv.Layer.from_workload(wl, flags=adakv.binding.ADAKV_FLAG_POOL_THEN_MEAN)))
    for v in described:
        if v["score"] == "mfma":
            seen.add((v["dtype"], int(v["d"]), int(v["mb"]), int(v["rs"]), int(v["kg"]), int(v["chunk"])))
            seen.add(("lse", v["lse"], int(v["d"])))
            seen.add(("pool", v["pool"], int(v["d"])))
        elif v["score"] == "mfma-pool-first":
            seen.add(("pool-first", v["dtype"], int(v["d"]), int(v["mb"]), int(v["rs"]), int(v["kg"]), int(v["chunk"])))
        else:
            seen.add((v["score"], v["dtype"], int(v["d"])))
    return seen


def test_gpu_shapes_reach_every_scoring_variant(lib):
    seen = _variants_reached()
    want = set()
    for dt, d in itertools.product(("bf16", "fp16"), (64, 128)):
        for mb, rs, kg, chunk in ((1, 1, 4, 2048), (2, 1, 4, 2048), (2, 2, 2, 512), (2, 2, 2, 1024),
                                  (2, 2, 2, 2048), (2, 2, 2, 4096), (2, 4, 1, 1024), (2, 4, 1, 2048)):
            want.add((dt, d, mb, rs, kg, chunk))
        if d == 128:
            want |= {(dt, d, 2, 8, 1, 2048), (dt, d, 2, 8, 1, 4096)}
        else:
            want.add((dt, d, 4, 4, 1, 1024))
    # the same instantiations once more for the other order of pooling and averaging
    want |= {("pool-first",) + v for v in set(want)}
    for d in (64, 128):
        want |= {("lse", "fused", d), ("lse", "kernel", d), ("pool", "fused", d), ("pool", "kernel", d)}
    for dt, d in itertools.product(("bf16", "fp16", "fp32"), (64, 128)):
        want.add(("fma", dt, d))
        if (dt, d) != ("fp32", 128):            # the other order is the same kernel per type and d;
            want.add(("fma-pool-first", dt, d)) # fp32 d = 128 is reached by the plain order only
    missing = sorted(map(str, want - seen))
    assert not missing, "no GPU parity shape reaches: " + ", ".join(missing)


def test_describe_follows_flags_and_rejects_what_score_rejects(lib):
    wl = synth.workload("llama8b_128k")
    plain = adakv.describe(adakv.Layer.from_workload(wl))
    assert plain["score"] == "mfma" and plain["chunk"] == "2048" and plain["topk"] == "separate"
    assert adakv.describe(adakv.Layer.from_workload(wl, flags=adakv.binding.ADAKV_FLAG_PIPELINE))["topk"] == "carried"
    assert adakv.describe(adakv.Layer.from_workload(wl), row_lse=True)["stats"] == "caller"
    first = adakv.describe(adakv.Layer.from_workload(wl, flags=adakv.binding.ADAKV_FLAG_POOL_THEN_MEAN))
    assert first["score"] == "mfma-pool-first" and first["pool"] == "rows"
    wl.pool_k = 17                                       # radius 8: beyond what that kernel pools across lanes
    assert adakv.describe(adakv.Layer.from_workload(wl, flags=adakv.binding.ADAKV_FLAG_POOL_THEN_MEAN))["score"] == "fma-pool-first"
    wl.pool_k = 4
    try:
        adakv.describe(adakv.Layer.from_workload(wl))
    except adakv.AdaKVError as e:
        assert e.status == -1
    else:
        raise AssertionError("an even pool kernel must be rejected")


def test_gpu_shapes_reach_every_decode_variant():
    """decode_attn_kernel<T, D, G> and decode_combine_kernel<D, G> are instantiated per element
    type, head dimension and group size; supported: three types, d 64 / 128, g 1 / 2 / 4 / 8."""
    shapes = list(GD.DECODE_SHAPES) + [s for s, _, _ in GD.decode_sweep_shapes()] + list(GD.DECODE_VARIANT_SHAPES)
    seen = {(dt, d, h_q // h) for h_q, h, d, _, _, _, dt, _ in shapes}
    want = set(itertools.product((torch.bfloat16, torch.float16, torch.float32), (64, 128), (1, 2, 4, 8)))
    missing = sorted(map(str, want - seen))
    assert not missing, "no GPU decode shape reaches: " + ", ".join(missing)
