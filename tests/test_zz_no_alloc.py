"""adakv_compress_static (the whole step with the library's built-in scratch array, for callers
that cannot allocate) against adakv_compress with a caller's workspace: same kernels, so every
output must be bit-identical.  Two calls in a row share the array; the second is smaller, so it
runs on whatever the first left behind."""
import pytest
import torch

import paper_2407_11550_amd as adakv
from paper_2407_11550_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _bufs(layer, wl):
    return dict(scores=torch.empty(layer.num_scores, dtype=torch.float32, device=DEV),
                budgets=torch.empty(layer.num_segments, dtype=torch.int32, device=DEV),
                cu_seqlens=torch.empty(layer.num_segments + 1, dtype=torch.int32, device=DEV),
                indices=torch.empty(layer.num_rows_out, dtype=torch.int32, device=DEV),
                K_out=torch.empty((layer.num_rows_out, wl.d), dtype=wl.dtype, device=DEV),
                V_out=torch.empty((layer.num_rows_out, wl.d), dtype=wl.dtype, device=DEV))


def test_static_scratch_entry_point_equals_the_workspace_one_on_two_calls_in_a_row():
    cases = [synth.small_workload(32, 8, 128, 32, 7, [9000, 4099, 700], [8 * 300, 8 * 250, 8 * 60],
                                  dtype=torch.bfloat16, seed=31),
             synth.small_workload(8, 2, 128, 16, 5, [1500], [2 * 100], dtype=torch.bfloat16, seed=32),
             synth.small_workload(4, 4, 64, 8, 7, [1024], [4 * 128], dtype=torch.float32, seed=33)]
    made = []
    for wl in cases:
        q, K, V = synth.generate(wl, device=DEV)
        layer = adakv.Layer.from_workload(wl)
        want = adakv.compress(layer, q, K, V)
        made.append((wl, layer, q, K, V, want, _bufs(layer, wl)))
    torch.cuda.synchronize()
    for rnd in range(2):                                   # the second round meets the array as the first left it
        for wl, layer, q, K, V, want, bufs in made:
            print(f"compress_static round {rnd} n {wl.n}", flush=True)
            for t in bufs.values():
                t.zero_()
            torch.cuda.synchronize()
            before = torch.cuda.memory_allocated()
            got = adakv.compress_static(layer, q, K, V, bufs=bufs)
            torch.cuda.synchronize()
            assert torch.cuda.memory_allocated() == before
            for key in want:
                assert torch.equal(got[key], want[key]), (rnd, wl.n, key)


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    wl = synth.workload("llama70b_128k")
    layer = adakv.Layer.from_workload(wl)
    assert adakv.workspace_bytes(layer) <= adakv.STATIC_SCRATCH_BYTES      # every named workload fits
    big = adakv.Layer(torch.bfloat16, 64, 8, 128, 64, 7, 0.2, [400000], [8 * 4096])
    assert adakv.workspace_bytes(big) > adakv.STATIC_SCRATCH_BYTES
    one = torch.zeros(16, dtype=torch.bfloat16, device=DEV)
    import ctypes
    lib = adakv.load_library()
    p = ctypes.c_void_p(one.data_ptr())
    st = lib.adakv_compress_static(ctypes.byref(big.c), p, p, p, None, p, p, p, p, p, p, None)
    assert st == -5 and b"scratch" in lib.adakv_strerror(st)
