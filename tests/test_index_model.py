"""A CPU model of the index arithmetic that decides which K rows the scoring kernel's lanes ask
for (chunks, halo, tile sets, the row clamp).  The kernel turns the clamped row, counted from
the tile set's first key, into a byte offset with an unsigned multiply, so the model checks, for
every chunk length, tile-set size, pool radius and ragged length the launcher can choose:
  * the clamped row is never negative and lies inside the sequence,
  * every row somebody needs (the chunk plus the pool radius on both sides) is read unclamped,
  * no tile set starts past the last needed key.
The formulas are retyped from csrc/score_mfma.hip (k0, k1, need_lo, need_hi, lim, lo); the test
documents the invariant and guards the arithmetic, it does not run the kernel."""
import pytest

TILE = 32
HALO = 32


def violations(n, chunk_len, kg, pool_r, halo, sweep):
    bad = 0
    for chunk in range((n + chunk_len - 1) // chunk_len):
        kc0 = chunk * chunk_len
        kc1 = min(n, kc0 + chunk_len)
        fused = sweep == 2 and halo
        pr = pool_r if fused else 0
        k0 = kc0 - HALO if (fused and kc0 > 0) else kc0
        k1 = min(n, kc1 + pr) if fused else kc1
        ntiles = (k1 - k0 + TILE - 1) // TILE
        iters = (ntiles + kg - 1) // kg
        need_lo, need_hi = max(kc0 - pr, 0), min(kc1 - 1 + pr, n - 1)
        for it in range(iters):
            key0 = k0 + it * kg * TILE
            bad += key0 > need_hi
            lim, lo = max(need_hi - key0, 0), max(need_lo - key0, 0)
            for rel in range(kg * TILE):
                row = max(min(rel, lim), lo)
                bad += row < 0 or not (0 <= key0 + row < n)
                bad += need_lo <= key0 + rel <= need_hi and row != rel
    return bad


@pytest.mark.parametrize("chunk_len", [512, 1024, 2048])
@pytest.mark.parametrize("kg", [1, 2, 4])
def test_row_clamp_stays_inside_the_needed_rows(chunk_len, kg):
    for n in [1, 5, 31, 32, 33, 300, 511, 512, 513, 2047, 2048, 2049, 2080, 4096, 4099, 6000, 6145]:
        for pool_r in [0, 1, 3, 16, 32]:
            for halo, sweep in [(1, 2), (0, 2), (0, 1)]:
                assert violations(n, chunk_len, kg, pool_r, halo, sweep) == 0, (n, pool_r, halo, sweep)


def pool_violations(n, chunk_len, nt, pool_r, halo):
    """The fused max-pool of sweep 2: thread tid pools keys kc0 + tid + i*nt (clamped to the
    chunk's last key) and reads offsets -r..r around them, clamped to the sequence, from the
    chunk's score array that starts at key k0 and holds span = k1 - k0 entries."""
    bad = 0
    r = pool_r if halo else 0
    for chunk in range((n + chunk_len - 1) // chunk_len):
        kc0 = chunk * chunk_len
        kc1 = min(n, kc0 + chunk_len)
        k0 = kc0 - HALO if (halo and kc0 > 0) else kc0
        k1 = min(n, kc1 + r) if halo else kc1
        span = k1 - k0
        bad += span > chunk_len + 2 * HALO
        for tid in (0, 1, nt // 2, nt - 1):
            for i in range(chunk_len // nt):
                pk = min(kc0 + tid + i * nt, kc1 - 1)
                for t in range(-r, r + 1):
                    idx = min(max(pk + t, 0), n - 1) - k0
                    bad += not (0 <= idx < span)
    return bad


@pytest.mark.parametrize("chunk_len,nt", [(512, 256), (1024, 256), (2048, 256), (1024, 512)])
def test_fused_pool_reads_stay_inside_the_chunk_array(chunk_len, nt):
    for n in [1, 5, 31, 33, 300, 511, 513, 2047, 2049, 2080, 4096, 4099, 6145]:
        for pool_r in [0, 1, 3, 16, 32]:
            for halo in (0, 1):
                assert pool_violations(n, chunk_len, nt, pool_r, halo) == 0, (n, pool_r, halo)


def interleaved_violations(n, chunk_len, kg):
    """Sweep 1: workgroup `chunk` of the nch = ceil(n / chunk_len) of a head takes the tile sets
    chunk, chunk + nch, ... of the whole sequence (a set = kg tiles of 32 keys).  Every set must be
    taken exactly once, every workgroup must have at least one, no set may start past the last
    key, and the row clamp (0 .. n-1-key0) must keep every lane inside the sequence."""
    bad = 0
    nch = (n + chunk_len - 1) // chunk_len
    ntiles = (n + TILE - 1) // TILE
    sets_all = (ntiles + kg - 1) // kg
    taken = [0] * sets_all
    for chunk in range(nch):
        iters = (sets_all - chunk + nch - 1) // nch
        bad += iters < 1
        for it in range(iters):
            s = chunk + it * nch
            bad += not (0 <= s < sets_all)
            if 0 <= s < sets_all:
                taken[s] += 1
            key0 = s * kg * TILE
            bad += key0 > n - 1
            lim = max(n - 1 - key0, 0)
            for rel in range(kg * TILE):
                row = max(min(rel, lim), 0)
                bad += not (0 <= key0 + row < n)
                bad += key0 + rel < n and row != rel
    bad += any(t != 1 for t in taken)
    return bad


@pytest.mark.parametrize("chunk_len", [512, 1024, 2048])
@pytest.mark.parametrize("kg", [1, 2, 4])
def test_interleaved_sets_of_sweep_one_cover_every_key_once(chunk_len, kg):
    for n in [1, 5, 31, 32, 33, 63, 64, 65, 300, 511, 512, 513, 2047, 2048, 2049, 2080, 4096, 4099, 6000, 6145, 20001]:
        assert interleaved_violations(n, chunk_len, kg) == 0, n
