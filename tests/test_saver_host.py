"""Two-stage saving, host side (no GPU): the daemon threads must leave the store in exactly
the state the oracle's chunk-store model reaches for the same continuous-batching schedule."""
import ctypes

import numpy as np
import pytest

import synthetic as syn
import oracle.hcache_oracle as oracle


@pytest.fixture(scope="module")
def hc():
    import paper_2410_05004_amd as hc
    return hc


def read_chunk(store, seq, layer, c, d):
    ptr, rows = store.chunk(seq, layer, c)
    buf = (ctypes.c_uint16 * (rows * d)).from_address(ptr)
    return np.frombuffer(buf, dtype=np.uint16).reshape(rows, d).copy()


def run_schedule(hc, seed, n_layers, d, chunk_tokens, n_threads, n_slots):
    steps, totals = syn.batching_schedule(seed)
    rng = np.random.default_rng(seed)
    hidden = {s: rng.integers(0, 65536, size=(n_layers, n, d), dtype=np.uint16) for s, n in totals.items()}
    cap = sum(-(-n // chunk_tokens) for n in totals.values()) * n_layers + 4
    store = hc.Store(n_layers, d, chunk_tokens, cap, pinned=False)
    max_rows = max(sum(n for _, _, n in st) for st in steps)
    saver = hc.Saver(store, max_rows, n_slots=n_slots, n_threads=n_threads)
    ref = oracle.ChunkStore(n_layers, d, chunk_tokens)
    for st in steps:
        row_seq = np.concatenate([np.full(n, s, dtype=np.int64) for s, _, n in st])
        for l in range(n_layers):                      # layer-before-token: all layers of this step
            rows = np.ascontiguousarray(np.concatenate([hidden[s][l, a:a + n] for s, a, n in st]))
            saver.save_layer_host(l, rows, len(rows), row_seq)
            oracle.save_step(ref, l, rows, row_seq)
    saver.flush()
    return store, saver, ref, totals, hidden


@pytest.mark.parametrize("n_threads,n_slots", [(1, 1), (4, 2), (8, 4)])
def test_saver_matches_oracle_store(hc, n_threads, n_slots):
    L, d, CT = 3, 16, 32
    store, saver, ref, totals, hidden = run_schedule(hc, 5, L, d, CT, n_threads, n_slots)
    for s, n in totals.items():
        for l in range(L):
            assert store.tokens(s, l) == n == ref.n_tokens(s, l)
            for c in range(ref.n_chunks(s, l)):
                assert np.array_equal(read_chunk(store, s, l, c, d), ref.chunk(s, l, c)), (s, l, c)
            # and both equal the source rows
            assert np.array_equal(ref.layer(s, l), hidden[s][l])
    saver.destroy()
    store.destroy()


def test_saver_reports_errors(hc):
    L, d, CT = 2, 8, 4
    store = hc.Store(L, d, CT, capacity_chunks=2, pinned=False)
    saver = hc.Saver(store, 16, n_slots=2, n_threads=2)
    rows = np.zeros((12, d), dtype=np.uint16)
    seq = np.full(12, 5, dtype=np.int64)
    # the index half of the save runs inside the call: a full arena is reported at once
    with pytest.raises(hc.HCacheError) as e:
        saver.save_layer_host(0, rows, 12, seq)        # needs 3 chunks, the arena has 2
    assert e.value.status == hc.HC_ERANGE and "arena" in str(e.value)
    assert store.tokens(5, 0) == 0
    # so is a layer that runs ahead of the layer below it
    with pytest.raises(hc.HCacheError) as e:
        saver.save_layer_host(1, rows[:1], 1, np.array([9], dtype=np.int64))
    assert e.value.status == hc.HC_ESTATE
    saver.flush()
    # argument checks
    for args, status in [((5, rows, 1, seq), hc.HC_ERANGE), ((0, rows, 17, seq), hc.HC_ERANGE),
                         ((0, None, 1, seq), hc.HC_EINVAL), ((0, rows, -1, seq), hc.HC_EINVAL)]:
        with pytest.raises(hc.HCacheError) as e:
            saver.save_layer_host(*args)
        assert e.value.status == status
    saver.save_layer_host(0, rows, 0, seq)             # empty batch: no-op
    saver.flush()
    saver.destroy()
    store.destroy()
    with pytest.raises(hc.HCacheError):
        hc.Saver(hc.Store(1, 8, 4, 1, pinned=False), 0)
