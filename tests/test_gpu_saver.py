"""Two-stage saving on the GPU: snapshots of device batches reach the store exactly as the
oracle's chunk-store model predicts, the activation buffer may be overwritten right after the
call, and a context saved this way restores to the KV the oracle computes."""
import ctypes

import numpy as np
import pytest

import synthetic as syn
import oracle.hcache_oracle as oracle
import gpu_harness as gh

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hc():
    import paper_2410_05004_amd as hc
    return hc


def read_chunk(store, seq, layer, c, d):
    ptr, rows = store.chunk(seq, layer, c)
    buf = (ctypes.c_uint16 * (rows * d)).from_address(ptr)
    return np.frombuffer(buf, dtype=np.uint16).reshape(rows, d).copy()


def test_save_then_restore_round_trip(hc):
    import torch
    L, d_model, n_kv, hd, B, CT = 3, 512, 2, 128, 16, 64
    steps, totals = syn.batching_schedule(11, n_seq=4, len_range=(100, 400), prefill_chunk=96)
    cases = {s: [gh.LayerCase(np.random.default_rng([41, s, l]), d_model, n_kv, hd, n) for l in range(L)]
             for s, n in totals.items()}
    cap = sum(-(-n // CT) for n in totals.values()) * L + 4
    store = hc.Store(L, d_model, CT, cap, pinned=True)
    max_rows = max(sum(n for _, _, n in st) for st in steps)
    saver = hc.Saver(store, max_rows, n_slots=3, n_threads=8)
    ref = oracle.ChunkStore(L, d_model, CT)
    dev = {s: [gh.to_dev_bf16(c.x_bits) for c in cs] for s, cs in cases.items()}
    compute = torch.cuda.current_stream()
    down = torch.cuda.Stream()
    act = torch.empty((max_rows, d_model), dtype=torch.bfloat16, device="cuda")   # the reused activation buffer
    scratch = torch.empty_like(act)
    for i, st in enumerate(steps):
        row_seq = np.concatenate([np.full(n, s, dtype=np.int64) for s, _, n in st])
        n_rows = len(row_seq)
        for l in range(L):
            torch.cat([dev[s][l][a:a + n] for s, a, n in st], out=act[:n_rows])
            if i % 2 == 0:
                saver.save_layer(l, act, n_rows, row_seq, compute.cuda_stream, down.cuda_stream)
            else:
                # the paper's pipeline: the layer runs beside its snapshot (here: it reads the
                # buffer), and the first operator that overwrites it waits for the copy
                saver.save_layer_deferred(l, act, n_rows, row_seq, compute.cuda_stream, down.cuda_stream)
                torch.mul(act, 2.0, out=scratch)
                saver.fence(compute.cuda_stream)
            act.fill_(-1.0)                             # the next layer overwrites the buffer at once
            rows = np.concatenate([cases[s][l].x_bits[a:a + n] for s, a, n in st])
            oracle.save_step(ref, l, rows, row_seq)
    saver.flush()
    for s, n in totals.items():
        for l in range(L):
            assert store.tokens(s, l) == n
            for c in range(ref.n_chunks(s, l)):
                assert np.array_equal(read_chunk(store, s, l, c, d_model), ref.chunk(s, l, c)), (s, l, c)
    # restore one saved context and compare with the oracle
    s0 = max(totals, key=totals.get)
    T = totals[s0]
    desc = gh.make_desc(hc, n_layers=L, d_model=d_model, n_q_heads=n_kv, n_kv_heads=n_kv,
                        head_dim=hd, block_size=B, max_position=T)
    ctx = hc.Context(desc)
    n_blocks = (T + B - 1) // B
    bt = np.random.default_rng(3).permutation(n_blocks + 3)[:n_blocks].astype(np.int32)
    d_bt = gh.to_dev_i32(bt)
    sh = gh.stream_handle()
    pools, keep = [], []
    for l in range(L):
        d_w, d_g = gh.to_dev_bf16(cases[s0][l].wkv_bits), gh.to_dev_bf16(cases[s0][l].gamma_bits)
        keep += [d_w, d_g]
        ctx.set_layer_weights(l, d_w, d_g, sh)
        pools.append(gh.new_pool(n_blocks + 3, B, n_kv, hd))
        ctx.set_kv_pool(l, pools[l], n_blocks + 3)
    ctx.restore_context(store, s0, 0, T, 0, d_bt, n_blocks, sh, down.cuda_stream)
    assert ctx.poll_device_error(sh) == 0
    torch.cuda.synchronize()
    pos = np.arange(T, dtype=np.int32)
    for l in range(L):
        ora = np.full((n_blocks + 3, 2, B, n_kv, hd), np.nan)
        c = cases[s0][l]
        oracle.restore_kv(ora, c.x, c.gamma, c.wkv, pos, bt, **gh.oracle_kw(desc))
        gh.compare_pool(gh.pool_bits(pools[l]), ora)
    ctx.destroy()
    saver.destroy()
    store.destroy()


def test_saver_argument_errors(hc):
    import torch
    store = hc.Store(2, 64, 8, 8, pinned=True)
    saver = hc.Saver(store, 16, n_slots=2, n_threads=2)
    x = torch.zeros((16, 64), dtype=torch.bfloat16, device="cuda")
    seq = np.zeros(16, dtype=np.int64)
    s = gh.stream_handle()
    other = torch.cuda.Stream().cuda_stream
    with pytest.raises(hc.HCacheError) as e:
        saver.save_layer(0, x, 16, seq, s, s)
    assert e.value.status == hc.HC_EINVAL
    with pytest.raises(hc.HCacheError) as e:
        saver.save_layer(0, x, 17, seq, s, other)
    assert e.value.status == hc.HC_ERANGE
    saver.save_layer(0, x, 16, seq, s, other)
    saver.flush()
    assert store.tokens(0, 0) == 16
    saver.destroy()
    store.destroy()


def test_saver_at_13b_width(hc):
    """Batches of the size the paper quotes for a 13B model (1024-row prefill chunks of
    d_model 5120, then 48-context decode steps) through the deferred-fence save path; the
    store must hold exactly what the oracle's model of the two stages holds."""
    import torch
    L, d_model, CT = 3, 5120, 64
    rng = np.random.default_rng(13)
    n_ctx, prefill, decode_steps = 48, 1024, 5
    store = hc.Store(L, d_model, CT, L * ((prefill + CT - 1) // CT + n_ctx) + n_ctx * L + 8 + 12 * L, pinned=True)
    saver = hc.Saver(store, 1024, n_slots=4, n_threads=8)
    ref = oracle.ChunkStore(L, d_model, CT)
    compute = torch.cuda.current_stream()
    down = torch.cuda.Stream()
    act = torch.empty((1024, d_model), dtype=torch.bfloat16, device="cuda")

    def save_step(row_seq, bits_per_layer):
        n = len(row_seq)
        for l in range(L):
            act[:n].copy_(gh.to_dev_bf16(bits_per_layer[l]))
            saver.save_layer_deferred(l, act, n, row_seq, compute.cuda_stream, down.cuda_stream)
            saver.fence(compute.cuda_stream)
            act.fill_(0.5)
            oracle.save_step(ref, l, bits_per_layer[l], row_seq)

    # context 100: one 1024-row prefill chunk
    save_step(np.full(prefill, 100, dtype=np.int64),
              [rng.integers(0, 1 << 16, size=(prefill, d_model), dtype=np.uint16) for _ in range(L)])
    # 48 contexts decode together (context 100 among them)
    ids = np.array([100] + list(range(1, n_ctx)), dtype=np.int64)
    for _ in range(decode_steps):
        save_step(ids, [rng.integers(0, 1 << 16, size=(n_ctx, d_model), dtype=np.uint16) for _ in range(L)])
    # fused steps (chunked prefill sharing a batch with decode rows): long runs of contexts 200
    # and 201 go from the device straight into their chunks (full chunks in one strided
    # transfer, the partial ones at either end on their own; the second step starts mid-chunk),
    # the single rows in between through the snapshot slot and the daemon threads
    for n200, n201 in ((300, 100), (200, 70)):
        ids = np.concatenate([np.full(n200, 200), np.arange(1, 11), np.full(n201, 201)]).astype(np.int64)
        save_step(ids, [rng.integers(0, 1 << 16, size=(len(ids), d_model), dtype=np.uint16) for _ in range(L)])
    saver.flush()
    for sid in (100, 1, n_ctx - 1, 200, 201, 10):
        for l in range(L):
            assert store.tokens(sid, l) == ref.n_tokens(sid, l)
            for c in range(ref.n_chunks(sid, l)):
                assert np.array_equal(read_chunk(store, sid, l, c, d_model), ref.chunk(sid, l, c)), (sid, l, c)
    saver.destroy()
    store.destroy()
