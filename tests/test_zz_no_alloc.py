"""hc_restore_context_static (the entry point that allocates nothing) against
hc_restore_context on the same stored context: bit-identical pools, on two calls in a row,
the second with a smaller input (the shared device-resident staging array keeps the first
call's rows), plus the size limit."""
import numpy as np
import pytest

import gpu_harness as gh

pytestmark = pytest.mark.gpu


def test_static_restore_matches_allocating_restore():
    import torch
    import paper_2410_05004_amd as hc

    L, d_model, n_kv, hd, B, CT = 4, 1024, 2, 128, 16, 64
    T_stored, pos_offset = 900, 1000
    assert hc.static_stage_bytes() == 8 * 1024 * 1024
    desc = gh.make_desc(hc, n_layers=L, d_model=d_model, n_q_heads=n_kv, n_kv_heads=n_kv,
                        head_dim=hd, block_size=B, max_position=pos_offset + T_stored)
    cases = [gh.LayerCase(np.random.default_rng([77, l]), d_model, n_kv, hd, T_stored) for l in range(L)]
    store = hc.Store(L, d_model, CT, capacity_chunks=L * ((T_stored + CT - 1) // CT) + 2, pinned=True)
    cuts = [0, 512, 700, 701, 900]                       # a prefill, then smaller appends
    for a, b in zip(cuts[:-1], cuts[1:]):
        for l in range(L):
            store.append(9, l, np.ascontiguousarray(cases[l].x_bits[a:b]), b - a)
    n_blocks = (pos_offset + T_stored + B - 1) // B
    num_pages = n_blocks + 5
    rng = np.random.default_rng(78)
    bt = rng.permutation(num_pages)[:n_blocks].astype(np.int32)
    d_bt = gh.to_dev_i32(bt)
    ctx = hc.Context(desc)
    s = gh.stream_handle()
    copy_stream = torch.cuda.Stream()
    keep = []
    for l in range(L):
        d_w, d_g = gh.to_dev_bf16(cases[l].wkv_bits), gh.to_dev_bf16(cases[l].gamma_bits)
        keep += [d_w, d_g]
        ctx.set_layer_weights(l, d_w, d_g, s)
    torch.cuda.synchronize()

    def run(fn, tok_begin, n_tok):
        pools = [gh.new_pool(num_pages, B, n_kv, hd) for _ in range(L)]
        for l in range(L):
            ctx.set_kv_pool(l, pools[l], num_pages)
        fn(store, 9, tok_begin, n_tok, pos_offset, d_bt, n_blocks, s, copy_stream.cuda_stream)
        assert ctx.poll_device_error(s) == 0
        torch.cuda.synchronize()
        return [gh.pool_bits(p) for p in pools]

    # two calls in a row through the static entry point, the second smaller and elsewhere
    ranges = [(30, 850), (200, 130)]
    got = [run(ctx.restore_context_static, a, n) for a, n in ranges]
    want = [run(ctx.restore_context, a, n) for a, n in ranges]
    for (a, n), g, w in zip(ranges, got, want):
        for l in range(L):
            assert np.any(w[l] != gh.SENTINEL)
            assert np.array_equal(g[l], w[l]), f"range ({a}, {n}) layer {l}: pools differ"
            written = (w[l] != gh.SENTINEL).all(axis=(3, 4)).sum()
            assert written == 2 * n, "the reference restore wrote an unexpected number of rows"

    # limits: rows beyond the static staging buffer, equal streams
    too_many = hc.static_stage_bytes() // (2 * d_model) + 1
    with pytest.raises(hc.HCacheError) as e:
        ctx.restore_context_static(store, 9, 0, too_many, 0, d_bt, n_blocks, s, copy_stream.cuda_stream)
    assert e.value.status == hc.HC_ERANGE
    with pytest.raises(hc.HCacheError) as e:
        ctx.restore_context_static(store, 9, 0, 10, 0, d_bt, n_blocks, s, s)
    assert e.value.status == hc.HC_EINVAL
    ctx.restore_context_static(store, 9, 0, 0, 0, d_bt, n_blocks, s, copy_stream.cuda_stream)   # empty
    ctx.destroy()
    store.destroy()
