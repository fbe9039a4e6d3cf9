"""GPU tests of the KV-offload complement (Section 4.1.2, layer-wise partition): the row <->
page copies and the whole-context restore that takes the first l_h layers from hidden states
and the rest from saved KV rows.  Everything goes through the C ABI; expected values come from
the fp64 oracle (projection) or are the saved bytes themselves (byte copies are bit-exact)."""
import numpy as np
import pytest

import gpu_harness as gh
import oracle.hcache_oracle as oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hc():
    import paper_2410_05004_amd as m
    return m


@pytest.fixture(scope="module")
def torch():
    return gh.torch_mod()


def rand_bf16_bits(rng, shape):
    """Finite, non-sentinel bf16 patterns."""
    b = rng.integers(0, 1 << 16, size=shape, dtype=np.uint16)
    b[(b & 0x7F80) == 0x7F80] &= 0xBFFF        # clear one exponent bit of inf / NaN patterns
    return b


@pytest.mark.parametrize("n_kv,hd,B", [(2, 128, 16), (1, 64, 8), (5, 128, 32)])
def test_scatter_gather_rows(hc, torch, n_kv, hd, B):
    """hc_scatter_kv places rows exactly where the oracle does, hc_gather_kv reads them back;
    arbitrary positions (unsorted, mid-page), invalid rows skipped and flagged."""
    rng = np.random.default_rng([77, n_kv, hd, B])
    d_kv = n_kv * hd
    n_blocks, num_pages = 40, 50
    n_tok = min(333, n_blocks * B - 7)
    desc = gh.make_desc(hc, n_layers=2, d_model=256, n_q_heads=n_kv, n_kv_heads=n_kv, head_dim=hd,
                        block_size=B, max_position=n_blocks * B)
    ctx = hc.Context(desc)
    s = gh.stream_handle()
    bt = rng.permutation(num_pages)[:n_blocks].astype(np.int32)
    pos = rng.permutation(n_blocks * B)[:n_tok].astype(np.int32)
    assert pos.shape == (n_tok,)
    rows = rand_bf16_bits(rng, (n_tok, 2 * d_kv))
    pool = gh.new_pool(num_pages, B, n_kv, hd)
    ctx.set_kv_pool(1, pool, num_pages)
    d_rows, d_pos, d_bt = gh.to_dev_bf16(rows), gh.to_dev_i32(pos), gh.to_dev_i32(bt)
    ctx.scatter_kv(1, d_rows, d_pos, n_tok, d_bt, n_blocks, s)
    assert ctx.poll_device_error(s) == 0
    want = np.full((num_pages, 2, B, n_kv, hd), gh.SENTINEL, dtype=np.uint16)
    oracle.scatter_kv(want, rows[:, :d_kv].reshape(n_tok, n_kv, hd),
                      rows[:, d_kv:].reshape(n_tok, n_kv, hd), pos, bt, B)
    assert np.array_equal(gh.pool_bits(pool), want)
    # read back in another order
    order = rng.permutation(n_tok)
    back = torch.zeros((n_tok, 2 * d_kv), dtype=torch.bfloat16, device="cuda")
    ctx.gather_kv(1, back, gh.to_dev_i32(pos[order]), n_tok, d_bt, n_blocks, s)
    assert ctx.poll_device_error(s) == 0
    got = back.view(torch.int16).cpu().numpy().view(np.uint16)
    k, v = oracle.gather_kv(want, pos[order], bt, B)
    assert np.array_equal(got[:, :d_kv], k.reshape(n_tok, d_kv))
    assert np.array_equal(got[:, d_kv:], v.reshape(n_tok, d_kv))
    # invalid rows: negative, beyond the table, unmapped block
    bt2 = bt.copy()
    bad_block = int(pos[5]) // B
    bt2[bad_block] = -1
    bad_pos = pos.copy()
    bad_pos[0], bad_pos[1] = -5, n_blocks * B + 1
    hit = np.nonzero(bad_pos // B == bad_block)[0]
    pool2 = gh.new_pool(num_pages, B, n_kv, hd)
    ctx.set_kv_pool(0, pool2, num_pages)
    ctx.scatter_kv(0, d_rows, gh.to_dev_i32(bad_pos), n_tok, gh.to_dev_i32(bt2), n_blocks, s)
    assert ctx.poll_device_error(s) == (hc.HC_DEV_BAD_POSITION | hc.HC_DEV_BAD_PAGE)
    good = np.ones(n_tok, dtype=bool)
    good[[0, 1]] = False
    good[hit] = False
    want2 = np.full_like(want, gh.SENTINEL)
    oracle.scatter_kv(want2, rows[good, :d_kv].reshape(-1, n_kv, hd),
                      rows[good, d_kv:].reshape(-1, n_kv, hd), bad_pos[good], bt2, B)
    assert np.array_equal(gh.pool_bits(pool2), want2)
    # host-side errors
    for call, args, st in [
        (ctx.scatter_kv, (2, d_rows, d_pos, n_tok, d_bt, n_blocks, s), hc.HC_ERANGE),
        (ctx.scatter_kv, (0, None, d_pos, n_tok, d_bt, n_blocks, s), hc.HC_EINVAL),
        (ctx.gather_kv, (0, d_rows.data_ptr() + 2, d_pos, n_tok, d_bt, n_blocks, s), hc.HC_EALIGN),
        (ctx.gather_kv, (0, d_rows, d_pos, -1, d_bt, n_blocks, s), hc.HC_EINVAL),
    ]:
        with pytest.raises(hc.HCacheError) as e:
            call(*args)
        assert e.value.status == st
    ctx.destroy()


MIXED_SHAPE = dict(L=5, d_model=512, n_kv=2, hd=128, T_stored=520, tok_begin=20, n_tok=490, pos_offset=200)


def mixed_cases(seed=39):
    """One LayerCase per layer, outlier channels included.  At d_model = 512 five x20 channels
    dominate every sum and the two bf16 roundings of the prescribed arithmetic alone use most of
    the 2e-2 x RMS budget; the seed is one for which they stay inside it on all five layers
    (tests/test_tolerance_model.py proves it on the CPU)."""
    m = MIXED_SHAPE
    return [gh.LayerCase(np.random.default_rng([seed, l]), m["d_model"], m["n_kv"], m["hd"], m["T_stored"])
            for l in range(m["L"])]


@pytest.mark.parametrize("l_h", [0, 3, 5])
def test_restore_context_mixed(hc, torch, l_h):
    """First l_h layers from the hidden-state store (checked against the oracle's projection),
    the others from a KV-row store filled with what a first restoration produced (checked
    bit-exactly against those bytes), into a pool with another block table."""
    rng = np.random.default_rng(41)
    L, d_model, n_kv, hd, B, CT = 5, 512, 2, 128, 16, 64
    d_kv = n_kv * hd
    T_stored, tok_begin, n_tok, pos_offset = 520, 20, 490, 200
    desc = gh.make_desc(hc, n_layers=L, d_model=d_model, n_q_heads=n_kv, n_kv_heads=n_kv,
                        head_dim=hd, block_size=B, max_position=pos_offset + T_stored)
    cases = mixed_cases()
    n_blocks = (pos_offset + T_stored + B - 1) // B
    num_pages = n_blocks + 7
    ctx = hc.Context(desc)
    s = gh.stream_handle()
    copy_stream = torch.cuda.Stream()
    keep = []
    for l in range(L):
        d_w, d_g = gh.to_dev_bf16(cases[l].wkv_bits), gh.to_dev_bf16(cases[l].gamma_bits)
        keep += [d_w, d_g]
        ctx.set_layer_weights(l, d_w, d_g, s)

    # generation time: the KV of every stored token exists in a cache; the offloaded layers'
    # rows are read out of it and saved
    bt_gen = rng.permutation(num_pages)[:n_blocks].astype(np.int32)
    d_bt_gen = gh.to_dev_i32(bt_gen)
    pos_all = (pos_offset + np.arange(T_stored)).astype(np.int32)
    d_pos_all = gh.to_dev_i32(pos_all)
    kv_rows = {}
    gen_pools = []
    for l in range(L):
        pool = gh.new_pool(num_pages, B, n_kv, hd)
        gen_pools.append(pool)
        ctx.set_kv_pool(l, pool, num_pages)
        ctx.restore_kv(l, gh.to_dev_bf16(cases[l].x_bits), d_pos_all, T_stored, d_bt_gen, n_blocks, s)
        if l >= l_h:
            rows = torch.zeros((T_stored, 2 * d_kv), dtype=torch.bfloat16, device="cuda")
            ctx.gather_kv(l, rows, d_pos_all, T_stored, d_bt_gen, n_blocks, s)
            kv_rows[l] = rows.view(torch.int16).cpu().numpy().view(np.uint16)
    assert ctx.poll_device_error(s) == 0

    cap = L * ((T_stored + CT - 1) // CT) + 2
    hstore = hc.Store(L, d_model, CT, capacity_chunks=cap) if l_h > 0 else None
    kstore = hc.Store(L - l_h, 2 * d_kv, CT, capacity_chunks=cap) if l_h < L else None
    cuts = [0, 300, 301, 520]
    for a, b in zip(cuts[:-1], cuts[1:]):
        for l in range(L):
            if hstore is not None:                       # a full hidden store; layers >= l_h unused
                hstore.append(9, l, np.ascontiguousarray(cases[l].x_bits[a:b]), b - a)
            if l >= l_h:
                kstore.append(9, l - l_h, np.ascontiguousarray(kv_rows[l][a:b]), b - a)

    # reuse time: another block table, fresh pools
    bt = rng.permutation(num_pages)[:n_blocks].astype(np.int32)
    d_bt = gh.to_dev_i32(bt)
    pools = []
    for l in range(L):
        pools.append(gh.new_pool(num_pages, B, n_kv, hd))
        ctx.set_kv_pool(l, pools[l], num_pages)
    torch.cuda.synchronize()
    for rep in range(2):
        ctx.restore_context_mixed(hstore, kstore, l_h, 9, tok_begin, n_tok, pos_offset, d_bt,
                                  n_blocks, s, copy_stream.cuda_stream)
    assert ctx.poll_device_error(s) == 0
    torch.cuda.synchronize()
    pos = pos_all[tok_begin:tok_begin + n_tok]
    for l in range(L):
        got = gh.pool_bits(pools[l])
        if l < l_h:
            ora = np.full((num_pages, 2, B, n_kv, hd), np.nan)
            c = cases[l]
            oracle.restore_kv(ora, c.x[tok_begin:tok_begin + n_tok], c.gamma, c.wkv, pos, bt,
                              **gh.oracle_kw(desc))
            gh.compare_pool(got, ora)
        else:
            want = np.full((num_pages, 2, B, n_kv, hd), gh.SENTINEL, dtype=np.uint16)
            r = kv_rows[l][tok_begin:tok_begin + n_tok]
            oracle.scatter_kv(want, r[:, :d_kv].reshape(n_tok, n_kv, hd),
                              r[:, d_kv:].reshape(n_tok, n_kv, hd), pos, bt, B)
            assert np.array_equal(got, want), f"layer {l}: offloaded KV not restored bit-exactly"
            # and those bytes are the projection of the hidden states (lossless either way)
            ora = np.full((num_pages, 2, B, n_kv, hd), np.nan)
            c = cases[l]
            oracle.restore_kv(ora, c.x[tok_begin:tok_begin + n_tok], c.gamma, c.wkv, pos, bt,
                              **gh.oracle_kw(desc))
            gh.compare_pool(got, ora)

    # host-side errors
    def status(*a):
        with pytest.raises(hc.HCacheError) as e:
            ctx.restore_context_mixed(*a)
        return e.value.status
    cs = copy_stream.cuda_stream
    assert status(hstore, kstore, L + 1, 9, 0, 10, 0, d_bt, n_blocks, s, cs) == hc.HC_ERANGE
    if 0 < l_h < L:
        assert status(hstore, None, l_h, 9, 0, 10, 0, d_bt, n_blocks, s, cs) == hc.HC_EINVAL
        assert status(None, kstore, l_h, 9, 0, 10, 0, d_bt, n_blocks, s, cs) == hc.HC_EINVAL
        assert status(hstore, hstore, l_h, 9, 0, 10, 0, d_bt, n_blocks, s, cs) == hc.HC_EINVAL
        assert status(hstore, kstore, l_h - 1, 9, 0, 10, 0, d_bt, n_blocks, s, cs) == hc.HC_EINVAL
        assert status(hstore, kstore, l_h, 8, 0, 10, 0, d_bt, n_blocks, s, cs) == hc.HC_ERANGE
        assert status(hstore, kstore, l_h, 9, 100, 500, 0, d_bt, n_blocks, s, cs) == hc.HC_ERANGE
    ctx.destroy()
    for st in (hstore, kstore):
        if st is not None:
            st.destroy()


def test_mixed_restore_at_7b_width(hc, torch):
    """The paper's schedule for Llama-2-7B is 31 layers from hidden states + 1 from KV offload
    (Table 3).  Full width (d_model 4096, 32 KV heads), 2048 tokens, streamed from pinned
    stores in 256-token chunks; three layers stand for the 32 (two projected, one offloaded):
    whole-pool indexing, sampled rows and a random projection for the projected layers, every
    byte for the offloaded one."""
    import synthetic as syn
    from test_gpu_fullsize import check_layer, sample_rows
    w = syn.WORKLOADS[1]
    T, B, CT = w.tokens, w.block_size, w.chunk_tokens
    model_layers = (0, 30, 31)                           # the last one comes from KV rows
    L, l_h = len(model_layers), 2
    desc = gh.make_desc(hc, n_layers=L, d_model=w.d_model, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads,
                        head_dim=w.head_dim, block_size=B, max_position=T, rope_theta=w.rope_theta,
                        rms_eps=w.rms_eps)
    ctx = hc.Context(desc)
    s = gh.stream_handle()
    copy_stream = torch.cuda.Stream()
    bt_gen, num_pages = syn.block_table(w, T, seq=1)
    bt, _ = syn.block_table(w, T, seq=0)
    d_bt_gen, d_bt = gh.to_dev_i32(bt_gen), gh.to_dev_i32(bt)
    pos = np.arange(T, dtype=np.int32)
    d_pos = gh.to_dev_i32(pos)
    data = []
    for i, l in enumerate(model_layers):
        wkv, gamma = syn.layer_weights(w, l)
        x = syn.layer_hidden(w, l)
        data.append((wkv, gamma, x))
        ctx.set_layer_weights(i, gh.to_dev_bf16(wkv), gh.to_dev_bf16(gamma), s)
        torch.cuda.synchronize()
    # generation time: the offloaded layer's KV exists in a cache under another block table
    gen_pool = gh.new_pool(num_pages, B, w.n_kv_heads, w.head_dim)
    ctx.set_kv_pool(2, gen_pool, num_pages)
    ctx.restore_kv(2, gh.to_dev_bf16(data[2][2]), d_pos, T, d_bt_gen, len(bt_gen), s)
    rows_dev = torch.zeros((T, 2 * w.d_kv), dtype=torch.bfloat16, device="cuda")
    ctx.gather_kv(2, rows_dev, d_pos, T, d_bt_gen, len(bt_gen), s)
    kv_rows = rows_dev.view(torch.int16).cpu().numpy().view(np.uint16)
    n_chunks = T // CT
    hstore = hc.Store(l_h, w.d_model, CT, l_h * n_chunks)
    kstore = hc.Store(1, 2 * w.d_kv, CT, n_chunks)
    for c in range(n_chunks):                            # arrival order: chunk by chunk, layer by layer
        for i in range(l_h):
            hstore.append(5, i, np.ascontiguousarray(data[i][2][c * CT:(c + 1) * CT]), CT)
        kstore.append(5, 0, np.ascontiguousarray(kv_rows[c * CT:(c + 1) * CT]), CT)
    pools = [gh.new_pool(num_pages, B, w.n_kv_heads, w.head_dim) for _ in range(L)]
    for i in range(L):
        ctx.set_kv_pool(i, pools[i], num_pages)
    ctx.restore_context_mixed(hstore, kstore, l_h, 5, 0, T, 0, d_bt, len(bt), s, copy_stream.cuda_stream)
    assert ctx.poll_device_error(s) == 0
    torch.cuda.synchronize()
    rng = np.random.default_rng(77)
    rows = sample_rows(rng, T, [256 * i for i in range(1, T // 256)], range(B), range(T - B, T), 256)
    for i in range(l_h):
        res = check_layer(w, desc, gh.pool_bits(pools[i]), data[i][2], data[i][0], data[i][1], pos,
                          np.zeros(T, dtype=np.int64), bt[None, :], rows, rng)
        print(f"layer {model_layers[i]} (from hidden states): sampled {res[0]:.4f} x RMS", flush=True)
    want = np.full((num_pages, 2, B, w.n_kv_heads, w.head_dim), gh.SENTINEL, dtype=np.uint16)
    oracle.scatter_kv(want, kv_rows[:, :w.d_kv].reshape(T, w.n_kv_heads, w.head_dim),
                      kv_rows[:, w.d_kv:].reshape(T, w.n_kv_heads, w.head_dim), pos, bt, B)
    assert np.array_equal(gh.pool_bits(pools[2]), want)
    # and those bytes are what projecting the layer's hidden states gives
    res = check_layer(w, desc, gh.pool_bits(pools[2]), data[2][2], data[2][0], data[2][1], pos,
                      np.zeros(T, dtype=np.int64), bt[None, :], rows, rng)
    print(f"layer 31 (from KV rows): sampled {res[0]:.4f} x RMS", flush=True)
    ctx.destroy()
    hstore.destroy()
    kstore.destroy()
