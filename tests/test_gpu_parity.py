"""GPU parity: the HIP restoration path, called through the C ABI, against the fp64 oracle
on the same seeded inputs.  Indexing (which page/slot is written) must match exactly;
values must agree within 2e-2 x the oracle's per-head RMS (bf16 inputs, fp32 accumulation,
one bf16 rounding of the output)."""
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


@pytest.fixture(scope="module")
def torch():
    import torch
    return torch


def run_single(hc, torch, case, desc, positions, block_table, num_pages, layer=0, split=None):
    ctx = hc.Context(desc)
    if split is not None:
        ctx.set_split(split)
    pool = gh.new_pool(num_pages, desc.block_size, desc.n_kv_heads, desc.head_dim)
    s = gh.stream_handle()
    d_w, d_g = gh.to_dev_bf16(case.wkv_bits), gh.to_dev_bf16(case.gamma_bits)
    ctx.set_layer_weights(layer, d_w, d_g, s)
    ctx.set_kv_pool(layer, pool, num_pages)
    d_x = gh.to_dev_bf16(case.x_bits) if len(case.x_bits) else None
    d_pos, d_bt = gh.to_dev_i32(positions), gh.to_dev_i32(block_table)
    ctx.restore_kv(layer, d_x, d_pos, len(positions), d_bt, len(block_table), s)
    flags = ctx.poll_device_error(s)
    bits = gh.pool_bits(pool)
    ctx.destroy()
    return bits, flags


def oracle_single(case, desc, positions, block_table, num_pages):
    pool = np.full((num_pages, 2, desc.block_size, desc.n_kv_heads, desc.head_dim), np.nan)
    oracle.restore_kv(pool, case.x, case.gamma, case.wkv, positions, block_table,
                      **gh.oracle_kw(desc))
    return pool


# ---------------------------------------------------------------------------------------
def test_tiny_workload_all_layers(hc, torch):
    """Workload 0 (2 layers, d=256, 4 KV heads of 64, T=128), every element."""
    w = syn.WORKLOADS[0]
    desc = gh.desc_of_workload(hc, w)
    ctx = hc.Context(desc)
    s = gh.stream_handle()
    bt, num_pages = syn.block_table(w, w.tokens)
    pos = np.arange(w.tokens, dtype=np.int32)
    d_pos, d_bt = gh.to_dev_i32(pos), gh.to_dev_i32(bt)
    keep = []
    for l in range(w.n_layers):
        wkv, gamma = syn.layer_weights(w, l)
        x = syn.layer_hidden(w, l)
        pool = gh.new_pool(num_pages, w.block_size, w.n_kv_heads, w.head_dim)
        d_w, d_g, d_x = gh.to_dev_bf16(wkv), gh.to_dev_bf16(gamma), gh.to_dev_bf16(x)
        keep += [d_w, d_g, d_x]
        ctx.set_layer_weights(l, d_w, d_g, s)
        ctx.set_kv_pool(l, pool, num_pages)
        ctx.restore_kv(l, d_x, d_pos, w.tokens, d_bt, len(bt), s)
        assert ctx.poll_device_error(s) == 0
        ora = np.full((num_pages, 2, w.block_size, w.n_kv_heads, w.head_dim), np.nan)
        oracle.restore_kv(ora, syn.bf16_bits_to_f64(x), syn.bf16_bits_to_f64(gamma),
                          syn.bf16_bits_to_f64(wkv), pos, bt, **gh.oracle_kw(desc))
        worst = gh.compare_pool(gh.pool_bits(pool), ora)
        print(f"layer {l}: worst err = {worst * gh.TOL:.3e} x RMS_head")
    ctx.destroy()


SHAPES = [
    # d_model, n_kv, hd, n_tok, style   (several token tiles + ragged tail; padded feature tiles)
    (1024, 6, 128, 600, 0),
    (512, 3, 64, 257, 0),      # d_kv = 192 -> part padded to 256 rows
    (512, 3, 64, 300, 1),      # interleaved RoPE
    (1024, 4, 128, 513, 1),
    (256, 1, 64, 1, 0),        # a single token, a single head
    (2048, 2, 128, 255, 0),
    (64, 1, 64, 70, 0),        # fewer d_model steps (2) than the weight ring is deep (4)
    (128, 2, 64, 300, 1),      # 4 steps: the ring is filled exactly once
    (192, 1, 64, 33, 0),
    # head dimensions other than 64 and 128: a tile's two pair groups are half a head (256) or
    # straddle heads (192), which the epilogue's write-out order has to follow
    (1024, 2, 256, 300, 0),
    (512, 2, 256, 100, 1),
    (1024, 2, 192, 280, 0),    # d_kv = 384: three pair groups per head, padded to 512 rows
    (512, 1, 192, 131, 1),
]


def shape_inputs(d_model, n_kv, hd, n_tok, style):
    """Seeded inputs of one SHAPES case (also read by the CPU feasibility test)."""
    rng = np.random.default_rng([11, d_model, n_kv, hd, n_tok, style])
    case = gh.LayerCase(rng, d_model, n_kv, hd, n_tok)
    B = 16
    offset = 1000                                   # starts mid-page: 1000 = 62*16 + 8
    n_blocks = (offset + n_tok + B - 1) // B
    num_pages = n_blocks + 7
    bt = rng.permutation(num_pages)[:n_blocks].astype(np.int32)
    # tokens in scrambled order: positions drive RoPE and the slot, not the row index
    pos = (offset + rng.permutation(n_tok)).astype(np.int32)
    return case, pos, bt, num_pages, offset


@pytest.mark.parametrize("d_model,n_kv,hd,n_tok,style", SHAPES)
def test_shapes_against_oracle(hc, torch, d_model, n_kv, hd, n_tok, style):
    case, pos, bt, num_pages, offset = shape_inputs(d_model, n_kv, hd, n_tok, style)
    desc = gh.make_desc(hc, n_layers=1, d_model=d_model, n_q_heads=n_kv * 2, n_kv_heads=n_kv,
                        head_dim=hd, block_size=16, max_position=offset + n_tok, rope_style=style,
                        rope_theta=500000.0)
    ora = oracle_single(case, desc, pos, bt, num_pages)
    model = gh.model_pool(desc, case.x, case.gamma, case.wkv, pos, bt, num_pages)
    # as the library launches it by default; then, where the shape allows it, with the d_model
    # loops of its tiles split (mode 2) and with every tile whole (mode 0)
    modes = [None] + ([2, 0] if hc.diag_split_plan(d_model, n_kv * hd, n_tok, 2)["split"] else [])
    for split in modes:
        bits, flags = run_single(hc, torch, case, desc, pos, bt, num_pages, split=split)
        assert flags == 0
        worst = gh.compare_pool(bits, ora)
        equal = gh.assert_close_to_model(bits, model)
        print(f"split mode {split}: worst err = {worst * gh.TOL:.3e} x RMS_head; {equal:.5f} of the outputs "
              f"equal the two-rounding arithmetic model")


SPLIT_SHAPES = [
    # d_model, n_kv, hd, n_tok, style, expected (token tiles computed whole, split tiles, workgroups per split tile)
    (2048, 2, 128, 700, 1, (0, 6, 4)),       # 2 x 3 tiles, every one split four ways
    (4096, 1, 64, 100, 0, (0, 1, 8)),        # one ragged tile, eight shares of 512 channels
]


@pytest.mark.parametrize("d_model,n_kv,hd,n_tok,style,expect", SPLIT_SHAPES)
def test_split_launch_against_oracle(hc, torch, d_model, n_kv, hd, n_tok, style, expect):
    """Launches that split the d_model loop of their tiles (split workgroups, then the finishing
    launch), every element against the oracle.  A launch with whole tiles and split tiles in
    one grid needs more than 256 tiles: tests/test_gpu_fullsize.py."""
    plan = hc.diag_split_plan(d_model, n_kv * hd, n_tok, 2)
    assert plan["split"] == 1 and (plan["nt_main"], plan["n_tail"], plan["n_split"]) == expect, plan
    case, pos, bt, num_pages, offset = shape_inputs(d_model, n_kv, hd, n_tok, style)
    desc = gh.make_desc(hc, n_layers=1, d_model=d_model, n_q_heads=n_kv * 2, n_kv_heads=n_kv,
                        head_dim=hd, block_size=16, max_position=offset + n_tok, rope_style=style,
                        rope_theta=500000.0)
    ora = oracle_single(case, desc, pos, bt, num_pages)
    for split in (2, 1, 0):
        bits, flags = run_single(hc, torch, case, desc, pos, bt, num_pages, split=split)
        assert flags == 0
        worst = gh.compare_pool(bits, ora)
        print(f"split={split}: worst err = {worst * gh.TOL:.3e} x RMS_head", flush=True)


def test_split_and_unsplit_launches_agree_on_random_shapes(hc, torch):
    """Twenty seeded shapes (odd numbers of feature tiles, padded K/V parts, ragged token tiles,
    one to twelve tiles split two to sixteen ways, all three RoPE styles): the split launch
    writes exactly the cache elements the unsplit launch writes, and every value within one
    bf16 step of it, or, for values that are small because their terms cancel, within 2^-9 of
    the RMS of all values (the two differ only in the order of fp32 additions).  The unsplit
    kernel is the one the other tests hold against the oracle at many shapes."""
    rng = np.random.default_rng(2024)
    done = 0
    while done < 20:
        d_model = int(rng.choice([1024, 2048, 4096, 8192]))
        hd = int(rng.choice([64, 128]))
        n_kv = int(rng.integers(1, 7))
        n_tok = int(rng.integers(1, 900))
        style = int(rng.integers(0, 3))
        plan = hc.diag_split_plan(d_model, n_kv * hd, n_tok, 2)
        if not plan["split"]:
            continue
        done += 1
        case = gh.LayerCase(rng, d_model, n_kv, hd, n_tok)
        B = 16
        offset = int(rng.integers(0, 64))
        n_blocks = (offset + n_tok + B - 1) // B
        num_pages = n_blocks + 3
        bt = rng.permutation(num_pages)[:n_blocks].astype(np.int32)
        pos = (offset + rng.permutation(n_tok)).astype(np.int32)
        desc = gh.make_desc(hc, n_layers=1, d_model=d_model, n_q_heads=n_kv, n_kv_heads=n_kv, head_dim=hd,
                            block_size=B, max_position=offset + n_tok, rope_style=style)
        got = []
        for split in (2, 0):
            bits, flags = run_single(hc, torch, case, desc, pos, bt, num_pages, split=split)
            assert flags == 0
            got.append(bits)
        a, b = got
        assert np.array_equal(a != gh.SENTINEL, b != gh.SENTINEL), (d_model, n_kv, hd, n_tok, style)
        m = a != gh.SENTINEL
        assert m.sum() == 2 * n_tok * n_kv * hd
        fa, fb = syn.bf16_bits_to_f64(a[m]), syn.bf16_bits_to_f64(b[m])
        step = np.maximum(np.abs(fa), np.abs(fb)) * 2.0 ** -7          # one bf16 step at the larger magnitude
        bad = np.abs(fa - fb) > np.maximum(step, np.sqrt(np.mean(fb * fb)) * 2.0 ** -9)
        assert not bad.any(), (d_model, n_kv, hd, n_tok, style, int(bad.sum()))
        print(f"d_model {d_model} heads {n_kv} x {hd} tokens {n_tok} style {style}: {plan['n_tail']} tiles x "
              f"{plan['n_split']}; {np.mean(a[m] == b[m]):.4f} of the values bit-identical", flush=True)


def test_block_sizes(hc, torch):
    for B in (8, 32):
        rng = np.random.default_rng([5, B])
        case = gh.LayerCase(rng, 512, 2, 128, 100)
        n_blocks = (100 + B - 1) // B
        bt = rng.permutation(n_blocks + 3)[:n_blocks].astype(np.int32)
        pos = np.arange(100, dtype=np.int32)
        desc = gh.make_desc(hc, n_layers=1, d_model=512, n_q_heads=2, n_kv_heads=2, head_dim=128,
                            block_size=B, max_position=128)
        bits, flags = run_single(hc, torch, case, desc, pos, bt, n_blocks + 3)
        assert flags == 0
        gh.compare_pool(bits, oracle_single(case, desc, pos, bt, n_blocks + 3))


def test_ragged_batch(hc, torch):
    rng = np.random.default_rng(17)
    d_model, n_kv, hd, B = 512, 2, 128, 16
    lens = np.array([37, 260, 1, 129, 300], dtype=np.int32)     # crosses token tiles mid-context
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(cu[-1])
    case = gh.LayerCase(rng, d_model, n_kv, hd, T)
    pos = np.concatenate([np.arange(n) for n in lens]).astype(np.int32)
    nblk = (lens + B - 1) // B
    num_pages = int(nblk.sum()) + 9
    perm = rng.permutation(num_pages).astype(np.int32)
    tables = np.full((len(lens), int(nblk.max())), -1, dtype=np.int32)
    at = 0
    for s, n in enumerate(nblk):
        tables[s, :n] = perm[at:at + n]
        at += n
    desc = gh.make_desc(hc, n_layers=1, d_model=d_model, n_q_heads=n_kv, n_kv_heads=n_kv,
                        head_dim=hd, block_size=B, max_position=512)
    ctx = hc.Context(desc)
    s = gh.stream_handle()
    pool = gh.new_pool(num_pages, B, n_kv, hd)
    d_w, d_g, d_x = gh.to_dev_bf16(case.wkv_bits), gh.to_dev_bf16(case.gamma_bits), gh.to_dev_bf16(case.x_bits)
    ctx.set_layer_weights(0, d_w, d_g, s)
    ctx.set_kv_pool(0, pool, num_pages)
    d_pos, d_cu, d_tab = gh.to_dev_i32(pos), gh.to_dev_i32(cu), gh.to_dev_i32(tables)
    ctx.restore_kv_ragged(0, d_x, d_pos, T, d_cu, len(lens), d_tab, tables.shape[1], s)
    assert ctx.poll_device_error(s) == 0
    ora = np.full((num_pages, 2, B, n_kv, hd), np.nan)
    oracle.restore_kv_ragged(ora, case.x, case.gamma, case.wkv, pos, cu, tables, **gh.oracle_kw(desc))
    gh.compare_pool(gh.pool_bits(pool), ora)
    ctx.destroy()


def test_ragged_batch_split_launch_with_bad_rows(hc, torch):
    """The ragged batch at d_model 2048 with the d_model loops split four ways (mode 2), so that
    the per-token lookups (context by row offset, page by block table) run in the workgroups of
    the finishing launch; one context's table has an unmapped block and one position lies past
    the table: those rows are skipped and flagged, the rest matches the oracle.  Then unsplit."""
    rng = np.random.default_rng(29)
    d_model, n_kv, hd, B = 2048, 2, 128, 16
    lens = np.array([37, 260, 1, 129, 300], dtype=np.int32)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(cu[-1])
    assert hc.diag_split_plan(d_model, n_kv * hd, T, 2)["n_split"] == 4
    case = gh.LayerCase(rng, d_model, n_kv, hd, T)
    pos = np.concatenate([rng.permutation(n) for n in lens]).astype(np.int32)
    nblk = (lens + B - 1) // B
    num_pages = int(nblk.sum()) + 9
    perm = rng.permutation(num_pages).astype(np.int32)
    tables = np.full((len(lens), int(nblk.max())), -1, dtype=np.int32)
    at = 0
    for i, n in enumerate(nblk):
        tables[i, :n] = perm[at:at + n]
        at += n
    tables[1, 3] = -1                                 # context 1: positions 48..63 unmapped
    pos[cu[4] + 7] = 400                              # context 4: block 25 is past its table
    desc = gh.make_desc(hc, n_layers=1, d_model=d_model, n_q_heads=n_kv, n_kv_heads=n_kv,
                        head_dim=hd, block_size=B, max_position=512)
    good = np.ones(T, dtype=bool)
    for i in range(len(lens)):
        for t in range(cu[i], cu[i + 1]):
            blk = pos[t] // B
            good[t] = blk < tables.shape[1] and tables[i, blk] >= 0
    assert (~good).sum() == 17
    ora = np.full((num_pages, 2, B, n_kv, hd), np.nan)
    seq_of = np.repeat(np.arange(len(lens)), lens)
    keep = np.nonzero(good)[0]
    cu_good = np.concatenate([[0], np.cumsum([good[cu[i]:cu[i + 1]].sum() for i in range(len(lens))])]).astype(np.int32)
    oracle.restore_kv_ragged(ora, case.x[keep], case.gamma, case.wkv, pos[keep], cu_good, tables, **gh.oracle_kw(desc))
    ctx = hc.Context(desc)
    s = gh.stream_handle()
    d_w, d_g, d_x = gh.to_dev_bf16(case.wkv_bits), gh.to_dev_bf16(case.gamma_bits), gh.to_dev_bf16(case.x_bits)
    ctx.set_layer_weights(0, d_w, d_g, s)
    d_pos, d_cu, d_tab = gh.to_dev_i32(pos), gh.to_dev_i32(cu), gh.to_dev_i32(tables)
    for split in (2, 0):
        ctx.set_split(split)
        pool = gh.new_pool(num_pages, B, n_kv, hd)
        ctx.set_kv_pool(0, pool, num_pages)
        ctx.restore_kv_ragged(0, d_x, d_pos, T, d_cu, len(lens), d_tab, tables.shape[1], s)
        assert ctx.poll_device_error(s) == (hc.HC_DEV_BAD_POSITION | hc.HC_DEV_BAD_PAGE)
        gh.compare_pool(gh.pool_bits(pool), ora)
    ctx.destroy()


def test_bad_rows_are_skipped_and_flagged(hc, torch):
    rng = np.random.default_rng(23)
    d_model, n_kv, hd, B, T = 256, 1, 64, 16, 40
    case = gh.LayerCase(rng, d_model, n_kv, hd, T)
    bt = np.array([3, -1, 1, 9], dtype=np.int32)     # block 1 unmapped, block 3 -> page outside pool
    num_pages = 5
    pos = np.arange(T, dtype=np.int32)               # 0..39 : blocks 0,1,2
    pos[5] = 70                                      # beyond the block table (block 4)
    pos[6] = -3
    pos[7] = 48                                      # block 3 -> page 9 >= num_pages
    desc = gh.make_desc(hc, n_layers=1, d_model=d_model, n_q_heads=1, n_kv_heads=1, head_dim=hd,
                        block_size=B, max_position=128)
    bits, flags = run_single(hc, torch, case, desc, pos, bt, num_pages)
    assert flags == (hc.HC_DEV_BAD_POSITION | hc.HC_DEV_BAD_PAGE)
    good = np.array([p >= 0 and p // B < 4 and 0 <= bt[p // B] < num_pages for p in pos])
    ora = np.full((num_pages, 2, B, n_kv, hd), np.nan)
    oracle.restore_kv(ora, case.x[good], case.gamma, case.wkv, pos[good], bt, **gh.oracle_kw(desc))
    gh.compare_pool(bits, ora)
    # position >= max_position is refused even when the table would cover it
    desc2 = gh.make_desc(hc, n_layers=1, d_model=d_model, n_q_heads=1, n_kv_heads=1, head_dim=hd,
                         block_size=B, max_position=16)
    bits, flags = run_single(hc, torch, case, desc2, np.arange(T, dtype=np.int32),
                             np.array([0, 1, 2], dtype=np.int32), num_pages)
    assert flags == hc.HC_DEV_BAD_POSITION
    assert np.all(bits[1:] == gh.SENTINEL) and np.all(bits[0] != gh.SENTINEL)


def test_host_side_errors(hc, torch):
    desc = gh.make_desc(hc, n_layers=2, d_model=256, n_q_heads=1, n_kv_heads=1, head_dim=64)
    ctx = hc.Context(desc)
    s = gh.stream_handle()
    x = torch.zeros(64, 256, dtype=torch.bfloat16, device="cuda")
    pos = torch.zeros(64, dtype=torch.int32, device="cuda")
    bt = torch.zeros(8, dtype=torch.int32, device="cuda")

    def status(fn, *a):
        with pytest.raises(hc.HCacheError) as e:
            fn(*a)
        return e.value.status

    assert status(ctx.restore_kv, 5, x, pos, 64, bt, 8, s) == hc.HC_ERANGE
    assert status(ctx.restore_kv, 0, x, pos, 64, bt, 8, s) == hc.HC_ESTATE      # no weights yet
    w = torch.zeros(128, 256, dtype=torch.bfloat16, device="cuda")
    g = torch.ones(256, dtype=torch.bfloat16, device="cuda")
    ctx.set_layer_weights(0, w, g, s)
    assert status(ctx.restore_kv, 0, x, pos, 64, bt, 8, s) == hc.HC_ESTATE      # no pool yet
    pool = gh.new_pool(4, 16, 1, 64)
    ctx.set_kv_pool(0, pool, 4)
    assert status(ctx.restore_kv, 0, None, pos, 64, bt, 8, s) == hc.HC_EINVAL
    assert status(ctx.restore_kv, 0, x.data_ptr() + 2, pos, 63, bt, 8, s) == hc.HC_EALIGN
    assert status(ctx.restore_kv, 0, x, pos, -1, bt, 8, s) == hc.HC_EINVAL
    assert status(ctx.set_kv_pool, 0, pool, 0) == hc.HC_ERANGE
    assert status(ctx.set_layer_weights, 0, None, g, s) == hc.HC_EINVAL
    ctx.restore_kv(0, x, pos, 0, bt, 8, s)                                      # empty: no-op
    assert ctx.poll_device_error(s) == 0
    assert np.all(gh.pool_bits(pool) == gh.SENTINEL)
    ctx.destroy()


@pytest.mark.parametrize("pinned,loader,d_model", [(True, 0, 512), (True, 1, 512), (False, 0, 512), (True, 0, 2048)],
                         ids=["copy-engines", "gather-kernel", "pageable-store", "split-launches"])
def test_restore_context_from_store(hc, torch, pinned, loader, d_model):
    """Whole-context pipelined restore from the chunk store: all layers, a token range that
    starts and ends inside chunks, positions offset so the first page is part filled; with
    the gather-kernel loader, the hipMemcpyAsync loader, and a store in pageable memory.  At
    d_model 2048 every layer's launch is a split launch (six tiles, four shares each, then the
    finishing launch), so the loader's events interleave with two kernels per layer that
    share the context's workspace."""
    rng = np.random.default_rng(31)
    L, n_kv, hd, B, CT = 5, 2, 128, 16, 64
    assert hc.diag_split_plan(d_model, n_kv * hd, 650)["n_split"] == (4 if d_model == 2048 else 1)
    T_stored, tok_begin, n_tok, pos_offset = 700, 30, 650, 1000
    desc = gh.make_desc(hc, n_layers=L, d_model=d_model, n_q_heads=n_kv, n_kv_heads=n_kv,
                        head_dim=hd, block_size=B, max_position=pos_offset + T_stored)
    cases = [gh.LayerCase(np.random.default_rng([31, l]), d_model, n_kv, hd, T_stored) for l in range(L)]
    store = hc.Store(L, d_model, CT, capacity_chunks=L * ((T_stored + CT - 1) // CT) + 2, pinned=pinned)
    # save order: a 512-token prefill, then smaller appends, layer by layer each time
    cuts = [0, 512, 600, 601, 700]
    for a, b in zip(cuts[:-1], cuts[1:]):
        for l in range(L):
            store.append(3, l, np.ascontiguousarray(cases[l].x_bits[a:b]), b - a)
    n_blocks = (pos_offset + T_stored + B - 1) // B
    num_pages = n_blocks + 5
    bt = rng.permutation(num_pages)[:n_blocks].astype(np.int32)
    ctx = hc.Context(desc)
    s = gh.stream_handle()
    copy_stream = torch.cuda.Stream()
    pools, keep = [], []
    for l in range(L):
        d_w, d_g = gh.to_dev_bf16(cases[l].wkv_bits), gh.to_dev_bf16(cases[l].gamma_bits)
        keep += [d_w, d_g]
        ctx.set_layer_weights(l, d_w, d_g, s)
        pools.append(gh.new_pool(num_pages, B, n_kv, hd))
        ctx.set_kv_pool(l, pools[l], num_pages)
    d_bt = gh.to_dev_i32(bt)
    ctx.set_loader(loader)
    torch.cuda.synchronize()
    for rep in range(2):                                # second call reuses the staging buffers
        ctx.restore_context(store, 3, tok_begin, n_tok, pos_offset, d_bt, n_blocks, s,
                            copy_stream.cuda_stream)
    assert ctx.poll_device_error(s) == 0
    torch.cuda.synchronize()
    pos = (pos_offset + tok_begin + np.arange(n_tok)).astype(np.int32)
    for l in range(L):
        ora = np.full((num_pages, 2, B, n_kv, hd), np.nan)
        c = cases[l]
        oracle.restore_kv(ora, c.x[tok_begin:tok_begin + n_tok], c.gamma, c.wkv, pos, bt,
                          **gh.oracle_kw(desc))
        gh.compare_pool(gh.pool_bits(pools[l]), ora)
    # errors
    with pytest.raises(hc.HCacheError) as e:
        ctx.restore_context(store, 3, 100, 700, 0, d_bt, n_blocks, s, copy_stream.cuda_stream)
    assert e.value.status == hc.HC_ERANGE
    with pytest.raises(hc.HCacheError) as e:
        ctx.restore_context(store, 3, 0, 10, 0, d_bt, n_blocks, s, s)
    assert e.value.status == hc.HC_EINVAL
    ctx.destroy()
    store.destroy()


SEVERAL_LENGTHS = np.array([200, 0, 1, 333, 64], dtype=np.int32)
SEVERAL_STORED = SEVERAL_LENGTHS + np.array([10, 5, 0, 0, 7])     # the store may hold more than is restored


def several_contexts_cases(seed=69, L=3, d_model=512, n_kv=2, hd=128):
    """cases[context][layer]; the seed is one for which the prescribed bf16 arithmetic itself
    stays inside the tolerance at this narrow width (tests/test_tolerance_model.py)."""
    return [[gh.LayerCase(np.random.default_rng([seed, i, l]), d_model, n_kv, hd, int(SEVERAL_STORED[i]))
             for l in range(L)] for i in range(len(SEVERAL_LENGTHS))]


def test_restore_several_contexts_from_store(hc, torch):
    """hc_restore_contexts: five stored contexts (one of them empty, one a single token) restored
    together, one ragged launch per layer, positions implied by the row offsets; against the
    oracle's ragged restore and against restoring each context on its own."""
    rng = np.random.default_rng(63)
    L, d_model, n_kv, hd, B, CT = 3, 512, 2, 128, 16, 64
    lengths, stored = SEVERAL_LENGTHS, SEVERAL_STORED
    ids = np.array([11, 5, 42, 7, 1000], dtype=np.int64)
    desc = gh.make_desc(hc, n_layers=L, d_model=d_model, n_q_heads=n_kv, n_kv_heads=n_kv, head_dim=hd,
                        block_size=B, max_position=512)
    cases = several_contexts_cases()
    store = hc.Store(L, d_model, CT, capacity_chunks=int(sum(-(-int(n) // CT) for n in stored)) * L + 4)
    # interleaved arrival: contexts take turns, 50 tokens at a time, layer by layer
    done = np.zeros(len(ids), dtype=int)
    while np.any(done < stored):
        for i in range(len(ids)):
            n = int(min(50, stored[i] - done[i]))
            if n > 0:
                for l in range(L):
                    store.append(int(ids[i]), l, np.ascontiguousarray(cases[i][l].x_bits[done[i]:done[i] + n]), n)
                done[i] += n
    max_blocks = 24
    num_pages = len(ids) * max_blocks + 3
    perm = rng.permutation(num_pages).astype(np.int32)
    tables = np.full((len(ids), max_blocks), -1, dtype=np.int32)
    at = 0
    for i, n in enumerate(lengths):
        nb = (int(n) + B - 1) // B
        tables[i, :nb] = perm[at:at + nb]
        at += nb
    ctx = hc.Context(desc)
    s = gh.stream_handle()
    copy_stream = torch.cuda.Stream()
    keep, pools = [], []
    # all contexts of a layer share the layer's weights: take context 0's
    for l in range(L):
        d_w, d_g = gh.to_dev_bf16(cases[0][l].wkv_bits), gh.to_dev_bf16(cases[0][l].gamma_bits)
        keep += [d_w, d_g]
        ctx.set_layer_weights(l, d_w, d_g, s)
        pools.append(gh.new_pool(num_pages, B, n_kv, hd))
        ctx.set_kv_pool(l, pools[l], num_pages)
    d_tables = gh.to_dev_i32(tables)
    for rep in range(2):
        ctx.restore_contexts(store, ids, lengths, d_tables, max_blocks, s, copy_stream.cuda_stream)
    assert ctx.poll_device_error(s) == 0
    torch.cuda.synchronize()
    cu = np.concatenate([[0], np.cumsum(lengths)])
    pos = np.concatenate([np.arange(n) for n in lengths]).astype(np.int32)
    for l in range(L):
        x = np.concatenate([cases[i][l].x[:lengths[i]] for i in range(len(ids))])
        ora = np.full((num_pages, 2, B, n_kv, hd), np.nan)
        oracle.restore_kv_ragged(ora, x, cases[0][l].gamma, cases[0][l].wkv, pos, cu, tables,
                                 **gh.oracle_kw(desc))
        gh.compare_pool(gh.pool_bits(pools[l]), ora)
    # bit for bit what restoring each context alone writes
    alone = [gh.new_pool(num_pages, B, n_kv, hd) for _ in range(L)]
    for l in range(L):
        ctx.set_kv_pool(l, alone[l], num_pages)
    for i, n in enumerate(lengths):
        if n:
            ctx.restore_context(store, int(ids[i]), 0, int(n), 0, gh.to_dev_i32(tables[i]), max_blocks, s,
                                copy_stream.cuda_stream)
    torch.cuda.synchronize()
    for l in range(L):
        assert np.array_equal(gh.pool_bits(alone[l]), gh.pool_bits(pools[l]))
    # errors
    def status(*a):
        with pytest.raises(hc.HCacheError) as e:
            ctx.restore_contexts(*a)
        return e.value.status
    cs = copy_stream.cuda_stream
    assert status(store, [11, 99], [10, 10], d_tables, max_blocks, s, cs) == hc.HC_ERANGE     # unknown context
    assert status(store, [11], [500], d_tables, max_blocks, s, cs) == hc.HC_ERANGE             # more than stored
    assert status(store, [11], [-1], d_tables, max_blocks, s, cs) == hc.HC_EINVAL
    assert status(store, [11], [10], d_tables, max_blocks, s, s) == hc.HC_EINVAL
    ctx.restore_contexts(store, [], [], d_tables, max_blocks, s, cs)                           # nothing to do
    ctx.destroy()
    store.destroy()
