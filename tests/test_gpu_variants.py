"""GPU parity of the layer-style variants of the restoration kernel against the fp64 oracle:
LayerNorm with shift, projection biases and no rotation (OPT-style, the paper's third test
model), and their combinations with RMSNorm and the two RoPE conventions."""
import numpy as np
import pytest

import synthetic as syn
import oracle.hcache_oracle as oracle
import gpu_harness as gh
from test_gpu_fullsize import check_layer, sample_rows

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hc():
    import paper_2410_05004_amd as m
    return m


def bf16(rng, shape, mean, std):
    return syn.f32_to_bf16_bits((mean + std * rng.standard_normal(shape)).astype(np.float32))


VARIANTS = [
    # norm_kind, rope_style, shift, bias
    (1, 2, True, True),        # OPT
    (1, 2, False, False),      # LayerNorm alone
    (1, 0, True, True),        # LayerNorm + rotary (GPT-NeoX-like)
    (1, 1, False, True),
    (0, 0, False, True),       # RMSNorm + K/V bias (Qwen-like)
    (0, 1, False, True),
    (0, 2, False, False),      # RMSNorm, no rotation
    (0, 2, False, True),
]


@pytest.mark.parametrize("norm_kind,rope_style,shift,with_bias", VARIANTS)
def test_variant_matches_oracle(hc, norm_kind, rope_style, shift, with_bias):
    """Every element of a 3-tile x 3-tile problem with ragged tails (d_kv = 640 pads the K and
    V parts), rows with a clearly non-zero mean, unsorted positions; once with each of the 15
    tiles' d_model loops split in two and finished by a second launch, once unsplit."""
    rng = np.random.default_rng([5, norm_kind, rope_style, shift, with_bias])
    d_model, n_kv, hd, B, T = 1024, 5, 128, 16, 600
    d_kv = n_kv * hd
    n_blocks = 64
    desc = gh.make_desc(hc, n_layers=1, d_model=d_model, n_q_heads=n_kv, n_kv_heads=n_kv, head_dim=hd,
                        block_size=B, max_position=n_blocks * B, rope_style=rope_style,
                        norm_kind=norm_kind)
    wkv = bf16(rng, (2 * d_kv, d_model), 0.0, 0.02)
    gamma = bf16(rng, (d_model,), 1.0, 0.1)
    beta = bf16(rng, (d_model,), 0.0, 0.05) if shift else None
    bias = bf16(rng, (2 * d_kv,), 0.0, 0.05) if with_bias else None
    x = bf16(rng, (T, d_model), 0.4, 1.0)
    pos = rng.permutation(n_blocks * B)[:T].astype(np.int32)
    num_pages = n_blocks + 9
    bt = rng.permutation(num_pages)[:n_blocks].astype(np.int32)
    assert hc.diag_split_plan(d_model, d_kv, T, 2)["n_split"] == 2
    ctx = hc.Context(desc)
    s = gh.stream_handle()
    dev = [gh.to_dev_bf16(a) if a is not None else None for a in (wkv, gamma, beta, bias)]
    if shift or with_bias or norm_kind == 1:
        ctx.set_layer_weights_affine(0, dev[0], dev[1], dev[2], dev[3], s)
    else:
        ctx.set_layer_weights(0, dev[0], dev[1], s)
    ora = np.full((num_pages, 2, B, n_kv, hd), np.nan)
    f = syn.bf16_bits_to_f64
    oracle.restore_kv(ora, f(x), f(gamma), f(wkv), pos, bt,
                      beta=None if beta is None else f(beta), bias=None if bias is None else f(bias),
                      **gh.oracle_kw(desc))
    for split in (2, 0):
        ctx.set_split(split)
        pool = gh.new_pool(num_pages, B, n_kv, hd)
        ctx.set_kv_pool(0, pool, num_pages)
        ctx.restore_kv(0, gh.to_dev_bf16(x), gh.to_dev_i32(pos), T, gh.to_dev_i32(bt), n_blocks, s)
        assert ctx.poll_device_error(s) == 0
        worst = gh.compare_pool(gh.pool_bits(pool), ora)
        print(f"variant norm={norm_kind} rope={rope_style} shift={shift} bias={with_bias} split={split}: "
              f"worst error {worst * gh.TOL:.4f} x RMS", flush=True)
    ctx.destroy()


def test_affine_argument_errors(hc):
    desc = gh.make_desc(hc, n_layers=1, d_model=256, n_q_heads=2, n_kv_heads=2, head_dim=64)
    ctx = hc.Context(desc)
    s = gh.stream_handle()
    rng = np.random.default_rng(3)
    w, g = gh.to_dev_bf16(bf16(rng, (256, 256), 0, 0.02)), gh.to_dev_bf16(bf16(rng, (256,), 1, 0.1))
    b = gh.to_dev_bf16(bf16(rng, (256,), 0, 0.1))
    with pytest.raises(hc.HCacheError) as e:               # a shift under RMSNorm
        ctx.set_layer_weights_affine(0, w, g, b, None, s)
    assert e.value.status == hc.HC_EINVAL
    ctx.set_layer_weights_affine(0, w, g, None, b, s)      # bias, then back to plain weights
    ctx.set_layer_weights(0, w, g, s)
    ctx.destroy()
    for bad in (dict(rope_style=3), dict(norm_kind=2), dict(norm_kind=-1)):
        with pytest.raises(hc.HCacheError) as e:
            hc.validate_desc(gh.make_desc(hc, n_layers=1, d_model=256, n_q_heads=2, n_kv_heads=2,
                                          head_dim=64, **bad))
        assert e.value.status == hc.HC_EINVAL


def test_opt30b_shape(hc):
    """The OPT-30B shape at full width (d_model 7168, 56 heads, 2048 tokens), first and last
    layer: whole-pool indexing, sampled rows element by element, random projection over all
    tokens."""
    import torch
    w = syn.WORKLOADS[5]
    T, B = w.tokens, w.block_size
    layers = (0, w.n_layers - 1)
    desc = gh.make_desc(hc, n_layers=len(layers), d_model=w.d_model, n_q_heads=w.n_q_heads,
                        n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, block_size=B,
                        max_position=T, rope_style=w.rope_style, rms_eps=w.rms_eps, norm_kind=1)
    ctx = hc.Context(desc)
    s = gh.stream_handle()
    bt, num_pages = syn.block_table(w, T)
    d_bt = gh.to_dev_i32(bt)
    pos = np.arange(T, dtype=np.int32)
    d_pos = gh.to_dev_i32(pos)
    rng = np.random.default_rng(55)
    rows = sample_rows(rng, T, [256 * i for i in range(1, T // 256)], range(B), range(T - B, T), 256)
    for i, l in enumerate(layers):
        wkv, gamma = syn.layer_weights(w, l)
        beta, bias = syn.layer_affine(w, l)
        x = syn.layer_hidden(w, l)
        ctx.set_layer_weights_affine(i, gh.to_dev_bf16(wkv), gh.to_dev_bf16(gamma),
                                     gh.to_dev_bf16(beta), gh.to_dev_bf16(bias), s)
        torch.cuda.synchronize()
        pool = gh.new_pool(num_pages, B, w.n_kv_heads, w.head_dim)
        ctx.set_kv_pool(i, pool, num_pages)
        ctx.restore_kv(i, gh.to_dev_bf16(x), d_pos, T, d_bt, len(bt), s)
        assert ctx.poll_device_error(s) == 0
        res = check_layer(w, desc, gh.pool_bits(pool), x, wkv, gamma, pos, np.zeros(T, dtype=np.int64),
                          bt[None, :], rows, rng, beta_bits=beta, bias_bits=bias)
        print(f"{w.name} layer {l}: sampled {res[0]:.4f} x RMS, projection {res[1]:.3f} / {res[2]:.3f} of limit",
              flush=True)
        del pool
    ctx.destroy()


@pytest.mark.parametrize("norm_kind", [0, 1])
def test_layers_in_one_launch(hc, norm_kind):
    """hc_restore_kv_layers over 35 layers (more than one launch holds; layers with and without
    a bias, so the kernel mode changes along the way) writes bit for bit what one
    hc_restore_kv per layer writes, and that is the oracle's result."""
    import torch
    rng = np.random.default_rng([9, norm_kind])
    L, d_model, n_kv, hd, B, T = 35, 256, 2, 64, 16, 300
    d_kv = n_kv * hd
    n_blocks = 24
    num_pages = n_blocks + 4
    desc = gh.make_desc(hc, n_layers=L, d_model=d_model, n_q_heads=n_kv, n_kv_heads=n_kv, head_dim=hd,
                        block_size=B, max_position=n_blocks * B, norm_kind=norm_kind)
    ctx = hc.Context(desc)
    s = gh.stream_handle()
    pos = rng.permutation(n_blocks * B)[:T].astype(np.int32)
    bt = rng.permutation(num_pages)[:n_blocks].astype(np.int32)
    d_pos, d_bt = gh.to_dev_i32(pos), gh.to_dev_i32(bt)
    f = syn.bf16_bits_to_f64
    hidden, pools_a, pools_b, params, keep = [], [], [], [], []
    for l in range(L):
        wkv, gamma = bf16(rng, (2 * d_kv, d_model), 0, 0.02), bf16(rng, (d_model,), 1, 0.1)
        bias = bf16(rng, (2 * d_kv,), 0, 0.05) if l % 5 in (1, 2) else None
        beta = bf16(rng, (d_model,), 0, 0.05) if norm_kind == 1 and l % 3 == 0 else None
        x = bf16(rng, (T, d_model), 0.3, 1.0)
        params.append((wkv, gamma, beta, bias, x))
        dev = [gh.to_dev_bf16(a) if a is not None else None for a in (wkv, gamma, beta, bias)]
        keep.append(dev)
        if beta is not None or bias is not None:
            ctx.set_layer_weights_affine(l, dev[0], dev[1], dev[2], dev[3], s)
        else:
            ctx.set_layer_weights(l, dev[0], dev[1], s)
        hidden.append(gh.to_dev_bf16(x))
        pools_a.append(gh.new_pool(num_pages, B, n_kv, hd))
        pools_b.append(gh.new_pool(num_pages, B, n_kv, hd))
    for l in range(L):
        ctx.set_kv_pool(l, pools_a[l], num_pages)
        ctx.restore_kv(l, hidden[l], d_pos, T, d_bt, n_blocks, s)
    for l in range(L):
        ctx.set_kv_pool(l, pools_b[l], num_pages)
    ctx.timing_begin()
    ctx.restore_kv_layers(0, hidden, d_pos, T, d_bt, n_blocks, s)
    _, launches = ctx.timing_end(s)
    assert ctx.poll_device_error(s) == 0
    # two tiles per layer: up to 32 layers go into one launch (short contexts fill the chip with layers)
    if norm_kind == 1:
        assert launches == 2                              # one mode: 32 + 3 layers
    else:
        assert launches > 2                               # the mode changes with the bias
    for l in (0, 1, 2, 3, 17, 31, 32, 34):
        a, b = gh.pool_bits(pools_a[l]), gh.pool_bits(pools_b[l])
        assert np.array_equal(a, b), f"layer {l}: fused launch differs from the single-layer launch"
        wkv, gamma, beta, bias, x = params[l]
        ora = np.full((num_pages, 2, B, n_kv, hd), np.nan)
        oracle.restore_kv(ora, f(x), f(gamma), f(wkv), pos, bt, beta=None if beta is None else f(beta),
                          bias=None if bias is None else f(bias), **gh.oracle_kw(desc))
        gh.compare_pool(b, ora)
    # a sub-range, and argument errors
    pools_c = [gh.new_pool(num_pages, B, n_kv, hd) for _ in range(3)]
    for i in range(3):
        ctx.set_kv_pool(10 + i, pools_c[i], num_pages)
    ctx.restore_kv_layers(10, hidden[10:13], d_pos, T, d_bt, n_blocks, s)
    for i in range(3):
        assert np.array_equal(gh.pool_bits(pools_c[i]), gh.pool_bits(pools_a[10 + i]))
    for args, st in [((30, hidden[:6], d_pos, T, d_bt, n_blocks, s), hc.HC_ERANGE),
                     ((-1, hidden[:2], d_pos, T, d_bt, n_blocks, s), hc.HC_ERANGE),
                     ((0, [hidden[0], None], d_pos, T, d_bt, n_blocks, s), hc.HC_EINVAL),
                     ((0, [hidden[0].data_ptr() + 2], d_pos, T, d_bt, n_blocks, s), hc.HC_EALIGN),
                     ((0, hidden[:2], None, T, d_bt, n_blocks, s), hc.HC_EINVAL)]:
        with pytest.raises(hc.HCacheError) as e:
            ctx.restore_kv_layers(*args)
        assert e.value.status == st
    ctx.restore_kv_layers(0, [], d_pos, T, d_bt, n_blocks, s)          # nothing to do
    torch.cuda.synchronize()
    ctx.destroy()


def test_opt_style_ragged_and_streamed(hc):
    """OPT-style layers through the other entry points: a ragged batch of four contexts in one
    launch, and a whole-context pipelined restore from the chunk store."""
    import torch
    rng = np.random.default_rng(21)
    L, d_model, n_kv, hd, B, CT = 2, 1024, 4, 128, 16, 64
    d_kv = n_kv * hd
    desc = gh.make_desc(hc, n_layers=L, d_model=d_model, n_q_heads=n_kv, n_kv_heads=n_kv, head_dim=hd,
                        block_size=B, max_position=1024, rope_style=2, norm_kind=1)
    ctx = hc.Context(desc)
    s = gh.stream_handle()
    f = syn.bf16_bits_to_f64
    params, keep = [], []
    for l in range(L):
        wkv, gamma = bf16(rng, (2 * d_kv, d_model), 0, 0.02), bf16(rng, (d_model,), 1, 0.1)
        beta, bias = bf16(rng, (d_model,), 0, 0.05), bf16(rng, (2 * d_kv,), 0, 0.05)
        params.append((wkv, gamma, beta, bias))
        dev = [gh.to_dev_bf16(a) for a in (wkv, gamma, beta, bias)]
        keep.append(dev)
        ctx.set_layer_weights_affine(l, *dev, s)
    # ragged: four contexts, one launch per layer
    lengths = np.array([130, 1, 257, 64])
    cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    T = int(cu[-1])
    max_blocks = 20
    num_pages = 4 * max_blocks + 5
    perm = rng.permutation(num_pages).astype(np.int32)
    tables = np.full((4, max_blocks), -1, dtype=np.int32)
    at = 0
    for i, n in enumerate(lengths):
        nb = (n + B - 1) // B
        tables[i, :nb] = perm[at:at + nb]
        at += nb
    pos = np.concatenate([np.arange(n, dtype=np.int32) for n in lengths])
    for l in range(L):
        x = bf16(rng, (T, d_model), 0.3, 1.0)
        pool = gh.new_pool(num_pages, B, n_kv, hd)
        ctx.set_kv_pool(l, pool, num_pages)
        ctx.restore_kv_ragged(l, gh.to_dev_bf16(x), gh.to_dev_i32(pos), T, gh.to_dev_i32(cu), 4,
                              gh.to_dev_i32(tables), max_blocks, s)
        assert ctx.poll_device_error(s) == 0
        wkv, gamma, beta, bias = params[l]
        ora = np.full((num_pages, 2, B, n_kv, hd), np.nan)
        oracle.restore_kv_ragged(ora, f(x), f(gamma), f(wkv), pos, cu, tables, beta=f(beta), bias=f(bias),
                                 **gh.oracle_kw(desc))
        gh.compare_pool(gh.pool_bits(pool), ora)
    # streamed: one context from the chunk store, positions offset into the first page
    T2, off = 300, 5
    xs = [bf16(rng, (T2, d_model), 0.3, 1.0) for _ in range(L)]
    store = hc.Store(L, d_model, CT, L * ((T2 + CT - 1) // CT) + 1)
    for a, b in ((0, 200), (200, 300)):
        for l in range(L):
            store.append(4, l, np.ascontiguousarray(xs[l][a:b]), b - a)
    n_blocks = (off + T2 + B - 1) // B
    bt = rng.permutation(n_blocks + 3)[:n_blocks].astype(np.int32)
    pools = []
    for l in range(L):
        pools.append(gh.new_pool(n_blocks + 3, B, n_kv, hd))
        ctx.set_kv_pool(l, pools[l], n_blocks + 3)
    copy_stream = torch.cuda.Stream()
    ctx.restore_context(store, 4, 0, T2, off, gh.to_dev_i32(bt), n_blocks, s, copy_stream.cuda_stream)
    assert ctx.poll_device_error(s) == 0
    torch.cuda.synchronize()
    pos2 = (off + np.arange(T2)).astype(np.int32)
    for l in range(L):
        wkv, gamma, beta, bias = params[l]
        ora = np.full((n_blocks + 3, 2, B, n_kv, hd), np.nan)
        oracle.restore_kv(ora, f(xs[l]), f(gamma), f(wkv), pos2, bt, beta=f(beta), bias=f(bias),
                          **gh.oracle_kw(desc))
        gh.compare_pool(gh.pool_bits(pools[l]), ora)
    ctx.destroy()
    store.destroy()
