"""Helpers for the GPU parity tests: device buffers via torch, calls through the C ABI
binding, comparison against the fp64 oracle.  (Test infrastructure; not product code.)"""
import numpy as np

import synthetic as syn
import oracle.hcache_oracle as oracle
import arith_model

SENTINEL = 0x7FC1          # bf16 NaN bit pattern pre-filled into every pool slot (never a result)
TOL = 2e-2                 # max |err| <= TOL * per-head RMS of the oracle (bf16 in, fp32 accumulate)


def torch_mod():
    import torch
    return torch


def to_dev_bf16(bits):
    torch = torch_mod()
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def to_dev_i32(a):
    torch = torch_mod()
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def new_pool(num_pages, block_size, n_kv_heads, head_dim):
    torch = torch_mod()
    t = torch.full((num_pages, 2, block_size, n_kv_heads, head_dim),
                   np.array(SENTINEL, dtype=np.uint16).view(np.int16).item(),
                   dtype=torch.int16, device="cuda")
    return t.view(torch.bfloat16)


def pool_bits(pool):
    torch = torch_mod()
    return pool.view(torch.int16).cpu().numpy().view(np.uint16)


def stream_handle():
    return torch_mod().cuda.current_stream().cuda_stream


def make_desc(hc, *, n_layers, d_model, n_q_heads, n_kv_heads, head_dim, block_size=16,
              max_position=4096, rope_style=0, rope_theta=10000.0, rms_eps=1e-5, norm_kind=0):
    return hc.ModelDesc(n_layers, d_model, n_q_heads, n_kv_heads, head_dim, block_size,
                        max_position, rope_style, rope_theta, rms_eps, norm_kind)


def desc_of_workload(hc, w, max_position=None, rope_style=0):
    if max_position is None:
        max_position = w.pos_offset + max(w.tokens, w.len_range[1]) + 1
    return make_desc(hc, n_layers=w.n_layers, d_model=w.d_model, n_q_heads=w.n_q_heads,
                     n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, block_size=w.block_size,
                     max_position=max_position, rope_style=rope_style, rope_theta=w.rope_theta,
                     rms_eps=w.rms_eps)


def oracle_kw(desc):
    # theta and eps as the float32 values the library received
    return dict(eps=float(np.float32(desc.rms_eps)), theta=float(np.float32(desc.rope_theta)),
                n_kv_heads=desc.n_kv_heads, head_dim=desc.head_dim, block_size=desc.block_size,
                rope_style=desc.rope_style, norm="layer" if desc.norm_kind == 1 else "rms")


def compare_pool(gpu_bits, ora_pool, tol=TOL):
    """gpu_bits: uint16 [P,2,B,H,hd]; ora_pool: float64, NaN where the oracle wrote nothing.
    Returns the worst error ratio (max |err| / (tol * RMS_head)); asserts indexing exactly."""
    written = ~np.isnan(ora_pool)
    assert np.array_equal(gpu_bits != SENTINEL, written), \
        "the set of cache elements written by the GPU differs from the oracle's"
    g = syn.bf16_bits_to_f64(gpu_bits)
    worst = 0.0
    H = ora_pool.shape[3]
    for kv in (0, 1):
        for h in range(H):
            m = written[:, kv, :, h, :]
            if not m.any():
                continue
            o = ora_pool[:, kv, :, h, :][m]
            gg = g[:, kv, :, h, :][m]
            assert np.all(np.isfinite(gg)), "non-finite value in restored KV"
            rms = np.sqrt(np.mean(o * o))
            err = np.max(np.abs(gg - o))
            worst = max(worst, err / (tol * rms))
    assert worst <= 1.0, f"max |err| = {worst * tol:.4g} x per-head RMS exceeds {tol}"
    return worst


def model_pool(desc, x, gamma, wkv, positions, block_table, num_pages):
    """Pool of bf16 bit patterns that the CPU model of the prescribed arithmetic (bf16 operands,
    exact sums, one output rounding; tests/arith_model.py) writes for one context; SENTINEL
    elsewhere.  RMSNorm layers only."""
    kw = oracle_kw(desc)
    k, v = arith_model.restore_rows(x, gamma, wkv, positions, eps=kw["eps"], theta=kw["theta"],
                                    n_kv_heads=desc.n_kv_heads, head_dim=desc.head_dim,
                                    rope_style=desc.rope_style)
    page, slot = oracle.page_slots(positions, block_table, desc.block_size)
    pool = np.full((num_pages, 2, desc.block_size, desc.n_kv_heads, desc.head_dim), SENTINEL, dtype=np.uint16)
    pool[page, 0, slot] = syn.f32_to_bf16_bits(k.astype(np.float32))
    pool[page, 1, slot] = syn.f32_to_bf16_bits(v.astype(np.float32))
    return pool


def assert_close_to_model(gpu_bits, model_bits, min_equal=0.98):
    """The GPU differs from the CPU model of its own arithmetic only by fp32 accumulation and
    the fp32 RoPE table (~1e-5 relative before the final rounding): every output is at most one
    bf16 step from the model's and nearly all are identical.  Far tighter than the tolerance
    against the unrounded oracle, and insensitive to where the outputs sit in their binades."""
    m = model_bits != SENTINEL
    assert np.array_equal(gpu_bits != SENTINEL, m)
    steps = arith_model.bf16_steps_apart(gpu_bits[m], model_bits[m])
    # near zero (|y| far below the head's RMS) one step is tiny and cancellation in the RoPE
    # sum can move a value by more than one; measure those in absolute terms instead
    far = steps > 1
    if far.any():
        g = syn.bf16_bits_to_f64(gpu_bits[m][far])
        e = syn.bf16_bits_to_f64(model_bits[m][far])
        scale = np.sqrt(np.mean(syn.bf16_bits_to_f64(model_bits[m]) ** 2))
        assert np.max(np.abs(g - e)) <= 1e-4 * scale, \
            f"{int(far.sum())} outputs more than one bf16 step from the arithmetic model"
    equal = float(np.mean(steps == 0))
    assert equal >= min_equal, f"only {equal:.4f} of the outputs equal the arithmetic model's"
    return equal


class LayerCase:
    """One layer's inputs on host (bf16 bits + fp64 decodes) for a given shape."""

    def __init__(self, rng, d_model, n_kv_heads, head_dim, n_tok, outliers=True):
        d_kv = n_kv_heads * head_dim
        self.wkv_bits = syn.f32_to_bf16_bits(rng.standard_normal((2 * d_kv, d_model), dtype=np.float32) * np.float32(0.02))
        self.gamma_bits = syn.f32_to_bf16_bits(1 + rng.standard_normal(d_model, dtype=np.float32) * np.float32(0.1))
        x = rng.standard_normal((n_tok, d_model), dtype=np.float32)
        if outliers and n_tok:
            ch = rng.choice(d_model, size=max(1, round(0.01 * d_model)), replace=False)
            x[:, ch] *= 20
        self.x_bits = syn.f32_to_bf16_bits(x)

    @property
    def wkv(self):
        return syn.bf16_bits_to_f64(self.wkv_bits)

    @property
    def gamma(self):
        return syn.bf16_bits_to_f64(self.gamma_bits)

    @property
    def x(self):
        return syn.bf16_bits_to_f64(self.x_bits)
