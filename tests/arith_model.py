"""CPU model of the arithmetic the restoration path is REQUIRED to use (bf16 operands, wide
accumulation, one bf16 rounding of the result) -- test infrastructure, built from the oracle's
functions and the bf16 helpers of `synthetic` only.

The fp64 oracle rounds nothing.  Any bf16 pipeline rounds at least twice: the operands of the
matrix product (here: the RMSNorm gain folded into the weights, one round-to-nearest-even
step; rounding the normalised activations instead is the same size of error) and the stored
result.  This module applies exactly those two roundings to the oracle's computation and
nothing else -- sums are fp64, so it is the *best* such a pipeline can do.  It serves two ends:

  * it says, for given inputs, how much of the 2e-2 x RMS_head budget the prescribed
    arithmetic itself uses (tests/test_tolerance_model.py), so that no GPU test has to narrow
    its inputs on an unproven claim;
  * the GPU result can be compared with it far more tightly than with the oracle: the only
    remaining differences are fp32 accumulation and the fp32 RoPE table (~1e-5 relative
    before the final rounding), i.e. a small fraction of outputs one bf16 step apart.
"""
import numpy as np

import synthetic as syn
import oracle.hcache_oracle as oracle


def round_bf16(a):
    """Nearest bf16 (ties to even) of fp64 values, returned as fp64."""
    return syn.bf16_bits_to_f64(syn.f32_to_bf16_bits(np.asarray(a, dtype=np.float64).astype(np.float32)))


def restore_rows(x, gamma, wkv, positions, *, eps, theta, n_kv_heads, head_dim, rope_style=0,
                 norm="rms", beta=None, bias=None, round_output=True):
    """(K, V) [T, H, hd] of the bf16 pipeline: gain folded into bf16 weights, exact sums,
    1/rms and RoPE in fp64, one rounding at the end (skipped when round_output is False)."""
    assert norm == "rms" and beta is None, "the model covers the RMSNorm path"
    gamma = np.asarray(gamma, dtype=np.float64)
    folded = round_bf16(np.asarray(wkv, dtype=np.float64) * gamma[None, :])
    k, v = oracle.project_kv(x, np.ones_like(gamma), folded, eps, n_kv_heads, head_dim, bias=bias)
    if rope_style != 2:
        k = oracle.apply_rope(k, positions, theta, rope_style)
    if round_output:
        k, v = round_bf16(k), round_bf16(v)
    return k, v


def error_ratio(ref, got):
    """max |got - ref| / RMS_head(ref), per head; ref, got [T, H, hd]."""
    rms = np.sqrt(np.mean(ref * ref, axis=(0, 2)))
    return np.max(np.abs(got - ref), axis=(0, 2)) / rms


def worst_ratio(x, gamma, wkv, positions, **kw):
    """Worst error of the bf16 pipeline against the oracle, in units of RMS_head (K and V)."""
    okw = {k: v for k, v in kw.items() if k in ("norm", "beta", "bias")}
    k, v = oracle.project_kv(x, gamma, wkv, kw["eps"], kw["n_kv_heads"], kw["head_dim"], **okw)
    if kw.get("rope_style", 0) != 2:
        k = oracle.apply_rope(k, positions, kw["theta"], kw.get("rope_style", 0))
    km, vm = restore_rows(x, gamma, wkv, positions, **kw)
    return float(max(error_ratio(k, km).max(), error_ratio(v, vm).max()))


def bf16_steps_apart(bits_a, bits_b):
    """Distance in representable bf16 values between two uint16 bit patterns (finite values)."""
    def key(b):
        b = b.astype(np.int32)
        return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)
    return np.abs(key(np.asarray(bits_a)) - key(np.asarray(bits_b)))
