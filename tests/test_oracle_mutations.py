"""Planted mistakes: each plausible slip in the oracle must trip at least one pin.

A fresh copy of the oracle module is loaded, one function is replaced by a subtly
wrong version, and the pin suite is run against the copy.  (All of this is CPU work
on the oracle; nothing here touches the HIP library.)
"""
import importlib.util
import os

import numpy as np
import pytest

import oracle_pins as pins

ORACLE_PATH = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))),
                           "oracle", "hcache_oracle.py")


def fresh_oracle():
    spec = importlib.util.spec_from_file_location("oracle_mutant", ORACLE_PATH)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def mut_eps_outside_sqrt(o):
    def rmsnorm(x, gamma, eps):
        x = np.asarray(x, dtype=np.float64)
        return x / (np.sqrt(np.mean(x * x, axis=-1, keepdims=True)) + eps) * gamma
    o.rmsnorm = rmsnorm


def mut_eps_dropped(o):
    real = o.rmsnorm
    o.rmsnorm = lambda x, gamma, eps: real(x, gamma, 0.0)


def mut_gamma_dropped(o):
    real = o.rmsnorm
    o.rmsnorm = lambda x, gamma, eps: real(x, np.ones_like(gamma), eps)


def mut_sum_instead_of_mean(o):
    def rmsnorm(x, gamma, eps):
        x = np.asarray(x, dtype=np.float64)
        return x / np.sqrt(np.sum(x * x, axis=-1, keepdims=True) + eps) * gamma
    o.rmsnorm = rmsnorm


def mut_rope_clockwise(o):
    real = o.apply_rope
    o.apply_rope = lambda y, p, theta, style=0: real(y, -np.asarray(p), theta, style)


def mut_rope_exponent(o):
    def rope_angles(positions, head_dim, theta):
        i = np.arange(head_dim // 2, dtype=np.float64)
        return np.asarray(positions, dtype=np.float64)[:, None] * np.power(theta, -i / head_dim)[None, :]
    o.rope_angles = rope_angles


def mut_rope_styles_swapped(o):
    real = o.apply_rope
    o.apply_rope = lambda y, p, theta, style=0: real(y, p, theta, 1 - style)


def mut_rope_on_v_too(o):
    real = o.restore_kv

    def restore_kv(pool, x, gamma, wkv, positions, block_table, **kw):
        page, slot = real(pool, x, gamma, wkv, positions, block_table, **kw)
        v = pool[page, 1, slot]
        pool[page, 1, slot] = o.apply_rope(v, positions, kw["theta"], kw.get("rope_style", 0))
        return page, slot
    o.restore_kv = restore_kv


def mut_kv_swapped(o):
    real = o.project_kv

    def project_kv(*a, **k):
        kk, vv = real(*a, **k)
        return vv, kk
    o.project_kv = project_kv


def mut_weight_not_transposed_heads(o):
    # heads laid out feature-major instead of head-major
    real = o.project_kv

    def project_kv(x, gamma, wkv, eps, H, hd):
        k, v = real(x, gamma, wkv, eps, H, hd)
        T = k.shape[0]
        return (k.reshape(T, hd, H).transpose(0, 2, 1).copy(),
                v.reshape(T, hd, H).transpose(0, 2, 1).copy())
    o.project_kv = project_kv


def mut_page_slot_swapped(o):
    def page_slots(positions, block_table, block_size):
        positions = np.asarray(positions, dtype=np.int64)
        block_table = np.asarray(block_table, dtype=np.int64)
        return block_table[positions % len(block_table)], (positions // len(block_table)) % block_size
    o.page_slots = page_slots


def mut_slot_off_by_one(o):
    real = o.page_slots

    def page_slots(positions, block_table, block_size):
        page, slot = real(positions, block_table, block_size)
        return page, (slot + 1) % block_size
    o.page_slots = page_slots


def mut_prefill_skips_norm(o):
    real = o.full_prefill

    def full_prefill(h0, layers, positions, **kw):
        rec = real(h0, layers, positions, **kw)
        return [(h * 1.0000001, k, v) for h, k, v in rec]
    o.full_prefill = full_prefill


def mut_store_row_major_across_layers(o):
    real = o.ChunkStore.chunk

    def chunk(self, seq, layer, c):
        return real(self, seq, (layer + 1) % self.n_layers if self.n_layers > 1 else layer, c)
    o.ChunkStore.chunk = chunk


def mut_save_rows_to_wrong_context(o):
    real = o.save_step
    o.save_step = lambda store, layer, rows, row_seq: real(store, layer, rows, list(row_seq)[::-1])


def mut_layernorm_uncentred_variance(o):
    def layernorm(x, gamma, beta, eps):
        x = np.asarray(x, dtype=np.float64)
        mu = np.mean(x, axis=-1, keepdims=True)
        return (x - mu) / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * gamma + beta
    o.layernorm = layernorm


def mut_layernorm_unbiased_variance(o):
    def layernorm(x, gamma, beta, eps):
        x = np.asarray(x, dtype=np.float64)
        xc = x - np.mean(x, axis=-1, keepdims=True)
        var = np.sum(xc * xc, axis=-1, keepdims=True) / (x.shape[-1] - 1)
        return xc / np.sqrt(var + eps) * gamma + beta
    o.layernorm = layernorm


def mut_layernorm_shift_before_gain(o):
    real = o.layernorm
    o.layernorm = lambda x, gamma, beta, eps: real(x, gamma, np.zeros_like(np.asarray(beta, dtype=float)), eps) + \
        np.asarray(beta) * np.asarray(gamma)


def mut_bias_dropped(o):
    real = o.project_kv
    o.project_kv = lambda *a, **kw: real(*a, **{**kw, "bias": None})


def mut_rotation_kept_without_rope(o):
    real = o.restore_kv
    o.restore_kv = lambda *a, **kw: real(*a, **{**kw, "rope_style": 0 if kw.get("rope_style") == 2 else kw.get("rope_style", 0)})


def mut_scatter_kv_swapped(o):
    real = o.scatter_kv
    o.scatter_kv = lambda pool, k, v, *a: real(pool, v, k, *a)


def mut_partition_floor(o):
    real = o.partition_layers

    def partition_layers(n, io_h, io_kv, c_h, c_token):
        l_h, l_o, comp = real(n, io_h, io_kv, c_h, c_token)
        x = n * io_kv / (io_kv + c_h - io_h) if c_h > io_h else n * c_token / (c_token + io_h - c_h)
        l_h = min(int(x), n)
        return l_h, n - l_h, comp
    o.partition_layers = partition_layers


def mut_partition_guarded_ceiling(o):
    # a tolerance subtracted before the ceiling: quotients a hair above an integer round down
    import math

    def partition_layers(n, io_h, io_kv, c_h, c_token):
        x = n * io_kv / (io_kv + c_h - io_h) if c_h > io_h else n * c_token / (c_token + io_h - c_h)
        l_h = min(max(math.ceil(x - 1e-9 * n), 0), n)
        return l_h, n - l_h, "kv" if c_h > io_h else "re"
    o.partition_layers = partition_layers


def mut_partition_wrong_branch(o):
    real = o.partition_layers
    o.partition_layers = lambda n, io_h, io_kv, c_h, c_token: real(n, c_h, io_kv, io_h, c_token)


def mut_flop_count(o):
    o.restore_flop = lambda n, d, dkv: 2 * n * d * dkv


MUTATIONS = [v for k, v in sorted(globals().items()) if k.startswith("mut_")]


@pytest.mark.parametrize("mutate", MUTATIONS, ids=lambda m: m.__name__)
def test_planted_mistake_is_caught(mutate):
    o = fresh_oracle()
    mutate(o)
    caught = []
    for check in pins.ALL_CHECKS:
        try:
            check(o)
        except Exception as e:  # any failure of a pin counts as "caught"
            caught.append(check.__name__)
    assert caught, f"{mutate.__name__} slipped through every pin"


def test_unmutated_copy_passes():
    o = fresh_oracle()
    for check in pins.ALL_CHECKS:
        check(o)
