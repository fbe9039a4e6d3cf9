"""Shapes and seeded tensors of the synthetic restoration workloads.

The first five workloads mirror the model shapes the paper evaluates (Llama-2-7B/13B,
Section 6 "Experimental Setup") and the context-length statistics it reports for
its traces (Section 2.3), plus a GQA and a 70B-shaped long-context case; the sixth has
the shape and layer style of OPT-30B, the paper's third test model.  All
tensors are random: the cost and the numerics of the restoration path depend on
shapes and value distributions only, not on trained weights.

Every tensor has its own random sub-stream keyed by (workload, tensor kind, layer),
so any layer can be generated alone and in any order.
"""
from dataclasses import dataclass
import numpy as np

from .bf16 import f32_to_bf16_bits

BASE_SEED = 20241005

# tensor-kind keys of the random sub-streams
_K_WKV, _K_GAMMA, _K_HIDDEN, _K_OUTLIER, _K_BLOCKS, _K_LENGTHS, _K_DENSE, _K_AFFINE = range(8)


@dataclass(frozen=True)
class Workload:
    index: int
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    rope_theta: float
    tokens: int                 # restored tokens (sum over contexts when ragged)
    pos_offset: int = 0         # absolute position of the first restored token
    chunk_tokens: int = 256     # tokens per chunk of the host store
    n_seq: int = 1              # independent contexts (ragged batch when > 1)
    len_range: tuple = (0, 0)   # inclusive length range of ragged contexts
    rms_eps: float = 1e-5
    block_size: int = 16
    d_ff: int = 0               # only the tiny workload runs a full forward pass
    norm: str = "rms"           # "rms" (Llama-style) or "layer" (OPT-style: shift and biases too)
    rope_style: int = 0         # 0 half-split, 1 interleaved, 2 none (learned absolute positions)
    hidden_mean: float = 0.0    # offset added to every hidden-state element

    @property
    def d_kv(self):
        return self.n_kv_heads * self.head_dim

    @property
    def n_out(self):            # fused K|V output width
        return 2 * self.d_kv

    @property
    def flop_per_token_layer(self):
        return 4 * self.d_model * self.d_kv


WORKLOADS = (
    Workload(0, "tiny-llama-2L-d256-T128", 2, 256, 4, 4, 64, 10000.0, 128,
             chunk_tokens=64, d_ff=704),
    Workload(1, "llama2-7b-T2048", 32, 4096, 32, 32, 128, 10000.0, 2048),
    Workload(2, "llama3-8b-gqa-T8192", 32, 4096, 32, 8, 128, 500000.0, 8192,
             chunk_tokens=256),
    Workload(3, "llama2-13b-ragged16", 40, 5120, 40, 40, 128, 10000.0, 0,
             n_seq=16, len_range=(512, 4096)),
    Workload(4, "70b-gqa-T32768", 80, 8192, 64, 8, 128, 500000.0, 32768,
             pos_offset=1000, chunk_tokens=512),
    # the paper's third test model (OPT-30B): LayerNorm, biases, no rotary embedding, MHA
    Workload(5, "opt30b-T2048", 48, 7168, 56, 56, 128, 10000.0, 2048,
             norm="layer", rope_style=2, hidden_mean=0.25),
)


def _rng(w, kind, layer=0, extra=0):
    return np.random.default_rng([BASE_SEED, w.index, kind, layer, extra])


def _normal_bf16(rng, shape, mean, std):
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    if mean != 0.0:
        x += np.float32(mean)
    return f32_to_bf16_bits(x)


def layer_weights(w, layer):
    """(W_kv, gamma) of one layer as bf16 bits.

    W_kv is [2*d_kv, d_model], nn.Linear layout; rows [0, d_kv) project to K and rows
    [d_kv, 2*d_kv) to V.  W ~ N(0, 0.02^2); gamma ~ 1 + N(0, 0.1^2).
    """
    wkv = _normal_bf16(_rng(w, _K_WKV, layer), (w.n_out, w.d_model), 0.0, 0.02)
    gamma = _normal_bf16(_rng(w, _K_GAMMA, layer), (w.d_model,), 1.0, 0.1)
    return wkv, gamma


def layer_affine(w, layer):
    """(beta [d_model], bias [2*d_kv]) of an OPT-style layer as bf16 bits: the LayerNorm shift
    ~ N(0, 0.05^2) and the K|V projection bias ~ N(0, 0.05^2)."""
    r = _rng(w, _K_AFFINE, layer)
    return _normal_bf16(r, (w.d_model,), 0.0, 0.05), _normal_bf16(r, (w.n_out,), 0.0, 0.05)


def outlier_channels(w, layer):
    """Sorted channel indices that carry the x20 outliers of this layer (1% of d_model)."""
    n = int(round(0.01 * w.d_model))
    return np.sort(_rng(w, _K_OUTLIER, layer).choice(w.d_model, size=n, replace=False))


def layer_hidden(w, layer, n_tokens=None, token_offset=0):
    """Saved hidden states of one layer, bf16 bits [n_tokens, d_model].

    N(0,1) with 1% of the channels (fixed per layer) scaled by 20, the pattern of
    LLM activation outliers.  `token_offset` selects a later slice of the same
    stream (rows are drawn in blocks of 256 tokens so slices are reproducible).
    """
    if n_tokens is None:
        n_tokens = w.tokens
    blk = 256
    first, last = token_offset // blk, (token_offset + n_tokens + blk - 1) // blk
    parts = []
    for b in range(first, last):
        parts.append(_rng(w, _K_HIDDEN, layer, b).standard_normal(
            size=(blk, w.d_model), dtype=np.float32))
    x = np.concatenate(parts, axis=0) if parts else np.zeros((0, w.d_model), np.float32)
    lo = token_offset - first * blk
    x = x[lo:lo + n_tokens]
    x[:, outlier_channels(w, layer)] *= np.float32(20.0)
    if w.hidden_mean != 0.0:
        x += np.float32(w.hidden_mean)
    return f32_to_bf16_bits(x)


def block_table(w, n_positions, seq=0, slack=1.25):
    """(block_table int32 [n_blocks], num_pages) for one context covering positions
    [0, n_positions): a seeded random permutation of a pool 25% larger than needed."""
    n_blocks = (n_positions + w.block_size - 1) // w.block_size
    num_pages = max(int(np.ceil(slack * n_blocks)), n_blocks + 1)
    perm = _rng(w, _K_BLOCKS, 0, seq).permutation(num_pages).astype(np.int32)
    return perm[:n_blocks].copy(), num_pages


def ragged_lengths(w):
    """Seeded context lengths of the ragged batch, int32 [n_seq], uniform in len_range."""
    lo, hi = w.len_range
    return _rng(w, _K_LENGTHS).integers(lo, hi, size=w.n_seq, endpoint=True).astype(np.int32)


def ragged_block_tables(w, lengths, slack=1.25):
    """(block_tables int32 [n_seq, max_blocks] padded with -1, num_pages) with disjoint
    page sets per context drawn from one shared pool."""
    lengths = np.asarray(lengths)
    nblk = (lengths + w.block_size - 1) // w.block_size
    total = int(nblk.sum())
    num_pages = max(int(np.ceil(slack * total)), total + 1)
    perm = _rng(w, _K_BLOCKS, 1).permutation(num_pages).astype(np.int32)
    max_blocks = int(nblk.max()) if len(nblk) else 0
    tables = np.full((len(lengths), max_blocks), -1, dtype=np.int32)
    at = 0
    for s, n in enumerate(nblk):
        tables[s, :n] = perm[at:at + n]
        at += n
    return tables, num_pages


def dense_model_weights(w, layer):
    """Remaining weights of a full transformer layer (tiny workload only), bf16 bits:
    Wq [Hq*hd, d], Wo [d, Hq*hd], W_gate/W_up [d_ff, d], W_down [d, d_ff], gamma2 [d]."""
    assert w.d_ff > 0, "only the tiny workload runs a full forward pass"
    r = _rng(w, _K_DENSE, layer)
    dq = w.n_q_heads * w.head_dim
    return {
        "wq": _normal_bf16(r, (dq, w.d_model), 0.0, 0.02),
        "wo": _normal_bf16(r, (w.d_model, dq), 0.0, 0.02),
        "w_gate": _normal_bf16(r, (w.d_ff, w.d_model), 0.0, 0.02),
        "w_up": _normal_bf16(r, (w.d_ff, w.d_model), 0.0, 0.02),
        "w_down": _normal_bf16(r, (w.d_model, w.d_ff), 0.0, 0.02),
        "gamma2": _normal_bf16(r, (w.d_model,), 1.0, 0.1),
    }


def batching_schedule(seed, n_seq=5, len_range=(40, 300), prefill_chunk=128, max_decode=24):
    """A seeded continuous-batching schedule (the shape of the paper's serving loop: chunked
    prefill fused with decode steps): a list of steps, each a list of (context id, first token,
    number of new tokens).  Contexts join one after another; a context first prefills its
    prompt in chunks of at most `prefill_chunk` tokens, then decodes one token per step."""
    rng = np.random.default_rng([BASE_SEED, 977, seed])
    prompt = rng.integers(len_range[0], len_range[1], size=n_seq, endpoint=True)
    decode = rng.integers(1, max_decode, size=n_seq, endpoint=True)
    start = np.sort(rng.integers(0, 6, size=n_seq))          # step at which each context arrives
    done = np.zeros(n_seq, dtype=np.int64)
    steps, t = [], 0
    while np.any(done < prompt + decode):
        step = []
        for s in range(n_seq):
            if t < start[s] or done[s] >= prompt[s] + decode[s]:
                continue
            if done[s] < prompt[s]:
                n = int(min(prefill_chunk, prompt[s] - done[s]))
            else:
                n = 1
            step.append((int(s) * 7 + 3, int(done[s]), n))    # sparse, non-contiguous ids
            done[s] += n
        if step:
            steps.append(step)
        t += 1
    totals = {int(s) * 7 + 3: int(prompt[s] + decode[s]) for s in range(n_seq)}
    return steps, totals
