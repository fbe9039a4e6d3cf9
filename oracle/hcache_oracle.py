"""CPU oracle for HCache KV restoration -- TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy statement of what the restoration path computes.  It exists
to check the HIP library; nothing in the product path may import it, and it imports
nothing from the product.  Inputs are float64 arrays (bf16 inputs are decoded
exactly by the caller); nothing is rounded on the way, outputs stay float64.

What the method computes (paper Section 3.1, the two restoration equations): for a
saved hidden state H_L^i -- the input of transformer layer L for token i -- the key
and value of that token at that layer are the layer's K and V projections of it,
exactly as a prefill would produce them (the paper calls the method lossless in
Section 7).  The paper's equations leave out normalisation and position embedding
(Section 2.1 says so explicitly); a Llama-style layer projects the RMS-normalised
input and rotates K, so restoration does the same, and Section 5 names the two
device steps: a GEMM, then a kernel that applies RoPE and copies into the KV cache.
Section 6 ("Baselines") says the KV cache is paged (PagedAttention).

Because the result has a plain definition, each function below is that definition
written out.  Readings chosen where the paper is silent:
  * hidden state = residual-stream input of the layer, before its input RMSNorm;
  * RMSNorm: eps is added to the mean square inside the square root, gamma
    multiplies the normalised value;
  * RoPE: angle = position * theta^(-2i/head_dim) for pair i, counter-clockwise
    rotation (RoFormer); style 0 pairs feature i with i + head_dim/2 ("half-split"),
    style 1 pairs 2i with 2i+1 ("interleaved");  applied to K only (and to Q in the
    full forward pass);
  * paged cache of one layer: pool[page, 0|1 (K|V), slot, kv_head, head_dim] with
    page = block_table[position // block_size], slot = position % block_size.

  * OPT-style layers (LayerNorm with shift, projection biases, no rotary embedding) are the
    same restoration with layernorm() in place of rmsnorm(), the bias added and no rotation.

Parity pins (tests/test_oracle_*.py): restored KV equals the KV of a naive full
prefill; pure-Python brute force on tiny inputs; closed forms for RMSNorm; RoPE
invariants plus a worked rotation; paging bijection/enumeration; store round trip.
Unpinned by the paper (fixed by this build's own convention): the default RoPE
pairing style, the page layout and the physical order of the chunk arena.
"""
import numpy as np


# --------------------------------------------------------------------------- norm
def rmsnorm(x, gamma, eps):
    """Root-mean-square normalisation of each row of x [T, d] with gain gamma [d].

    The paper folds normalisation into the modules it does not spell out
    (Section 2.1); this is the Llama form: x * gamma / sqrt(mean(x^2) + eps).
    """
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(gamma, dtype=np.float64)


def layernorm(x, gamma, beta, eps):
    """Layer normalisation of each row of x [T, d]: (x - mean) / sqrt(var + eps) * gamma + beta
    with the biased variance var = mean((x - mean)^2).  The normalisation of OPT-style
    models (the paper evaluates OPT-30B, Section 6 "Models"), whose layers also carry biases
    and use learned absolute position embeddings instead of RoPE."""
    x = np.asarray(x, dtype=np.float64)
    mu = np.mean(x, axis=-1, keepdims=True)
    xc = x - mu
    var = np.mean(xc * xc, axis=-1, keepdims=True)
    return xc / np.sqrt(var + eps) * np.asarray(gamma, dtype=np.float64) + np.asarray(beta, dtype=np.float64)


# --------------------------------------------------------------------------- RoPE
def rope_angles(positions, head_dim, theta):
    """angle[t, i] = positions[t] * theta^(-2 i / head_dim), i in [0, head_dim/2)."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    inv_freq = np.power(float(theta), -2.0 * i / head_dim)
    return np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]


def apply_rope(y, positions, theta, style=0):
    """Rotate y [T, heads, head_dim] by each token's absolute position (Section 5:
    RoPE is applied to the re-projected K before it is copied into the cache)."""
    y = np.asarray(y, dtype=np.float64)
    T, H, hd = y.shape
    ang = rope_angles(positions, hd, theta)           # [T, hd/2]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    out = np.empty_like(y)
    if style == 0:
        a, b = y[..., : hd // 2], y[..., hd // 2:]
        out[..., : hd // 2] = a * c - b * s
        out[..., hd // 2:] = b * c + a * s
    elif style == 1:
        a, b = y[..., 0::2], y[..., 1::2]
        out[..., 0::2] = a * c - b * s
        out[..., 1::2] = b * c + a * s
    else:
        raise ValueError("rope style must be 0 (half-split) or 1 (interleaved)")
    return out


# ----------------------------------------------------------------- restoration
def project_kv(x, gamma, wkv, eps, n_kv_heads, head_dim, *, norm="rms", beta=None, bias=None):
    """K (before RoPE) and V of every token: the restoration equations of Section 3.1
    applied to the normalised hidden state.  wkv is [2*d_kv, d] (nn.Linear layout),
    rows [0, d_kv) = W_k, rows [d_kv, 2 d_kv) = W_v.  Returns ([T,H,hd], [T,H,hd]).

    norm = "rms" (Llama-style, default) or "layer" (OPT-style, with shift beta [d]);
    bias [2*d_kv], when given, is the projections' bias (b_k then b_v)."""
    d_kv = n_kv_heads * head_dim
    wkv = np.asarray(wkv, dtype=np.float64)
    assert wkv.shape[0] == 2 * d_kv
    if norm == "rms":
        assert beta is None
        xh = rmsnorm(x, gamma, eps)
    elif norm == "layer":
        xh = layernorm(x, gamma, np.zeros(wkv.shape[1]) if beta is None else beta, eps)
    else:
        raise ValueError("norm must be 'rms' or 'layer'")
    y = xh @ wkv.T                                     # [T, 2 d_kv]
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64)
    T = y.shape[0]
    k = y[:, :d_kv].reshape(T, n_kv_heads, head_dim)
    v = y[:, d_kv:].reshape(T, n_kv_heads, head_dim)
    return k, v


def page_slots(positions, block_table, block_size):
    """(page, slot) of each token: page = block_table[pos // B], slot = pos % B.
    Raises if a position falls outside the block table or on an unmapped (-1) block."""
    positions = np.asarray(positions, dtype=np.int64)
    block_table = np.asarray(block_table, dtype=np.int64)
    blk = positions // block_size
    if positions.size and (positions.min() < 0 or blk.max() >= block_table.size):
        raise IndexError("position outside the block table")
    page = block_table[blk]
    if (page < 0).any():
        raise IndexError("position maps to an unallocated block")
    return page, positions % block_size


def restore_kv(pool, x, gamma, wkv, positions, block_table, *, eps, theta,
               n_kv_heads, head_dim, block_size, rope_style=0, norm="rms", beta=None, bias=None):
    """Restore one layer's K/V for the tokens of one context into its paged cache.

    pool: float64 [num_pages, 2, block_size, n_kv_heads, head_dim], modified in place
    (only the slots of the given positions are written).  Returns (page, slot).
    rope_style 2 = no rotation (models with learned absolute position embeddings: the
    position is already part of the hidden state)."""
    k, v = project_kv(x, gamma, wkv, eps, n_kv_heads, head_dim, norm=norm, beta=beta, bias=bias)
    if rope_style != 2:
        k = apply_rope(k, positions, theta, rope_style)
    page, slot = page_slots(positions, block_table, block_size)
    if page.size and page.max() >= pool.shape[0]:
        raise IndexError("block table names a page outside the pool")
    pool[page, 0, slot] = k
    pool[page, 1, slot] = v
    return page, slot


def restore_kv_ragged(pool, x, gamma, wkv, positions, cu_seqlens, block_tables, **kw):
    """Ragged batch: the tokens of several contexts concatenated; context s owns rows
    cu_seqlens[s]..cu_seqlens[s+1]-1 and row s of block_tables (padded with -1)."""
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    out = []
    for s in range(len(cu) - 1):
        a, b = cu[s], cu[s + 1]
        out.append(restore_kv(pool, x[a:b], gamma, wkv, positions[a:b],
                              block_tables[s], **kw))
    return out


def gather_kv(pool, positions, block_table, block_size):
    """Read back (K, V) [T, H, hd] of the given positions from a paged pool."""
    page, slot = page_slots(positions, block_table, block_size)
    return pool[page, 0, slot], pool[page, 1, slot]


def scatter_kv(pool, k, v, positions, block_table, block_size):
    """KV-offload restoration of one layer (Section 4.1.2, layer-wise partition): the saved
    K and V rows [T, H, hd] of the given positions go back into the pages the block table
    names.  No arithmetic: the values are the cache's own."""
    page, slot = page_slots(positions, block_table, block_size)
    for t in range(len(page)):
        pool[page[t], 0, slot[t]] = k[t]
        pool[page[t], 1, slot[t]] = v[t]


# -------------------------------------------------------------- full forward pass
def full_prefill(h0, layers, positions, *, eps, theta, n_q_heads, n_kv_heads,
                 head_dim, rope_style=0):
    """Naive prefill of a Llama-style stack (paper Section 2.1: attention then FFN per
    layer, with the residual connections, norms and position embedding the paper's
    equations omit).  Causal attention includes the token itself and scales scores by
    1/sqrt(head_dim); grouped-query attention maps query head q to KV head
    q // (n_q_heads // n_kv_heads).

    layers: list of dicts with float64 'wkv', 'gamma', 'wq', 'wo', 'w_gate', 'w_up',
    'w_down', 'gamma2'.  Returns a list, per layer, of (H_l, K_l roped, V_l): the
    hidden states a serving system would save and the KV cache it would hold.
    """
    h = np.asarray(h0, dtype=np.float64)
    T = h.shape[0]
    group = n_q_heads // n_kv_heads
    d_kv = n_kv_heads * head_dim
    causal = np.tril(np.ones((T, T), dtype=bool))
    record = []
    for lw in layers:
        xh = rmsnorm(h, lw["gamma"], eps)
        q = (xh @ lw["wq"].T).reshape(T, n_q_heads, head_dim)
        k = (xh @ lw["wkv"][:d_kv].T).reshape(T, n_kv_heads, head_dim)
        v = (xh @ lw["wkv"][d_kv:].T).reshape(T, n_kv_heads, head_dim)
        q = apply_rope(q, positions, theta, rope_style)
        k = apply_rope(k, positions, theta, rope_style)
        record.append((h.copy(), k.copy(), v.copy()))
        att = np.empty((T, n_q_heads, head_dim))
        for qh in range(n_q_heads):
            kh = qh // group
            s = (q[:, qh] @ k[:, kh].T) / np.sqrt(head_dim)
            s = np.where(causal, s, -np.inf)
            s = s - s.max(axis=-1, keepdims=True)
            p = np.exp(s)
            p /= p.sum(axis=-1, keepdims=True)
            att[:, qh] = p @ v[:, kh]
        h = h + att.reshape(T, -1) @ lw["wo"].T
        xh2 = rmsnorm(h, lw["gamma2"], eps)
        g = xh2 @ lw["w_gate"].T
        u = xh2 @ lw["w_up"].T
        h = h + ((g / (1.0 + np.exp(-g))) * u) @ lw["w_down"].T
    return record


def full_prefill_opt(h0, layers, *, eps, n_heads, head_dim):
    """Naive prefill of an OPT-style stack (pre-LayerNorm decoder, multi-head attention,
    biases on every projection, ReLU feed-forward, no rotary embedding: h0 already holds
    token plus learned position embeddings).  layers: dicts with float64 'wkv' [2d, d],
    'bkv' [2d], 'gamma', 'beta', 'wq', 'bq', 'wo', 'bo', 'gamma2', 'beta2', 'w1', 'b1',
    'w2', 'b2'.  Returns per layer (H_l, K_l, V_l) like full_prefill."""
    h = np.asarray(h0, dtype=np.float64)
    T = h.shape[0]
    d_kv = n_heads * head_dim
    causal = np.tril(np.ones((T, T), dtype=bool))
    record = []
    for lw in layers:
        xh = layernorm(h, lw["gamma"], lw["beta"], eps)
        q = (xh @ lw["wq"].T + lw["bq"]).reshape(T, n_heads, head_dim)
        k = (xh @ lw["wkv"][:d_kv].T + lw["bkv"][:d_kv]).reshape(T, n_heads, head_dim)
        v = (xh @ lw["wkv"][d_kv:].T + lw["bkv"][d_kv:]).reshape(T, n_heads, head_dim)
        record.append((h.copy(), k.copy(), v.copy()))
        att = np.empty((T, n_heads, head_dim))
        for hh in range(n_heads):
            s = (q[:, hh] @ k[:, hh].T) / np.sqrt(head_dim)
            s = np.where(causal, s, -np.inf)
            s = s - s.max(axis=-1, keepdims=True)
            p = np.exp(s)
            p /= p.sum(axis=-1, keepdims=True)
            att[:, hh] = p @ v[:, hh]
        h = h + att.reshape(T, -1) @ lw["wo"].T + lw["bo"]
        xh2 = layernorm(h, lw["gamma2"], lw["beta2"], eps)
        h = h + np.maximum(xh2 @ lw["w1"].T + lw["b1"], 0.0) @ lw["w2"].T + lw["b2"]
    return record


# ------------------------------------------------------------------- host store
class ChunkStore:
    """Reference model of the chunk-based hidden-state store (Section 4.2.1): the
    hidden states of one layer of one context are kept in fixed-size token chunks,
    each chunk contiguous.  States arrive in generation order -- for each batch of
    new tokens, layer 0 first, then layer 1, ... (layer-before-token, Section 3.2
    challenge C2) -- and are read back one whole layer at a time."""

    def __init__(self, n_layers, d_model, chunk_tokens):
        self.n_layers, self.d_model, self.chunk_tokens = n_layers, d_model, chunk_tokens
        self.rows = {}          # (seq, layer) -> list of row arrays
        self.count = {}         # (seq, layer) -> tokens appended

    def append(self, seq, layer, rows):
        rows = np.asarray(rows)
        assert rows.ndim == 2 and rows.shape[1] == self.d_model
        n_prev = self.count.get((seq, layer), 0)
        if layer > 0 and self.count.get((seq, layer - 1), 0) < n_prev + len(rows):
            raise RuntimeError("layer appended before the layer below it")
        self.rows.setdefault((seq, layer), []).extend(rows)
        self.count[(seq, layer)] = n_prev + len(rows)

    def n_tokens(self, seq, layer):
        return self.count.get((seq, layer), 0)

    def n_chunks(self, seq, layer):
        return -(-self.n_tokens(seq, layer) // self.chunk_tokens)

    def chunk(self, seq, layer, c):
        """Rows of chunk c (the last chunk may be partly filled)."""
        r = self.rows[(seq, layer)]
        lo = c * self.chunk_tokens
        if lo >= len(r) or c < 0:
            raise IndexError("no such chunk")
        return np.stack(r[lo: lo + self.chunk_tokens])

    def layer(self, seq, layer):
        return np.concatenate([self.chunk(seq, layer, c)
                               for c in range(self.n_chunks(seq, layer))])


def save_step(store, layer, rows, row_seq):
    """Stage 2 of the two-stage saving (Section 4.2.2): the snapshot of one layer's inputs
    for the whole running batch is taken apart row by row, each row appended to the chunk
    list of its own context."""
    rows = np.asarray(rows)
    for r, s in zip(rows, row_seq):
        store.append(int(s), layer, r[None, :])


# ------------------------------------------------------------ bubble-free partition
def restoration_time(l_h, n_layers, io_h, io_kv, c_h, c_token):
    """Pipelined restoration time when l_h layers come from hidden states and the rest from
    the complementary method (Section 4.1.2).  Compute-bound platform (c_h > io_h): the
    complement is KV offload, which only adds transfer: max(c_h*l_h, io_h*l_h + io_kv*l_o),
    the paper's min-max objective.  Transfer-bound platform: the complement is token
    recomputation, which only adds compute: max(c_h*l_h + c_token*l_o, io_h*l_h)."""
    l_o = n_layers - l_h
    if c_h > io_h:
        return max(c_h * l_h, io_h * l_h + io_kv * l_o)
    return max(c_h * l_h + c_token * l_o, io_h * l_h)


def partition_layers(n_layers, io_h, io_kv, c_h, c_token):
    """The closed forms of Section 4.1.2: (l_h, l_o, complement), complement 'kv' or 're'.
    Premises of the method: io_kv > io_h and c_token > c_h.  The ceiling is the exact one:
    the given times are taken as the rational numbers they are, so no rounding of the
    quotient can move the result across an integer."""
    import math
    from fractions import Fraction
    assert io_kv > io_h and c_token > c_h
    n = Fraction(int(n_layers))
    io_h, io_kv, c_h, c_token = (Fraction(float(t)) for t in (io_h, io_kv, c_h, c_token))
    if c_h > io_h:
        l_h = math.ceil(n * io_kv / (io_kv + c_h - io_h))
        comp = "kv"
    else:
        l_h = math.ceil(n * c_token / (c_token + io_h - c_h))
        comp = "re"
    l_h = min(max(l_h, 0), int(n_layers))
    return l_h, int(n_layers) - l_h, comp


# --------------------------------------------------------------- cost accounting
def restore_flop(n_tokens, d_model, d_kv):
    """Floating-point operations of one layer's projection, one multiply-add = 2
    (Section 3.2, C_hidden numerator: 4 N D^2 when d_kv = D)."""
    return 4 * n_tokens * d_model * d_kv


def hidden_bytes(n_tokens, d_model, n_layers, elem=2):
    return n_tokens * d_model * n_layers * elem


def kv_bytes(n_tokens, d_kv, n_layers, elem=2):
    return 2 * n_tokens * d_kv * n_layers * elem
