"""Floating-point side of a serving step (test infrastructure).

Follows the layer description of Sec. 2.1 ("LLM Inference Workflow"): RMS
normalisation and a residual connection around each module; the attention
module makes query, key and value vectors from the normalised input and
computes Softmax(Q K^T / sqrt(d)) V against the keys and values of all previous
tokens; its output goes through the O-projection; the feed-forward network is
an up projection, a gate projection, an activation and a down projection.  The
evaluated model family (Sec. 5.1, "Model and GPU") uses grouped-query
attention, rotary position embedding and a SiLU-gated feed-forward network.
The batch is the mixed one of Sec. 2.4: one chunk of prefill tokens plus one
token per running decode request, all sequences concatenated along the token
axis.

Readings fixed where the text is silent:
pre-norm placement, eps = 1e-5 unless given, half-split rotary pairing
(j, j + d/2) with theta_j = base^(-2j/d) and no long-context rescale, keys
cached after rotation, softmax scale 1/sqrt(head_dim), a token attends to
positions 0..its own inclusive, query head h reads KV head h // (nq/nkv), no
biases.

Everything is dense and naive on purpose.  Arithmetic runs in `dtype`
(float32 by default, float64 for the tighter self-checks); the only rounding to
bfloat16 is the KV-cache write, because the cache's storage format is part of
what is specified.  Attention always reads keys and values back from the paged
pool, so one-shot prefill, chunked prefill and decode share one code path.
"""
from dataclasses import dataclass

import numpy as np

from . import bf16

PAGE = 16


@dataclass
class Shape:
    hidden: int
    n_q: int
    n_kv: int
    head_dim: int
    ffn: int
    rope_base: float = 10000.0
    rms_eps: float = 1e-5


@dataclass
class Seq:
    n_new: int          # tokens fed this step
    kv_len: int         # attended span after the step (new tokens included)
    pages: list         # physical page ids, len >= ceil(kv_len / 16)


class PagedKV:
    """Paged KV cache: bfloat16 bit patterns, 16 tokens per page.

    bits[slot, page, 0] holds keys and bits[slot, page, 1] values, each
    [16 tokens][n_kv][head_dim].  `slot` is a physical KV layer slot; layer l of
    a stack uses slot l mod n_slots.
    """

    def __init__(self, n_pages, n_slots, n_kv, head_dim):
        self.bits = np.zeros((n_slots, n_pages, 2, PAGE, n_kv, head_dim), dtype=np.uint16)

    def write_bits(self, slot, pages, pos0, k_bits, v_bits):
        """Store bfloat16 patterns [n][n_kv][d] at logical positions pos0..pos0+n-1."""
        for i in range(k_bits.shape[0]):
            p = pos0 + i
            page = int(pages[p // PAGE])
            self.bits[slot, page, 0, p % PAGE] = k_bits[i]
            self.bits[slot, page, 1, p % PAGE] = v_bits[i]

    def write(self, slot, pages, pos0, k, v):
        """Round float keys/values [n][n_kv][d] to bfloat16 (RNE) and store them."""
        self.write_bits(slot, pages, pos0, bf16.to_bits(k), bf16.to_bits(v))

    def gather(self, slot, pages, length, dtype=np.float32):
        """Keys and values of logical positions 0..length-1 as [length][n_kv][d]."""
        n_pg = (length + PAGE - 1) // PAGE
        idx = np.asarray(pages[:n_pg], dtype=np.int64)
        blk = self.bits[slot, idx]                       # [n_pg, 2, 16, n_kv, d]
        k = blk[:, 0].reshape(n_pg * PAGE, *blk.shape[3:])[:length]
        v = blk[:, 1].reshape(n_pg * PAGE, *blk.shape[3:])[:length]
        return bf16.from_bits(k, dtype), bf16.from_bits(v, dtype)


def rmsnorm(x, gain, eps):
    """x * rsqrt(mean(x^2) + eps) * gain, row-wise over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + x.dtype.type(eps)) * gain


def rope(u, pos, base):
    """Rotary embedding on u [T][heads][d] at integer positions pos [T].

    Pair (j, j + d/2) is rotated by angle pos * base^(-2j/d); angles, sines and
    cosines are formed in float64 and then cast to u's dtype.
    """
    d = u.shape[-1]
    half = d // 2
    j = np.arange(half, dtype=np.float64)
    theta = np.float64(base) ** (-2.0 * j / d)
    phi = np.asarray(pos, dtype=np.float64)[:, None] * theta[None, :]      # [T][half]
    c = np.cos(phi).astype(u.dtype)[:, None, :]
    s = np.sin(phi).astype(u.dtype)[:, None, :]
    lo, hi = u[..., :half], u[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def softmax_rows(s):
    """Max-subtracted softmax along the last axis (-inf entries get weight 0)."""
    m = np.max(s, axis=-1, keepdims=True)
    w = np.exp(s - m)
    return w / np.sum(w, axis=-1, keepdims=True)


def attention_paged(q, seqs, pool, slot, n_kv):
    """Causal attention of every new token against its sequence's paged cache.

    q is [T][n_q][d] (rotated).  The new tokens' own keys/values must already
    be in the pool.  Token i of a sequence (position p = kv_len - n_new + i)
    attends to cache positions 0..p inclusive.  Returns [T][n_q][d].
    """
    T, n_q, d = q.shape
    group = n_q // n_kv
    out = np.zeros_like(q)
    scale = q.dtype.type(1.0 / np.sqrt(d))
    t0 = 0
    for sq in seqs:
        prefix = sq.kv_len - sq.n_new
        K, V = pool.gather(slot, sq.pages, sq.kv_len, q.dtype)      # [L][n_kv][d]
        key_pos = np.arange(sq.kv_len)
        q_pos = prefix + np.arange(sq.n_new)
        visible = key_pos[None, :] <= q_pos[:, None]                # [n_new][L]
        for h in range(n_q):
            kh = h // group
            s = (q[t0:t0 + sq.n_new, h] @ K[:, kh].T) * scale       # [n_new][L]
            s = np.where(visible, s, -np.inf)
            out[t0:t0 + sq.n_new, h] = softmax_rows(s) @ V[:, kh]
        t0 += sq.n_new
    return out


def silu(z):
    return z / (1.0 + np.exp(-z))


def layer_forward(x, w, seqs, pool, slot, shape, taps=None, bf16_activations=False):
    """One decoder layer over the concatenated new tokens.

    x [T][hidden] float; w maps names to float arrays in math layout [in][out]
    (w_qkv has q, k, v column blocks in that order; w_o, w_gate, w_up, w_down;
    gains g_attn, g_ffn).  Appends this step's keys/values to pool[slot] and
    returns the layer output [T][hidden].  `taps`, if a dict, receives the
    intermediates by name.

    bf16_activations=False is the definition.  With True, the tensors that a
    bf16-storage implementation feeds to its matrix units (normalised inputs,
    rotated queries, attention output, gated activation) are additionally rounded
    to bfloat16 where they are produced, everything else unchanged; comparing an
    implementation against this variant separates "rounds in the stated places"
    from "computes something else".
    """
    def stored(a):
        return bf16.round_trip(a.astype(np.float32)).astype(a.dtype) if bf16_activations else a

    T = x.shape[0]
    nq, nkv, d = shape.n_q, shape.n_kv, shape.head_dim
    dt = x.dtype
    assert sum(s.n_new for s in seqs) == T

    pos = np.concatenate([np.arange(s.kv_len - s.n_new, s.kv_len) for s in seqs]) if seqs else np.zeros(0, int)

    xn = stored(rmsnorm(x, w["g_attn"].astype(dt), shape.rms_eps))
    qkv = xn @ w["w_qkv"].astype(dt)
    q = qkv[:, :nq * d].reshape(T, nq, d)
    k = qkv[:, nq * d:(nq + nkv) * d].reshape(T, nkv, d)
    v = qkv[:, (nq + nkv) * d:].reshape(T, nkv, d)
    q = stored(rope(q, pos, shape.rope_base))
    k = rope(k, pos, shape.rope_base)

    t0 = 0
    for sq in seqs:                                   # KV append (bf16 RNE at the write)
        pool.write(slot, sq.pages, sq.kv_len - sq.n_new,
                   k[t0:t0 + sq.n_new].astype(np.float32), v[t0:t0 + sq.n_new].astype(np.float32))
        t0 += sq.n_new

    attn = stored(attention_paged(q, seqs, pool, slot, nkv))
    o = attn.reshape(T, nq * d) @ w["w_o"].astype(dt)
    x1 = x + o

    xn2 = stored(rmsnorm(x1, w["g_ffn"].astype(dt), shape.rms_eps))
    gate = xn2 @ w["w_gate"].astype(dt)
    up = xn2 @ w["w_up"].astype(dt)
    act = stored(silu(gate) * up)
    f = act @ w["w_down"].astype(dt)
    out = x1 + f

    if taps is not None:
        taps.update(xn=xn, q=q, k=k, v=v, attn=attn, o=o, x1=x1, xn2=xn2, act=act, ffn=f, out=out)
    return out


def stack_forward(x, layers, seqs, pool, shape, taps=None, bf16_activations=False):
    """Run `layers` (a list of weight dicts) in order; layer l uses KV slot
    l mod n_slots.  Activations stay in x's dtype between layers."""
    n_slots = pool.bits.shape[0]
    for l, w in enumerate(layers):
        t = {} if taps is not None else None
        x = layer_forward(x, w, seqs, pool, l % n_slots, shape, t, bf16_activations)
        if taps is not None:
            taps[l] = t
    return x
