"""Pins for the CPU oracle: it is checked against things other than itself.

Brute force on tiny inputs, torch library routines as special cases, closed
forms and invariants.  Each test says which mistake it would catch.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import bf16, layer
from oracle.layer import PagedKV, Seq, Shape

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- bf16
def test_bf16_round_matches_torch_cast():
    rng = np.random.default_rng(0)
    x = np.concatenate([
        rng.standard_normal(200000).astype(np.float32) * np.float32(10.0) ** rng.integers(-30, 30, 200000).astype(np.float32),
        np.array([0.0, -0.0, 1.0, -1.0, np.inf, -np.inf, 3.3895314e38, 1e-40, -1e-45], dtype=np.float32),
    ]).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bf16.to_bits(x), want)


def test_bf16_ties_to_even_closed_form():
    # 1 + 2^-8 is exactly half-way between 1 and 1 + 2^-7: even mantissa (1.0) wins;
    # 1 + 3*2^-8 is half-way between 1+2^-7 (odd) and 1+2^-6 (even): rounds up.
    x = np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -20], dtype=np.float32)
    got = bf16.from_bits(bf16.to_bits(x))
    assert got.tolist() == [1.0, 1 + 2.0 ** -6, 1 + 2.0 ** -7]


def test_bf16_nan_and_roundtrip():
    assert np.isnan(bf16.from_bits(bf16.to_bits(np.array([np.nan], dtype=np.float32))))[0]
    bits = np.arange(0, 0x7F80, 37, dtype=np.uint16)          # all finite positive patterns (sampled)
    assert np.array_equal(bf16.to_bits(bf16.from_bits(bits)), bits)


# ------------------------------------------------------------------- helpers for attention
def _random_pool_case(rng, n_kv, d, lens_new, n_pages_extra=5):
    """Random sequences with scattered pages; returns pool, seqs and the dense K/V."""
    need = [(L + 15) // 16 for _, L in lens_new]
    n_pages = sum(need) + n_pages_extra
    perm = rng.permutation(n_pages)
    pool = PagedKV(n_pages, 1, n_kv, d)
    seqs, dense, at = [], [], 0
    for (n_new, L), k in zip(lens_new, need):
        pages = perm[at:at + k].tolist()
        at += k
        K = rng.standard_normal((L, n_kv, d)).astype(np.float32)
        V = rng.standard_normal((L, n_kv, d)).astype(np.float32)
        pool.write(0, pages, 0, K, V)
        seqs.append(Seq(n_new, L, pages))
        dense.append((bf16.round_trip(K).astype(np.float64), bf16.round_trip(V).astype(np.float64)))
    return pool, seqs, dense


def _brute_force_attention(q, seqs, dense, n_kv):
    """Scalar loops straight from Softmax(q.k/sqrt(d)) v over positions 0..p."""
    T, n_q, d = q.shape
    G = n_q // n_kv
    out = np.zeros((T, n_q, d))
    t = 0
    for sq, (K, V) in zip(seqs, dense):
        for i in range(sq.n_new):
            p = sq.kv_len - sq.n_new + i
            for h in range(n_q):
                logits = [float(np.dot(q[t, h], K[j, h // G])) / math.sqrt(d) for j in range(p + 1)]
                m = max(logits)
                w = [math.exp(l - m) for l in logits]
                z = sum(w)
                acc = np.zeros(d)
                for j in range(p + 1):
                    acc += (w[j] / z) * V[j, h // G]
                out[t, h] = acc
            t += 1
    return out


@pytest.mark.parametrize("n_q,n_kv,d", [(4, 2, 16), (4, 4, 8), (8, 1, 32)])
def test_paged_attention_vs_brute_force(n_q, n_kv, d):
    # catches: wrong page gather, off-by-one causal boundary, wrong GQA map, missing scale
    rng = np.random.default_rng(1)
    lens_new = [(7, 23), (1, 1), (1, 17), (5, 5), (1, 64), (33, 50)]
    pool, seqs, dense = _random_pool_case(rng, n_kv, d, lens_new)
    T = sum(n for n, _ in lens_new)
    q = rng.standard_normal((T, n_q, d))
    got = layer.attention_paged(q, seqs, pool, 0, n_kv)
    want = _brute_force_attention(q, seqs, dense, n_kv)
    assert np.max(np.abs(got - want)) < 1e-12
    got32 = layer.attention_paged(q.astype(np.float32), seqs, pool, 0, n_kv)
    assert np.max(np.abs(got32 - want)) < 1e-5


def test_paged_attention_vs_torch_sdpa():
    # library special case: explicit boolean mask, KV heads expanded to MHA
    rng = np.random.default_rng(2)
    n_q, n_kv, d = 8, 2, 32
    lens_new = [(40, 100), (1, 77), (16, 16)]
    pool, seqs, dense = _random_pool_case(rng, n_kv, d, lens_new)
    T = sum(n for n, _ in lens_new)
    q = rng.standard_normal((T, n_q, d))
    got = layer.attention_paged(q, seqs, pool, 0, n_kv)
    t = 0
    for sq, (K, V) in zip(seqs, dense):
        qs = torch.from_numpy(q[t:t + sq.n_new]).permute(1, 0, 2)                   # [n_q][n][d]
        Ks = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(n_q // n_kv, 0)  # [n_q][L][d]
        Vs = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(n_q // n_kv, 0)
        qpos = torch.arange(sq.kv_len - sq.n_new, sq.kv_len)[:, None]
        mask = torch.arange(sq.kv_len)[None, :] <= qpos
        want = torch.nn.functional.scaled_dot_product_attention(qs, Ks, Vs, attn_mask=mask).permute(1, 0, 2).numpy()
        assert np.max(np.abs(got[t:t + sq.n_new] - want)) < 1e-12
        t += sq.n_new


def test_page_permutation_invariance_bit_exact():
    rng = np.random.default_rng(3)
    n_kv, d, n_q = 2, 16, 4
    L, n_new = 75, 9
    K = rng.standard_normal((L, n_kv, d)).astype(np.float32)
    V = rng.standard_normal((L, n_kv, d)).astype(np.float32)
    q = rng.standard_normal((n_new, n_q, d)).astype(np.float32)
    outs = []
    for s in range(3):
        pages = np.random.default_rng(100 + s).permutation(11)[:5].tolist()
        pool = PagedKV(11, 1, n_kv, d)
        pool.write(0, pages, 0, K, V)
        outs.append(layer.attention_paged(q, [Seq(n_new, L, pages)], pool, 0, n_kv))
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


def test_decode_with_one_key_returns_v_exactly():
    rng = np.random.default_rng(4)
    n_q, n_kv, d = 4, 2, 16
    pool = PagedKV(3, 1, n_kv, d)
    k = rng.standard_normal((1, n_kv, d)).astype(np.float32)
    v = rng.standard_normal((1, n_kv, d)).astype(np.float32)
    pool.write(0, [2], 0, k, v)
    q = rng.standard_normal((1, n_q, d)).astype(np.float32)
    out = layer.attention_paged(q, [Seq(1, 1, [2])], pool, 0, n_kv)
    want = bf16.round_trip(v)[0]                         # [n_kv][d]
    for h in range(n_q):
        assert np.array_equal(out[0, h], want[h // 2])


def test_softmax_properties():
    rng = np.random.default_rng(5)
    n_q, n_kv, d, L = 4, 2, 16, 40
    s = rng.standard_normal((6, 50)) * 5
    s[0, 10:] = -np.inf
    w = layer.softmax_rows(s)
    assert np.allclose(w.sum(-1), 1.0, atol=1e-14) and np.all(w[0, 10:] == 0)
    big = layer.softmax_rows(np.array([[1000.0, 1000.0 + np.log(3.0)]]))      # would overflow without the max shift
    assert np.allclose(big, [[0.25, 0.75]], atol=1e-12)
    # all keys equal -> uniform weights -> output = running mean of V
    pool = PagedKV(4, 1, n_kv, d)
    K = np.tile(rng.standard_normal((1, n_kv, d)), (L, 1, 1)).astype(np.float32)
    V = rng.standard_normal((L, n_kv, d)).astype(np.float32)
    pool.write(0, [3, 0, 2], 0, K, V)
    q = rng.standard_normal((L, n_q, d))
    out = layer.attention_paged(q, [Seq(L, L, [3, 0, 2])], pool, 0, n_kv)
    Vb = bf16.round_trip(V).astype(np.float64)
    for i in (0, 1, 15, 16, 39):
        want = Vb[:i + 1].mean(0)                        # [n_kv][d]
        assert np.allclose(out[i, 0], want[0], atol=1e-12) and np.allclose(out[i, 3], want[1], atol=1e-12)
    # convex combination: inside the per-coordinate range of the visible values
    q2 = rng.standard_normal((L, n_q, d)) * 3
    pool.write(0, [3, 0, 2], 0, rng.standard_normal((L, n_kv, d)).astype(np.float32), V)
    o2 = layer.attention_paged(q2, [Seq(L, L, [3, 0, 2])], pool, 0, n_kv)
    for i in (3, 20, 39):
        assert np.all(o2[i, 1] <= Vb[:i + 1, 0].max(0) + 1e-12) and np.all(o2[i, 1] >= Vb[:i + 1, 0].min(0) - 1e-12)


def test_gqa_equals_expanded_mha():
    rng = np.random.default_rng(6)
    n_q, n_kv, d = 8, 2, 16
    lens_new = [(6, 30), (1, 19)]
    pool, seqs, dense = _random_pool_case(rng, n_kv, d, lens_new)
    T = 7
    q = rng.standard_normal((T, n_q, d))
    got = layer.attention_paged(q, seqs, pool, 0, n_kv)
    pool2 = PagedKV(pool.bits.shape[1], 1, n_q, d)
    for sq, (K, V) in zip(seqs, dense):
        pool2.write(0, sq.pages, 0, np.repeat(K, 4, axis=1).astype(np.float32), np.repeat(V, 4, axis=1).astype(np.float32))
    want = layer.attention_paged(q, seqs, pool2, 0, n_q)
    assert np.max(np.abs(got - want)) < 1e-13


# ----------------------------------------------------------------------------- RoPE
def test_rope_complex_closed_form_and_isometry():
    # (u_j + i u_{j+d/2}) * exp(i p theta_j): pins pairing, direction and frequency
    rng = np.random.default_rng(7)
    d, base = 64, 10000.0
    u = rng.standard_normal((5, 3, d))
    pos = np.array([0, 1, 17, 4095, 16383])
    got = layer.rope(u, pos, base)
    z = u[..., :d // 2] + 1j * u[..., d // 2:]
    theta = np.array([base ** (-(2.0 * j) / d) for j in range(d // 2)])
    zr = z * np.exp(1j * pos[:, None, None] * theta[None, None, :])
    # one ulp of theta times position 16383 is ~4e-12 of phase: 1e-10 still pins every index and sign
    assert np.max(np.abs(got[..., :d // 2] - zr.real)) < 1e-10
    assert np.max(np.abs(got[..., d // 2:] - zr.imag)) < 1e-10
    assert np.array_equal(got[0], u[0])                                  # position 0 is the identity
    assert np.allclose(np.linalg.norm(got, axis=-1), np.linalg.norm(u, axis=-1), rtol=1e-12)
    g32 = layer.rope(u.astype(np.float32), pos, base)
    assert np.allclose(np.linalg.norm(g32, axis=-1), np.linalg.norm(u, axis=-1), rtol=1e-6)


def test_rope_d2_is_plane_rotation():
    u = np.array([[[1.0, 0.0]], [[0.0, 1.0]]])
    got = layer.rope(u, np.array([1, 2]), 10000.0)         # d = 2: theta_0 = 1 rad per position
    assert np.allclose(got[0, 0], [math.cos(1), math.sin(1)], atol=1e-15)
    assert np.allclose(got[1, 0], [-math.sin(2), math.cos(2)], atol=1e-15)


def test_rope_inner_product_depends_on_offset_only():
    rng = np.random.default_rng(8)
    d = 32
    q = rng.standard_normal((1, 1, d))
    k = rng.standard_normal((1, 1, d))
    dots = []
    for m, n in [(5, 2), (103, 100), (4003, 4000)]:
        dots.append(float(np.sum(layer.rope(q, [m], 500000.0) * layer.rope(k, [n], 500000.0))))
    assert abs(dots[0] - dots[1]) < 1e-10 and abs(dots[0] - dots[2]) < 1e-9


# ------------------------------------------------------------------- small dense pieces
def test_rmsnorm_and_silu_vs_torch():
    rng = np.random.default_rng(9)
    x = rng.standard_normal((7, 96)) * 3
    g = rng.standard_normal(96)
    got = layer.rmsnorm(x, g, 1e-5)
    want = torch.nn.functional.rms_norm(torch.from_numpy(x), (96,), torch.from_numpy(g), 1e-5).numpy()
    assert np.max(np.abs(got - want)) < 1e-13
    unit = layer.rmsnorm(x, np.ones(96), 0.0)
    assert np.allclose(np.mean(unit * unit, -1), 1.0, atol=1e-13)
    z = np.linspace(-30, 30, 601)
    assert np.max(np.abs(layer.silu(z) - torch.nn.functional.silu(torch.from_numpy(z)).numpy())) < 1e-14
    assert layer.silu(np.zeros(1))[0] == 0.0 and abs(layer.silu(np.array([40.0]))[0] - 40.0) < 1e-12


# ------------------------------------------------------------------- whole layer
def _tiny_shape():
    return Shape(hidden=64, n_q=4, n_kv=2, head_dim=16, ffn=96, rope_base=10000.0, rms_eps=1e-5)


def _tiny_weights(rng, sh, std=0.2, gains=True):
    H, nq, nkv, d, F = sh.hidden, sh.n_q, sh.n_kv, sh.head_dim, sh.ffn
    w = {
        "w_qkv": rng.standard_normal((H, (nq + 2 * nkv) * d)) * std,
        "w_o": rng.standard_normal((nq * d, H)) * std,
        "w_gate": rng.standard_normal((H, F)) * std,
        "w_up": rng.standard_normal((H, F)) * std,
        "w_down": rng.standard_normal((F, H)) * std,
        "g_attn": 1 + 0.1 * rng.standard_normal(H) if gains else np.ones(H),
        "g_ffn": 1 + 0.1 * rng.standard_normal(H) if gains else np.ones(H),
    }
    return w


def _torch_block_one_shot(x, w, sh):
    """A standard pre-norm GQA decoder block composed from torch library routines
    (rms_norm, complex-multiply rotary, scaled_dot_product_attention with
    is_causal and enable_gqa, silu), valid for one-shot prefill from an empty cache."""
    F = torch.nn.functional
    T = x.shape[0]
    nq, nkv, d = sh.n_q, sh.n_kv, sh.head_dim
    tx = torch.from_numpy(x)
    tw = {k: torch.from_numpy(np.asarray(v, dtype=np.float64)) for k, v in w.items()}
    xn = F.rms_norm(tx, (sh.hidden,), tw["g_attn"], sh.rms_eps)
    qkv = xn @ tw["w_qkv"]
    q, k, v = qkv.split([nq * d, nkv * d, nkv * d], dim=-1)
    inv = sh.rope_base ** (-torch.arange(0, d, 2, dtype=torch.float64) / d)
    ang = torch.arange(T, dtype=torch.float64)[:, None] * inv[None, :]
    rot = torch.polar(torch.ones_like(ang), ang)[:, None, :]

    def rotary(u, nh):
        u = u.reshape(T, nh, d)
        z = torch.complex(u[..., :d // 2], u[..., d // 2:]) * rot
        return torch.cat([z.real, z.imag], dim=-1)

    q, k = rotary(q, nq), rotary(k, nkv)
    v = v.reshape(T, nkv, d)
    k = k.to(torch.float32).to(torch.bfloat16).to(torch.float64)       # cache stores bf16
    v = v.to(torch.float32).to(torch.bfloat16).to(torch.float64)
    a = F.scaled_dot_product_attention(q.permute(1, 0, 2)[None], k.permute(1, 0, 2)[None], v.permute(1, 0, 2)[None],
                                       is_causal=True, enable_gqa=True)[0].permute(1, 0, 2).reshape(T, nq * d)
    x1 = tx + a @ tw["w_o"]
    xn2 = F.rms_norm(x1, (sh.hidden,), tw["g_ffn"], sh.rms_eps)
    out = x1 + (F.silu(xn2 @ tw["w_gate"]) * (xn2 @ tw["w_up"])) @ tw["w_down"]
    return out.numpy(), k.numpy(), v.numpy()


def test_layer_one_shot_prefill_vs_torch_block():
    # catches: dropped residual, norm in the wrong place, transposed weight, gate/up swapped
    # (silu(up)*gate differs), q/k/v column blocks in the wrong order, missing rotary on k
    rng = np.random.default_rng(10)
    sh = _tiny_shape()
    w = _tiny_weights(rng, sh)
    T = 37
    x = rng.standard_normal((T, sh.hidden))
    pages = [4, 1, 3]
    pool = PagedKV(6, 1, sh.n_kv, sh.head_dim)
    out = layer.layer_forward(x, w, [Seq(T, T, pages)], pool, 0, sh)
    want, k_want, v_want = _torch_block_one_shot(x, w, sh)
    assert np.max(np.abs(out - want)) < 1e-9
    K, V = pool.gather(0, pages, T, np.float64)
    # the float64 -> float32 hop before the bf16 rounding can flip a tie: allow <= 1 ulp, rarely
    assert np.mean(K != k_want) < 2e-3 and np.max(np.abs(K - k_want)) <= np.max(np.abs(k_want)) * 2.0 ** -7
    assert np.mean(V != v_want) < 2e-3


def _prefill_in_chunks(x, w, sh, chunks, pages, dtype):
    pool = PagedKV(max(pages) + 1, 1, sh.n_kv, sh.head_dim)
    outs, done = [], 0
    for c in chunks:
        outs.append(layer.layer_forward(x[done:done + c].astype(dtype), w, [Seq(c, done + c, pages)], pool, 0, sh))
        done += c
    return np.concatenate(outs), pool


def test_chunked_prefill_equals_one_shot():
    # Sec. 2.1/2.4: chunking a prompt is a scheduling choice, not a numerical one
    rng = np.random.default_rng(11)
    sh = _tiny_shape()
    w = _tiny_weights(rng, sh)
    L = 128
    x = rng.standard_normal((L, sh.hidden))
    pages = rng.permutation(12)[:8].tolist()
    ref, pool_ref = _prefill_in_chunks(x, w, sh, [L], pages, np.float64)
    for chunks in ([64, 64], [1, 127], [17, 111], [16] * 8, [1] * 128):
        out, pool = _prefill_in_chunks(x, w, sh, chunks, pages, np.float64)
        assert np.array_equal(pool.bits, pool_ref.bits)
        assert np.max(np.abs(out - ref)) < 1e-10
    out32, pool32 = _prefill_in_chunks(x, w, sh, [17, 111], pages, np.float32)
    assert np.max(np.abs(out32 - ref)) < 1e-4 * np.sqrt(np.mean(ref ** 2)) * 10
    assert np.mean(pool32.bits != pool_ref.bits) < 5e-3


def test_chunk_patterns_of_the_papers_worked_example():
    # Sec. 4.7: 2050-token prompt, budget 1024 -> 1+1024+1024+1, or 1024+1026 under dynamic chunking
    prompt, patterns = None, []
    for line in open(os.path.join(GOLDEN, "dynamic_chunking_example.txt")):
        f = line.split()
        if not f or f[0].startswith("#"):
            continue
        if f[0] == "prompt":
            prompt = int(f[1])
        elif f[0] == "pattern":
            patterns.append([int(v) for v in f[1:]])
    assert prompt == 2050 and [1, 1024, 1024, 1] in patterns and [1024, 1026] in patterns
    assert all(sum(p) == prompt for p in patterns)
    rng = np.random.default_rng(12)
    sh = Shape(hidden=32, n_q=2, n_kv=1, head_dim=16, ffn=48)
    w = _tiny_weights(rng, sh)
    x = rng.standard_normal((prompt, sh.hidden))
    pages = rng.permutation(140)[:129].tolist()
    ref, pool_ref = _prefill_in_chunks(x, w, sh, [prompt], pages, np.float64)
    for chunks in patterns:
        out, pool = _prefill_in_chunks(x, w, sh, chunks, pages, np.float64)
        assert np.array_equal(pool.bits, pool_ref.bits)
        assert np.max(np.abs(out - ref)) < 1e-9


def test_decode_is_a_one_token_chunk_and_mixed_batch_is_separable():
    # a mixed batch gives each sequence what it would get alone (requests do not interact)
    rng = np.random.default_rng(13)
    sh = _tiny_shape()
    w = _tiny_weights(rng, sh)
    specs = [(20, 52), (1, 17), (1, 64), (1, 1)]
    pages_all = rng.permutation(16)
    seqs, at = [], 0
    for n, L in specs:
        k = (L + 15) // 16
        seqs.append(Seq(n, L, pages_all[at:at + k].tolist()))
        at += k
    T = sum(n for n, _ in specs)
    x = rng.standard_normal((T, sh.hidden))

    def fresh_pool():
        r = np.random.default_rng(99)
        pool = PagedKV(16, 1, sh.n_kv, sh.head_dim)
        for sq in seqs:
            p = sq.kv_len - sq.n_new
            pool.write(0, sq.pages, 0, r.standard_normal((p, sh.n_kv, sh.head_dim)).astype(np.float32),
                       r.standard_normal((p, sh.n_kv, sh.head_dim)).astype(np.float32))
        return pool

    pool = fresh_pool()
    mixed = layer.layer_forward(x, w, seqs, pool, 0, sh)
    t = 0
    for sq in seqs:
        alone_pool = fresh_pool()
        alone = layer.layer_forward(x[t:t + sq.n_new], w, [sq], alone_pool, 0, sh)
        assert np.max(np.abs(alone - mixed[t:t + sq.n_new])) < 1e-12
        t += sq.n_new


def test_layer_degenerate_weights():
    rng = np.random.default_rng(14)
    sh = _tiny_shape()
    w = _tiny_weights(rng, sh)
    x = rng.standard_normal((5, sh.hidden))
    w0 = dict(w, w_o=np.zeros_like(w["w_o"]), w_down=np.zeros_like(w["w_down"]))
    pool = PagedKV(2, 1, sh.n_kv, sh.head_dim)
    assert np.array_equal(layer.layer_forward(x, w0, [Seq(5, 5, [1])], pool, 0, sh), x)
    # kv_len 1, FFN switched off: out = x + expand(v) @ W_o, with v = bf16(rmsnorm(x) @ W_v)
    w1 = dict(w, w_down=np.zeros_like(w["w_down"]))
    pool = PagedKV(2, 1, sh.n_kv, sh.head_dim)
    x1 = x[:1]
    out = layer.layer_forward(x1, w1, [Seq(1, 1, [0])], pool, 0, sh)
    xn = x1 / np.sqrt(np.mean(x1 ** 2) + 1e-5) * w["g_attn"]
    v = bf16.round_trip((xn @ w["w_qkv"][:, (sh.n_q + sh.n_kv) * sh.head_dim:]).astype(np.float32)).astype(np.float64)
    v = v.reshape(sh.n_kv, sh.head_dim)
    a = np.concatenate([v[h // 2] for h in range(sh.n_q)])[None, :]
    assert np.max(np.abs(out - (x1 + a @ w["w_o"]))) < 1e-12


def test_stack_uses_kv_slot_per_layer():
    rng = np.random.default_rng(15)
    sh = _tiny_shape()
    ws = [_tiny_weights(rng, sh) for _ in range(3)]
    x = rng.standard_normal((9, sh.hidden))
    seqs = [Seq(9, 9, [2])]
    pool = PagedKV(3, 3, sh.n_kv, sh.head_dim)
    out = layer.stack_forward(x, ws, seqs, pool, sh)
    y = x
    for l in range(3):
        p = PagedKV(3, 1, sh.n_kv, sh.head_dim)
        y = layer.layer_forward(y, ws[l], seqs, p, 0, sh)
        assert np.array_equal(p.bits[0], pool.bits[l])
    assert np.array_equal(out, y)


def test_bf16_activation_variant_stays_within_rounding_of_the_definition():
    rng = np.random.default_rng(16)
    sh = _tiny_shape()
    w = _tiny_weights(rng, sh)
    x = rng.standard_normal((40, sh.hidden))
    pages = [0, 2, 1]
    seqs = [Seq(40, 40, pages)]
    ta, tb = {}, {}
    a = layer.layer_forward(x, w, seqs, PagedKV(3, 1, sh.n_kv, sh.head_dim), 0, sh, ta)
    b = layer.layer_forward(x, w, seqs, PagedKV(3, 1, sh.n_kv, sh.head_dim), 0, sh, tb, bf16_activations=True)
    rms = np.sqrt(np.mean(a * a))
    assert 0 < np.max(np.abs(a - b)) < 5e-2 * rms      # these test weights (std 0.2) amplify every rounding ~4x
    for name in ("xn", "q", "attn", "xn2", "act"):
        stored = tb[name]
        assert np.array_equal(bf16.round_trip(stored.astype(np.float32)).astype(np.float64), stored)   # exactly bf16 values
    assert np.max(np.abs(tb["xn"] - ta["xn"])) <= 2.0 ** -8 * np.max(np.abs(ta["xn"]))                  # half an ulp
