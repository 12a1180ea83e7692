"""Pins of oracle/head.py against things other than itself: torch's own embedding / rms_norm / linear /
argmax, closed forms, and brute force on tiny inputs."""
import numpy as np
import torch

from oracle import bf16 as obf
from oracle import head as oh
from oracle import layer as ol
from oracle import run as orun
from paper_2507_17769_amd import workloads as W


def test_embed_is_torch_embedding_and_rejects_bad_ids():
    rng = np.random.default_rng(0)
    table = rng.standard_normal((50, 8))
    ids = rng.integers(0, 50, size=23)
    want = torch.nn.functional.embedding(torch.from_numpy(ids), torch.from_numpy(table)).numpy()
    assert np.array_equal(oh.embed(ids, table), want)
    for bad in ([-1], [50]):
        try:
            oh.embed(bad, table)
            assert False
        except ValueError:
            pass


def test_last_token_rows():
    seqs = [ol.Seq(5, 9, []), ol.Seq(1, 3, []), ol.Seq(2, 2, [])]
    assert oh.last_token_rows(seqs) == [4, 5, 7]


def test_logits_vs_torch_and_only_last_tokens_matter():
    rng = np.random.default_rng(1)
    H, V = 16, 37
    x = rng.standard_normal((8, H))
    g = rng.uniform(0.5, 1.5, H)
    w = rng.standard_normal((H, V))
    seqs = [ol.Seq(5, 5, []), ol.Seq(1, 4, []), ol.Seq(2, 2, [])]
    got = oh.logits(x, seqs, g, w, 1e-5)
    rows = torch.from_numpy(x[[4, 5, 7]])
    want = torch.nn.functional.linear(torch.nn.functional.rms_norm(rows, (H,), torch.from_numpy(g), 1e-5), torch.from_numpy(w.T)).numpy()
    assert got.shape == (3, V) and np.allclose(got, want, rtol=0, atol=1e-12)
    x2 = x.copy()
    x2[[0, 1, 2, 3, 6]] += 100.0       # tokens that generate nothing
    assert np.array_equal(oh.logits(x2, seqs, g, w, 1e-5), got)
    # closed form: a one-hot output column picks one normalised coordinate
    e = np.zeros((H, 1)); e[3, 0] = 1.0
    one = oh.logits(x, seqs, np.ones(H), e, 0.0)
    assert np.allclose(one[:, 0], x[[4, 5, 7], 3] / np.sqrt((x[[4, 5, 7]] ** 2).mean(1)), atol=1e-12)


def test_greedy_first_maximum_both_paths_and_torch():
    rng = np.random.default_rng(2)
    lg = rng.integers(-3, 4, size=(40, 11)).astype(np.float64)      # many ties
    want = np.array([int(np.flatnonzero(r == r.max())[0]) for r in lg], dtype=np.int32)
    assert np.array_equal(oh.greedy(lg), want)
    assert np.array_equal(oh.greedy_rows(lg), want)
    wide = rng.standard_normal((3, 5000))
    assert np.array_equal(oh.greedy(wide), torch.argmax(torch.from_numpy(wide), dim=1).numpy())
    assert oh.greedy(np.array([[1.0, 1.0, 1.0]]))[0] == 0


def test_run_model_composes_embedding_stack_and_head():
    m = dict(W.MODELS["tiny"])
    V = 96
    rng = np.random.default_rng(3)
    head_bits = {"embedding": W.normal_bf16(rng, (V, m["hidden"])), "g_final": obf.to_bits(np.ones(m["hidden"], np.float32)),
                 "w_out": W.normal_bf16(rng, (m["hidden"], V), 0.05)}
    layers = [W.layer_weights(m, 4, l) for l in range(2)]
    b = W.custom_batch("tiny", 5, 6, 0, [3, 9])
    ids = rng.integers(0, V, size=b.n_tokens)
    pool = orun.make_pool(m, b.n_pool_pages, 2)
    for i, s in enumerate(b.seqs):
        if s.prefix > 0:
            k, v = b.prefix_kv(i, 0)
            for slot in range(2):
                pool.write_bits(slot, [int(p) for p in s.pages], 0, k, v)
    import copy
    pool2 = copy.deepcopy(pool)
    nxt, lg, hidden = orun.run_model(m, head_bits, layers, b.seqs, ids, pool, np.float64)
    # the same thing by hand: rows of the table through run_step, then the head
    x_bits = head_bits["embedding"][ids]
    hidden2, _ = orun.run_step(m, layers, b.seqs, x_bits, pool2, np.float64)
    assert np.array_equal(hidden, hidden2)
    hw = orun.widen_weights(head_bits, np.float64)
    lg2 = oh.logits(hidden2, orun.to_seqs(b.seqs), hw["g_final"], hw["w_out"], 1e-5)
    assert np.array_equal(lg, lg2) and np.array_equal(nxt, np.argmax(lg2, axis=1))
    assert nxt.dtype == np.int32 and nxt.shape == (len(b.seqs),)
