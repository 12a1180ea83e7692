"""Full-model step (tokens in, greedy token out) through the C ABI against oracle/run.run_model."""
import copy

import numpy as np
import pytest
import torch

from oracle import bf16 as obf
from oracle import head as oh
from oracle import run as orun
from paper_2507_17769_amd import binding as B
from paper_2507_17769_amd import workloads as W
from paper_2507_17769_amd.runner import Engine, bits_to_dev
from gpu_harness import TOL, rel_err, row_score

pytestmark = pytest.mark.gpu


def _setup(model, b, n_layers, vocab, seed=31, n_kv_layers=None):
    m = W.MODELS[model] if isinstance(model, str) else model
    n_kv_layers = n_kv_layers or n_layers
    layers = [W.layer_weights(m, seed, l) for l in range(n_layers)]
    head = W.head_weights(m, vocab, seed)
    eng = Engine(m, b.n_pool_pages, n_layers, n_kv_layers, max_position=max(s.kv_len for s in b.seqs) + 16)
    for l, w in enumerate(layers):
        eng.load_layer(l, w)
    eng.load_head(head)
    pool = orun.make_pool(m, b.n_pool_pages, n_kv_layers)
    for slot in range(n_kv_layers):
        for i, s in enumerate(b.seqs):
            if s.prefix > 0:
                k, v = b.prefix_kv(i, slot)
                eng.write_kv(slot, s.pages, 0, k, v)
                pool.write_bits(slot, [int(p) for p in s.pages], 0, k, v)
    return m, layers, head, eng, pool


def _check_tokens(got_next, got_logits, want_logits, tag):
    """The greedy pick is exact integer work on the logits the device computed; against the oracle it is
    unique only where the oracle's best logit leads by more than both sides' rounding."""
    first_max = np.array([int(np.flatnonzero(r == r.max())[0]) for r in got_logits], dtype=np.int32)
    assert np.array_equal(got_next, first_max), f"{tag}: not the first maximum of the device's own logits"
    want = oh.greedy(want_logits)
    rms = float(np.sqrt(np.mean(want_logits.astype(np.float64) ** 2)))
    for i, (g, w) in enumerate(zip(got_next, want)):
        lead = np.sort(want_logits[i])[-1] - np.sort(want_logits[i])[-2]
        if lead > 2 * TOL * rms:
            assert g == w, f"{tag}: sequence {i}: token {g}, oracle {w} leads by {lead:.4f}"
        else:   # near-tie: any token within the rounding band of the best is a valid pick
            assert want_logits[i, g] >= want_logits[i, w] - 2 * TOL * rms, f"{tag}: sequence {i}: token {g} is not near the best"


@pytest.mark.parametrize("spec,n_layers,vocab", [
    ((40, 24, [1, 17, 100]), 3, 1024),        # mixed batch, three layers
    ((0, 0, [5, 33, 64, 200] * 20), 2, 4096),  # 80 decode sequences: the output projection takes the tiled GEMM
    ((7, 0, []), 1, 64),                      # one short prefill, smallest vocabulary
])
def test_model_step_against_oracle(spec, n_layers, vocab):
    b = W.custom_batch("tiny", 29, *spec, name="model")
    m, layers, head, eng, pool = _setup("tiny", b, n_layers, vocab)
    ids = W.token_ids(vocab, b.n_tokens, 7)
    pool_b = copy.deepcopy(pool)
    out = eng.step_tokens(b.seqs, ids, want_hidden=True)
    eng.ctx.sync()
    got_next, got_logits, got_hidden = out["next"].cpu().numpy(), out["logits"].cpu().numpy(), out["hidden"].cpu().numpy()
    want_next, want_logits, want_hidden = orun.run_model(m, head, layers, b.seqs, ids, pool, np.float32)
    _, want_logits_b, want_hidden_b = orun.run_model(m, head, layers, b.seqs, ids, pool_b, np.float32, bf16_activations=True)
    assert rel_err(got_hidden, want_hidden) <= TOL, rel_err(got_hidden, want_hidden)
    assert rel_err(got_logits, want_logits) <= TOL, rel_err(got_logits, want_logits)
    assert row_score(got_logits, want_logits_b, TOL, 0.0) <= 1.0
    _check_tokens(got_next, got_logits, want_logits, str(spec))
    # the step without optional outputs picks the same tokens
    out2 = eng.step_tokens(b.seqs, ids, want_logits=False)
    eng.ctx.sync()
    assert np.array_equal(out2["next"].cpu().numpy(), got_next)
    eng.close()


def test_generation_loop_prefill_then_decode_steps():
    """Three requests served the way an instance serves them: one step prefills the prompts, every further step
    feeds each request the token it generated and appends to its pages.  The oracle gets the same token ids (the
    device's own picks), so that both sides stay on one trajectory; logits and picks are compared at every step and
    the caches at the end."""
    m, vocab, n_layers, n_steps = W.MODELS["tiny"], 256, 2, 7
    prompts = [20, 7, 33]
    rng = np.random.Generator(np.random.PCG64(77))
    need = [(p + n_steps + 15) // 16 for p in prompts]
    perm = rng.permutation(sum(need) + 5).astype(np.int32)
    pages, at = [], 0
    for k in need:
        pages.append(perm[at:at + k].copy())
        at += k
    layers = [W.layer_weights(m, 13, l) for l in range(n_layers)]
    head = W.head_weights(m, vocab, 13)
    eng = Engine(m, len(perm), n_layers, n_layers, max_position=64)
    for l, w in enumerate(layers):
        eng.load_layer(l, w)
    eng.load_head(head)
    pool = orun.make_pool(m, len(perm), n_layers)
    ids = W.token_ids(vocab, sum(prompts), 3)
    kv = list(prompts)
    for step in range(n_steps):
        seqs = [W.SeqSpec(req_id=100 + i, n_new=(prompts[i] if step == 0 else 1), kv_len=kv[i], pages=pages[i]) for i in range(3)]
        out = eng.step_tokens(seqs, ids)
        eng.ctx.sync()
        got_next, got_logits = out["next"].cpu().numpy(), out["logits"].cpu().numpy()
        _, want_logits, _ = orun.run_model(m, head, layers, seqs, ids, pool, np.float32)
        assert rel_err(got_logits, want_logits) <= TOL, (step, rel_err(got_logits, want_logits))
        _check_tokens(got_next, got_logits, want_logits, f"step {step}")
        ids = got_next.astype(np.int32)      # each request continues with the token it generated
        kv = [k + 1 for k in kv]
    # the caches hold the same keys and values after the loop (up to one bf16 rounding flip)
    for i in range(3):
        n = prompts[i] + n_steps - 1
        for l in range(n_layers):
            k, v = eng.read_kv(l, pages[i], 0, n)
            wk, wv = pool.gather(l, [int(p) for p in pages[i]], n)
            for g, w in ((k, wk), (v, wv)):
                g64, w64 = obf.from_bits(g).astype(np.float64), np.asarray(w, dtype=np.float64)
                assert np.all(np.abs(g64 - w64) <= 2.0 ** -7 * np.abs(w64) + 2e-2 * np.sqrt(np.mean(w64 * w64)))
    eng.close()


def test_equal_logits_pick_the_lowest_index():
    # an output matrix with repeated columns gives bit-identical logits in different tiles, wavefronts and blocks
    b = W.custom_batch("tiny", 3, 0, 0, [9, 40], name="ties")
    m = W.MODELS["tiny"]
    vocab = 512
    head = W.head_weights(m, vocab, 5)
    base = head["w_out"][:, :8].copy()
    head["w_out"] = np.tile(base, (1, vocab // 8))       # column j == column j % 8
    eng = Engine(m, b.n_pool_pages, 1, 1, max_position=64)
    eng.load_layer(0, W.layer_weights(m, 1, 0))
    eng.load_head(head)
    eng.load_prefixes(b)
    out = eng.step_tokens(b.seqs, W.token_ids(vocab, b.n_tokens, 1))
    eng.ctx.sync()
    lg, nxt = out["logits"].cpu().numpy(), out["next"].cpu().numpy()
    assert np.array_equal(lg, np.tile(lg[:, :8], (1, vocab // 8)))
    assert np.all(nxt < 8) and np.array_equal(nxt, np.argmax(lg[:, :8], axis=1))
    eng.close()


def test_model_step_state_and_range_errors():
    b = W.custom_batch("tiny", 3, 0, 0, [9], name="err")
    m = W.MODELS["tiny"]
    eng = Engine(m, b.n_pool_pages, 2, 1, max_position=64)
    for l in range(2):
        eng.load_layer(l, W.layer_weights(m, 1, l))
    eng.load_prefixes(b)
    eng.vocab = 128
    with pytest.raises(B.PolystepError) as e:
        eng.step_tokens(b.seqs, [0])
    assert e.value.status == B.PS_ESTATE            # no head yet
    bad = W.head_weights(m, 128, 5)
    dev = {k: bits_to_dev(v, eng.device) for k, v in bad.items()}
    with pytest.raises(B.PolystepError) as e:
        eng.ctx.init_head(dev["embedding"].data_ptr(), dev["g_final"].data_ptr(), dev["w_out"].data_ptr(), 100)
    assert e.value.status == B.PS_EINVAL            # vocabulary not a multiple of 64
    eng.load_head(bad)
    for tok in (-1, 128):
        with pytest.raises(B.PolystepError) as e:
            eng.step_tokens(b.seqs, [tok])
        assert e.value.status == B.PS_ERANGE
    eng.ctx.set_option("only_layer", 1)
    with pytest.raises(B.PolystepError) as e:
        eng.step_tokens(b.seqs, [5])
    assert e.value.status == B.PS_ESTATE
    eng.ctx.set_option("only_layer", -1)
    out = eng.step_tokens(b.seqs, [5], want_parts=True)
    assert len(out["parts_ms"]) == 3 and all(x >= 0 for x in out["parts_ms"])
    eng.close()
