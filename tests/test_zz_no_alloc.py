"""ps_step_static, the step for callers that cannot allocate device memory: its buffers are pieces of a device
array that is part of the library image.  It runs the kernels of ps_step, so for the same batch its output and
the cache contents must be bit-identical to ps_step's; the array keeps the previous call's contents, so a second,
smaller call right after a larger one must be just as exact."""
import numpy as np
import pytest
import torch

from paper_2507_17769_amd import binding as B
from paper_2507_17769_amd import workloads as W
from paper_2507_17769_amd.runner import Engine, bits_to_dev, dev_to_bits

pytestmark = pytest.mark.gpu


def _both_ways(eng, batch, x_bits):
    """(output, appended K, appended V) of ps_step and of ps_step_static on the same batch."""
    res = []
    x = bits_to_dev(x_bits, eng.device)
    for static in (False, True):
        out = torch.zeros_like(x)
        if static:
            eng.ctx.step_static(batch.seqs, x.data_ptr(), out.data_ptr())
        else:
            eng.ctx.step(batch.seqs, x.data_ptr(), out.data_ptr())
        eng.ctx.sync()
        kv = [eng.read_kv(l, s.pages, s.prefix, s.n_new) for l in range(eng.n_kv_layers) for s in batch.seqs]
        res.append((dev_to_bits(out), kv))
        # wipe what the step appended, so that the second run cannot pass on the first one's cache writes
        for l in range(eng.n_kv_layers):
            for s in batch.seqs:
                z = np.zeros((s.n_new, eng.model["n_kv"], eng.model["head_dim"]), dtype=np.uint16)
                eng.write_kv(l, s.pages, s.prefix, z, z)
    return res


def _assert_same(res, tag):
    (o0, kv0), (o1, kv1) = res
    assert np.array_equal(o0, o1), f"{tag}: output differs from ps_step"
    for (k0, v0), (k1, v1) in zip(kv0, kv1):
        assert np.array_equal(k0, k1) and np.array_equal(v0, v1), f"{tag}: appended cache entries differ from ps_step"
    assert o0.any(), tag


def test_static_step_matches_ps_step_twice_in_a_row_second_call_smaller():
    m = W.MODELS["tiny"]
    big = W.custom_batch("tiny", 51, 100, 37, [5, 250, 1000], name="static_big")
    small = W.custom_batch("tiny", 52, 0, 0, [3, 40], name="static_small")
    n_layers = 3
    eng = Engine(m, max(big.n_pool_pages, small.n_pool_pages), n_layers, n_layers, max_position=2048)
    eng.n_kv_layers = n_layers
    for l in range(n_layers):
        eng.load_layer(l, W.layer_weights(m, 51, l))
    try:
        for b in (big, small):
            for l in range(n_layers):
                eng.load_prefixes(b, layer=l, slot_tag=l)
            _assert_same(_both_ways(eng, b, b.activations()), b.name)
        # beyond the array: refused before anything is launched, with the sizes in the message
        huge = W.custom_batch("tiny", 53, 70000, 0, [], name="static_huge")
        eng2 = Engine(m, huge.n_pool_pages, 1, 1, max_position=70016)
        eng2.load_layer(0, W.layer_weights(m, 51, 0))
        x = torch.zeros((huge.n_tokens, m["hidden"]), dtype=torch.int16, device=eng2.device)
        with pytest.raises(B.PolystepError) as e:
            eng2.ctx.step_static(huge.seqs, x.data_ptr(), x.data_ptr())
        assert e.value.status == B.PS_ERANGE and "static" in str(e.value)
        eng2.ctx.step_static([], 0, 0)       # an empty step is valid here too
        eng2.close()
    finally:
        eng.close()


def test_static_step_8b_layer_decode_batch_then_a_smaller_one():
    """The 64-decode batch of the 8B-shaped layer (about 40 MiB of the array: split partials of 2048 attention
    workers, six fp32 partial sums of the QKV projection), then 8 decodes on the same context."""
    b = W.config_batch(1, seed=0)
    eng = Engine(b.model, b.n_pool_pages, 1, 1, max_position=max(s.kv_len for s in b.seqs) + 16)
    eng.n_kv_layers = 1
    eng.load_layer(0, W.layer_weights(b.model, 0, 0))
    try:
        eng.load_prefixes(b)
        x_bits = b.activations()
        _assert_same(_both_ways(eng, b, x_bits), "64 decodes")
        import copy
        small = copy.copy(b)
        small.seqs = b.seqs[:8]
        _assert_same(_both_ways(eng, small, x_bits[:8]), "8 decodes")
    finally:
        eng.close()
