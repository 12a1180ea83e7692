"""Run the oracle on a batch given as plain arrays (test infrastructure).

Inputs are bf16 bit patterns (uint16) exactly as handed to the GPU path; they are widened to
`dtype` here.  Nothing in this file knows how the inputs were drawn.
"""
import numpy as np

from . import bf16, layer


def shape_from(model):
    return layer.Shape(hidden=model["hidden"], n_q=model["n_q"], n_kv=model["n_kv"], head_dim=model["head_dim"],
                       ffn=model["ffn"], rope_base=model["rope_base"], rms_eps=model.get("rms_eps", 1e-5))


def widen_weights(weights_bits, dtype=np.float32):
    return {k: bf16.from_bits(v, dtype) for k, v in weights_bits.items()}


def make_pool(model, n_pages, n_slots=1):
    return layer.PagedKV(n_pages, n_slots, model["n_kv"], model["head_dim"])


def to_seqs(seqs):
    return [layer.Seq(int(s.n_new), int(s.kv_len), [int(p) for p in s.pages]) for s in seqs]


def run_step(model, layers_bits, seqs, x_bits, pool, dtype=np.float32, want_taps=False, bf16_activations=False):
    """One step over all layers.  Returns (out [T][hidden] in dtype, taps or None)."""
    sh = shape_from(model)
    x = bf16.from_bits(x_bits, dtype)
    ws = [widen_weights(w, dtype) for w in layers_bits]
    taps = {} if want_taps else None
    out = layer.stack_forward(x, ws, to_seqs(seqs), pool, sh, taps, bf16_activations)
    return out, taps


def run_layer_from(model, weights_bits, seqs, x, pool, slot, dtype=np.float32, bf16_activations=False):
    """One layer from a float residual-stream input x [T][hidden] (teacher forcing: x is the
    input the layer actually received inside a deeper stack).  Appends to pool[slot]."""
    sh = shape_from(model)
    return layer.layer_forward(np.asarray(x, dtype=dtype), widen_weights(weights_bits, dtype), to_seqs(seqs), pool, slot, sh,
                               None, bf16_activations)


def run_model(model, head_bits, layers_bits, seqs, token_ids, pool, dtype=np.float32, bf16_activations=False):
    """Full step: token ids -> embedding -> layer stack -> final norm -> logits of every sequence's last
    token -> greedy next token.  head_bits: {"embedding" [vocab][hidden], "g_final" [hidden],
    "w_out" [hidden][vocab]} as bf16 bit patterns.  Returns (next tokens [n_seqs] int32,
    logits [n_seqs][vocab], final hidden states [T][hidden])."""
    from . import head
    sh = shape_from(model)
    hw = widen_weights(head_bits, dtype)
    x = head.embed(token_ids, hw["embedding"])
    ws = [widen_weights(w, dtype) for w in layers_bits]
    sq = to_seqs(seqs)
    hidden = layer.stack_forward(x, ws, sq, pool, sh, None, bf16_activations)
    stored = (lambda a: bf16.round_trip(a.astype(np.float32)).astype(a.dtype)) if bf16_activations else None
    lg = head.logits(hidden, sq, hw["g_final"], hw["w_out"], sh.rms_eps, stored)
    return head.greedy(lg), lg, hidden
