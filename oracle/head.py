"""What surrounds the layer stack in a full serving step (test infrastructure).

Sec. 2.1 ("LLM Inference Workflow"): a request's tokens enter the layers as embedding vectors,
the prefill ends by generating the first output token, and every decode step takes the previous
token and generates the next one until the end of the sequence.  The paper says nothing about
how the token is picked; the reading taken here is the plainest one that makes a step
deterministic:

  * embedding: row `token id` of a [vocab][hidden] table, as stored (bf16 values);
  * after the last layer: RMS normalisation with its own gain (the model family of Sec. 5.1
    ends with one), in `dtype`;
  * logits = normalised hidden state of the sequence's LAST new token times the [hidden][vocab]
    output matrix, no bias; only that token's logits exist, because only it generates a token;
  * next token = the index of the largest logit, the lowest index among equal ones (greedy).

Everything is dense and naive on purpose.
"""
import numpy as np

from . import layer


def embed(token_ids, table):
    """token_ids [T] int -> [T][hidden] rows of `table` ([vocab][hidden], any float dtype)."""
    token_ids = np.asarray(token_ids, dtype=np.int64)
    if token_ids.size and (token_ids.min() < 0 or token_ids.max() >= table.shape[0]):
        raise ValueError("token id outside the vocabulary")
    out = np.empty((len(token_ids), table.shape[1]), dtype=table.dtype)
    for i, t in enumerate(token_ids):
        out[i] = table[t]
    return out


def last_token_rows(seqs):
    """Index, in the concatenated token axis, of the last new token of every sequence."""
    rows, t0 = [], 0
    for s in seqs:
        rows.append(t0 + s.n_new - 1)
        t0 += s.n_new
    return rows


def logits(x, seqs, g_final, w_out, eps, stored=None):
    """x [T][hidden] (output of the last layer) -> [n_seqs][vocab].  `stored`, if given, is applied to the
    normalised rows (the variant that keeps activations in bf16 rounds them there)."""
    rows = x[last_token_rows(seqs)]
    xn = layer.rmsnorm(rows, g_final.astype(x.dtype), eps)
    if stored is not None:
        xn = stored(xn)
    return xn @ w_out.astype(x.dtype)


def greedy(lg):
    """[n][vocab] -> [n] int32: first index of each row's maximum."""
    if lg.shape[1] > 4096:
        return greedy_rows(lg)
    out = np.empty(len(lg), dtype=np.int32)
    for i, row in enumerate(lg):
        best, arg = row[0], 0
        for j in range(1, len(row)):
            if row[j] > best:
                best, arg = row[j], j
        out[i] = arg
    return out


def greedy_rows(lg):
    """Same as greedy() for wide rows: numpy's argmax also returns the first maximum."""
    return np.argmax(lg, axis=1).astype(np.int32)
