"""Seeded synthetic inputs for the mixed-batch serving step.

This module only draws numbers and lays them out; it contains none of the
step's arithmetic and is the one piece shared by the HIP path's tests, the
benchmark and the CPU oracle's tests.  bfloat16 values are produced by torch's
own float32 -> bfloat16 cast and handed around as uint16 bit patterns.

The shapes follow the model family the paper evaluates (Sec. 5.1, "Model and
GPU": an 8B-parameter GQA decoder) and its batch structure (Sec. 2.4: all
running decodes plus one prefill chunk).  Request lengths stand in for the
paper's traces (Table 1), which are not redistributable here: decode KV lengths
are uniform or log-normal, the chunk sits at a given prefix offset.
"""
from dataclasses import dataclass, field

import numpy as np
import torch

PAGE = 16

MODELS = {
    # hidden, q heads, kv heads, head_dim, ffn, rope base, layers
    "tiny": dict(hidden=256, n_q=4, n_kv=2, head_dim=64, ffn=704, rope_base=10000.0, n_layers=1),
    "8b": dict(hidden=4096, n_q=32, n_kv=8, head_dim=128, ffn=14336, rope_base=500000.0, n_layers=1),
    "70b": dict(hidden=8192, n_q=64, n_kv=8, head_dim=128, ffn=28672, rope_base=500000.0, n_layers=80),
}
RMS_EPS = 1e-5
WEIGHT_STD = 0.02


def _to_bf16_bits(x_f32):
    t = torch.from_numpy(np.ascontiguousarray(x_f32, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def normal_bf16(rng, shape, std=1.0):
    """N(0, std^2) samples rounded to bfloat16, as uint16 bit patterns."""
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return _to_bf16_bits(x)


def head_weights(model, vocab, seed, std=WEIGHT_STD):
    """Embedding table [vocab][hidden] ~ N(0, 1) (the scale of the configurations' input activations),
    final gain 1, output matrix [hidden][vocab] ~ N(0, std^2); bf16 bit patterns."""
    rng = np.random.Generator(np.random.PCG64([int(seed), 86028121, int(vocab)]))
    H = model["hidden"]
    return {"embedding": normal_bf16(rng, (vocab, H)), "g_final": _to_bf16_bits(np.ones(H, dtype=np.float32)),
            "w_out": normal_bf16(rng, (H, vocab), std)}


def token_ids(vocab, n, seed, tag=0):
    rng = np.random.Generator(np.random.PCG64([int(seed), 49979687, int(tag)]))
    return rng.integers(0, vocab, size=n, dtype=np.int32)


def layer_weights(model, seed, layer=0, std=WEIGHT_STD):
    """bfloat16 N(0, std^2) weights (std 0.02 by default) in math layout [in][out]; unit gains."""
    m = MODELS[model] if isinstance(model, str) else model
    rng = np.random.Generator(np.random.PCG64([int(seed), 7919, int(layer)]))
    H, nq, nkv, d, F = m["hidden"], m["n_q"], m["n_kv"], m["head_dim"], m["ffn"]
    one = np.uint16(0x3F80)
    return {
        "w_qkv": normal_bf16(rng, (H, (nq + 2 * nkv) * d), std),
        "w_o": normal_bf16(rng, (nq * d, H), std),
        "w_gate": normal_bf16(rng, (H, F), std),
        "w_up": normal_bf16(rng, (H, F), std),
        "w_down": normal_bf16(rng, (F, H), std),
        "g_attn": np.full(H, one, dtype=np.uint16),
        "g_ffn": np.full(H, one, dtype=np.uint16),
    }


@dataclass
class SeqSpec:
    req_id: int
    n_new: int
    kv_len: int
    pages: np.ndarray            # int32 physical page ids, len = ceil(kv_len/16)

    @property
    def prefix(self):
        return self.kv_len - self.n_new


@dataclass
class Batch:
    model: str
    seed: int
    seqs: list
    n_pool_pages: int
    name: str = ""
    _rng_tag: int = 0
    extra: dict = field(default_factory=dict)

    @property
    def n_tokens(self):
        return sum(s.n_new for s in self.seqs)

    @property
    def total_kv(self):
        return sum(s.kv_len for s in self.seqs)

    def activations(self):
        """Token activations [T][hidden], bfloat16 bits of N(0,1)."""
        rng = np.random.Generator(np.random.PCG64([self.seed, 104729, self._rng_tag]))
        return normal_bf16(rng, (self.n_tokens, MODELS[self.model]["hidden"]))

    def prefix_kv(self, s, slot=0):
        """Cached keys and values of sequence index s: two [prefix][n_kv][d]
        arrays of bfloat16 bits, N(0,1).  `slot` varies the draw per KV layer slot."""
        m = MODELS[self.model]
        sq = self.seqs[s]
        rng = np.random.Generator(np.random.PCG64([self.seed, 1299709, self._rng_tag, s, slot]))
        shape = (sq.prefix, m["n_kv"], m["head_dim"])
        return normal_bf16(rng, shape), normal_bf16(rng, shape)


def _assign_pages(rng, n_new_kv, slack=0.125, min_extra=3):
    """Give every sequence distinct pages from one permutation of the pool."""
    need = [(L + PAGE - 1) // PAGE for _, L in n_new_kv]
    total = sum(need)
    n_pool = total + max(min_extra, int(total * slack))
    perm = rng.permutation(n_pool).astype(np.int32)
    seqs, at = [], 0
    for i, ((n, L), k) in enumerate(zip(n_new_kv, need)):
        seqs.append(SeqSpec(req_id=1000 + i, n_new=int(n), kv_len=int(L), pages=perm[at:at + k].copy()))
        at += k
    return seqs, n_pool


def lognormal_lengths(rng, n, median, sigma, lo, hi):
    """Log-normal lengths with the given median, clipped to [lo, hi], rounded to int."""
    x = np.exp(np.log(float(median)) + sigma * rng.standard_normal(n))
    return np.rint(np.clip(x, lo, hi)).astype(np.int64)


def custom_batch(model, seed, chunk, chunk_prefix, decode_kv, name="custom", tag=0):
    """One prefill chunk (chunk = 0 for none) at prefix `chunk_prefix`, then one
    decode token per entry of decode_kv (each the KV length after the step)."""
    rng = np.random.Generator(np.random.PCG64([int(seed), 15485863, int(tag)]))
    spec = []
    if chunk > 0:
        spec.append((int(chunk), int(chunk_prefix) + int(chunk)))
    spec += [(1, int(L)) for L in decode_kv]
    seqs, n_pool = _assign_pages(rng, spec)
    return Batch(model=model, seed=int(seed), seqs=seqs, n_pool_pages=n_pool, name=name, _rng_tag=int(tag))


def multi_batch(model, seed, chunks, decode_kv, name="multi", tag=0):
    """Several prefill chunks in one iteration (the budget shared by more than one prefill request,
    Sec. 4.7 of the paper's dynamic-chunking discussion) plus decodes.  chunks: (n_new, prefix) per
    prefill request; decode_kv: KV length after the step per decode request.  The order is the one
    given: chunks first, then decodes."""
    rng = np.random.Generator(np.random.PCG64([int(seed), 15485863, int(tag), 1]))
    spec = [(int(n), int(p) + int(n)) for n, p in chunks] + [(1, int(L)) for L in decode_kv]
    seqs, n_pool = _assign_pages(rng, spec)
    return Batch(model=model, seed=int(seed), seqs=seqs, n_pool_pages=n_pool, name=name, _rng_tag=int(tag))


def config_batch(cfg, seed=0):
    """The benchmark configurations, by index.

    0  tiny layer: 64-token chunk at prefix 64 + decodes with KV lengths 17, 64, 100, 128
    1  8B layer: 64 decodes, KV lengths uniform in [512, 4096]
    2  8B layer: 512-token chunk at prefix 2048 + 128 decodes, KV log-normal
       (median 1024, sigma 0.8) clipped to [16, 8192]
    4  70B layer shape: 1024-token chunk at prefix 4096 + 256 decodes, KV
       log-normal (median 2048, sigma 0.8) clipped to [16, 16384]
    (3 is the latency grid: see grid_cell_batch.)
    """
    rng = np.random.Generator(np.random.PCG64([int(seed), 32452843, int(cfg)]))
    if cfg == 0:
        return custom_batch("tiny", seed, 64, 64, [17, 64, 100, 128], name="cfg0")
    if cfg == 1:
        kv = rng.integers(512, 4096, size=64, endpoint=True)
        return custom_batch("8b", seed, 0, 0, kv, name="cfg1")
    if cfg == 2:
        kv = lognormal_lengths(rng, 128, 1024, 0.8, 16, 8192)
        return custom_batch("8b", seed, 512, 2048, kv, name="cfg2")
    if cfg == 4:
        kv = lognormal_lengths(rng, 256, 2048, 0.8, 16, 16384)
        return custom_batch("70b", seed, 1024, 4096, kv, name="cfg4")
    raise ValueError("cfg must be 0, 1, 2 or 4")


GRID_CHUNKS = (0, 128, 256, 512, 1024, 2048)
GRID_DECODES = (0, 16, 64, 256)
GRID_SEEDS = (0, 1, 2, 3, 4)


def grid_cell_lengths(chunk, n_decode, seed):
    """(chunk prefix offset, decode KV lengths) of one latency-grid cell draw:
    offset uniform integer in [0, 4096]; decode lengths log-normal (median 1024,
    sigma 0.8) clipped to [16, 8192]."""
    rng = np.random.Generator(np.random.PCG64([int(seed), 49979687, int(chunk), int(n_decode)]))
    off = int(rng.integers(0, 4096, endpoint=True)) if chunk > 0 else 0
    kv = lognormal_lengths(rng, n_decode, 1024, 0.8, 16, 8192)
    return off, kv


def grid_cell_batch(chunk, n_decode, seed, model="8b"):
    off, kv = grid_cell_lengths(chunk, n_decode, seed)
    return custom_batch(model, seed, chunk, off, kv, name=f"grid_c{chunk}_d{n_decode}", tag=chunk * 1000 + n_decode)


SIM_TPOTS_MS = (20.0, 30.0, 50.0, 100.0)
SIM_TTFTS_MS = (300.0, 500.0, 1000.0)
SIM_TIER_PROBS = (0.1, 0.2, 0.3, 0.4)


def sim_trace(seed, n, rate_per_ms, max_prompt, max_output, burst=False):
    """Synthetic request trace of the paper's kind (Sec. 5.1, 5.3): Poisson arrivals at rate_per_ms, input lengths
    uniform in [1, max_prompt] and output lengths uniform in [1, max_output] (`uniform_512_512` = 1024 / 1024,
    `uniform_4096_1024` = 8192 / 2048), TTFT drawn uniformly from 300 / 500 / 1000 ms, TPOT tier 20 / 30 / 50 / 100 ms
    with probabilities 10 / 20 / 30 / 40 %; burst: the second half of the requests draws the tiers with the
    probabilities reversed.  Returns plain lists."""
    rng = np.random.Generator(np.random.PCG64([int(seed), 67867967, int(n)]))
    arrival = np.cumsum(rng.exponential(1.0 / float(rate_per_ms), n))
    prompt = rng.integers(1, max_prompt, size=n, endpoint=True)
    output = rng.integers(1, max_output, size=n, endpoint=True)
    ttft = rng.choice(np.array(SIM_TTFTS_MS), size=n)
    tier = rng.choice(len(SIM_TPOTS_MS), size=n, p=SIM_TIER_PROBS)
    if burst:
        late = rng.choice(len(SIM_TPOTS_MS), size=n, p=SIM_TIER_PROBS[::-1])
        tier[n // 2:] = late[n // 2:]
    return {"arrival": arrival.tolist(), "prompt": prompt.tolist(), "output": output.tolist(), "ttft": ttft.tolist(),
            "tier": tier.tolist()}
