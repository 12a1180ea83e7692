"""Convenience wrapper used by the tests, the smoke entry and the benchmark: owns a library
context plus the torch tensors (device memory only) that feed it.  All computation happens in
libpolystep; torch allocates buffers and moves bytes."""
import numpy as np
import torch

from . import binding as B
from . import workloads as W


def bits_to_dev(bits, device):
    """uint16 bf16 bit patterns (numpy) -> int16 device tensor holding the same bits."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device)


def dev_to_bits(t):
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


class Engine:
    def __init__(self, model, n_pool_pages, n_layers=1, n_kv_layers=1, max_position=None, perm_seed=0, device="cuda:0"):
        if not torch.cuda.is_available():
            raise RuntimeError("Engine needs a GPU: there is no CPU fallback")
        self.model = dict(W.MODELS[model]) if isinstance(model, str) else dict(model)
        m = self.model
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.stream = torch.cuda.current_stream(self.device)
        self.n_layers = n_layers
        if max_position is None:
            max_position = 16 * n_pool_pages
        self.ctx = B.Context(m["hidden"], m["n_q"], m["n_kv"], m["head_dim"], m["ffn"], n_layers, max_position,
                             W.RMS_EPS, m["rope_base"], stream=self.stream.cuda_stream)
        self.ctx.kv_alloc(n_pool_pages, n_kv_layers, perm_seed)
        self.n_pool_pages = n_pool_pages

    def close(self):
        self.ctx.destroy()

    def load_layer(self, layer, weights_bits):
        dev = {k: bits_to_dev(v, self.device) for k, v in weights_bits.items()}
        self.ctx.init_layer(layer, **{k: t.data_ptr() for k, t in dev.items()})
        self.ctx.sync()

    def load_head(self, head_bits):
        """head_bits: {"embedding" [vocab][hidden], "g_final" [hidden], "w_out" [hidden][vocab]} as bf16 bit patterns."""
        dev = {k: bits_to_dev(v, self.device) for k, v in head_bits.items()}
        self.vocab = int(head_bits["embedding"].shape[0])
        self.ctx.init_head(dev["embedding"].data_ptr(), dev["g_final"].data_ptr(), dev["w_out"].data_ptr(), self.vocab)
        self.ctx.sync()

    def step_tokens(self, seqs, token_ids, want_logits=True, want_hidden=False, want_stats=False, want_parts=False):
        """Full-model step.  Returns dict with "next" (int32 tensor [n_seqs]), optionally "logits" (fp32
        [n_seqs][vocab]) and "hidden" (fp32 [T][hidden]), "stats", "parts_ms"."""
        n, T = len(seqs), sum(int(s.n_new) for s in seqs)
        out = {"next": torch.empty(n, dtype=torch.int32, device=self.device)}
        if want_logits:
            out["logits"] = torch.empty((n, self.vocab), dtype=torch.float32, device=self.device)
        if want_hidden:
            out["hidden"] = torch.empty((T, self.model["hidden"]), dtype=torch.float32, device=self.device)
        out["stats"], out["parts_ms"] = self.ctx.step_tokens(
            seqs, token_ids, out["next"].data_ptr(), out["logits"].data_ptr() if want_logits else None,
            out["hidden"].data_ptr() if want_hidden else None, want_stats, want_parts)
        return out

    def write_kv(self, layer, pages, pos0, k_bits, v_bits):
        n = k_bits.shape[0]
        if n == 0:
            return
        k, v = bits_to_dev(k_bits, self.device), bits_to_dev(v_bits, self.device)
        self.ctx.kv_write(layer, pages, pos0, n, k.data_ptr(), v.data_ptr())
        self.ctx.sync()

    def read_kv(self, layer, pages, pos0, n):
        m = self.model
        k = torch.empty((n, m["n_kv"], m["head_dim"]), dtype=torch.int16, device=self.device)
        v = torch.empty_like(k)
        self.ctx.kv_read(layer, pages, pos0, n, k.data_ptr(), v.data_ptr())
        self.ctx.sync()
        return dev_to_bits(k), dev_to_bits(v)

    def load_prefixes(self, batch, layer=0, slot_tag=0):
        for i, s in enumerate(batch.seqs):
            if s.prefix > 0:
                k, v = batch.prefix_kv(i, slot_tag)
                self.write_kv(layer, s.pages, 0, k, v)

    def alloc_taps(self, T):
        m = self.model
        i16 = dict(dtype=torch.int16, device=self.device)
        return {
            "xn": torch.zeros((T, m["hidden"]), **i16),
            "q": torch.zeros((T, m["n_q"], m["head_dim"]), **i16),
            "attn": torch.zeros((T, m["n_q"] * m["head_dim"]), **i16),
            "x1": torch.zeros((T, m["hidden"]), dtype=torch.float32, device=self.device),
            "xn2": torch.zeros((T, m["hidden"]), **i16),
            "act": torch.zeros((T, m["ffn"]), **i16),
            "x_in": torch.zeros((T, m["hidden"]), dtype=torch.float32, device=self.device),
            "x_out": torch.zeros((T, m["hidden"]), dtype=torch.float32, device=self.device),
        }

    def step(self, seqs, x_dev, out_dev=None, want_stats=False):
        """x_dev: int16 device tensor [T][hidden] of bf16 bits.  Returns (out_dev, stats)."""
        if out_dev is None:
            out_dev = torch.empty_like(x_dev)
        stats = self.ctx.step(seqs, x_dev.data_ptr(), out_dev.data_ptr(), want_stats)
        return out_dev, stats
