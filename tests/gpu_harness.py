"""Shared code of the GPU parity tests: run one batch through libpolystep and through the
oracle on the same seeded inputs, and compare."""
import numpy as np
import torch

from oracle import bf16 as obf
from oracle import run as orun
from paper_2507_17769_amd import workloads as W
from paper_2507_17769_amd.runner import Engine, bits_to_dev, dev_to_bits

# max |gpu - oracle| <= TOL * RMS(oracle tensor): the stated bound for bf16 inputs with fp32 accumulate
TOL = 2e-2


def f32(bits):
    return obf.from_bits(bits, np.float32)


def rel_err(got, want):
    want = np.asarray(want, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    rms = float(np.sqrt(np.mean(want * want))) or 1.0
    return float(np.max(np.abs(got - want))) / rms if want.size else 0.0


# Against the oracle variant that rounds activations to bf16 in the same places as the kernels,
# what is left is fp32 summation order, exp2-vs-exp, the bf16 rounding of the softmax weights
# (up to 2^-8 relative per weight, coherent across a row's head_dim outputs) and rounding flips:
# a stored activation that lands on the other side of a bf16 rounding boundary differs by a whole
# ulp, and a handful of such flips in the input row of a GEMM moves a small output row by about
# 1e-2 of its RMS.  Which elements flip depends on the summation order, i.e. on the attention split
# plan and the GEMM split, so intermediates are held to the stated factor per row, not to less.
TIGHT = TOL


def row_score(got, want, tol=TOL, ulps=1.0):
    """Intermediates, judged per token row: max_ij |err_ij| / (tol * RMS(row i) + ulps * 2^-8 * |want_ij|).
    2^-8 |v| is half a bf16 ulp at the bottom of a binade: `ulps` = 1 allows for the rounding that
    storing a tensor as bf16 adds no matter how it was computed, 2 for one rounding flip between two
    bf16 tensors, 0 for fp32 tensors.  A score <= 1 passes.  Rows are the unit because tokens differ
    widely in scale (a token that attends to one key carries a raw value vector, one that attends
    to thousands an average of them)."""
    want = np.asarray(want, dtype=np.float64)
    want = want.reshape(len(want), -1)
    got = np.asarray(got, dtype=np.float64).reshape(want.shape)
    if want.size == 0:
        return 0.0
    rms = np.sqrt(np.mean(want * want, axis=1, keepdims=True))
    rms = np.where(rms > 0, rms, 1.0)
    allow = tol * rms + ulps * 2.0 ** -8 * np.abs(want)
    return float(np.max(np.abs(got - want) / allow))


def bf16_ulp_distance(a_bits, b_bits):
    """Distance in representable bf16 values (sign-magnitude order)."""
    def key(b):
        b = b.astype(np.int32)
        return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)
    return np.abs(key(a_bits) - key(b_bits))


class Case:
    """One batch on both sides.  After run(): self.err maps tensor name -> max|err|/RMS."""

    def __init__(self, batch, n_layers=1, n_kv_layers=1, weight_seed=0, options=None, model_override=None,
                 weight_std=W.WEIGHT_STD):
        self.batch = batch
        self.model = model_override or W.MODELS[batch.model]
        self.n_layers, self.n_kv_layers = n_layers, n_kv_layers
        self.layers = [W.layer_weights(self.model, weight_seed, l, weight_std) for l in range(n_layers)]
        self.eng = Engine(self.model, batch.n_pool_pages, n_layers, n_kv_layers,
                          max_position=max(16 * 8, max(s.kv_len for s in batch.seqs) + 16))
        for k, v in (options or {}).items():
            self.eng.ctx.set_option(k, v)
        for l, w in enumerate(self.layers):
            self.eng.load_layer(l, w)
        self.pool = orun.make_pool(self.model, batch.n_pool_pages, n_kv_layers)
        # cached prefixes: same bits to both sides, one draw per physical KV slot
        for slot in range(n_kv_layers):
            for i, s in enumerate(batch.seqs):
                if s.prefix > 0:
                    k, v = batch.prefix_kv(i, slot)
                    self.eng.write_kv(slot, s.pages, 0, k, v)
                    self.pool.write_bits(slot, [int(p) for p in s.pages], 0, k, v)
        self.x_bits = batch.activations()

    def run(self, tap_layer=0, dtype=np.float32, tight=TIGHT):
        """tight: per-row tolerance against the bf16-activation variant of the oracle."""
        b, eng = self.batch, self.eng
        T = b.n_tokens
        taps = eng.alloc_taps(T)
        eng.ctx.set_taps(tap_layer, **{k: t.data_ptr() for k, t in taps.items()})
        x_dev = bits_to_dev(self.x_bits, eng.device)
        # the step twice (it is idempotent for a fixed batch): fp32 output with taps, then bf16 output
        out32_dev = torch.empty((T, self.model["hidden"]), dtype=torch.float32, device=eng.device)
        eng.ctx.set_option("out_f32", 1)
        _, self.stats = eng.step(b.seqs, x_dev, out32_dev, want_stats=True)
        eng.ctx.sync()
        eng.ctx.set_taps(0)
        eng.ctx.set_option("out_f32", 0)
        out_dev, _ = eng.step(b.seqs, x_dev)
        eng.ctx.sync()
        self.out_bits = dev_to_bits(out_dev)
        self.out32 = out32_dev.cpu().numpy()
        # the bf16 output is the fp32 output rounded once, nothing else
        assert np.array_equal(self.out_bits, obf.to_bits(self.out32)), "bf16 x_out is not RNE(fp32 x_out)"
        import copy
        pool_b = self.pool_b = copy.deepcopy(self.pool)
        want, otaps = orun.run_step(self.model, self.layers, b.seqs, self.x_bits, self.pool, dtype, want_taps=True)
        want_b, otaps_b = orun.run_step(self.model, self.layers, b.seqs, self.x_bits, pool_b, dtype, want_taps=True,
                                        bf16_activations=True)
        self.want, self.want_b = want, want_b
        ot, otb = otaps[tap_layer], otaps_b[tap_layer]
        got = {k: f32(dev_to_bits(taps[k])) for k in ("xn", "q", "attn", "xn2", "act")}
        got["x1"] = taps["x1"].cpu().numpy()
        got["out"] = self.out32
        self.got = got
        ot["out"], otb["out"] = want, want_b
        # final output against the definition: the stated bar, max |err| <= TOL x RMS over the whole
        # tensor, for the fp32 output; the bf16 output additionally carries its own storage rounding
        # (half a bf16 ulp of each value), which alone is > TOL/2 x RMS on the largest elements
        w64 = np.asarray(want, dtype=np.float64)
        rms = float(np.sqrt(np.mean(w64 * w64))) or 1.0
        self.err = {"out": rel_err(self.out32, want),
                    "out_bf16": float(np.max(np.abs(f32(self.out_bits) - w64) / (TOL * rms + 2.0 ** -8 * np.abs(w64)))) * TOL}
        self.score = {}
        for k, v in got.items():
            fp32_tensor = k in ("x1", "out")
            # vs the definition: reported, and enforced only at ten times the bar as a gross-error
            # catch (a 200-token chunk at prefix 1000 on the 8B shape reached 6.5 times the bar on one
            # attention row while agreeing with the bf16-activation variant within the bar itself).
            # The rounding of the bf16 tensors an intermediate is computed FROM is not
            # proportional to its own size: a softmax over ~100 effective keys turns 2^-9 relative
            # noise on q into several percent of a (small) attention output row, and silu(g)*u is
            # heavy-tailed.  The definition evaluated with bf16 activations shows the same deviations.
            self.score[k] = 0.1 * row_score(v, ot[k], TOL, 0.0 if fp32_tensor else 2.0)
            # vs the same arithmetic with bf16 activations: a rounding flip (one ulp) plus TIGHT
            self.score[k + "|bf16"] = row_score(v, otb[k], tight, 0.0 if fp32_tensor else 2.0)
        if tap_layer == 0:
            # the attention branch on its own scale: x1 - x against the O-projection output
            ob = got["x1"].astype(np.float64) - f32(self.x_bits)
            self.score["o_branch"] = 0.1 * row_score(ob, ot["o"], TOL, 0.0)
            self.score["o_branch|bf16"] = row_score(ob, otb["o"], TOL, 0.0)
        self.err.update({k + ":score": v * TOL for k, v in self.score.items()})
        return self.err

    def check_pool(self):
        """Cache contents after the step.  Every slot that the step did not write is bit-identical
        to the oracle's pool (prefix and untouched pages alike).  Appended keys and values: against
        the oracle variant with bf16 activations they are one bf16 rounding of the same fp32
        arithmetic, so they agree up to one rounding flip (one bf16 ulp of the value, 2^-7 relative,
        plus 3e-3 x RMS for entries that cancel to near zero: the normalised input itself carries bf16
        rounding flips against the oracle's, each moving a sum by about 2^-8 / sqrt(hidden) of its RMS;
        over 480 random batches the largest excess seen was 2.3e-3 x RMS, on one entry);
        against the definition they are held
        to the floating-point bar.  Returns the fraction of appended entries that differ at all from
        the bf16-activation variant."""
        eng, b = self.eng, self.batch
        all_pages = np.arange(b.n_pool_pages, dtype=np.int32)
        new_mask = np.zeros(b.n_pool_pages * 16, dtype=bool)
        for s in b.seqs:
            for p in range(s.prefix, s.kv_len):
                new_mask[int(s.pages[p // 16]) * 16 + p % 16] = True
        worst = 0.0
        for slot in range(self.n_kv_layers):
            k, v = eng.read_kv(slot, all_pages, 0, b.n_pool_pages * 16)
            for which, got, name in ((0, k, "K"), (1, v, "V")):
                want = self.pool.bits[slot, :, which].reshape(b.n_pool_pages * 16, *got.shape[1:])
                want_b = self.pool_b.bits[slot, :, which].reshape(want.shape)
                assert np.array_equal(got[~new_mask], want[~new_mask]), f"{name}: a slot outside the append set changed"
                if not new_mask.any():
                    continue
                g = f32(got[new_mask]).astype(np.float64)
                w, wb = f32(want[new_mask]).astype(np.float64), f32(want_b[new_mask]).astype(np.float64)
                assert row_score(g, w, TOL, 2.0) <= 1.0, f"{name}: appended entries off the definition"
                if slot > 0:      # deeper layers see inputs that already differ by earlier flips
                    assert row_score(g, wb, TOL, 2.0) <= 1.0, f"{name}: appended entries off (slot {slot})"
                    continue
                rms = float(np.sqrt(np.mean(wb * wb))) or 1.0
                over = np.abs(g - wb) - (2.0 ** -7 * np.abs(wb) + 3e-3 * rms)
                assert over.max() <= 0, f"{name}: appended entries differ by more than one bf16 rounding flip"
                worst = max(worst, float(np.mean(g != wb)))
        return worst

    def stagewise(self, tol=1e-2):
        """Every stage of layer 0 on its own: the oracle's step applied to the tensors the kernels
        actually produced as that stage's input (read back through the taps and ps_kv_read), so
        that no deviation is carried from one stage into the next.  Needs run() first (taps on layer
        0, one layer).  Returns name -> row_score at `tol` (<= 1 passes); bf16 tensors get one
        rounding flip on top."""
        from oracle import layer as ol
        sh = orun.shape_from(self.model)
        b, g, w = self.batch, self.got, orun.widen_weights(self.layers[0], np.float64)
        seqs = orun.to_seqs(b.seqs)
        nq, nkv, d = sh.n_q, sh.n_kv, sh.head_dim
        T = b.n_tokens
        x = f32(self.x_bits).astype(np.float64)
        pos = np.concatenate([np.arange(s.kv_len - s.n_new, s.kv_len) for s in seqs])
        rt = lambda a: obf.round_trip(a.astype(np.float32)).astype(np.float64)
        out = {}
        out["xn<-x"] = row_score(g["xn"], rt(ol.rmsnorm(x, w["g_attn"], sh.rms_eps)), tol, 2.0)
        qkv = g["xn"].astype(np.float64) @ w["w_qkv"]
        q = rt(ol.rope(qkv[:, :nq * d].reshape(T, nq, d), pos, sh.rope_base))
        out["q<-xn"] = row_score(g["q"].reshape(T, -1), q.reshape(T, -1), tol, 2.0)
        # attention over the cache as the device holds it after the step
        pool = orun.make_pool(self.model, b.n_pool_pages, 1)
        all_pages = np.arange(b.n_pool_pages, dtype=np.int32)
        k, v = self.eng.read_kv(0, all_pages, 0, b.n_pool_pages * 16)
        pool.write_bits(0, [int(p) for p in all_pages], 0, k, v)
        attn = rt(ol.attention_paged(g["q"].astype(np.float64).reshape(T, nq, d), seqs, pool, 0, nkv))
        out["attn<-q,cache"] = row_score(g["attn"].reshape(T, -1), attn.reshape(T, -1), tol, 2.0)
        o = g["attn"].astype(np.float64).reshape(T, nq * d) @ w["w_o"]
        out["o<-attn"] = row_score(g["x1"].astype(np.float64) - x, o, tol, 0.0)
        out["xn2<-x1"] = row_score(g["xn2"], rt(ol.rmsnorm(g["x1"].astype(np.float64), w["g_ffn"], sh.rms_eps)), tol, 2.0)
        xn2 = g["xn2"].astype(np.float64)
        act = rt(ol.silu(xn2 @ w["w_gate"]) * (xn2 @ w["w_up"]))
        out["act<-xn2"] = row_score(g["act"], act, tol, 2.0)
        f = g["act"].astype(np.float64) @ w["w_down"]
        out["ffn<-act"] = row_score(g["out"].astype(np.float64) - g["x1"].astype(np.float64), f, tol, 0.0)
        return out

    def close(self):
        self.eng.close()
