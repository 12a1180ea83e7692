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


# ---------------------------------------------------------------------------------------------------
# The tolerance rule, the same for every case (nothing below is switched by what a case happens to show):
#
#  R   the layer of Sec. 2.1 as the oracle defines it (rounding to bf16 only at the cache write);
#  R_b the same definition with the operands of its contractions in bf16, which is what "bf16 inputs,
#      fp32 accumulate" means for a layer whose matrix units take bf16: the normalised inputs, the
#      rotated queries, the attention output and the gated activation are rounded where they are
#      produced (oracle: bf16_activations=True).
#
#  (A) final output, whole tensor:  max|got - R_b| <= TOL x RMS(R_b)
#  (B) final output against R:       max|got - R|   <= TOL x RMS(R) + gap,  gap = max|R_b - R| computed
#      on the CPU from the two oracle runs of that case (no kernel involved); (B) follows from (A) by the
#      triangle inequality and is asserted as a guard of the harness itself.
#  (C) every stage on its own, per token row: the oracle's stage applied to the tensors the kernels actually
#      produced as that stage's input; max over the row |got - want| <= TOL x RMS(row), plus one bf16 ulp of
#      the value for tensors stored as bf16 (a value on the other side of a rounding boundary).  Rows are the
#      unit because tokens differ widely in scale (a token that attends to one key carries a raw value
#      vector, one that attends to thousands an average of them).
#  (D) appended keys and values, from the normalised input the kernels produced: one bf16 rounding flip plus
#      the rounding-error bound of an fp32 sum of K products, K x 2^-23 x (|A| |W|) elementwise.
#  End-to-end deviations of the intermediates from R_b and R are reported (Case.report), not asserted:
#  they are the stage's own deviation (C) plus what the oracle's stage makes of its input's deviation.
# ---------------------------------------------------------------------------------------------------


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
                 weight_std=W.WEIGHT_STD, guard=True):
        """guard: the library fills its workspaces with bf16 NaN before every step, the harness does the same with
        every output and tap buffer, and the pool gets one more page at either end, filled with a seeded pattern that
        no sequence owns (the batch's page ids are shifted by one): a kernel that reads what the step has not written,
        or writes a page too far at either end of the pool, fails the comparisons that follow."""
        self.guard = guard
        if guard:
            import dataclasses
            batch = dataclasses.replace(batch, seqs=[dataclasses.replace(s, pages=(np.asarray(s.pages) + 1).astype(np.int32)) for s in batch.seqs],
                                        n_pool_pages=batch.n_pool_pages + 2)
        self.batch = batch
        self.model = model_override or W.MODELS[batch.model]
        self.n_layers, self.n_kv_layers = n_layers, n_kv_layers
        self.layers = [W.layer_weights(self.model, weight_seed, l, weight_std) for l in range(n_layers)]
        self.eng = Engine(self.model, batch.n_pool_pages, n_layers, n_kv_layers,
                          max_position=max(16 * 8, max(s.kv_len for s in batch.seqs) + 16))
        if guard:
            self.eng.ctx.set_option("poison_workspaces", 1)
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
        if guard:   # the two pages nobody owns
            rng = np.random.default_rng(12345)
            m = self.model
            for slot in range(n_kv_layers):
                for page in (0, batch.n_pool_pages - 1):
                    k = rng.integers(0, 0x7F80, size=(16, m["n_kv"], m["head_dim"])).astype(np.uint16)
                    v = rng.integers(0, 0x7F80, size=(16, m["n_kv"], m["head_dim"])).astype(np.uint16)
                    self.eng.write_kv(slot, np.array([page], dtype=np.int32), 0, k, v)
                    self.pool.write_bits(slot, [page], 0, k, v)
        self.x_bits = batch.activations()

    def run(self, tap_layer=0, dtype=np.float32, stages=True):
        """Runs the step on the device (fp32 output with taps on `tap_layer`, then bf16 output) and both oracle
        evaluations.  Returns self.err: name -> value that passes when <= TOL (rules A, B of the header, the bf16
        output, and with `stages` the per-stage rows of rule C and the appended cache entries of rule D)."""
        b, eng = self.batch, self.eng
        T = b.n_tokens
        self.tap_layer = tap_layer
        taps = eng.alloc_taps(T)
        if self.guard:
            for t in taps.values():
                t.fill_(float("nan") if t.dtype == torch.float32 else 0x7FC0)
        eng.ctx.set_taps(tap_layer, **{k: t.data_ptr() for k, t in taps.items()})
        x_dev = bits_to_dev(self.x_bits, eng.device)
        # the step twice (it is idempotent for a fixed batch): fp32 output with taps, then bf16 output
        out32_dev = torch.full((T, self.model["hidden"]), float("nan"), dtype=torch.float32, device=eng.device)
        eng.ctx.set_option("out_f32", 1)
        _, self.stats = eng.step(b.seqs, x_dev, out32_dev, want_stats=True)
        eng.ctx.sync()
        eng.ctx.set_taps(0)
        eng.ctx.set_option("out_f32", 0)
        out_dev, _ = eng.step(b.seqs, x_dev, torch.full_like(x_dev, 0x7FC0))
        eng.ctx.sync()
        self.out_bits = dev_to_bits(out_dev)
        self.out32 = out32_dev.cpu().numpy()
        assert np.isfinite(self.out32).all() and np.isfinite(f32(self.out_bits)).all(), "NaN in the step's output"
        for k in ("xn", "q", "attn", "xn2", "act", "x1"):
            tv = taps[k].cpu().numpy()
            assert np.isfinite(tv if tv.dtype == np.float32 else f32(tv.view(np.uint16))).all(), f"NaN in the {k} tap: something read an unwritten buffer"

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
        got["x_in"] = taps["x_in"].cpu().numpy() if tap_layer > 0 else f32(self.x_bits)
        last = tap_layer == self.n_layers - 1
        got["out"] = self.out32 if last else taps["x_out"].cpu().numpy()
        self.got = got
        ot["out"], otb["out"] = (want, want_b) if last else (ot["out"], otb["out"])
        w64, wb64 = np.asarray(want, dtype=np.float64), np.asarray(want_b, dtype=np.float64)
        rms = float(np.sqrt(np.mean(w64 * w64))) or 1.0
        rms_b = float(np.sqrt(np.mean(wb64 * wb64))) or 1.0
        self.gap = float(np.max(np.abs(wb64 - w64))) / rms if w64.size else 0.0
        self.err = {
            # (A) against the definition with bf16 contraction operands
            "out": rel_err(self.out32, want_b),
            # (B) against the plain definition: what is left of the distance after the CPU-only gap between the two
            "out_vs_plain_minus_gap": max(0.0, rel_err(self.out32, want) - self.gap),
            # the bf16 output additionally carries its own storage rounding (half a bf16 ulp of each value)
            "out_bf16": float(np.max(np.abs(f32(self.out_bits) - wb64) / (TOL * rms_b + 2.0 ** -8 * np.abs(wb64)))) * TOL,
        }
        # end-to-end deviations of the intermediates, per token row, in units of the bar: reported only
        self.report = {"out_vs_plain": rel_err(self.out32, want), "gap_plain_vs_bf16_operands": self.gap}
        for k in ("xn", "q", "attn", "x1", "xn2", "act", "out"):
            ulps = 0.0 if k in ("x1", "out") else 2.0
            self.report[k + "|rows_vs_bf16_operands"] = row_score(got[k], otb[k], TOL, ulps)
            self.report[k + "|rows_vs_plain"] = row_score(got[k], ot[k], TOL, ulps)
        if stages:
            for k, v in self.stagewise().items():
                self.err["stage " + k] = v * TOL
        return self.err

    def slot_is_intact(self):
        """The tapped layer's KV slot still holds what that layer appended (no later layer of an aliased stack wrote it)."""
        return self.tap_layer + self.n_kv_layers >= self.n_layers

    def check_pool(self):
        """Cache contents after the step.  Every slot that the step did not write is bit-identical to the oracle's
        pool (prefix and untouched pages alike).  Appended keys and values against both oracle evaluations, per
        token row at the bar plus one bf16 rounding flip (they are bf16 roundings of fp32 sums; rule D in run()
        holds them tighter, from the kernels' own normalised input).  Returns the fraction of appended entries that
        differ at all from the evaluation with bf16 operands."""
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
                assert row_score(g, wb, TOL, 2.0) <= 1.0, f"{name}: appended entries off the definition with bf16 operands (slot {slot})"
                gap = np.abs(wb - w).reshape(len(w), -1).max(axis=1, keepdims=True)
                rms = np.sqrt(np.mean(w.reshape(len(w), -1) ** 2, axis=1, keepdims=True))
                allow = TOL * np.where(rms > 0, rms, 1.0) + gap + 2.0 ** -7 * np.abs(w.reshape(len(w), -1))
                assert np.all(np.abs(g - w).reshape(len(w), -1) <= allow), f"{name}: appended entries off the plain definition (slot {slot})"
                worst = max(worst, float(np.mean(g != wb)))
        return worst

    def kv_sum_bounds(self):
        """Rounding-error bound of the fp32 sums behind the appended keys and values, elementwise [T][n_kv][d]:
        any order of summing K products in fp32 stays within K x 2^-23 x sum |a_k| |w_k| of the exact sum (2^-23
        covers adders that truncate).  A rotated key entry is a combination of a pair (j, j + d/2) with
        |cos|, |sin| <= 1, so its bound is the sum of the pair's."""
        sh = orun.shape_from(self.model)
        nq, nkv, d, T = sh.n_q, sh.n_kv, sh.head_dim, self.batch.n_tokens
        w = orun.widen_weights(self.layers[self.tap_layer], np.float64)["w_qkv"][:, nq * d:]
        xn = self.got["xn"].astype(np.float64)
        bound = (sh.hidden * 2.0 ** -23) * (np.abs(xn) @ np.abs(w))      # [T][2 nkv d]
        kb = bound[:, :nkv * d].reshape(T, nkv, d)
        kb = kb + np.concatenate([kb[..., d // 2:], kb[..., :d // 2]], axis=-1)
        # the rotation itself in fp32 with fp32 sines and cosines: two products and a sum, each rounded, on factors
        # that are themselves rounded: a few 2^-24 of |lo| + |hi|
        ka = np.abs((xn @ w[:, :nkv * d]).reshape(T, nkv, d))
        kb = kb + 2.0 ** -21 * (ka + np.concatenate([ka[..., d // 2:], ka[..., :d // 2]], axis=-1))
        return kb, bound[:, nkv * d:].reshape(T, nkv, d)

    def stagewise(self, tol=TOL):
        """Rule C: every stage of the tapped layer on its own, the oracle's stage applied to the tensors the kernels
        actually produced as that stage's input (read back through the taps and ps_kv_read), so that no deviation
        is carried from one stage into the next; and rule D for the appended keys and values.  Needs run() first.
        Returns name -> row score at `tol` (<= 1 passes); bf16 tensors get one rounding flip on top."""
        from oracle import layer as ol
        sh = orun.shape_from(self.model)
        b, g, w = self.batch, self.got, orun.widen_weights(self.layers[self.tap_layer], np.float64)
        seqs = orun.to_seqs(b.seqs)
        nq, nkv, d = sh.n_q, sh.n_kv, sh.head_dim
        T = b.n_tokens
        x = g["x_in"].astype(np.float64)
        pos = np.concatenate([np.arange(s.kv_len - s.n_new, s.kv_len) for s in seqs])
        rt = lambda a: obf.round_trip(a.astype(np.float32)).astype(np.float64)
        out = {}
        out["xn<-x"] = row_score(g["xn"], rt(ol.rmsnorm(x, w["g_attn"], sh.rms_eps)), tol, 2.0)
        xn = g["xn"].astype(np.float64)
        qkv = xn @ w["w_qkv"]
        q = rt(ol.rope(qkv[:, :nq * d].reshape(T, nq, d), pos, sh.rope_base))
        out["q<-xn"] = row_score(g["q"].reshape(T, -1), q.reshape(T, -1), tol, 2.0)
        if self.slot_is_intact():
            slot = self.tap_layer % self.n_kv_layers
            # (D) appended keys and values: bf16(fp32 sum) against bf16(exact sum) of the same operands
            kb, vb = self.kv_sum_bounds()
            k_want = rt(ol.rope(qkv[:, nq * d:(nq + nkv) * d].reshape(T, nkv, d), pos, sh.rope_base))
            v_want = rt(qkv[:, (nq + nkv) * d:].reshape(T, nkv, d))
            worst, t0 = 0.0, 0
            for s in b.seqs:
                kg, vg = self.eng.read_kv(slot, s.pages, s.prefix, s.n_new)
                for got_bits, want_v, bnd in ((kg, k_want, kb), (vg, v_want, vb)):
                    gv, wv, bv = f32(got_bits).astype(np.float64), want_v[t0:t0 + s.n_new], bnd[t0:t0 + s.n_new]
                    worst = max(worst, float(np.max(np.abs(gv - wv) / (2.0 ** -7 * np.abs(wv) + bv + 1e-30))))
                t0 += s.n_new
            out["appended kv<-xn"] = worst
            # attention over the cache as the device holds it after the step
            pool = orun.make_pool(self.model, b.n_pool_pages, 1)
            all_pages = np.arange(b.n_pool_pages, dtype=np.int32)
            k, v = self.eng.read_kv(slot, all_pages, 0, b.n_pool_pages * 16)
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
