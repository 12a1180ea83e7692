"""CPU-side tests of the C-ABI library: it loads, exports what the header declares, and its
host logic (validation, index arrays, allocator, attention work list) agrees bit for bit with
the oracle.  No device is touched: contexts are created host-only."""
import ctypes
import os
import re

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle import indices as oi
from paper_2507_17769_amd import binding as B
from paper_2507_17769_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def host_ctx(model="tiny", max_position=20000):
    m = W.MODELS[model]
    return B.Context(m["hidden"], m["n_q"], m["n_kv"], m["head_dim"], m["ffn"], 1, max_position, 1e-5,
                     m["rope_base"], host_only=True)


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "polystep.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = sorted(set(re.findall(r"\b(ps_[a-z_]+)\s*\(", text)))
    assert declared == B.EXPORTS, (declared, B.EXPORTS)
    for name in declared:
        assert getattr(B.lib, name) is not None


def test_create_rejects_bad_shapes():
    for kw in (dict(head_dim=96), dict(n_q_heads=6, n_kv_heads=4), dict(hidden=100), dict(n_q_heads=12, n_kv_heads=4)):
        args = dict(hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=704)
        args.update(kw)
        with pytest.raises(B.PolystepError) as e:
            B.Context(**args, host_only=True)
        assert e.value.status == B.PS_EINVAL
    d = B.ps_model_desc(256, 4, 2, 64, 704, 1, 8, 128, 1e-5, 1e4, 1)     # page_size 8
    h = ctypes.c_void_p()
    assert B.lib.ps_create(ctypes.byref(d), None, ctypes.byref(h)) == B.PS_EINVAL
    assert b"page_size" in B.lib.ps_last_error(None)


def test_host_only_context_refuses_device_calls():
    c = host_ctx()
    with pytest.raises(B.PolystepError) as e:
        c.step([(1, 1, 1, [0])], 0, 0)
    assert e.value.status == B.PS_ESTATE
    with pytest.raises(B.PolystepError) as e:
        c.init_layer(0, w_qkv=1, w_o=1, w_gate=1, w_up=1, w_down=1, g_attn=1, g_ffn=1)
    assert e.value.status == B.PS_ESTATE


@pytest.mark.parametrize("cfg", [0, 1, 2])
def test_step_indices_match_oracle_on_configs(cfg):
    b = W.config_batch(cfg, seed=3)
    c = host_ctx(b.model)
    cu, pos, slots = c.step_indices(b.seqs)
    n_new = [s.n_new for s in b.seqs]
    kv = [s.kv_len for s in b.seqs]
    pages = [s.pages for s in b.seqs]
    assert np.array_equal(cu, oi.cu_seqlens(n_new))
    assert np.array_equal(pos, oi.positions(n_new, kv))
    assert np.array_equal(slots, oi.slot_mapping(n_new, kv, pages))


@settings(max_examples=150, deadline=None)
@given(st.lists(st.tuples(st.integers(1, 70), st.integers(0, 90)), min_size=0, max_size=7), st.integers(0, 2 ** 32))
def test_step_indices_match_oracle_fuzz(spec, seed):
    n_new = [n for n, _ in spec]
    kv = [n + p for n, p in spec]
    need = [oi.pages_needed(L) for L in kv]
    perm = np.random.default_rng(seed).permutation(sum(need) + 2)
    pages, at = [], 0
    for k in need:
        pages.append(perm[at:at + k].astype(np.int32))
        at += k
    c = host_ctx()
    cu, pos, slots = c.step_indices([(i, n, L, p) for i, (n, L, p) in enumerate(zip(n_new, kv, pages))])
    assert np.array_equal(cu, oi.cu_seqlens(n_new))
    assert np.array_equal(pos, oi.positions(n_new, kv))
    assert np.array_equal(slots, oi.slot_mapping(n_new, kv, pages))


def test_batch_validation_errors():
    c = host_ctx(max_position=256)
    c.kv_alloc(8, 1, 0)                              # host-only pool: allocator state only
    ok = [(1, 4, 20, [0, 1]), (2, 1, 5, [2])]
    c.step_indices(ok)
    cases = [
        ([(1, 0, 5, [0])], B.PS_EINVAL, "n_new"),
        ([(1, 6, 5, [0])], B.PS_EINVAL, "kv_len"),
        ([(1, 1, 257, list(range(8)) * 3)], B.PS_ERANGE, "max_position"),
        ([(1, 1, 17, [0])], B.PS_EINVAL, "shorter"),
        ([(1, 1, 5, [8])], B.PS_ERANGE, "outside"),
        ([(1, 1, 5, [-1])], B.PS_ERANGE, "outside"),
        ([(1, 1, 5, [3]), (2, 1, 5, [3])], B.PS_EINVAL, "twice"),
        ([(1, 1, 20, [3, 3])], B.PS_EINVAL, "twice"),
        ([(1, 1, 5, [3]), (1, 1, 5, [4])], B.PS_EINVAL, "duplicate req_id"),
    ]
    for seqs, status, word in cases:
        with pytest.raises(B.PolystepError) as e:
            c.step_indices(seqs)
        assert e.value.status == status and word in str(e.value), (seqs, str(e.value))
        c.step_indices(ok)                           # a failed call leaves the context usable
    # empty batch is valid
    cu, pos, slots = c.step_indices([])
    assert cu.tolist() == [0] and len(pos) == 0


def test_allocator_matches_oracle_bit_exact():
    rng = np.random.default_rng(5)
    for n_pages, seed in [(29, 0), (64, 2 ** 63 + 5), (1000, 123456789)]:
        c = host_ctx(max_position=1 << 20)
        c.kv_alloc(n_pages, 1, seed)
        o = oi.PageAllocator(n_pages, seed)
        live = {}
        for step in range(300):
            rid = int(rng.integers(0, 12))
            if rid in live and rng.random() < 0.3:
                c.kv_release(rid)
                o.release(rid)
                del live[rid]
            else:
                kv_len = int(live.get(rid, 0) + rng.integers(0, 40))
                want = o.reserve(rid, kv_len)
                if want is None:
                    with pytest.raises(B.PolystepError) as e:
                        c.kv_reserve(rid, kv_len)
                    assert e.value.status == B.PS_ENOMEM
                else:
                    got = c.kv_reserve(rid, kv_len)
                    assert got.tolist() == want
                    live[rid] = kv_len
            assert c.kv_free_pages() == o.n_free()
    with pytest.raises(B.PolystepError) as e:
        c.kv_release(777)
    assert e.value.status == B.PS_EINVAL


TEAM_TILES = 12   # query tiles of a team item: four wavefronts with three tiles each


def _check_plan_covers(b, c, workers=None):
    """Every (sequence, kv head, query token, kv page needed by that token) is covered by exactly
    one work item, ranges start on even pages, partial slots do not collide, items are listed by
    worker, and the workers' KV weights are balanced."""
    m = W.MODELS[b.model]
    G = m["n_q"] // m["n_kv"]
    if workers is not None:
        c.set_option("attn_workers", workers)
    items = c.plan_attention(b.seqs)
    cover = {}
    slots_used = set()
    per_seg = {}
    for seq, h, q0, qn, p0, p1, part, worker in items.tolist():
        s = b.seqs[seq]
        assert 0 <= h < m["n_kv"] and 0 <= q0 and qn >= 1 and q0 + qn <= s.n_new
        need = oi.pages_needed(s.prefix + q0 + qn)
        assert 0 <= p0 < p1 <= need and p0 % 2 == 0
        full = (p0 == 0 and p1 == need)
        assert (part < 0) == full
        per_seg.setdefault((seq, h, q0), []).append((p0, p1, part))
        if part >= 0:
            nt = 1 if s.n_new <= 16 // G else TEAM_TILES
            for k in range(nt):
                assert part + k not in slots_used
                slots_used.add(part + k)
        for q in range(q0, q0 + qn):
            for p in range(p0, p1):
                key = (seq, h, q, p)
                assert key not in cover
                cover[key] = 1
    for si, s in enumerate(b.seqs):
        for h in range(m["n_kv"]):
            for q in {0, s.n_new // 2, s.n_new - 1}:
                for p in range(oi.pages_needed(s.prefix + q + 1)):
                    assert (si, h, q, p) in cover
    assert np.all(np.diff(items[:, 7]) >= 0)                     # listed worker by worker
    for ranges in per_seg.values():                              # splits of a stream tile it in order
        assert all(a[1] == b_[0] for a, b_ in zip(ranges, ranges[1:]))
    return items





def _worker_weights(items, b, G):
    """page pairs per worker, for the team workers (prefill query blocks) and the single-wavefront workers (decodes)"""
    team, wave = {}, {}
    for seq, h, q0, qn, p0, p1, part, worker in items.tolist():
        w = team if b.seqs[seq].n_new > 16 // G else wave
        w[worker] = w.get(worker, 0) + (p1 - p0 + 1) // 2
    assert not team or not wave or max(team) < min(wave)       # team workers come first
    return np.array(list(team.values())), np.array(list(wave.values()))


def test_attention_plan_covers_everything_once():
    c = host_ctx()
    b = W.config_batch(0)
    for workers in (0, 1, 2, 3, 7, 1000):
        _check_plan_covers(b, c, workers)
    b = W.custom_batch("tiny", 1, 37, 1000, [1, 15, 16, 17, 500, 2000], name="odd")
    for workers in (0, 1, 5, 64, 100000):
        _check_plan_covers(b, c, workers)
    c8 = host_ctx("8b")
    for cfg in (1, 2):
        b8 = W.config_batch(cfg)
        items = _check_plan_covers(b8, c8)
        team, wave = _worker_weights(items, b8, 4)
        # all 512 resident blocks are used: a team is one block, four single-wavefront workers share one
        assert len(team) + len(wave) // 4 == 512 and len(wave) % 4 == 0, (len(team), len(wave))
        assert (len(team) > 0) == (cfg == 2)
        for w in (team, wave):
            assert len(w) == 0 or w.max() - w.min() <= 2, (len(w), w.min(), w.max())
