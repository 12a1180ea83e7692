"""Pins for the oracle's integer side: closed forms, a published generator vector,
an independently written shuffle, and randomised structural properties."""
import os

import numpy as np
from hypothesis import given, settings, strategies as st

from oracle import indices
from oracle.indices import PageAllocator, SplitMix64

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_splitmix64_published_vector():
    want = [int(l) for l in open(os.path.join(GOLDEN, "splitmix64_seed1234567.txt")) if l.strip() and not l.startswith("#")]
    r = SplitMix64(1234567)
    assert [r.next() for _ in range(len(want))] == want and len(want) == 5


def test_cu_seqlens_and_positions_closed_forms():
    n_new = [64, 1, 1, 1, 1]
    kv = [128, 17, 64, 100, 128]
    assert indices.cu_seqlens(n_new).tolist() == [0, 64, 65, 66, 67, 68]
    pos = indices.positions(n_new, kv)
    assert pos[:64].tolist() == list(range(64, 128)) and pos[64:].tolist() == [16, 63, 99, 127]
    assert pos.dtype == np.int32 and indices.cu_seqlens([]).tolist() == [0]


def test_slot_mapping_hand_example():
    # KV lengths 17, 64, 100, 128 put the decode token in page slot 0 (fresh page), 15, 3, 15
    pages = [[7, 3], [9, 8, 1, 0], [2, 4, 6, 10, 12, 14, 5], [11, 13, 15, 16, 17, 18, 19, 20]]
    got = indices.slot_mapping([1, 1, 1, 1], [17, 64, 100, 128], pages)
    assert got.tolist() == [3 * 16 + 0, 0 * 16 + 15, 5 * 16 + 3, 20 * 16 + 15]
    # a 5-token chunk straddling a page boundary: positions 14..18
    got = indices.slot_mapping([5], [19], [[40, 2]])
    assert got.tolist() == [40 * 16 + 14, 40 * 16 + 15, 2 * 16 + 0, 2 * 16 + 1, 2 * 16 + 2]


@settings(max_examples=200, deadline=None)
@given(st.lists(st.tuples(st.integers(1, 40), st.integers(0, 70)), min_size=1, max_size=6), st.integers(0, 2 ** 32))
def test_slot_mapping_properties(spec, seed):
    n_new = [n for n, _ in spec]
    kv = [n + p for n, p in spec]
    need = [indices.pages_needed(L) for L in kv]
    perm = np.random.default_rng(seed).permutation(sum(need) + 3)
    pages, at = [], 0
    for k in need:
        pages.append(perm[at:at + k].tolist())
        at += k
    slots = indices.slot_mapping(n_new, kv, pages)
    pos = indices.positions(n_new, kv)
    cu = indices.cu_seqlens(n_new)
    assert len(set(slots.tolist())) == len(slots) == cu[-1]            # all distinct
    for s in range(len(spec)):
        sl, ps = slots[cu[s]:cu[s + 1]], pos[cu[s]:cu[s + 1]]
        assert ps.tolist() == list(range(kv[s] - n_new[s], kv[s]))
        assert all(int(v) // 16 in pages[s] for v in sl)               # inside the sequence's pages
        assert all(int(v) % 16 == int(p) % 16 for v, p in zip(sl, ps))
        assert all(pages[s].index(int(v) // 16) == int(p) // 16 for v, p in zip(sl, ps))


def _second_fisher_yates(n, seed):
    """Written again from the sentence: i from n-1 down to 1, j = next() mod (i+1), swap."""
    state = seed & 0xFFFFFFFFFFFFFFFF
    a = np.arange(n)
    i = n - 1
    while i >= 1:
        state = (state + 0x9E3779B97F4A7C15) % (1 << 64)
        z = state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) % (1 << 64)
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) % (1 << 64)
        z ^= z >> 31
        j = z % (i + 1)
        a[i], a[j] = a[j], a[i]
        i -= 1
    return a.tolist()


def test_allocator_initial_order_vs_second_implementation():
    for n, seed in [(1, 5), (2, 0), (29, 42), (1000, 2 ** 63 + 11)]:
        a = PageAllocator(n, seed)
        assert a.free == _second_fisher_yates(n, seed)
        assert sorted(a.free) == list(range(n))


def test_allocator_shuffle_is_uniform_on_three_pages():
    counts = {}
    for seed in range(6000):
        key = tuple(PageAllocator(3, seed).free)
        counts[key] = counts.get(key, 0) + 1
    assert len(counts) == 6 and min(counts.values()) > 850 and max(counts.values()) < 1150


def test_allocator_reserve_grow_release_semantics():
    a = PageAllocator(10, 7)
    order = list(a.free)
    assert a.reserve(1, 17) == order[0:2]
    assert a.reserve(2, 1) == order[2:3]
    assert a.reserve(1, 32) == order[0:2]                 # already covered: no new page
    assert a.reserve(1, 33) == order[0:2] + order[3:4]    # grows by one, popped from the front
    assert a.n_free() == 6
    assert a.reserve(3, 16 * 7) is None and a.n_free() == 6 and 3 not in a.owned   # all-or-nothing
    a.release(1)
    assert a.n_free() == 9
    got = a.reserve(4, 16 * 9)                             # remaining fresh pages, then the released ones in hand-out order
    assert got == order[4:10] + order[0:2] + order[3:4]
    assert a.n_free() == 0


@settings(max_examples=100, deadline=None)
@given(st.integers(1, 60), st.integers(0, 2 ** 64 - 1),
       st.lists(st.tuples(st.integers(0, 5), st.integers(0, 200), st.booleans()), max_size=30))
def test_allocator_never_double_allocates(n_pages, seed, ops):
    a = PageAllocator(n_pages, seed)
    for rid, kv_len, rel in ops:
        if rel and rid in a.owned:
            a.release(rid)
        else:
            got = a.reserve(rid, kv_len)
            if got is not None:
                assert len(got) >= indices.pages_needed(kv_len)
        held = [p for v in a.owned.values() for p in v]
        free = a.free[a.head:]
        assert sorted(held + free) == list(range(n_pages))
