"""Integer side of a serving step (test infrastructure; exactly one right answer).

A step batches, per Sec. 2.4 ("Prefill-Decode Disaggregation and Chunked
Prefill"), every running decode request (one new token each) with a chunk of
prefill tokens.  Each sequence s in the batch is described by

    n_new[s]    tokens fed this step (1 for a decode, the chunk size for a prefill)
    kv_len[s]   attended span AFTER the step, the new tokens included
    pages[s]    physical page ids; logical token position p lives in
                page pages[s][p // 16], slot p % 16

so the cached prefix is kv_len - n_new and the new tokens sit at positions
prefix ... kv_len-1.  A decode is the n_new = 1 case: each decode iteration feeds
the one token generated last (Sec. 2.1).
"""
import numpy as np

PAGE = 16
_MASK64 = (1 << 64) - 1


def cu_seqlens(n_new):
    """Exclusive prefix sum of new-token counts, length n_seqs + 1."""
    out = np.zeros(len(n_new) + 1, dtype=np.int32)
    for s, n in enumerate(n_new):
        out[s + 1] = out[s] + int(n)
    return out


def positions(n_new, kv_len):
    """Logical position of every new token, sequences concatenated in order."""
    out = []
    for n, L in zip(n_new, kv_len):
        prefix = int(L) - int(n)
        for i in range(int(n)):
            out.append(prefix + i)
    return np.asarray(out, dtype=np.int32)


def slot_mapping(n_new, kv_len, pages):
    """Flat cache slot (page id * 16 + position % 16) of every new token."""
    out = []
    for n, L, pt in zip(n_new, kv_len, pages):
        prefix = int(L) - int(n)
        for i in range(int(n)):
            p = prefix + i
            out.append(int(pt[p // PAGE]) * PAGE + p % PAGE)
    return np.asarray(out, dtype=np.int32)


def pages_needed(kv_len):
    return (int(kv_len) + PAGE - 1) // PAGE


class SplitMix64:
    """splitmix64 (Steele, Lea & Flood 2014; Vigna's public-domain reference)."""

    def __init__(self, seed):
        self.state = int(seed) & _MASK64

    def next(self):
        self.state = (self.state + 0x9E3779B97F4A7C15) & _MASK64
        z = self.state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
        return z ^ (z >> 31)


class PageAllocator:
    """Seeded page allocator.

    The free list starts as the Fisher-Yates shuffle of 0..n_pages-1 driven by
    splitmix64(seed): for i = n_pages-1 down to 1, j = next() mod (i+1), swap
    entries i and j.  reserve() pops from the front, in call order, until the
    request owns ceil(kv_len/16) pages; release() appends the request's pages to
    the back in the order they were handed out.
    """

    def __init__(self, n_pages, seed):
        order = list(range(int(n_pages)))
        rng = SplitMix64(seed)
        for i in range(len(order) - 1, 0, -1):
            j = rng.next() % (i + 1)
            order[i], order[j] = order[j], order[i]
        self.free = order
        self.head = 0
        self.owned = {}

    def n_free(self):
        return len(self.free) - self.head

    def reserve(self, req_id, kv_len):
        """Grow req_id to cover kv_len tokens; returns its full page list or
        None (state unchanged) when the pool cannot cover the growth."""
        have = self.owned.get(req_id, [])
        need = pages_needed(kv_len) - len(have)
        if need > self.n_free():
            return None
        if need > 0:
            have = have + self.free[self.head:self.head + need]
            self.head += need
        self.owned[req_id] = have
        return list(have)

    def release(self, req_id):
        pages = self.owned.pop(req_id)
        self.free.extend(pages)
