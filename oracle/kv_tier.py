"""CPU oracle for the KV-cache movement.  TEST INFRASTRUCTURE ONLY (see
layer_math.py for who may import this package).

What the paper fixes (section 4.2 "Tiered KV cache buffering" and the
re-sharding paragraph with its figure; section 5.2 "Bandwidth-aware KV cache
layout"):
  * during swap-out every GPU pushes the shard it holds under the prefill
    layout into one CPU store shared by all GPUs; the shards together form
    the complete cache;
  * during swap-in every GPU pulls the shard it needs under the decode layout;
  * the CPU store keeps each K and V tensor as (num_heads, seq_len, head_dim),
    because tensor parallelism slices along heads.
Paging, the order of the outer dimensions, and the allocation policy are not
in the paper; the readings used here are spelled out next to each function.

All movement is written as the index formula applied element by element (numpy
fancy indexing over the full index grid): pure copies on arrays of any dtype,
so results are compared bit for bit.
"""
import numpy as np


# --------------------------------------------------------------------------
# host tier: canonical complete cache
# --------------------------------------------------------------------------
def tier_index(n_kv, d, s, l, c, g, p, e):
    """Element offset, relative to the sequence's base, of (layer l, c in {0:K,
    1:V}, kv head g, position p, element e) for a sequence of exactly s tokens.
    Per (layer, K|V) the block is heads x seq_len x head_dim."""
    return (((l * 2 + c) * n_kv + g) * s + p) * d + e


def tier_seq_elems(n_layers, n_kv, d, s):
    return n_layers * 2 * n_kv * s * d


def _grid(layers, heads, s, d):
    l = np.arange(*layers)[:, None, None, None, None]
    c = np.arange(2)[None, :, None, None, None]
    g = np.arange(*heads)[None, None, :, None, None]
    p = np.arange(s)[None, None, None, :, None]
    e = np.arange(d)[None, None, None, None, :]
    return l, c, g, p, e


def tier_put(tier, base, content, n_kv, layers, heads):
    """Swap-out of one sequence's shard: content [n_layers_local, 2,
    n_heads_local, s, d] holds layers [layers[0], layers[1]) and kv heads
    [heads[0], heads[1]) and lands at its place in the complete cache."""
    s, d = content.shape[3], content.shape[4]
    l, c, g, p, e = _grid(layers, heads, s, d)
    tier[base + tier_index(n_kv, d, s, l, c, g, p, e)] = content


def tier_get(tier, base, s, n_kv, d, layers, heads):
    """Swap-in of one sequence's shard: the inverse gather."""
    l, c, g, p, e = _grid(layers, heads, s, d)
    return tier[base + tier_index(n_kv, d, s, l, c, g, p, e)]


class TierAllocator:
    """Placement of sequence slots in the host tier: first fit at the lowest
    free address; a released block merges with free neighbours.  A sequence that
    fits nowhere means the tier is full (the paper's trigger for leaving the
    prefill phase); once every live sequence is released the tier is one free
    block again and placement restarts at 0 (the trigger for leaving decode).
    Keeping holes reusable lets the swap-out of one batch overlap the drain of
    the previous one."""

    def __init__(self, capacity_elems):
        self.capacity = capacity_elems
        self.free = [(0, capacity_elems)]        # sorted (offset, length)
        self.base = {}

    @property
    def used(self):
        return sum(n for _, n in self.base.values())

    def place(self, seq, elems):
        if seq in self.base:
            return self.base[seq][0]
        for j, (off, length) in enumerate(self.free):
            if length >= elems:
                self.free[j:j + 1] = [(off + elems, length - elems)] if length > elems else []
                self.base[seq] = (off, elems)
                return off
        raise MemoryError("host tier full")

    def release(self, seq):
        off, elems = self.base.pop(seq)
        blocks = sorted(self.free + [(off, elems)])
        merged = [blocks[0]]
        for o, n in blocks[1:]:
            po, pn = merged[-1]
            if po + pn == o:
                merged[-1] = (po, pn + n)
            else:
                merged.append((o, n))
        self.free = merged


# --------------------------------------------------------------------------
# device staging format used by the export / import entry points
# --------------------------------------------------------------------------
def staging_offsets(lens, n_layers_local, n_heads_local, d):
    """Element offset of every sequence in a staging buffer laid out as
    [seq][layer_local][K|V][head_local][position][d], sequences back to back at
    their exact lengths."""
    per_tok = n_layers_local * 2 * n_heads_local * d
    return np.concatenate([[0], np.cumsum(np.asarray(lens, dtype=np.int64) * per_tok)])


# --------------------------------------------------------------------------
# paged device store (logical model)
# --------------------------------------------------------------------------
class PageAllocator:
    """Deterministic policy: the free list starts as 0,1,2,...; an allocation
    takes the lowest free page id; freed pages return to the list, which is
    kept sorted.  A sequence of s tokens owns ceil(s/page) pages, appended in
    order as it grows."""

    def __init__(self, n_pages, page_size=16):
        self.page_size = page_size
        self.free = list(range(n_pages))
        self.tables = {}

    def pages_needed(self, length):
        return -(-length // self.page_size)

    def ensure(self, seq, length):
        table = self.tables.setdefault(seq, [])
        need = self.pages_needed(length) - len(table)
        if need > len(self.free):
            raise MemoryError("page pool exhausted")
        for _ in range(max(need, 0)):
            table.append(self.free.pop(0))
        return table

    def release(self, seq):
        pages = self.tables.pop(seq)
        self.free = sorted(self.free + pages)


class PagedStore:
    """Logical paged cache of one shard: token p of a sequence lives in page
    table[p // page] at slot p % page, the same page id in every local layer
    and for K and V."""

    def __init__(self, n_pages, n_layers_local, n_heads_local, d, dtype, page_size=16):
        self.alloc = PageAllocator(n_pages, page_size)
        self.pool = np.zeros((n_layers_local, 2, n_pages, n_heads_local, page_size, d), dtype=dtype)
        self.lens = {}

    def write(self, seq, content, start=0):
        """content [n_layers_local, 2, n_heads_local, n, d] -> positions start..start+n-1."""
        n = content.shape[3]
        table = self.alloc.ensure(seq, start + n)
        ps = self.alloc.page_size
        for j in range(n):
            p = start + j
            self.pool[:, :, table[p // ps], :, p % ps, :] = content[:, :, :, j, :]
        self.lens[seq] = max(self.lens.get(seq, 0), start + n)

    def read(self, seq):
        s = self.lens[seq]
        table = self.alloc.tables[seq]
        ps = self.alloc.page_size
        out = np.zeros(self.pool.shape[:2] + (self.pool.shape[3], s, self.pool.shape[5]),
                       dtype=self.pool.dtype)
        for p in range(s):
            out[:, :, :, p, :] = self.pool[:, :, table[p // ps], :, p % ps, :]
        return out

    def release(self, seq):
        self.alloc.release(seq)
        del self.lens[seq]


def reshard(src_store, dst_store, tier, tier_alloc, seqs, n_layers, n_kv, d,
            src_layers, src_heads, dst_layers, dst_heads):
    """Swap-out under the source layout followed by swap-in under the target
    layout, sequence by sequence.  Only what the source wrote can be pulled:
    the caller is responsible for all source shards having pushed first."""
    for seq in seqs:
        s = src_store.lens[seq]
        base = tier_alloc.place(seq, tier_seq_elems(n_layers, n_kv, d, s))
        tier_put(tier, base, src_store.read(seq), n_kv, src_layers, src_heads)
    for seq in seqs:
        s = src_store.lens[seq]
        base = tier_alloc.base[seq][0]
        dst_store.write(seq, tier_get(tier, base, s, n_kv, d, dst_layers, dst_heads))
