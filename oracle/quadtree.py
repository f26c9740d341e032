"""Oracle for the paper's own batch generator: quad-tree + Density First Search.

TEST INFRASTRUCTURE ONLY: one flat table of requests and range queries over
it; every counter is recomputed from the table on every query; shares no code
with the C++ library.

Paper Section 3.3.  In-flight requests live in the leaves of a quad-tree keyed
on prefix length.  Every internal node covers a range of prefix lengths that
is split into four equal sub-ranges for its children and carries a
(request counter, block counter) pair describing its sub-tree.  Algorithm 1
(Density First Search) produces one batch: starting at the root,
  case 1  the sub-tree fits the block budget B_max and holds at least K_min
          requests            -> the whole sub-tree is the batch;
  case 2  it exceeds B_max    -> descend into the child with the largest
          request counter;
  case 3  it fits but holds fewer than K_min requests -> widen with requests
          of the nearest siblings (left siblings if there are any, scanned
          from the nearest outwards; otherwise the right siblings), stopping
          at the first request that would exceed the remaining block budget,
          and keep at most K_min - |batch| of them.
Section 4.1: the tree covers prefix lengths [1, 65536], longer prefixes are
treated as 65536; B_max = 40 % of the GPU's blocks, K_min = 36.
Section 3.5 (starvation): every internal node remembers when its sub-tree last
produced a batch; a sub-tree whose age exceeds a threshold is served first.

Readings where the paper is silent (listed in the design notes):
  * leaf width is a parameter (default 16 tokens = one KV block);
  * requests inside a node are ordered by (length, id); a scan "from the
    nearest" walks the left siblings in descending and the right siblings in
    ascending (length, id) order;
  * equal request counters: the leftmost child wins;
  * case 2 at a leaf (no children to descend into): requests are taken in
    ascending order while they fit B_max, and at least one is taken;
  * case 3 widens on one side only, as the paper's algorithm states it: the
    left siblings if the node has any (even empty ones), else the right ones;
  * a starving sub-tree is served by starting the search at that node: the
    non-empty internal node with the largest age above the threshold (ties:
    the deeper, then the leftmost node); the node where a search ends and all
    its ancestors are stamped with the current time; a node is also stamped
    when the first request arrives in its empty sub-tree.

Pins (tests/test_oracle_quadtree.py): three hand-worked trees, one per case
(tests/golden/quadtree_cases.json), and invariants over random inputs (block
budget respected, case-1 batches are whole sub-trees, case-3 batches have at
most K_min members and come from one parent's children, every request is
emitted exactly once).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Tuple


@dataclass
class Request:
    id: int
    length: int     # clamped prefix length, the tree key
    blocks: int


@dataclass(frozen=True)
class Span:
    """A node of the quad-tree, named by the inclusive range of prefix lengths
    it covers.  The tree is implicit: a span of width w > leaf_width has four
    children of width w / 4; the root is [1, max_len]."""
    lo: int
    hi: int
    max_len: int
    leaf_width: int

    @property
    def width(self) -> int:
        return self.hi - self.lo + 1

    def is_leaf(self) -> bool:
        return self.width == self.leaf_width

    @property
    def depth(self) -> int:
        d, w = 0, self.max_len
        while w > self.width:
            w //= 4
            d += 1
        return d

    @property
    def children(self) -> List["Span"]:
        if self.is_leaf():
            return []
        q = self.width // 4
        return [Span(self.lo + i * q, self.lo + (i + 1) * q - 1, self.max_len, self.leaf_width) for i in range(4)]

    @property
    def parent(self) -> Optional["Span"]:
        if self.width == self.max_len:
            return None
        w = self.width * 4
        lo = 1 + (self.lo - 1) // w * w
        return Span(lo, lo + w - 1, self.max_len, self.leaf_width)

    @property
    def slot(self) -> int:
        """Position among the parent's four children (0 = leftmost)."""
        return (self.lo - 1) // self.width % 4

    def holds(self, length: int) -> bool:
        return self.lo <= length <= self.hi


class QuadTree:
    def __init__(self, max_len: int = 65536, leaf_width: int = 16):
        if max_len < leaf_width or leaf_width < 1:
            raise ValueError("bad tree geometry")
        span = max_len
        while span > leaf_width:
            if span % 4:
                raise ValueError("max_len / leaf_width must be a power of four")
            span //= 4
        if span != leaf_width:
            raise ValueError("max_len / leaf_width must be a power of four")
        self.max_len = max_len
        self.leaf_width = leaf_width
        self.root = Span(1, max_len, max_len, leaf_width)
        self.table: Dict[int, Request] = {}              # every request in the tree, by id
        self.served: Dict[Tuple[int, int], float] = {}   # (lo, hi) of a node -> time stamp (Section 3.5)
        self.last_case = None        # 1, 2 (leaf overflow) or 3: how the last batch ended
        self.last_node: Optional[Span] = None

    # -- the table and the counters derived from it ------------------------
    def clamp(self, length: int) -> int:
        return max(1, min(int(length), self.max_len))

    def collect(self, node: Span) -> List[Request]:
        """The requests whose key falls in the node's range, in ascending (length, id)."""
        return sorted((r for r in self.table.values() if node.holds(r.length)), key=lambda r: (r.length, r.id))

    def request_counter(self, node: Span) -> int:
        return len(self.collect(node))

    def block_counter(self, node: Span) -> int:
        return sum(r.blocks for r in self.collect(node))

    def _path(self, key: int) -> List[Span]:
        """Root-to-leaf chain of the nodes whose range holds `key`."""
        chain, node = [self.root], self.root
        while not node.is_leaf():
            node = next(c for c in node.children if c.holds(key))
            chain.append(node)
        return chain

    def insert(self, rid: int, length: int, blocks: int, now: float = 0.0) -> None:
        if rid in self.table:
            raise ValueError(f"request {rid} is already in the tree")
        if blocks < 1 or length < 1:
            raise ValueError("length and blocks must be positive")
        key = self.clamp(length)
        for node in self._path(key):
            if self.request_counter(node) == 0:
                self.served[(node.lo, node.hi)] = now    # age counts from the first arrival
        self.table[rid] = Request(rid, key, int(blocks))

    def remove(self, rid: int) -> None:
        del self.table[rid]

    def __len__(self) -> int:
        return len(self.table)

    # -- one batch (Section 3.3) --------------------------------------------
    def _widen(self, node: Span, budget: int, want: int) -> List[Request]:
        """Case 3: up to `want` requests of the node's siblings, nearest in prefix length first,
        ending at the first one whose blocks no longer fit `budget`."""
        parent = node.parent
        if parent is None:
            return []
        family = self.collect(parent)
        if node.slot > 0:      # there are siblings to the left: only they are searched, longest first
            pool = [r for r in reversed(family) if r.length < node.lo]
        else:                  # leftmost child: the siblings to the right, shortest first
            pool = [r for r in family if r.length > node.hi]
        taken: List[Request] = []
        for r in pool:
            if len(taken) == want or r.blocks > budget:
                break
            taken.append(r)
            budget -= r.blocks
        return taken

    def _search(self, node: Span, b_max: int, k_min: int) -> List[Request]:
        while True:
            own = self.collect(node)
            load = sum(r.blocks for r in own)
            if load > b_max and not node.is_leaf():
                # case 2: too many blocks here -> the child that holds the most requests (leftmost on ties)
                node = max(node.children, key=lambda c: (self.request_counter(c), -c.lo))
                continue
            self.last_node = node
            if load > b_max:
                # case 2 with nothing below: requests in order while they fit, never fewer than one
                self.last_case = 2
                batch, room = [], b_max
                for r in own:
                    if batch and r.blocks > room:
                        break
                    batch.append(r)
                    room -= r.blocks
                return batch
            if len(own) >= k_min:
                self.last_case = 1                       # case 1: fits and is large enough
                return own
            self.last_case = 3                           # case 3: fits but is too small
            return own + self._widen(node, b_max - load, k_min - len(own))

    def _starving(self, now: float, threshold: float) -> Optional[Span]:
        """The non-empty internal node that has waited longest beyond the threshold
        (ties: the deeper one, then the leftmost)."""
        seen, best = set(), None
        for r in self.table.values():
            for node in self._path(r.length)[:-1]:       # internal nodes only
                if (node.lo, node.hi) in seen:
                    continue
                seen.add((node.lo, node.hi))
                age = now - self.served.get((node.lo, node.hi), 0.0)
                if age > threshold:
                    rank = (age, node.depth, -node.lo)
                    if best is None or rank > best[0]:
                        best = (rank, node)
        return None if best is None else best[1]

    def next_batch(self, b_max: int, k_min: int, now: float = 0.0,
                   starve_after: Optional[float] = None) -> List[int]:
        """Generate one batch, remove its requests from the tree, return their
        ids in emission order ([] when the tree is empty)."""
        if not self.table:
            return []
        start = self.root
        if starve_after is not None:
            start = self._starving(now, starve_after) or self.root
        batch = self._search(start, b_max, k_min)
        node = self.last_node
        while node is not None:                          # the node where the search ended, and its ancestors
            self.served[(node.lo, node.hi)] = now
            node = node.parent
        for r in batch:
            self.remove(r.id)
        return [r.id for r in batch]


def dfs_batches(kv_lens, blocks, b_max: int, k_min: int, max_len: int = 65536, leaf_width: int = 16):
    """All requests inserted, then batches generated until the tree is empty.
    Returns (order, batch_offsets) like the sort-and-chunk batcher."""
    t = QuadTree(max_len, leaf_width)
    for i, (l, b) in enumerate(zip(kv_lens, blocks)):
        t.insert(i, int(l), int(b))
    order, offsets = [], [0]
    while len(t):
        ids = t.next_batch(b_max, k_min)
        order.extend(ids)
        offsets.append(len(order))
    return order, offsets
