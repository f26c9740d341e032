"""Oracle for the paper's own batch generator: quad-tree + Density First Search.

TEST INFRASTRUCTURE ONLY: plain Python objects and recursion, counters
recomputed from scratch on every query; shares no code with the C++ library.

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
  * case 3 follows the listing literally: one side only (left if present);
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

from dataclasses import dataclass, field
from typing import List, Optional


@dataclass
class Request:
    id: int
    length: int     # clamped prefix length, the tree key
    blocks: int


@dataclass
class Node:
    lo: int
    hi: int                      # inclusive range of prefix lengths
    depth: int
    parent: Optional["Node"] = None
    slot: int = 0                # index among the parent's children
    children: List["Node"] = field(default_factory=list)   # empty for a leaf
    requests: List[Request] = field(default_factory=list)  # leaves only
    last_served: float = 0.0

    def is_leaf(self) -> bool:
        return not self.children


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
        self.root = self._build(1, max_len, 0, None, 0)
        self._by_id = {}
        self.last_case = None        # 1, 2 (leaf overflow) or 3: how the last batch ended
        self.last_node = None

    def _build(self, lo, hi, depth, parent, slot) -> Node:
        n = Node(lo=lo, hi=hi, depth=depth, parent=parent, slot=slot)
        width = hi - lo + 1
        if width > self.leaf_width:
            q = width // 4
            n.children = [self._build(lo + i * q, lo + (i + 1) * q - 1, depth + 1, n, i) for i in range(4)]
        return n

    # -- bookkeeping ------------------------------------------------------
    def clamp(self, length: int) -> int:
        return max(1, min(int(length), self.max_len))

    def insert(self, rid: int, length: int, blocks: int, now: float = 0.0) -> None:
        if rid in self._by_id:
            raise ValueError(f"request {rid} is already in the tree")
        if blocks < 1 or length < 1:
            raise ValueError("length and blocks must be positive")
        key = self.clamp(length)
        node = self.root
        while True:
            if self.request_counter(node) == 0:
                node.last_served = now       # age counts from the first arrival
            if node.is_leaf():
                break
            q = (node.hi - node.lo + 1) // 4
            node = node.children[(key - node.lo) // q]
        r = Request(rid, key, int(blocks))
        node.requests.append(r)
        self._by_id[rid] = (r, node)

    def remove(self, rid: int) -> None:
        r, leaf = self._by_id.pop(rid)
        leaf.requests.remove(r)

    def __len__(self) -> int:
        return len(self._by_id)

    def collect(self, node: Node) -> List[Request]:
        """CollectRequests: the sub-tree's requests in ascending (length, id)."""
        if node.is_leaf():
            return sorted(node.requests, key=lambda r: (r.length, r.id))
        out: List[Request] = []
        for c in node.children:
            out.extend(self.collect(c))
        return out

    def request_counter(self, node: Node) -> int:
        return len(self.collect(node))

    def block_counter(self, node: Node) -> int:
        return sum(r.blocks for r in self.collect(node))

    # -- Algorithm 1 ------------------------------------------------------
    def recursive_dfs(self, node: Node, b_max: int, k_min: int) -> List[Request]:
        batch = self.collect(node)
        b_used = sum(r.blocks for r in batch)
        if b_used <= b_max and len(batch) >= k_min:                    # case 1
            self.last_case, self.last_node = 1, node
            return batch
        if b_used > b_max:                                              # case 2
            if node.is_leaf():
                taken, used = [], 0
                for r in batch:          # the first request is always taken
                    if taken and used + r.blocks > b_max:
                        break
                    taken.append(r)
                    used += r.blocks
                self.last_case, self.last_node = 2, node
                return taken
            counts = [self.request_counter(c) for c in node.children]
            c_max = node.children[counts.index(max(counts))]
            return self.recursive_dfs(c_max, b_max, k_min)
        b_left = b_max - b_used                                         # case 3
        k_left = k_min - len(batch)
        addition: List[Request] = []
        if node.parent is not None:
            sibs = node.parent.children
            left, right = sibs[:node.slot], sibs[node.slot + 1:]
            if left:
                addition = self.r_search(left, b_left, k_left)
            else:
                addition = self.l_search(right, b_left, k_left)
        self.last_case, self.last_node = 3, node
        return batch + addition[:min(k_left, len(addition))]

    def r_search(self, siblings: List[Node], b_left: int, k_left: int) -> List[Request]:
        selected: List[Request] = []
        for s in reversed(siblings):                       # right to left: nearest first
            for r in reversed(self.collect(s)):            # longest (nearest) first
                if r.blocks + sum(x.blocks for x in selected) <= b_left:
                    selected.append(r)
                else:
                    return selected
        return selected

    def l_search(self, siblings: List[Node], b_left: int, k_left: int) -> List[Request]:
        selected: List[Request] = []
        for s in siblings:                                 # left to right: nearest first
            for r in self.collect(s):                      # shortest (nearest) first
                if r.blocks + sum(x.blocks for x in selected) <= b_left:
                    selected.append(r)
                else:
                    return selected
        return selected

    # -- batch generation --------------------------------------------------
    def _internal_nodes(self, node: Node):
        if node.is_leaf():
            return
        yield node
        for c in node.children:
            yield from self._internal_nodes(c)

    def next_batch(self, b_max: int, k_min: int, now: float = 0.0,
                   starve_after: Optional[float] = None) -> List[int]:
        """Generate one batch, remove its requests from the tree, return their
        ids in emission order ([] when the tree is empty)."""
        if len(self) == 0:
            return []
        start = self.root
        if starve_after is not None:
            best = None
            for n in self._internal_nodes(self.root):
                if self.request_counter(n) == 0:
                    continue
                age = now - n.last_served
                if age > starve_after:
                    key = (age, n.depth, -n.lo)
                    if best is None or key > best[0]:
                        best = (key, n)
            if best is not None:
                start = best[1]
        batch = self.recursive_dfs(start, b_max, k_min)
        n = self.last_node
        while n is not None:
            n.last_served = now
            n = n.parent
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
