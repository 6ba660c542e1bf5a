"""TEST INFRASTRUCTURE -- plain Python statement of the pack stage, for checking the planner.

Not part of the product path; shares no code with the C++ planner.  Pure-Python recursion and
lists, meant for small and medium batches.

What is written out here, in the paper's order and notation:

* ``build_forest`` -- the tree-structured block table (sec. "Pack Scheduler", paragraph
  "Tree Structure Block Table"): rows of the block table are compressed on identical leading
  page ids into a forest; an internal node is a run of pages shared by the same set of
  queries, with ``l`` = its KV length and ``s`` = the number of queries under it; every query
  ends in one leaf that holds its non-shared pages.
* ``tree_heuristic`` -- Algorithm 1 (TreeHeuristic): a leaf becomes a pack of its own; for
  every child the inter-node profit rule picks Scheme 1 (split) or Scheme 2 (merge the
  parent's blocks into the child's packs and take the child's queries out of the parent);
  last, the node's remaining queries are packed with the node's blocks.
* ``model_cost`` -- the memory-access count behind the profit model (paragraphs "Intra-node
  profit" and "Inter-node profit", Eq. 1 and Eq. 2): a pack of ``s`` queries over ``l`` tokens
  loads ``l*d`` KV elements and moves ``4*s*d`` elements of fp32 intermediates.
* ``long_kv_split`` -- sec. "Multi Kernel Forward", paragraph "Long KV Split": packs longer
  than the mean pack KV length are cut into equal parts no longer than the mean.

Readings where the paper is silent or garbled (also listed in the design notes):
  - Algorithm 1's test ``4 x c.size < root.len``: ``len`` is the token length of the ``blocks``
    argument of the current call (the node's run plus every ancestor run merged into it),
    because that is the KV a merged child would load again.  Ties merge, as the algorithm's
    else-branch does.
  - Only pages that a request fills completely can be shared; a trailing partial page is
    private to its request even when another row names the same page id.
  - Packs without queries or without pages are dropped.
  - The split mean is taken once over the packs before splitting, in tokens; a pack of
    ``len > mean`` is cut into ``ceil(len/mean)`` parts (at most one part per page) whose page
    counts differ by at most one, longer parts first.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from fractions import Fraction
from typing import Dict, List, Sequence, Tuple

import numpy as np


@dataclass
class Node:
    queries: List[int]            # request ids under this node, ascending
    start: int                    # index of the node's first page in the block-table rows
    blocks: List[int]             # page ids owned by this node
    children: List["Node"] = field(default_factory=list)
    is_leaf: bool = False

    @property
    def size(self) -> int:        # the paper's s
        return len(self.queries)


@dataclass(frozen=True)
class Pack:
    queries: Tuple[int, ...]      # ascending request ids
    start: int                    # first page index (same in every query's row)
    num_pages: int
    kv_len: int                   # valid tokens in the pack's pages


def _row_pages(kv_len: int, P: int) -> int:
    return -(-kv_len // P)


def build_forest(block_tables: np.ndarray, kv_lens: Sequence[int], P: int) -> List[Node]:
    """Compress block-table rows into a forest of shared-page runs."""
    B = len(kv_lens)
    rows = [[int(x) for x in block_tables[r, :_row_pages(int(kv_lens[r]), P)]] for r in range(B)]
    full = [int(kv_lens[r]) // P for r in range(B)]       # pages that may be shared

    def leaf(r: int, depth: int) -> Node:
        return Node([r], depth, rows[r][depth:], [], True)

    def grow(reqs: List[int], depth: int) -> List[Node]:
        """Nodes for requests that agree on pages [0, depth)."""
        out: List[Node] = []
        groups: Dict[int, List[int]] = {}
        singles: List[int] = []
        for r in reqs:
            if depth < full[r]:
                groups.setdefault(rows[r][depth], []).append(r)
            else:
                singles.append(r)
        made = {}
        for pid, members in groups.items():
            if len(members) == 1:
                made[members[0]] = leaf(members[0], depth)
                continue
            # longest run of identical, fully filled pages shared by all members
            run = 0
            while all(depth + run < full[r] for r in members) and \
                    len({rows[r][depth + run] for r in members}) == 1:
                run += 1
            node = Node(sorted(members), depth, rows[members[0]][depth:depth + run])
            node.children = grow(sorted(members), depth + run)
            made[members[0]] = node
        for r in singles:
            made[r] = leaf(r, depth)
        # keep the order of first appearance in the batch
        for r in reqs:
            if r in made:
                out.append(made[r])
        return out

    return grow(list(range(B)), 0)


def tree_heuristic(root: Node, blocks_start: int, blocks_pages: int, kv_lens: Sequence[int],
                   P: int, decisions: List = None) -> List[Pack]:
    """Algorithm 1.  ``blocks`` is always a contiguous range of row page indices
    [blocks_start, blocks_start + blocks_pages) because merged runs are adjacent.
    ``decisions`` (optional) collects (parent_start, child first query, 'split'|'merge')."""
    def pack(queries: List[int], start: int, pages: int) -> List[Pack]:
        if not queries or pages == 0:
            return []
        if len(queries) == 1:
            n = min(int(kv_lens[queries[0]]), (start + pages) * P) - start * P
        else:
            n = pages * P
        return [Pack(tuple(sorted(queries)), start, pages, n)]

    if root.is_leaf:
        return pack(root.queries, blocks_start, blocks_pages)
    packs: List[Pack] = []
    remaining = list(root.queries)
    blocks_len = blocks_pages * P                     # shared pages are always full
    for c in root.children:
        if 4 * c.size < blocks_len:
            # Scheme 1: split
            packs += tree_heuristic(c, c.start, len(c.blocks), kv_lens, P, decisions)
            if decisions is not None:
                decisions.append((root.start, c.queries[0], "split"))
        else:
            # Scheme 2: merge this node's blocks into the child's
            packs += tree_heuristic(c, blocks_start, blocks_pages + len(c.blocks), kv_lens, P,
                                    decisions)
            remaining = [q for q in remaining if q not in set(c.queries)]
            if decisions is not None:
                decisions.append((root.start, c.queries[0], "merge"))
    packs += pack(remaining, blocks_start, blocks_pages)
    return packs


def naive_packs(forest: List[Node], kv_lens: Sequence[int], P: int) -> List[Pack]:
    """One pack per tree node (the ablation the paper calls naive packing)."""
    out: List[Pack] = []

    def walk(n: Node):
        pages = len(n.blocks)
        if pages:
            if n.is_leaf:
                r = n.queries[0]
                tok = min(int(kv_lens[r]), (n.start + pages) * P) - n.start * P
            else:
                tok = pages * P
            out.append(Pack(tuple(n.queries), n.start, pages, tok))
        for c in n.children:
            walk(c)

    for t in forest:
        walk(t)
    return out


def plan_packs(block_tables: np.ndarray, kv_lens: Sequence[int], P: int) -> List[Pack]:
    """Forest, then TreeHeuristic on every tree."""
    packs: List[Pack] = []
    for t in build_forest(block_tables, kv_lens, P):
        packs += tree_heuristic(t, t.start, len(t.blocks), kv_lens, P)
    return packs


def model_cost(packs: Sequence[Pack], d: int = 1) -> int:
    """Memory accesses in the paper's unit (elements): KV loads ``l*d`` per pack plus fp32
    intermediates written and read, ``4*s*d`` per pack."""
    return sum(p.kv_len * d + 4 * len(p.queries) * d for p in packs)


def long_kv_split(packs: Sequence[Pack], kv_lens: Sequence[int], P: int) -> List[Pack]:
    """Cut every pack longer than the mean pack length into equal page-aligned parts, as many as it
    takes to bring every part of more than one page under the mean."""
    if not packs:
        return []
    mean = Fraction(sum(p.kv_len for p in packs), len(packs))
    out: List[Pack] = []
    for p in packs:
        if Fraction(p.kv_len) <= mean:
            out.append(p)
            continue
        q = Fraction(p.kv_len) / mean
        parts = -(-q.numerator // q.denominator)          # ceil(len / mean)
        parts = min(parts, p.num_pages)
        # parts are whole pages: while the longest part (the first: full pages) is still over the
        # mean and a part has more than one page, cut once more
        while parts < p.num_pages and Fraction(-(-p.num_pages // parts) * P) > mean:
            parts += 1
        base, extra = divmod(p.num_pages, parts)
        start = p.start
        for i in range(parts):
            n = base + (1 if i < extra else 0)
            end_tok = (start + n - p.start) * P
            tok = min(p.kv_len, end_tok) - (start - p.start) * P
            out.append(Pack(p.queries, start, n, tok))
            start += n
    return out


def cover_multiset(items: Sequence[Tuple[Sequence[int], int, int]]):
    """Sorted list of (request, page index) pairs covered by items = (queries, start, pages)."""
    pairs = []
    for queries, start, pages in items:
        for r in queries:
            pairs.extend((int(r), i) for i in range(start, start + pages))
    pairs.sort()
    return pairs


def expected_cover(kv_lens: Sequence[int], P: int):
    pairs = []
    for r, n in enumerate(kv_lens):
        pairs.extend((r, i) for i in range(_row_pages(int(n), P)))
    return pairs
