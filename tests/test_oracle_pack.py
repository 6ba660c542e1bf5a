"""Pins for the plain pack-stage statement in oracle/pack.py: a hand-worked example, the
paper's closed forms re-derived from an explicit traffic count, forest round trips, exact
cover, and the structure counts the benchmark shapes fix."""
import json
import os
import random

from fractions import Fraction

import numpy as np
import pytest

from oracle import pack as op
from paper_2511_22333_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden", "tree_heuristic_worked_example.json")


def _load_gold():
    g = json.load(open(GOLD))
    rows = g["block_tables"]
    width = max(len(r) for r in rows)
    bt = np.full((len(rows), width), -1, np.int32)
    for i, r in enumerate(rows):
        bt[i, :len(r)] = r
    return g, bt, np.array(g["kv_lens"], np.int32)


def _canon(packs):
    return sorted((tuple(p.queries), p.start, p.num_pages, p.kv_len) for p in packs)


def test_hand_worked_example_packs_and_split():
    g, bt, kl = _load_gold()
    packs = op.plan_packs(bt, kl, g["page_size"])
    want = sorted((tuple(q), s, n, t) for q, s, n, t in g["packs"])
    assert _canon(packs) == want
    items = op.long_kv_split(packs, kl, g["page_size"])
    want_items = sorted((tuple(q), s, n, t) for q, s, n, t in g["split_items"])
    assert _canon(items) == want_items


def _walk(nodes):
    for n in nodes:
        yield n
        yield from _walk(n.children)


def _check_forest(bt, kl, P):
    forest = op.build_forest(bt, kl, P)
    B = len(kl)
    # root-to-leaf concatenation reconstructs each row (sec. "Pack Scheduler",
    # "Tree Structure Block Table")
    seen = set()

    def down(n, prefix):
        blocks = prefix + n.blocks
        assert n.start == len(prefix)
        if n.is_leaf:
            r = n.queries[0]
            assert blocks == [int(x) for x in bt[r, : -(-int(kl[r]) // P)]]
            assert r not in seen
            seen.add(r)
            assert not n.children
        else:
            assert n.size >= 2 and len(n.blocks) >= 1
            assert sorted(q for c in n.children for q in c.queries) == n.queries
            # maximal run: no page after the run is shared (as a full page) by all queries
            nxt = len(blocks)
            if all(nxt < int(kl[r]) // P for r in n.queries):
                assert len({int(bt[r, nxt]) for r in n.queries}) > 1
            # siblings start with different pages (or are leaves without shareable pages)
            firsts = [int(bt[c.queries[0], nxt]) for c in n.children
                      if nxt < int(kl[c.queries[0]]) // P]
            assert len(firsts) == len(set(firsts))
            for c in n.children:
                down(c, blocks)

    for t in forest:
        down(t, [])
    assert seen == set(range(B))
    return forest


@pytest.mark.parametrize("seed", range(25))
def test_forest_round_trip_and_exact_cover_random(seed):
    b = wl.random_forest_batch(seed, duplicate_rows=(seed % 3 == 0))
    P = b.page_size
    _check_forest(b.block_tables, b.kv_lens, P)
    packs = op.plan_packs(b.block_tables, b.kv_lens, P)
    want = op.expected_cover(b.kv_lens, P)
    assert op.cover_multiset([(p.queries, p.start, p.num_pages) for p in packs]) == want
    items = op.long_kv_split(packs, b.kv_lens, P)
    assert op.cover_multiset([(p.queries, p.start, p.num_pages) for p in items]) == want
    # tokens per request add up
    tok = np.zeros(b.num_requests, np.int64)
    for p in items:
        assert p.num_pages >= 1 and p.kv_len >= 1
        if len(p.queries) > 1:
            assert p.kv_len == p.num_pages * P
        for r in p.queries:
            tok[r] += p.kv_len
    assert np.array_equal(tok, b.kv_lens.astype(np.int64))
    # every query of a pack really holds the same page ids on the pack's range
    for p in items:
        ref = b.block_tables[p.queries[0], p.start:p.start + p.num_pages]
        for r in p.queries[1:]:
            assert np.array_equal(b.block_tables[r, p.start:p.start + p.num_pages], ref)
    # merging never costs more than one pack per node under the paper's own count
    naive = op.naive_packs(op.build_forest(b.block_tables, b.kv_lens, P), b.kv_lens, P)
    assert op.model_cost(packs) <= op.model_cost(naive)
    assert op.cover_multiset([(p.queries, p.start, p.num_pages) for p in naive]) == want


def test_intra_node_profit_closed_form():
    # packing s queries over l shared tokens saves (s-1) l d loads and costs 8 s d of
    # intermediates (4 s d at the node, 4 s d at the leaves): ratio >= l/16.
    # Counted explicitly from pack lists rather than from the formula.
    rnd = random.Random(1)
    for _ in range(200):
        s, l, d = rnd.randint(2, 64), 16 * rnd.randint(1, 300), rnd.choice([64, 128])
        leaf = [rnd.randint(1, 500) for _ in range(s)]
        kv = [l + x for x in leaf]
        packed = [op.Pack(tuple(range(s)), 0, l // 16, l)] + \
                 [op.Pack((i,), l // 16, -(-leaf[i] // 16), leaf[i]) for i in range(s)]
        separate = [op.Pack((i,), 0, -(-kv[i] // 16), kv[i]) for i in range(s)]
        kv_saved = sum(p.kv_len for p in separate) * d - sum(p.kv_len for p in packed) * d
        assert kv_saved == (s - 1) * l * d
        inter = 4 * d * sum(len(p.queries) for p in packed)      # every pack writes and reads
        assert inter == 8 * s * d
        assert kv_saved * 16 >= l * inter * (s - 1) // s          # r = (s-1) l / (8 s) >= l/16
        assert (s - 1) * l * d / (8 * s * d) >= l / 16 - 1e-12


def test_inter_node_scheme_difference_matches_eq1_eq2():
    # Scheme 2 minus Scheme 1 = 4 s_i d - l_u d, from explicit pack lists
    rnd = random.Random(2)
    for _ in range(300):
        d = 128
        l_u = 16 * rnd.randint(1, 40)
        kids = [(rnd.randint(1, 12), 16 * rnd.randint(1, 40)) for _ in range(rnd.randint(2, 5))]
        s_u = sum(s for s, _ in kids)
        base = 0
        qid = []
        for s, _ in kids:
            qid.append(tuple(range(base, base + s)))
            base += s
        i = rnd.randrange(len(kids))
        pu = l_u // 16

        def child_pack(k, merged):
            s, l = kids[k]
            if merged:
                return op.Pack(qid[k], 0, pu + l // 16, l_u + l)
            return op.Pack(qid[k], pu, l // 16, l)

        scheme1 = [op.Pack(tuple(range(s_u)), 0, pu, l_u)] + \
                  [child_pack(k, False) for k in range(len(kids))]
        rest = tuple(q for k in range(len(kids)) if k != i for q in qid[k])
        scheme2 = [op.Pack(rest, 0, pu, l_u)] + \
                  [child_pack(k, k == i) for k in range(len(kids))]
        s_i = kids[i][0]
        delta = op.model_cost(scheme1, d) - op.model_cost(scheme2, d)     # profit2 - profit1
        assert delta == 4 * s_i * d - l_u * d
        # Eq. 1 as printed: profit of scheme 1 relative to one query per CTA for node u's level
        # (children's own intermediates are common to both sides and cancel in the difference)
        eq1 = (s_u - 1) * l_u * d - 4 * s_u * d + sum((s - 1) * l * d for s, l in kids)
        eq2 = ((s_u - s_i - 1) * l_u * d - 4 * (s_u - s_i) * d
               + sum((s - 1) * l * d for k, (s, l) in enumerate(kids) if k != i)
               + (s_i - 1) * (l_u + kids[i][1]) * d)
        assert eq2 - eq1 == delta


# ---- brute force over every split/merge assignment of small trees --------------------------------
# An assignment says, for every edge into an INTERNAL child, whether the child is merged (Scheme 2)
# or split (Scheme 1); edges into leaves are split (merging a single query never pays once the
# blocks are longer than 4 tokens).  _packs_of turns an assignment into its explicit pack list with
# nothing of Algorithm 1's rule in it, and the cost is counted from that list.

def _tree_P1(spec, next_q, start=0):
    """Tree with one token per page from a nested spec (length, [children]) / (length,) for a leaf."""
    length, kids = spec[0], (spec[1] if len(spec) > 1 else None)
    if kids is None:
        q = next_q[0]
        next_q[0] += 1
        return op.Node([q], start, list(range(length)), [], True)
    children = [_tree_P1(k, next_q, start + length) for k in kids]
    return op.Node(sorted(q for c in children for q in c.queries), start, list(range(length)), children)


def _kv_lens(root):
    lens = {}

    def walk(n, acc):
        acc += len(n.blocks)
        if n.is_leaf:
            lens[n.queries[0]] = acc
        for c in n.children:
            walk(c, acc)

    walk(root, 0)
    return [lens[q] for q in sorted(lens)]


def _internal_edges(root):
    out = []

    def walk(n):
        for c in n.children:
            if not c.is_leaf:
                out.append(c)
                walk(c)

    walk(root)
    return out


def _packs_of(root, merged):
    """Explicit packs of an assignment: merged = set of id(child) for merged internal children."""
    out = []

    def visit(n, start, pages):
        if n.is_leaf:
            if pages:
                out.append((tuple(n.queries), start, pages))
            return
        remaining = set(n.queries)
        for c in n.children:
            if id(c) in merged:
                visit(c, start, pages + len(c.blocks))
                remaining -= set(c.queries)
            else:
                visit(c, c.start, len(c.blocks))
        if remaining and pages:
            out.append((tuple(sorted(remaining)), start, pages))

    visit(root, root.start, len(root.blocks))
    return out


def _cost(packs):
    return sum(pages + 4 * len(q) for q, _, pages in packs)        # P = 1: pages are tokens


def _blocks_len_seen_by(root, merged):
    """Length of the blocks each internal child's PARENT call holds under an assignment."""
    seen = {}

    def visit(n, pages):
        for c in n.children:
            if c.is_leaf:
                continue
            seen[id(c)] = pages
            visit(c, pages + len(c.blocks) if id(c) in merged else len(c.blocks))

    visit(root, len(root.blocks))
    return seen


def _random_small_tree(rng):
    """At most 6 internal edges; leaves long enough that merging a node into a leaf never pays."""
    budget = [int(rng.integers(1, 7))]

    def grow(depth):
        kids = []
        for _ in range(int(rng.integers(1, 4))):
            if budget[0] > 0 and depth < 3 and rng.random() < 0.7:
                budget[0] -= 1
                kids.append(grow(depth + 1))
            else:
                kids.append((int(rng.integers(5, 30)),))
        if sum(1 for k in kids if len(k) == 1) == 0 and rng.random() < 0.5:
            kids.append((int(rng.integers(5, 30)),))
        return (int(rng.integers(5, 30)), kids)          # > 4 tokens: no leaf is tempted to merge

    return grow(0)


@pytest.mark.parametrize("seed", range(40))
def test_algorithm_1_is_the_one_assignment_that_obeys_the_rule_at_every_edge(seed):
    # Among all 2^E assignments exactly one has, at every edge, "merged iff 4 s_child >= length of
    # the blocks the parent's call holds" (the blocks include every ancestor run merged so far);
    # its explicit pack list is what tree_heuristic returns.  A wrong accumulated length, a
    # query not taken out of the parent, a flipped comparison or a mishandled tie changes it.
    rng = np.random.default_rng(seed)
    root = _tree_P1(_random_small_tree(rng), [0])
    lens = _kv_lens(root)
    edges = _internal_edges(root)
    assert len(edges) <= 6
    consistent = []
    for mask in range(1 << len(edges)):
        merged = {id(c) for k, c in enumerate(edges) if mask >> k & 1}
        seen = _blocks_len_seen_by(root, merged)
        if all((id(c) in merged) == (4 * c.size >= seen[id(c)]) for c in edges):
            consistent.append(merged)
    assert len(consistent) == 1
    want = sorted(_packs_of(root, consistent[0]))
    got = sorted((p.queries, p.start, p.num_pages)
                 for p in op.tree_heuristic(root, root.start, len(root.blocks), lens, 1))
    assert got == want
    assert op.model_cost(op.tree_heuristic(root, root.start, len(root.blocks), lens, 1)) == _cost(want)


@pytest.mark.parametrize("seed", range(30))
def test_heuristic_cost_is_the_minimum_where_the_profit_model_applies(seed):
    # Eq. 1 / Eq. 2 compare the two schemes for ONE child with the parent's pack still there and
    # everything below unchanged.  That is the whole story for a node whose internal children have
    # long runs of their own (nothing below is tempted to merge): the children's decisions are
    # then independent, and the heuristic's modelled traffic is the minimum over all assignments
    # that leave the parent a pack.
    rng = np.random.default_rng(100 + seed)
    kids = []
    for _ in range(int(rng.integers(2, 7))):                 # 2..6 internal children
        s = int(rng.integers(1, 9))
        kids.append((200, [(int(rng.integers(5, 30)),) for _ in range(s)]))
    kids.append((int(rng.integers(5, 30)),))                 # one direct leaf: the pack stays
    root = _tree_P1((int(rng.integers(5, 40)), kids), [0])
    lens = _kv_lens(root)
    edges = _internal_edges(root)
    best = min(_cost(_packs_of(root, {id(c) for k, c in enumerate(edges) if mask >> k & 1}))
               for mask in range(1 << len(edges)))
    got = op.model_cost(op.tree_heuristic(root, root.start, len(root.blocks), lens, 1))
    assert got == best


def test_where_the_per_child_rule_is_not_the_global_minimum():
    # The rule prices one child at a time.  When EVERY child of a node merges, the node's own pack
    # disappears, which the per-child comparison does not see: a 16-token node over two groups of
    # three queries is split by the rule (4 * 3 < 16), although merging both groups would save
    # 16 + 4 * 6 of the node's pack for 2 * 16 of repeated loads, 8 less in total.  (A heuristic,
    # as the paper calls it.)
    root = _tree_P1((16, [(200, [(20,)] * 3), (200, [(20,)] * 3)]), [0])
    lens = _kv_lens(root)
    edges = _internal_edges(root)
    got = op.model_cost(op.tree_heuristic(root, root.start, len(root.blocks), lens, 1))
    split_all = _cost(_packs_of(root, set()))
    merge_all = _cost(_packs_of(root, {id(c) for c in edges}))
    assert got == split_all and merge_all == split_all - 8


@pytest.mark.parametrize("seed", range(10))
def test_merging_into_a_single_query_never_pays(seed):
    # edges into leaves: Scheme 2 for a child of one query repeats the blocks to save 4
    rng = np.random.default_rng(200 + seed)
    l_u, n = int(rng.integers(5, 60)), int(rng.integers(2, 6))
    leaves = [int(rng.integers(1, 50)) for _ in range(n)]
    split = l_u + 4 * n + sum(x + 4 for x in leaves)
    for k in range(n):                                       # leaf k reads the node's blocks itself
        merged = l_u + 4 * (n - 1) + sum(x + 4 for x in leaves) + l_u
        assert merged - split == l_u - 4 > 0
    root = _tree_P1((l_u, [(x,) for x in leaves]), [0])
    got = op.model_cost(op.tree_heuristic(root, root.start, len(root.blocks), _kv_lens(root), 1))
    assert got == split


@pytest.mark.parametrize("l_u", [1, 2, 3, 4])
def test_blocks_of_at_most_four_tokens_are_merged_into_single_queries(l_u):
    # 4 * 1 >= l_u: every leaf takes the node's blocks along (ties merge), the node's pack is gone,
    # and no assignment of the leaf edges is cheaper
    leaves = [7, 12, 30]
    root = _tree_P1((l_u, [(x,) for x in leaves]), [0])
    packs = op.tree_heuristic(root, root.start, len(root.blocks), _kv_lens(root), 1)
    assert sorted((p.queries, p.start, p.num_pages) for p in packs) == \
        [((k,), 0, l_u + x) for k, x in enumerate(leaves)]
    costs = []
    for mask in range(8):
        merged = [mask >> k & 1 for k in range(3)]
        rest = sum(1 for m in merged if not m)
        costs.append((l_u + 4 * rest if rest else 0) + sum(x + 4 + (l_u if m else 0) for x, m in zip(leaves, merged)))
    assert op.model_cost(packs) == min(costs)


def test_merge_fires_on_short_parents_and_not_on_long_ones():
    # root of 16 tokens over 8 requests in 2 groups of 4 -> 4*4 >= 16 both merge, root vanishes
    b = wl.tree_batch([1, 2, 8], [16, 32, 40], num_q_heads=4, num_kv_heads=4, seed=3)
    packs = op.plan_packs(b.block_tables, b.kv_lens, 16)
    multi = [p for p in packs if len(p.queries) > 1]
    assert sorted((len(p.queries), p.start, p.num_pages) for p in multi) == [(4, 0, 3), (4, 0, 3)]
    # same shape with a long root: 4*4 < 1024 -> split, root kept as a pack of 8
    b = wl.tree_batch([1, 2, 8], [1024, 32, 40], num_q_heads=4, num_kv_heads=4, seed=3)
    packs = op.plan_packs(b.block_tables, b.kv_lens, 16)
    multi = sorted((len(p.queries), p.start, p.num_pages) for p in packs if len(p.queries) > 1)
    assert multi == [(4, 64, 2), (4, 64, 2), (8, 0, 64)]


@pytest.mark.parametrize("name,n_packs", [("C1", 5), ("C2", 33), ("C3", 137), ("C4", 273),
                                          ("C5", 512)])
def test_benchmark_shapes_pack_one_per_node(name, n_packs):
    # every shared node of the benchmark shapes has l >= 256 >> 4 s of any child
    b = wl.config(name)
    packs = op.plan_packs(b.block_tables, b.kv_lens, b.page_size)
    assert len(packs) == n_packs
    assert sum(p.kv_len for p in packs) == b.unique_kv_tokens()
    items = op.long_kv_split(packs, b.kv_lens, b.page_size)
    mean = sum(p.kv_len for p in packs) / len(packs)
    for it in items:
        assert it.kv_len <= mean or it.num_pages == 1       # "under the mean value", page permitting
    assert sum(p.kv_len for p in items) == b.unique_kv_tokens()


@pytest.mark.parametrize("seed", range(20))
def test_split_takes_the_fewest_equal_parts_that_stay_under_the_mean(seed):
    # sec. "Multi Kernel Forward", "Long KV Split": a pack over the mean is cut into equal parts that keep the
    # length under the mean.  Stated without the ceil(len/mean) shortcut: try 2, 3, ... parts of page counts as
    # equal as possible, longer first, and take the first count whose every part has at most `mean` tokens --
    # or one page per part where not even that brings them under.
    rng = np.random.default_rng(900 + seed)
    P = int(rng.choice([1, 4, 16]))
    lens = [int(x) for x in rng.integers(1, 40 * P, int(rng.integers(2, 12)))]
    if seed % 3 == 0:
        lens.append(int(rng.integers(100 * P, 400 * P)))          # one very long pack drags the mean up
    packs = [op.Pack((i,), 0, -(-n // P), n) for i, n in enumerate(lens)]
    mean = Fraction(sum(lens), len(lens))
    got = op.long_kv_split(packs, lens, P)
    k = 0
    for i, n in enumerate(lens):
        pages = -(-n // P)
        want = None
        if n <= mean:
            want = [(0, pages, n)]
        else:
            for parts in range(2, pages + 1):
                base, extra = divmod(pages, parts)
                cuts, start = [], 0
                for j in range(parts):
                    c = base + (1 if j < extra else 0)
                    cuts.append((start, c, min(n, (start + c) * P) - start * P))
                    start += c
                if all(t <= mean for _, _, t in cuts) or parts == pages:
                    want = cuts
                    break
            if want is None:                                      # a single page cannot be cut
                want = [(0, pages, n)]
        for s0, c, t in want:
            assert (got[k].queries, got[k].start, got[k].num_pages, got[k].kv_len) == ((i,), s0, c, t)
            k += 1
    assert k == len(got)


def test_partial_last_page_is_never_shared():
    # two rows name the same page id where request 1 only half fills it
    bt = np.array([[5, 6, 7], [5, 6, -1]], np.int32)
    kl = np.array([48, 24], np.int32)
    packs = op.plan_packs(bt, kl, 16)
    assert _canon(packs) == sorted([((0, 1), 0, 1, 16), ((0,), 1, 2, 32), ((1,), 1, 1, 8)])
