"""Planner (pat_plan) against the plain pack-stage statement in oracle/pack.py, bit-exactly,
plus the invariants every schedule must keep (exact cover, slots, rows, tiles) and the
error behaviour of the C ABI.  CPU only: no kernel is launched."""
import dataclasses
import json
import os
import re

import numpy as np
import pytest

from oracle import pack as op
from paper_2511_22333_amd import binding as pb
from paper_2511_22333_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _items(ex):
    out = []
    for i in range(ex["num_items"]):
        reqs = tuple(int(x) for x in ex["item_req_ids"][ex["item_req_off"][i]:ex["item_req_off"][i + 1]])
        n_pages = int(ex["item_page_off"][i + 1] - ex["item_page_off"][i])
        out.append((reqs, int(ex["item_page_start"][i]), n_pages, int(ex["item_kv_len"][i])))
    return out


def check_schedule(batch, plan):
    """Invariants of any valid schedule.  Returns the exported view."""
    ex = plan.export()
    st = plan.stats()
    P, B, G = batch.page_size, batch.num_requests, batch.group_size
    items = _items(ex)
    # exact cover of (request, page index), bit-exact
    assert op.cover_multiset([(q, s, n) for q, s, n, _ in items]) == op.expected_cover(batch.kv_lens, P)
    tok = np.zeros(B, np.int64)
    for i, (reqs, start, n_pages, kv_len) in enumerate(items):
        assert list(reqs) == sorted(set(reqs)) and len(reqs) >= 1 and n_pages >= 1
        ids = ex["item_page_ids"][ex["item_page_off"][i]:ex["item_page_off"][i + 1]]
        for r in reqs:      # every request of the item holds exactly these pages there
            assert np.array_equal(batch.block_tables[r, start:start + n_pages], ids)
            tok[r] += kv_len
        if len(reqs) > 1:
            assert kv_len == n_pages * P
            for r in reqs:  # shared pages are completely filled in every sharing request
                assert int(batch.kv_lens[r]) >= (start + n_pages) * P
        else:
            r = reqs[0]
            assert kv_len == min(int(batch.kv_lens[r]), (start + n_pages) * P) - start * P
        assert (n_pages - 1) * P < kv_len <= n_pages * P
    assert np.array_equal(tok, batch.kv_lens.astype(np.int64))
    assert st.unique_kv_tokens == sum(it[3] for it in items)
    assert st.total_kv_tokens == int(batch.kv_lens.astype(np.int64).sum())
    # slots: one per (item, request) of requests with more than one item; -1 otherwise
    parts = np.zeros(B, np.int64)
    for reqs, *_ in items:
        for r in reqs:
            parts[r] += 1
    slots_seen = []
    per_req = {r: [] for r in range(B)}
    for i, (reqs, *_rest) in enumerate(items):
        sl = ex["item_req_slot"][ex["item_req_off"][i]:ex["item_req_off"][i + 1]]
        for r, s in zip(reqs, sl):
            if parts[r] == 1:
                assert s == -1
            else:
                assert s >= 0
                slots_seen.append(int(s))
                per_req[r].append(int(s))
    assert sorted(slots_seen) == list(range(st.num_slots)) == list(range(ex["num_slots"]))
    for r in range(B):
        got = sorted(int(x) for x in ex["req_slot_ids"][ex["req_slot_off"][r]:ex["req_slot_off"][r + 1]])
        assert got == sorted(per_req[r])
    assert st.num_merge_requests == int((parts > 1).sum())
    # entries: row blocks tile each item's rows exactly once, within the tile's m
    rows_seen = {}
    for e in range(ex["num_entries"]):
        it = int(ex["entry_item"][e])
        rc, m, n = pb.pat_tile_info(int(ex["entry_tile"][e]))
        assert rc == 0
        assert 1 <= ex["entry_num_rows"][e] <= m
        rows_seen.setdefault(it, []).append((int(ex["entry_row_begin"][e]), int(ex["entry_num_rows"][e])))
    assert set(rows_seen) == set(range(len(items)))
    for it, blocks in rows_seen.items():
        blocks.sort()
        pos = 0
        for b0, n in blocks:
            assert b0 == pos
            pos += n
        assert pos == len(items[it][0]) * G
    assert st.num_entries == ex["num_entries"]
    # packed tiles (m > 16): one workgroup per KV head; 16-row tiles: one per pair of KV heads,
    # or per head where the device-aware split asked for it
    want_wgs = 0
    for e in range(ex["num_entries"]):
        _, m, _ = pb.pat_tile_info(int(ex["entry_tile"][e]))
        hp = int(ex["entry_heads_per_wg"][e])
        assert hp == 1 if m > 16 else hp in (1, 2)
        want_wgs += (batch.num_kv_heads + hp - 1) // hp
    assert st.num_workgroups == want_wgs
    assert sum(st.tile_histogram) == st.num_entries
    assert st.workspace_bytes >= st.num_slots * batch.num_q_heads * (batch.head_dim + 1) * 4
    return ex


def _canon(items):
    return sorted(items)


@pytest.mark.parametrize("seed", range(30))
def test_planner_equals_plain_statement_on_random_forests(seed):
    b = wl.random_forest_batch(seed, duplicate_rows=(seed % 4 == 0), max_requests=14)
    want_packs = op.plan_packs(b.block_tables, b.kv_lens, b.page_size)
    # no split: packs themselves
    plan = pb.plan_for_batch(b, split_policy=pb.PAT_SPLIT_NONE)
    ex = check_schedule(b, plan)
    assert _canon(_items(ex)) == _canon((p.queries, p.start, p.num_pages, p.kv_len) for p in want_packs)
    assert plan.stats().num_packs == len(want_packs)
    # paper's mean split
    plan = pb.plan_for_batch(b, split_policy=pb.PAT_SPLIT_MEAN)
    ex = check_schedule(b, plan)
    want = op.long_kv_split(want_packs, b.kv_lens, b.page_size)
    assert _canon(_items(ex)) == _canon((p.queries, p.start, p.num_pages, p.kv_len) for p in want)


@pytest.mark.parametrize("seed", range(100, 130))
def test_planner_equals_plain_statement_on_larger_forests(seed):
    # deeper and wider forests, longer nodes, other head settings: packs (split NONE),
    # the paper's mean split and the one-pack-per-node mode all equal the plain statement
    hq, hkv = [(8, 2), (32, 8), (64, 8), (16, 8), (32, 32)][seed % 5]
    b = wl.random_forest_batch(seed, duplicate_rows=(seed % 4 == 1), max_requests=48, max_depth=6,
                               max_node_tokens=[64, 400, 1200][seed % 3], num_q_heads=hq, num_kv_heads=hkv)
    want_packs = op.plan_packs(b.block_tables, b.kv_lens, b.page_size)
    plan = pb.plan_for_batch(b, split_policy=pb.PAT_SPLIT_NONE)
    ex = check_schedule(b, plan)
    assert _canon(_items(ex)) == _canon((p.queries, p.start, p.num_pages, p.kv_len) for p in want_packs)
    plan = pb.plan_for_batch(b, split_policy=pb.PAT_SPLIT_MEAN)
    ex = check_schedule(b, plan)
    want = op.long_kv_split(want_packs, b.kv_lens, b.page_size)
    assert _canon(_items(ex)) == _canon((p.queries, p.start, p.num_pages, p.kv_len) for p in want)
    naive = op.naive_packs(op.build_forest(b.block_tables, b.kv_lens, b.page_size), b.kv_lens, b.page_size)
    plan = pb.plan_for_batch(b, mode=pb.PAT_MODE_NAIVE_PER_NODE, split_policy=pb.PAT_SPLIT_NONE)
    ex = check_schedule(b, plan)
    assert _canon(_items(ex)) == _canon((p.queries, p.start, p.num_pages, p.kv_len) for p in naive)
    # the default (device-aware) plan: invariants only
    check_schedule(b, pb.plan_for_batch(b))


def test_planner_reproduces_hand_worked_example():
    g = json.load(open(os.path.join(ROOT, "tests", "golden", "tree_heuristic_worked_example.json")))
    rows = g["block_tables"]
    bt = np.full((len(rows), max(len(r) for r in rows)), -1, np.int32)
    for i, r in enumerate(rows):
        bt[i, :len(r)] = r
    kl = np.array(g["kv_lens"], np.int32)
    kw = dict(page_size=16, num_pages=300, num_q_heads=8, num_kv_heads=2, head_dim=128, dtype="bf16")
    plan = pb.pat_plan(bt, kl, split_policy=pb.PAT_SPLIT_NONE, **kw)
    assert _canon(_items(plan.export())) == _canon((tuple(q), s, n, t) for q, s, n, t in g["packs"])
    assert plan.stats().num_merged_children == 2
    plan = pb.pat_plan(bt, kl, split_policy=pb.PAT_SPLIT_MEAN, **kw)
    assert _canon(_items(plan.export())) == _canon((tuple(q), s, n, t) for q, s, n, t in g["split_items"])


@pytest.mark.parametrize("name", wl.CONFIG_NAMES)
def test_benchmark_shapes(name):
    b = wl.config(name)
    want_packs = op.plan_packs(b.block_tables, b.kv_lens, b.page_size)
    plan = pb.plan_for_batch(b, split_policy=pb.PAT_SPLIT_MEAN)
    ex = check_schedule(b, plan)
    want = op.long_kv_split(want_packs, b.kv_lens, b.page_size)
    assert _canon(_items(ex)) == _canon((p.queries, p.start, p.num_pages, p.kv_len) for p in want)
    st = plan.stats()
    assert st.unique_kv_tokens == b.unique_kv_tokens()
    assert st.num_merged_children == 0
    # default policy and the baseline mode keep the invariants too
    check_schedule(b, pb.plan_for_batch(b))
    base = pb.plan_for_batch(b, mode=pb.PAT_MODE_NO_SHARING)
    check_schedule(b, base)
    assert base.stats().unique_kv_tokens == b.total_kv_tokens()


@pytest.mark.parametrize("seed", range(8))
def test_modes_and_policies_keep_exact_cover(seed):
    b = wl.random_forest_batch(200 + seed, max_requests=20, max_node_tokens=200)
    for mode in (pb.PAT_MODE_PAT, pb.PAT_MODE_NAIVE_PER_NODE, pb.PAT_MODE_NO_SHARING):
        for pol, tgt in ((pb.PAT_SPLIT_AUTO, 0), (pb.PAT_SPLIT_MEAN, 0), (pb.PAT_SPLIT_NONE, 0),
                         (pb.PAT_SPLIT_TARGET, 16), (pb.PAT_SPLIT_TARGET, 100)):
            plan = pb.plan_for_batch(b, mode=mode, split_policy=pol, split_target_tokens=tgt)
            ex = check_schedule(b, plan)
            if pol == pb.PAT_SPLIT_TARGET:
                # parts as equal as pages allow, never more than a page over the target
                assert max(ex["item_kv_len"]) <= tgt + 2 * b.page_size
    naive = pb.plan_for_batch(b, mode=pb.PAT_MODE_NAIVE_PER_NODE, split_policy=pb.PAT_SPLIT_NONE)
    forest = op.build_forest(b.block_tables, b.kv_lens, b.page_size)
    want = op.naive_packs(forest, b.kv_lens, b.page_size)
    assert _canon(_items(naive.export())) == _canon((p.queries, p.start, p.num_pages, p.kv_len) for p in want)


def test_merge_factor_changes_decisions_only():
    b = wl.tree_batch([1, 2, 8], [64, 32, 40], num_q_heads=4, num_kv_heads=4, seed=3)
    never = pb.plan_for_batch(b, merge_factor=1, split_policy=pb.PAT_SPLIT_NONE)     # 1*4 < 64
    always = pb.plan_for_batch(b, merge_factor=1000, split_policy=pb.PAT_SPLIT_NONE)
    check_schedule(b, never)
    check_schedule(b, always)
    assert never.stats().num_merged_children == 0
    assert always.stats().num_merged_children > 0
    assert always.stats().num_packs == 8          # everything merged down to the leaves
    assert always.stats().unique_kv_tokens == b.total_kv_tokens()


def test_explicit_tree_matches_derived_forest():
    b = wl.config("C3")
    # rebuild the generating tree in ABI form
    P = b.page_size
    parent = np.array([nd.parent for nd in b.nodes], np.int32)
    pages = np.array([-(-nd.num_tokens // P) for nd in b.nodes], np.int32)
    leaf = np.zeros(b.num_requests, np.int32)
    for i, nd in enumerate(b.nodes):
        if nd.is_leaf:
            leaf[nd.request] = i
    plan_e = pb.plan_for_batch(b, split_policy=pb.PAT_SPLIT_MEAN, node_parent=parent,
                               node_num_pages=pages, req_leaf_node=leaf)
    plan_d = pb.plan_for_batch(b, split_policy=pb.PAT_SPLIT_MEAN)
    check_schedule(b, plan_e)
    assert _canon(_items(plan_e.export())) == _canon(_items(plan_d.export()))
    # a tree that claims sharing the block tables do not have is refused
    bt = b.block_tables.copy()
    bt[5, 3] = bt[5, 3] + 1 if bt[5, 3] + 1 < b.num_pages else bt[5, 3] - 1
    with pytest.raises(pb.PatError) as ei:
        pb.pat_plan(bt, b.kv_lens, page_size=P, num_pages=b.num_pages, num_q_heads=32,
                    num_kv_heads=8, head_dim=128, dtype="bf16", node_parent=parent,
                    node_num_pages=pages, req_leaf_node=leaf)
    assert ei.value.status == -9


def test_row_blocks_when_rows_exceed_the_tile():
    b = wl.tree_batch([1, 40], [64, 20], num_q_heads=8, num_kv_heads=2, seed=1)   # 40*4 = 160 rows
    plan = pb.plan_for_batch(b, split_policy=pb.PAT_SPLIT_NONE)
    ex = check_schedule(b, plan)
    big = [e for e in range(ex["num_entries"]) if len(_items(ex)[ex["entry_item"][e]][0]) == 40]
    assert len(big) >= 2
    rows = [int(ex["entry_num_rows"][e]) for e in big]
    assert sum(rows) == 160 and max(rows) - min(rows) <= 1
    _, m, _ = pb.pat_tile_info(int(ex["entry_tile"][big[0]]))
    assert max(rows) <= m


def test_items_are_ordered_heaviest_first():
    b = wl.config("C5")
    ex = pb.plan_for_batch(b).export()
    kv = ex["item_kv_len"]
    assert all(kv[i] >= kv[i + 1] for i in range(len(kv) - 1))


def test_plan_time_is_roughly_linear():
    import time
    ts = []
    for n in (128, 512):
        b = wl.tree_batch([n], [2048], seed=5)
        t0 = time.perf_counter()
        for _ in range(3):
            pb.plan_for_batch(b)
        ts.append((time.perf_counter() - t0) / 3)
    assert ts[1] < ts[0] * 16 + 0.05      # 4x the pages: far from quadratic


@pytest.mark.parametrize("mutate,status", [
    (lambda kw: kw.__setitem__("num_q_heads", 7), -1),
    (lambda kw: kw.__setitem__("head_dim", 64), -4),
    (lambda kw: kw.__setitem__("page_size", 32), -4),
    (lambda kw: kw.__setitem__("dtype", 5), -4),
    (lambda kw: kw.__setitem__("num_pages", 3), -2),
    (lambda kw: kw.__setitem__("force_tile", 99), -1),
    (lambda kw: kw.__setitem__("split_policy", 9), -1),
    (lambda kw: kw.__setitem__("mode", 7), -1),
])
def test_errors_are_status_codes(mutate, status):
    b = wl.config("C1")
    kw = dict(page_size=16, num_pages=b.num_pages, num_q_heads=4, num_kv_heads=4, head_dim=128,
              dtype="fp16")
    mutate(kw)
    with pytest.raises(pb.PatError) as ei:
        pb.pat_plan(b.block_tables, b.kv_lens, **kw)
    assert ei.value.status == status


def test_bad_rows_are_refused():
    b = wl.config("C1")
    kw = dict(page_size=16, num_pages=b.num_pages, num_q_heads=4, num_kv_heads=4, head_dim=128,
              dtype="fp16")
    kl = b.kv_lens.copy()
    kl[2] = 0
    with pytest.raises(pb.PatError) as ei:
        pb.pat_plan(b.block_tables, kl, **kw)
    assert ei.value.status == -3
    kl[2] = 16 * b.block_tables.shape[1] + 1
    with pytest.raises(pb.PatError) as ei:
        pb.pat_plan(b.block_tables, kl, **kw)
    assert ei.value.status == -3
    bt = b.block_tables.copy()
    bt[1, 0] = -5
    with pytest.raises(pb.PatError) as ei:
        pb.pat_plan(bt, b.kv_lens, **kw)
    assert ei.value.status == -2
    # entries past a row's last page are ignored, whatever they hold
    bt = b.block_tables.copy()
    kl = b.kv_lens.copy()
    kl[0] = 40
    bt[0, 3:] = 10 ** 6
    check_schedule(wl.DecodeBatch("x", 4, 4, 4, 128, 16, "fp16", bt, kl, b.num_pages),
                   pb.pat_plan(bt, kl, **kw))


def test_gpu_calls_refuse_a_plan_that_was_not_uploaded():
    b = wl.config("C1")
    plan = pb.plan_for_batch(b)
    rc = pb.lib.pat_forward(plan.handle, 16, 16, 16, 8, 8, 8, 1.0, 16, None, 256, 1 << 20, None)
    assert rc == -6
    assert pb.lib.pat_merge(plan.handle, 16, None, 256, 1 << 20, None) == -6
    assert pb.lib.pat_forward(None, 16, 16, 16, 8, 8, 8, 1.0, 16, None, 256, 1 << 20, None) == -1


@pytest.mark.parametrize("scale", [0.0, -0.5, float("nan"), float("inf")])
def test_forward_refuses_a_scale_that_is_not_positive_and_finite(scale):
    # the packed tiles take row maxima on unscaled scores, which needs scale > 0
    b = wl.config("C1")
    plan = pb.plan_for_batch(b)
    for fn in (pb.lib.pat_forward, pb.lib.pat_decode_attention):
        assert fn(plan.handle, 16, 16, 16, 8, 8, 8, scale, 16, None, 256, 1 << 20, None) == -1


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "pat.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(pat_[a-z_]+)\s*\(", hdr))
    assert declared == set(pb.EXPORTED)
    for name in declared:
        assert hasattr(pb.lib, name), name
    assert pb.pat_version().startswith("pat-")
    assert pb.pat_strerror(-2)
    assert pb.lib.pat_num_tiles() >= 1


# ---- lazy update (pat_plan_advance) ---------------------------------------------------------
def _roomy(batch, extra=4096):
    """The same batch in a pool with `extra` free pages (decode steps take pages from them)."""
    return dataclasses.replace(batch, num_pages=batch.num_pages + extra)


def _tails_are_private(batch):
    """True when no request shares its very last page with another request."""
    last = {}
    for r in range(batch.num_requests):
        n = -(-int(batch.kv_lens[r]) // batch.page_size)
        last.setdefault(int(batch.block_tables[r, n - 1]), []).append(r)
    return all(len(v) == 1 for v in last.values())


@pytest.mark.parametrize("seed", range(12))
def test_advance_keeps_the_schedule_valid_over_decode_steps(seed):
    b = _roomy(wl.random_forest_batch(300 + seed, max_requests=12, max_node_tokens=150))
    if not _tails_are_private(b):
        pytest.skip("covered by test_advance_is_refused_for_shared_tails")
    plan = pb.plan_for_batch(b)
    n_items = plan.stats().num_items
    cur = b
    for step in range(1, 70):                    # crosses several page boundaries per request
        cur = wl.decode_steps(cur, 1)
        pb.pat_plan_advance(plan, cur.kv_lens, cur.block_tables)
        if step % 7 == 0 or step == 69:
            ex = check_schedule(cur, plan)
            assert ex["num_items"] == n_items    # same packs, only tails grew
    # a fresh plan of the final batch covers the same (request, page) pairs
    fresh = check_schedule(cur, pb.plan_for_batch(cur))
    cover = lambda ex: op.cover_multiset([(q, s, n) for q, s, n, _ in _items(ex)])
    assert cover(plan.export()) == cover(fresh)


def test_advance_of_a_subset_and_by_many_tokens():
    b = _roomy(wl.config("C2"))
    plan = pb.plan_for_batch(b)
    grow = np.arange(b.num_requests) % 3 == 0
    cur = wl.decode_steps(b, 100, grow)          # 100 tokens at once: 6-7 new pages each
    pb.pat_plan_advance(plan, cur.kv_lens, cur.block_tables)
    check_schedule(cur, plan)
    st = plan.stats()
    assert st.total_kv_tokens == int(cur.kv_lens.astype(np.int64).sum())
    assert st.unique_kv_tokens == cur.unique_kv_tokens()


def test_advance_runs_out_of_reserve_and_other_refusals():
    b = _roomy(wl.config("C1"))
    plan = pb.plan_for_batch(b, tail_reserve_pages=2)
    ok = wl.decode_steps(b, 32)                  # exactly two more pages per request
    pb.pat_plan_advance(plan, ok.kv_lens, ok.block_tables)
    check_schedule(ok, plan)
    too_far = wl.decode_steps(ok, 1)
    with pytest.raises(pb.PatError) as ei:
        pb.pat_plan_advance(plan, too_far.kv_lens, too_far.block_tables)
    assert ei.value.status == pb.PAT_ERR_PLAN_STALE
    check_schedule(ok, plan)                     # a refused advance changes nothing
    with pytest.raises(pb.PatError) as ei:       # shrinking is not an advance
        pb.pat_plan_advance(plan, b.kv_lens, ok.block_tables)
    assert ei.value.status == pb.PAT_ERR_PLAN_STALE
    none = pb.plan_for_batch(b, tail_reserve_pages=-1)
    one_page = wl.decode_steps(b, b.page_size)
    with pytest.raises(pb.PatError) as ei:
        pb.pat_plan_advance(none, one_page.kv_lens, one_page.block_tables)
    assert ei.value.status == pb.PAT_ERR_PLAN_STALE
    bad = wl.decode_steps(b, 16)
    bad.block_tables[0, -(-int(bad.kv_lens[0]) // 16) - 1] = bad.num_pages + 5
    fresh = pb.plan_for_batch(b)
    with pytest.raises(pb.PatError) as ei:
        pb.pat_plan_advance(fresh, bad.kv_lens, bad.block_tables)
    assert ei.value.status == pb.PAT_ERR_BAD_PAGE_ID


def test_advance_is_refused_for_shared_tails():
    # two identical rows: both requests end inside shared pages, neither has an item of its own
    bt = np.array([[3, 4, 5], [3, 4, 5]], np.int32)
    kl = np.array([48, 48], np.int32)
    kw = dict(page_size=16, num_pages=16, num_q_heads=8, num_kv_heads=2, head_dim=128, dtype="bf16")
    plan = pb.pat_plan(bt, kl, **kw)
    bt2 = np.array([[3, 4, 5, 6], [3, 4, 5, 7]], np.int32)
    with pytest.raises(pb.PatError) as ei:
        pb.pat_plan_advance(plan, kl + 1, bt2)
    assert ei.value.status == pb.PAT_ERR_PLAN_STALE


def test_own_run_time_model_keeps_the_invariants():
    b = wl.config("C2")
    default = pb.plan_for_batch(b)
    check_schedule(b, default)
    # a model that makes packed workgroups look cheap gives them longer chunks
    cheap = pb.plan_for_batch(b, model_ns=(1000, 5, 4000, 20))
    check_schedule(b, cheap)
    assert list(cheap.stats().tile_histogram)[4] < list(default.stats().tile_histogram)[4]
    for bad in ((-1, 26, 4000, 20), (13000, 0, 4000, 20), (13000, 26, 4000, 0)):
        with pytest.raises(pb.PatError) as ei:
            pb.plan_for_batch(b, model_ns=bad)
        assert ei.value.status == pb.PAT_ERR_INVALID_ARG


def test_many_round_batches_are_cut_only_where_the_launch_would_wait_for_one_workgroup():
    # C4: a document node (8192 tokens, one packed workgroup per KV head) runs about as long as the
    # whole launch is estimated to take and starts first: it stays whole, while a finer cut
    # would add partials to write and merge
    b = wl.config("C4")
    plan = pb.plan_for_batch(b)
    ex = check_schedule(b, plan)
    assert int(np.max(ex["item_kv_len"])) == 8192
    # one request far longer than a CU's share of the batch would keep the launch waiting: cut
    rng = np.random.default_rng(5)
    lens = np.concatenate([[32768], rng.integers(400, 600, 200)])
    long_one = wl.tree_batch([201], [lambda r, n: lens], num_q_heads=32, num_kv_heads=8, dtype="bf16", seed=5)
    plan = pb.plan_for_batch(long_one)
    ex = check_schedule(long_one, plan)
    assert plan.stats().num_items >= 201 + 7 and int(np.max(ex["item_kv_len"])) <= 4096
    # with few slots the same request is no longer than the launch: nothing is cut
    plan = pb.plan_for_batch(long_one, num_cus=4)
    check_schedule(long_one, plan)
    assert plan.stats().num_items == 201


def test_background_planning_gives_the_same_plan():
    batches = [wl.random_forest_batch(500 + i, max_requests=16) for i in range(6)] + [wl.config("C3")]
    jobs = [pb.plan_for_batch(b, background=True) for b in batches]
    for b, job in zip(batches, jobs):
        got = job.finish()
        want = pb.plan_for_batch(b)
        check_schedule(b, got)
        a, c = got.export(), want.export()
        assert all(np.array_equal(a[k], c[k]) for k in a if isinstance(a[k], np.ndarray))
    # errors of the planner come back from finish(); a job that is dropped is cleaned up
    bad = batches[0]
    bt = bad.block_tables.copy()
    bt[0, 0] = bad.num_pages + 7
    job = pb.pat_plan(bt, bad.kv_lens, page_size=16, num_pages=bad.num_pages, num_q_heads=bad.num_q_heads,
                      num_kv_heads=bad.num_kv_heads, head_dim=128, dtype=bad.dtype, background=True)
    with pytest.raises(pb.PatError) as ei:
        job.finish()
    assert ei.value.status == pb.PAT_ERR_BAD_PAGE_ID
    del jobs
    pb.plan_for_batch(batches[1], background=True)      # never finished: discarded on collection


def test_tile_solver_admits_every_tile_that_is_built():
    # the constraints of sec. "Multi-tile Kernel" restated for a CU of this GPU (LDS, bytes in
    # flight against latency x bandwidth, registers): every tile the library holds a kernel for
    # (the VALU cross-check tile aside) is in the feasible set, and oversized ones are not
    from paper_2511_22333_amd import calibrate
    tiles, need = calibrate.tile_solver()
    feasible = {(t["m"], t["n"]) for t in tiles if t["feasible"]}
    assert 32 * 1024 < need < 128 * 1024
    for tid, m, n in calibrate.built_tiles():
        if (m, n) != (16, 4):
            assert (m, n) in feasible, (tid, m, n)
    assert (256, 256) not in feasible and (128, 256) not in feasible      # LDS and registers
    assert (128, 16) not in feasible                                      # too little in flight


def test_short_unshared_batches_run_as_wavefront_items():
    # tile n follows the KV length: a launch of many rounds made of nothing but unshared requests
    # of up to 384 tokens takes the n = 32 tile (one wavefront per request and KV head, no cuts);
    # one long request, or a shared prefix, keeps the n = 128 tile
    rng = np.random.default_rng(9)
    lens = rng.integers(20, 385, 2048)
    short = wl.tree_batch([2048], [lambda r, n: lens], num_q_heads=32, num_kv_heads=8, dtype="bf16", seed=9)
    plan = pb.plan_for_batch(short)
    check_schedule(short, plan)
    st = plan.stats()
    assert st.num_wave_items == 2048 * 8 and st.num_workers == 256 and st.num_slots == 0
    assert list(st.tile_histogram)[:3] == [0, 0, 2048]
    lens2 = lens.copy()
    lens2[7] = 385
    longer = wl.tree_batch([2048], [lambda r, n: lens2], num_q_heads=32, num_kv_heads=8, dtype="bf16", seed=9)
    assert pb.plan_for_batch(longer).stats().num_wave_items == 0
    assert pb.plan_for_batch(short, wave_kv_tokens=-1).stats().num_wave_items == 0
    for name in ("C2", "C3", "C4", "C5"):
        assert pb.plan_for_batch(wl.config(name)).stats().num_wave_items == 0


def test_very_short_leaves_run_as_wavefront_items_beside_packed_tiles():
    # 16-row packs of at most 96 tokens that would fill more than one round of workgroups by themselves
    # run as wavefront items whatever else the launch holds; the shared prefix keeps its packed tile
    b = wl.tree_batch([1, 256], [2048, 64], num_q_heads=32, num_kv_heads=8, dtype="fp16", seed=3)
    plan = pb.plan_for_batch(b)
    check_schedule(b, plan)
    st = plan.stats()
    hist = list(st.tile_histogram)
    assert st.num_wave_items == 256 * 8 and hist[2] == 256 and hist[1] == 0 and hist[4] > 0
    # leaves of 128 tokens, or few enough leaves for one round: 16-row workgroups as before
    for B, L in (([1, 256], [2048, 128]), ([1, 48], [2048, 64])):
        other = wl.tree_batch(B, L, num_q_heads=32, num_kv_heads=8, dtype="fp16", seed=3)
        assert pb.plan_for_batch(other).stats().num_wave_items == 0
    assert pb.plan_for_batch(b, wave_kv_tokens=-1).stats().num_wave_items == 0


# ---- plan cache keyed by the block table ---------------------------------------------------------
def test_plan_cache_hits_advances_and_evicts():
    cache = pb.PlanCache(2)
    b = _roomy(wl.tree_batch([1, 3, 9], [96, 48, lambda rng, n: rng.integers(5, 120, n)],
                             num_q_heads=16, num_kv_heads=4, dtype="bf16", seed=31), extra=64)
    p0, how = cache.get(b)
    assert how == 0
    check_schedule(b, p0)
    p1, how = cache.get(b)                                     # the same batch: the same plan
    assert how == 1 and p1.handle.value == p0.handle.value
    wide = dataclasses.replace(b, block_tables=np.pad(b.block_tables, ((0, 0), (0, 5)), constant_values=-1))
    p1, how = cache.get(wide)                                  # unused entries are not part of the key
    assert how == 1 and p1.handle.value == p0.handle.value
    p2, how = cache.get(b, mode=pb.PAT_MODE_NO_SHARING)        # other options: another plan
    assert how == 0 and p2.handle.value != p0.handle.value
    grown = wl.decode_steps(b, 3)
    p3, how = cache.get(grown)                                 # decode steps later: advanced in place
    assert how == 2 and p3.handle.value == p0.handle.value
    check_schedule(grown, p3)
    p4, how = cache.get(grown)
    assert how == 1
    # a changed page id in the middle of a row is neither the same batch nor a successor
    other = dataclasses.replace(grown, block_tables=grown.block_tables.copy())
    other.block_tables[2, 1] = (int(other.block_tables[2, 1]) + 1) % other.num_pages
    p5, how = cache.get(other)
    assert how == 0
    check_schedule(other, p5)
    # capacity 2: the no-sharing plan was the least recently used and is gone; asking again plans anew
    _, how = cache.get(b, mode=pb.PAT_MODE_NO_SHARING)
    assert how in (0, 2)
    # a request that got shorter is not a successor
    shorter = dataclasses.replace(other, kv_lens=other.kv_lens - 1)
    _, how = cache.get(shorter)
    assert how == 0
    cache.close()
    with pytest.raises(pb.PatError):
        pb.PlanCache(0)
