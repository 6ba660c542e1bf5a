"""GPU parity: the HIP path through the C ABI against the fp64 oracle, element by element,
on the same seeded inputs.  Tolerances: max-abs 2e-3 (fp16), 1e-2 (bf16) on out; 1e-4 on lse (scaled
with |lse| above 32: gpu_util.lse_tol)."""
import numpy as np
import pytest
import torch

from paper_2511_22333_amd import binding as pb
from paper_2511_22333_amd import workloads as wl

from gpu_util import compare, compare_all_requests_in_groups, parity, run_hip, run_oracle, to_gpu

pytestmark = pytest.mark.gpu


def _log(msg):
    print(msg, flush=True)


def test_c1_tiny_fp16():
    _log("case C1")
    (err, lerr), plan = parity(wl.config("C1"))
    _log(f"C1 err={err:.2e} lse_err={lerr:.2e} items={plan.stats().num_items}")


@pytest.mark.parametrize("layout", ["NHD", "HND"])
@pytest.mark.parametrize("seed", [0, 1, 2, 3, 4, 5])
def test_random_forests_poisoned(seed, layout):
    dtype = "bf16" if seed % 2 else "fp16"
    b = wl.random_forest_batch(seed, duplicate_rows=(seed % 3 == 0), dtype=dtype,
                               max_requests=14, max_node_tokens=150)
    _log(f"case forest seed={seed} layout={layout} dtype={dtype} B={b.num_requests}")
    parity(b, layout=layout)


@pytest.mark.parametrize("kv", [1, 2, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 257, 1000])
def test_single_request_ragged_lengths(kv):
    _log(f"case single kv={kv}")
    b = wl.tree_batch([1], [kv], num_q_heads=8, num_kv_heads=2, dtype="bf16", seed=kv)
    parity(b)


@pytest.mark.parametrize("heads", [(4, 4), (8, 8), (16, 8), (32, 8), (64, 8), (8, 1), (32, 32),
                                   # odd head counts and group sizes that are no power of two: a last
                                   # workgroup with one KV head, a merge wavefront with one q head
                                   (3, 3), (6, 3), (3, 1), (5, 5), (12, 4), (1, 1),
                                   # groups wider than a 16-row block, up to more rows per request than
                                   # one packed tile of 64 holds
                                   (32, 1), (64, 2), (71, 1), (40, 5)])
def test_head_configurations(heads):
    hq, hkv = heads
    _log(f"case heads {hq}/{hkv}")
    b = wl.tree_batch([1, 3, 9], [64, 48, lambda rng, n: rng.integers(1, 200, n)],
                      num_q_heads=hq, num_kv_heads=hkv, dtype="fp16", seed=7)
    parity(b)


def test_deep_tree_and_forced_merges():
    _log("case deep tree")
    b = wl.tree_batch([1, 2, 4, 8, 16], [16, 16, 32, 16, lambda rng, n: rng.integers(1, 90, n)],
                      num_q_heads=8, num_kv_heads=2, dtype="bf16", seed=11)
    (_, _), plan = parity(b)
    assert plan.stats().num_merged_children > 0


def test_rows_exceed_largest_tile():
    _log("case rows > m")
    b = wl.tree_batch([1, 70], [256, lambda rng, n: rng.integers(1, 40, n)],
                      num_q_heads=16, num_kv_heads=2, dtype="bf16", seed=13)    # 560 rows
    parity(b)


@pytest.mark.parametrize("mode", [pb.PAT_MODE_PAT, pb.PAT_MODE_NAIVE_PER_NODE, pb.PAT_MODE_NO_SHARING])
@pytest.mark.parametrize("policy,target", [(pb.PAT_SPLIT_AUTO, 0), (pb.PAT_SPLIT_MEAN, 0),
                                           (pb.PAT_SPLIT_NONE, 0), (pb.PAT_SPLIT_TARGET, 16),
                                           (pb.PAT_SPLIT_TARGET, 48)])
def test_result_does_not_depend_on_the_plan(mode, policy, target):
    # sec. "Output Merge": any partition of the KV merges to the same attention
    _log(f"case plan-invariance mode={mode} policy={policy} target={target}")
    b = wl.tree_batch([2, 4, 12], [96, 64, lambda rng, n: rng.integers(1, 300, n)],
                      num_q_heads=8, num_kv_heads=2, dtype="fp16", seed=17)
    parity(b, mode=mode, split_policy=policy, split_target_tokens=target)


@pytest.mark.parametrize("tile", [0, 1, 2, 3, 4])
def test_every_tile_gives_the_same_attention(tile):
    # force_tile runs the whole batch through one tile family (rows are cut to its m)
    _log(f"case force_tile={tile}")
    b = wl.tree_batch([1, 3, 12], [128, 80, lambda rng, n: rng.integers(1, 150, n)],
                      num_q_heads=8, num_kv_heads=2, dtype="bf16", seed=23)
    (_, _), plan = parity(b, force_tile=tile)
    hist = list(plan.stats().tile_histogram)
    assert hist[tile] == plan.stats().num_entries


@pytest.mark.parametrize("s_req", [9, 24])          # 36 rows -> 64-row tile, 96 rows -> 128-row tile
@pytest.mark.parametrize("node_tokens", [16, 32, 48, 64, 80, 128, 144, 192, 208, 256, 272, 336, 528])
def test_packed_tiles_over_tile_counts(node_tokens, s_req):
    # one shared node of 1..9 tiles (a page count that is no multiple of four ends in a
    # partial tile), kept whole, so every path of the packed tile's pipeline is taken
    _log(f"case packed node_tokens={node_tokens} s={s_req}")
    b = wl.tree_batch([1, s_req], [node_tokens, lambda rng, n: rng.integers(1, 40, n)],
                      num_q_heads=8, num_kv_heads=2, dtype="bf16", seed=node_tokens + s_req)
    (_, _), plan = parity(b, split_policy=pb.PAT_SPLIT_NONE)
    hist = list(plan.stats().tile_histogram)
    assert hist[3 if s_req == 9 else 4] == 1


@pytest.mark.parametrize("loud_half", [0, 1])
@pytest.mark.parametrize("s_req", [9, 24])
def test_packed_tile_row_maximum_spans_both_token_halves(s_req, loud_half):
    # The packed tile splits the 32 tokens a wavefront handles over its two lane halves (half h
    # holds tokens 4h .. 4h + 3 of every eight); the running maximum has to be the maximum over
    # both.  The keys of one half are made 40 times louder than the rest, so the scores there
    # exceed the other half's by far more than an exponential taken against the wrong maximum
    # can hold.
    _log(f"case packed loud half={loud_half} s={s_req}")
    b = wl.tree_batch([1, s_req], [256, lambda rng, n: rng.integers(1, 40, n)],
                      num_q_heads=8, num_kv_heads=2, dtype="bf16", seed=91 + s_req)
    q, kp, vp, strides = wl.make_tensors(b, poison=True)
    P = b.page_size
    for j in range(256 // P):
        pid = int(b.block_tables[0, j])
        for t in range(P):
            if ((t >> 2) & 1) == loud_half:
                kp[pid, t] *= 40.0
    want, want_lse = run_oracle(b, (q, kp, vp, strides))
    out, lse, plan = run_hip(b, to_gpu((q, kp, vp, strides)), split_policy=pb.PAT_SPLIT_NONE)
    assert list(plan.stats().tile_histogram)[3 if s_req == 9 else 4] == 1
    compare(b, out, lse, want, want_lse)


@pytest.mark.parametrize("tile", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("kind", ["loud", "identical"])
def test_extreme_scores_on_every_tile(tile, kind):
    # loud: keys 30 times N(0,1), so the softmax is close to one-hot and scores differ by hundreds;
    # identical: every key of a request's context is the same vector, so the output is the mean of
    # the values whatever the query (and every running maximum stays where the first tile put it)
    _log(f"case extreme scores tile={tile} kind={kind}")
    b = wl.tree_batch([1, 3, 12], [128, 80, lambda rng, n: rng.integers(1, 150, n)],
                      num_q_heads=8, num_kv_heads=2, dtype="bf16", seed=29)
    q, kp, vp, strides = wl.make_tensors(b, poison=True)
    live = torch.from_numpy(b.referenced_pages().astype(np.int64))
    if kind == "loud":
        kp[live] *= 30.0
    else:
        kp[live] = kp[live][0, 0].clone()          # one [Hkv, d] row everywhere
    want, want_lse = run_oracle(b, (q, kp, vp, strides))
    out, lse, plan = run_hip(b, to_gpu((q, kp, vp, strides)), force_tile=tile)
    compare(b, out, lse, want, want_lse)


@pytest.mark.parametrize("lens", [[700] + [20] * 9, [700] * 4, [300, 40, 40]])
def test_merge_mappings_for_short_and_long_partial_lists(lens):
    # The merge kernel maps a (request, head pair) or a (request, head) to a wavefront depending
    # on the mean length of the partial lists, and takes lists of more than 28 partials in
    # chunks: one long list among short ones, long lists only, and a few partials each.
    _log(f"case merge lists {lens[:3]}..")
    b = wl.tree_batch([len(lens)], [lambda rng, n: np.array(lens)], num_q_heads=8, num_kv_heads=2,
                      dtype="fp16", seed=len(lens))
    (_, _), plan = parity(b, split_policy=pb.PAT_SPLIT_TARGET, split_target_tokens=16)
    ex = plan.export()
    n_parts = np.diff(ex["req_slot_off"])
    assert n_parts.max() == -(-max(lens) // 16)


@pytest.mark.parametrize("layout", ["NHD", "HND"])
@pytest.mark.parametrize("wave_kv", [16, 48, 100000])
def test_wavefront_items_on_forests(wave_kv, layout):
    # the 16-row packs of a forest cut into parts of at most wave_kv tokens, every (part, KV head)
    # walked by one wavefront of a persistent workgroup next to the packed tiles of the shared
    # nodes: parts of one stage, of several stages with a ragged last one, and whole packs
    for seed in (3, 4, 8):
        b = wl.random_forest_batch(seed, dtype="bf16" if seed % 2 else "fp16", max_requests=40,
                                   max_node_tokens=400, num_q_heads=16, num_kv_heads=4)
        _log(f"case wave items seed={seed} wave_kv={wave_kv} layout={layout} B={b.num_requests}")
        (_, _), plan = parity(b, layout=layout, wave_kv_tokens=wave_kv, wave_max_tokens=100000)
        st = plan.stats()
        assert st.num_wave_items > 0 and st.num_workers > 0
        assert list(st.tile_histogram)[2] > 0


def test_short_unshared_batch_takes_the_wavefront_tile_by_itself():
    # the planner's own choice of n = 32: 2048 unshared requests of up to 384 tokens, every request
    # against the oracle
    rng = np.random.default_rng(9)
    lens = rng.integers(1, 385, 2048)
    b = wl.tree_batch([2048], [lambda r, n: lens], num_q_heads=16, num_kv_heads=4, dtype="bf16", seed=61)
    _log("case short unshared batch")
    tensors = wl.make_tensors(b, device="cuda")
    out, lse, plan = run_hip(b, tensors)
    st = plan.stats()
    assert st.num_wave_items == 2048 * 4 and list(st.tile_histogram)[2] == 2048
    err, lerr = compare_all_requests_in_groups(b, out, lse, tensors, group=512)
    _log(f"short unshared: err={err:.2e} lse_err={lerr:.2e}")


@pytest.mark.parametrize("case", [
    # (B, L, heads, dtype): hundreds of very short leaves under packed prefixes -- the leaves run as
    # wavefront items by the planner's own rule, the prefix as packed tiles cut by the few-round search
    ([1, 320], [1008, (1, 96)], (32, 8), "bf16"),
    ([2, 300], [(300, 1500), (1, 64)], (64, 8), "fp16"),           # ragged prefixes: leaves of up to 79
    ([1, 4, 288], [704, 160, (1, 96)], (16, 8), "bf16"),
    ([1, 260], [2048, (40, 96)], (8, 8), "fp16"),
    # the same shapes with leaves too long for that rule: 16-row workgroups, cut searched the same way
    ([1, 320], [1008, (1, 200)], (32, 8), "bf16"),
    ([1, 96], [4096, (100, 160)], (64, 8), "fp16"),
])
def test_batches_of_a_few_rounds_with_short_leaves(case):
    B, L, (hq, hkv), dtype = case
    spec = [(lambda rng, n, lo=x[0], hi=x[1]: rng.integers(lo, hi + 1, n)) if isinstance(x, tuple) else x for x in L]
    b = wl.tree_batch(B, spec, num_q_heads=hq, num_kv_heads=hkv, dtype=dtype, seed=hq + len(B))
    _log(f"case few rounds B={B} L={L} heads={hq}/{hkv} {dtype}")
    tensors = wl.make_tensors(b, device="cuda", poison=True)
    out, lse, plan = run_hip(b, tensors)
    st = plan.stats()
    short = all(not isinstance(x, tuple) or x[1] <= 96 for x in L[-1:])
    assert (st.num_wave_items > 0) == short, (st.num_wave_items, short)
    err, lerr = compare_all_requests_in_groups(b, out, lse, tensors, group=128)
    _log(f"  items={st.num_items} workgroups={st.num_workgroups} wave_items={st.num_wave_items} "
         f"tiles={list(st.tile_histogram)[:5]} err={err:.2e} lse_err={lerr:.2e}")


@pytest.mark.parametrize("seed", range(12))
def test_random_trees_under_the_default_plan(seed):
    # (B, L) trees drawn at random -- one to three shared levels, 24 to 384 requests, node lengths from
    # one page to thousands of tokens, the paper's head settings, both dtypes, both layouts -- under
    # the planner's own choices (one round, a few rounds, many rounds, wavefront items), every request
    # against the oracle
    rng = np.random.default_rng(4000 + seed)
    levels = int(rng.integers(1, 4))
    B = [int(rng.choice([1, 2, 4]))]
    for _ in range(levels - 1):
        B.append(B[-1] * int(rng.choice([1, 2, 4])))
    B.append(B[-1] * int(rng.choice([6, 12, 24])))
    hi = [int(rng.choice([16, 64, 400, 3000])) for _ in B]
    L = [(lambda r, n, h=h: r.integers(1, h + 1, n)) for h in hi]
    hq, hkv = [(64, 8), (32, 8), (16, 8), (32, 32)][seed % 4]
    dtype, layout = ("bf16", "fp16")[seed % 2], ("NHD", "HND")[(seed // 2) % 2]
    b = wl.tree_batch(B, L, num_q_heads=hq, num_kv_heads=hkv, dtype=dtype, seed=4000 + seed)
    _log(f"case random tree seed={seed} B={B} max L={hi} heads={hq}/{hkv} {dtype} {layout} "
         f"{b.unique_kv_bytes() / 1e6:.1f} MB")
    tensors = wl.make_tensors(b, device="cuda", poison=True, layout=layout)
    out, lse, plan = run_hip(b, tensors)
    st = plan.stats()
    err, lerr = compare_all_requests_in_groups(b, out, lse, tensors, group=128)
    _log(f"  items={st.num_items} workgroups={st.num_workgroups} wave_items={st.num_wave_items} "
         f"tiles={list(st.tile_histogram)[:5]} err={err:.2e} lse_err={lerr:.2e}")


def test_wavefront_items_many_per_wavefront():
    # far more items than the 8 x 4 wavefronts of four persistent workgroups: every wavefront walks a
    # list of items, requesting the next item's rows while it finishes the current one
    rng = np.random.default_rng(3)
    lens = rng.integers(1, 700, 96)
    b = wl.tree_batch([96], [lambda r, n: lens], num_q_heads=8, num_kv_heads=2, dtype="bf16", seed=53)
    _log("case wave items, long lists")
    (_, _), plan = parity(b, wave_kv_tokens=64, wave_max_tokens=100000, num_cus=4)
    st = plan.stats()
    assert st.num_workers == 4 and st.num_wave_items > 20 * 32


@pytest.mark.parametrize("node_tokens", [16, 32, 48, 240])
def test_tile_follows_the_kv_length_of_a_small_group(node_tokens):
    # 5 requests x 4 heads = 20 rows: below the crossover the node runs as two 16-row blocks,
    # from it on as one 64-row packed workgroup per KV head; same attention either way
    _log(f"case 20 rows over {node_tokens} tokens")
    b = wl.tree_batch([1, 5], [node_tokens, lambda rng, n: rng.integers(1, 40, n)],
                      num_q_heads=8, num_kv_heads=2, dtype="bf16", seed=node_tokens)
    (_, _), plan = parity(b, split_policy=pb.PAT_SPLIT_NONE)
    ex = plan.export()
    shared = [e for e in range(ex["num_entries"]) if ex["item_kv_len"][ex["entry_item"][e]] == node_tokens
              and np.diff(ex["item_req_off"])[ex["entry_item"][e]] == 5]
    tiles = sorted(int(ex["entry_tile"][e]) for e in shared)
    assert tiles == ([1, 1] if node_tokens < 48 else [3])


@pytest.mark.parametrize("layout", ["NHD", "HND"])
def test_two_kernel_launch_on_forests_and_in_a_graph(layout):
    # dual_launch: packed tiles as 512-thread workgroups on the caller's stream, 16-row tiles as
    # 256-thread workgroups of one KV head on the plan's own stream, forked from and joined to the
    # caller's (sec. "Multi-Stream Forward"); eagerly, and captured in a HIP graph that is replayed
    # three times with eager work in between
    for seed in (1, 2, 6):
        b = wl.random_forest_batch(seed, dtype="bf16" if seed % 2 else "fp16", max_requests=30,
                                   max_node_tokens=300, num_q_heads=16, num_kv_heads=4,
                                   duplicate_rows=(seed % 3 == 0))
        _log(f"case two kernels seed={seed} layout={layout} B={b.num_requests}")
        cpu = wl.make_tensors(b, poison=True, layout=layout)
        want, want_lse = run_oracle(b, cpu)
        q, kp, vp, st = to_gpu(cpu)
        plan = pb.plan_for_batch(b, dual_launch=1)
        dev, ws = pb.alloc_plan_buffers(plan)
        pb.pat_plan_upload(plan, dev)
        out = torch.full_like(q, float("nan"))
        lse = torch.full((b.num_requests, b.num_q_heads), float("nan"), dtype=torch.float32, device="cuda")
        pb.pat_decode_attention(plan, q, kp, vp, st, b.softmax_scale, out, lse, ws)
        torch.cuda.synchronize()
        compare(b, out, lse, want, want_lse)
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=side):
            pb.pat_decode_attention(plan, q, kp, vp, st, b.softmax_scale, out, lse, ws)
        for _ in range(3):
            out.fill_(float("nan"))
            lse.fill_(float("nan"))
            ws.fill_(0xFF)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            compare(b, out, lse, want, want_lse)


@pytest.mark.parametrize("spin_limit", [0, 3, -1])
@pytest.mark.parametrize("fused", [1, -1])
def test_merge_inside_the_forward_launch(fused, spin_limit):
    # fused_merge: the forward launch merges (arrival counters; in launches of one round, claimed
    # and bounded waits).  spin_limit 0 makes every claimed wait give up at once, so the arrival that
    # completes a request merges it (the fallback); 3 mixes both; -1 is the default.  Against the
    # oracle, twice per plan (the state words and counters must be back to their initial values).
    pb.pat_debug_set_spin_limit(spin_limit)
    try:
        cases = [wl.random_forest_batch(s, dtype="bf16" if s % 2 else "fp16", max_requests=30,
                                        max_node_tokens=300, num_q_heads=16, num_kv_heads=4,
                                        duplicate_rows=(s % 3 == 0)) for s in (0, 1, 5)]
        cases.append(wl.tree_batch([1, 24], [1024, lambda rng, n: rng.integers(1, 300, n)],
                                   num_q_heads=32, num_kv_heads=8, dtype="bf16", seed=71))     # one round
        cases.append(wl.tree_batch([2, 8, 400], [512, 256, lambda rng, n: rng.integers(1, 200, n)],
                                   num_q_heads=16, num_kv_heads=8, dtype="bf16", seed=72))     # many rounds
        for b in cases:
            _log(f"case fused merge={fused} spin={spin_limit} B={b.num_requests}")
            cpu = wl.make_tensors(b, poison=True)
            want, want_lse = run_oracle(b, cpu)
            q, kp, vp, st = to_gpu(cpu)
            plan = pb.plan_for_batch(b, fused_merge=fused)
            assert (plan.stats().fused_merge != 0) == (fused == 1)
            dev, ws = pb.alloc_plan_buffers(plan)
            pb.pat_plan_upload(plan, dev)
            for _ in range(2):
                out = torch.full_like(q, float("nan"))
                lse = torch.full((b.num_requests, b.num_q_heads), float("nan"), dtype=torch.float32, device="cuda")
                ws.fill_(0xFF)
                pb.pat_decode_attention(plan, q, kp, vp, st, b.softmax_scale, out, lse, ws)
                torch.cuda.synchronize()
                compare(b, out, lse, want, want_lse)
    finally:
        pb.pat_debug_set_spin_limit(-1)


def test_debug_trace_records_every_workgroup():
    b = wl.config("C1")
    q, kp, vp, st = to_gpu(wl.make_tensors(b))
    plan = pb.plan_for_batch(b)
    dev, ws = pb.alloc_plan_buffers(plan)
    pb.pat_plan_upload(plan, dev)
    n = plan.stats().num_workgroups
    tr = torch.zeros(n * 8, dtype=torch.int64, device="cuda")
    out = torch.empty_like(q)
    pb.pat_debug_set_trace(tr)
    try:
        pb.pat_forward(plan, q, kp, vp, st, b.softmax_scale, out, None, ws)
        torch.cuda.synchronize()
    finally:
        pb.pat_debug_set_trace(None)
    t = tr.cpu().numpy().reshape(n, 8)
    assert (t[:, 0] > 0).all() and (t[:, 1] >= t[:, 0]).all()
    assert set((t[:, 3] >> 32).tolist()) <= {0, 1, 2, 3, 4}
    tr.zero_()
    pb.pat_forward(plan, q, kp, vp, st, b.softmax_scale, out, None, ws)     # switched off again
    torch.cuda.synchronize()
    assert int(tr.abs().sum()) == 0


def test_lazy_update_follows_decode_steps():
    # plan once, then advance the plan instead of planning again (sec. "Pack Scheduler")
    import dataclasses
    _log("case lazy update")
    b = wl.tree_batch([1, 3, 9], [96, 48, lambda rng, n: rng.integers(5, 120, n)],
                      num_q_heads=16, num_kv_heads=4, dtype="bf16", seed=31)
    b = dataclasses.replace(b, num_pages=b.num_pages + 64)      # free pages to grow into
    plan = pb.plan_for_batch(b)
    dev, ws = pb.alloc_plan_buffers(plan)
    cur = b
    for steps in (0, 1, 15, 40):
        if steps:
            cur = wl.decode_steps(cur, steps)
            pb.pat_plan_advance(plan, cur.kv_lens, cur.block_tables)
            q0, kp0, vp0, st0 = to_gpu(wl.make_tensors(cur))
            with pytest.raises(pb.PatError) as ei:                  # the device copy is stale
                pb.pat_decode_attention(plan, q0, kp0, vp0, st0, cur.softmax_scale,
                                        torch.empty_like(q0), None, ws)
            assert ei.value.status == pb.PAT_ERR_PLAN_NOT_UPLOADED
        pb.pat_plan_upload(plan, dev)
        cpu = wl.make_tensors(cur, poison=True)
        want, want_lse = run_oracle(cur, cpu)
        q, kp, vp, st = to_gpu(cpu)
        out = torch.full_like(q, float("nan"))
        lse = torch.full((cur.num_requests, cur.num_q_heads), float("nan"), dtype=torch.float32,
                         device="cuda")
        ws.fill_(0xFF)
        pb.pat_decode_attention(plan, q, kp, vp, st, cur.softmax_scale, out, lse, ws)
        torch.cuda.synchronize()
        compare(cur, out, lse, want, want_lse)


def test_separate_stages_and_null_lse():
    b = wl.config("C1")
    cpu = wl.make_tensors(b, poison=True)
    want, want_lse = run_oracle(b, cpu)
    out, lse, _ = run_hip(b, to_gpu(cpu), separate_stages=True)
    compare(b, out, lse, want, want_lse)
    out, lse, _ = run_hip(b, to_gpu(cpu), with_lse=False)
    compare(b, out, None, want, want_lse)


def test_plan_reuse_across_calls_and_new_values():
    # one plan serves many calls (lazy update, sec. "Pack Scheduler")
    b = wl.tree_batch([1, 6], [128, lambda rng, n: rng.integers(1, 100, n)], num_q_heads=8,
                      num_kv_heads=2, dtype="bf16", seed=19)
    plan = pb.plan_for_batch(b)
    dev, ws = pb.alloc_plan_buffers(plan)
    pb.pat_plan_upload(plan, dev)
    for seed in (1, 2, 3):
        cpu = wl.make_tensors(b, seed=seed, poison=True)
        q, kp, vp, st = to_gpu(cpu)
        out = torch.empty_like(q)
        lse = torch.empty(b.num_requests, b.num_q_heads, dtype=torch.float32, device="cuda")
        pb.pat_decode_attention(plan, q, kp, vp, st, b.softmax_scale, out, lse, ws)
        torch.cuda.synchronize()
        want, want_lse = run_oracle(b, cpu)
        compare(b, out, lse, want, want_lse)


def test_non_default_stream():
    b = wl.config("C1")
    cpu = wl.make_tensors(b)
    want, want_lse = run_oracle(b, cpu)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        out, lse, _ = run_hip(b, to_gpu(cpu))
    compare(b, out, lse, want, want_lse)


def test_small_workspace_is_refused():
    b = wl.config("C1")
    q, kp, vp, st = to_gpu(wl.make_tensors(b))
    plan = pb.plan_for_batch(b)
    dev, ws = pb.alloc_plan_buffers(plan)
    pb.pat_plan_upload(plan, dev)
    out = torch.empty_like(q)
    with pytest.raises(pb.PatError) as ei:
        pb.pat_decode_attention(plan, q, kp, vp, st, 1.0, out, None, ws[:256])
    assert ei.value.status == -5
    with pytest.raises(pb.PatError) as ei:
        pb.pat_decode_attention(plan, q, kp, vp, (st[0], st[1] + 1, st[2]), 1.0, out, None, ws)
    assert ei.value.status == -1


@pytest.mark.parametrize("name", ["C2", "C3", "T3", "H32", "H16"])
def test_full_size_configs_all_requests(name):
    _log(f"case {name} full")
    b = wl.config(name)
    (err, lerr), plan = parity(b, poison=False)
    st = plan.stats()
    _log(f"{name} err={err:.2e} lse_err={lerr:.2e} items={st.num_items} wgs={st.num_workgroups}")


@pytest.mark.parametrize("name", ["C4", "C5"])
def test_largest_configs_all_requests(name):
    # the two largest shapes at the benchmark's full size and in its launch configuration (default
    # plan: row blocks over the 2048-row root on C4, the unit queue on C5), every request against
    # the oracle, whose pages are gathered from the GPU pools 32 requests at a time
    _log(f"case {name} full, all requests")
    b = wl.config(name)
    tensors = wl.make_tensors(b, device="cuda")
    out, lse, plan = run_hip(b, tensors)
    assert torch.isfinite(out.float()).all() and torch.isfinite(lse).all()
    err, lerr = compare_all_requests_in_groups(b, out, lse, tensors)
    st = plan.stats()
    _log(f"{name} all {b.num_requests} requests err={err:.2e} lse_err={lerr:.2e} "
         f"wgs={st.num_workgroups} tiles={list(st.tile_histogram)[:5]}")


def test_unit_queue_gives_the_same_result_on_every_launch():
    # A batch of many rounds of long unshared requests runs its 16-row units through the forward
    # kernel's queue (persistent workgroups drawing from an atomic counter that the last one to
    # leave resets): several launches of one plan must agree bit for bit, also with a fresh upload
    # in between, and every request must agree with the oracle.
    _log("case unit queue")
    rng = np.random.default_rng(17)
    lens = rng.integers(1900, 2400, 140)
    b = wl.tree_batch([140], [lambda r, n: lens], num_q_heads=16, num_kv_heads=8, dtype="bf16", seed=41)
    q, kp, vp, st = wl.make_tensors(b, device="cuda")
    plan = pb.plan_for_batch(b)
    assert plan.stats().num_workgroups >= 512
    dev, ws = pb.alloc_plan_buffers(plan)
    pb.pat_plan_upload(plan, dev)
    outs = []
    for i in range(3):
        out = torch.full_like(q, float("nan"))
        lse = torch.full((b.num_requests, b.num_q_heads), float("nan"), dtype=torch.float32, device="cuda")
        pb.pat_decode_attention(plan, q, kp, vp, st, b.softmax_scale, out, lse, ws)
        torch.cuda.synchronize()
        outs.append((out, lse))
        if i == 1:
            pb.pat_plan_upload(plan, dev)               # counters start from zero again
    for out, lse in outs[1:]:
        assert torch.equal(out, outs[0][0]) and torch.equal(lse, outs[0][1])
    err, lerr = compare_all_requests_in_groups(b, outs[0][0], outs[0][1], (q, kp, vp, st), group=70)
    _log(f"unit queue: all 140 requests err={err:.2e} lse_err={lerr:.2e}")
