"""Offline derivation of the tile family and of the planner's constants on the GPU at hand
(sec. "Multi-tile Kernel": latency-versus-size microbenchmark, constraints on feasible tiles,
kernel-equivalence run, KV-length decision; sec. "Tile Selection").

    python -m paper_2511_22333_amd.calibrate latency       # L and B of the memory system
    python -m paper_2511_22333_amd.calibrate solver        # feasible (m, n) under the constraints
    python -m paper_2511_22333_amd.calibrate equivalence   # every tile on a no-prefix batch, KV 1024
    python -m paper_2511_22333_amd.calibrate sweep-kv      # KV-length thresholds of the selector
    python -m paper_2511_22333_amd.calibrate model         # run-time model of the split (default)
    python -m paper_2511_22333_amd.calibrate grid          # (B, L) trees x head settings x modes
    python -m paper_2511_22333_amd.calibrate timeline C3   # per-workgroup timeline of one forward launch

The run-time model:

The device-aware split (PAT_SPLIT_AUTO) balances one-round batches with a linear model of a
workgroup's run time: packed workgroup = a + b * tokens, 16-row workgroup = c + d * tokens *
KV heads (ns); the 64-row packed tile takes fixed fractions of a and b.  The paper derives its tile table and split thresholds offline from latency
microbenchmarks on the target GPU (sec. "Multi-tile Kernel", "Tile Selection"); this is that step
for the model used here: it runs tree-shaped batches that fill the chip once, reads every
workgroup's start and end time from the kernel's timeline records (pat_debug_set_trace) and fits
the four constants by least squares.  The result can be passed to pat_plan through
pat_plan_opts.model_ns (binding: model_ns=...).

    python -m paper_2511_22333_amd.calibrate            # prints the fit and one JSON line
"""
from __future__ import annotations

import json
import sys

import numpy as np
import torch

from . import binding as pb
from . import workloads as wl


def _one_round_batches(num_q_heads: int = 32):
    """(B, L) trees in the shape of the Llama-3-8B benchmark layer: one shared root, 32 leaves."""
    out = []
    for seed, (root, lo, hi) in enumerate([(2048, 64, 512), (4096, 64, 512), (4096, 256, 1024),
                                           (8192, 64, 512), (1024, 32, 256), (6144, 128, 768)]):
        out.append(wl.tree_batch([1, 32], [root, lambda rng, n, lo=lo, hi=hi: rng.integers(lo, hi + 1, n)],
                                 num_q_heads=num_q_heads, num_kv_heads=8, dtype="bf16", seed=7000 + seed,
                                 name=f"cal{seed}"))
    return out


def workgroup_times(batch, launches: int = 6, model_ns=None):
    """[(tile rows m, tokens, heads, ns)] for every workgroup of `launches` traced forward launches,
    each on its own copy of the KV pools (so nothing is found in a cache)."""
    plan = pb.plan_for_batch(batch, model_ns=model_ns)
    ex, st = plan.export(), plan.stats()
    dev, ws = pb.alloc_plan_buffers(plan)
    pb.pat_plan_upload(plan, dev)
    # workgroup -> entry, in launch order: ceil(Hkv / heads per workgroup) units per entry
    wg_entry = []
    for e in range(ex["num_entries"]):
        hp = int(ex["entry_heads_per_wg"][e])
        wg_entry += [e] * (-(-batch.num_kv_heads // hp))
    assert len(wg_entry) == st.num_workgroups
    copies = [wl.make_tensors(batch, seed=i, device="cuda") for i in range(launches + 2)]
    out = torch.empty_like(copies[0][0])
    trace = torch.zeros(st.num_workgroups * 8, dtype=torch.int64, device="cuda")
    rows = []
    for i in range(launches + 2):
        q, kp, vp, strides = copies[i]
        if i >= 2:                                   # two untraced launches first
            trace.zero_()
            pb.pat_debug_set_trace(trace)
        try:
            pb.pat_forward(plan, q, kp, vp, strides, batch.softmax_scale, out, None, ws)
            torch.cuda.synchronize()
        finally:
            pb.pat_debug_set_trace(None)
        if i < 2:
            continue
        t = trace.cpu().numpy().reshape(-1, 8)
        for wg, e in enumerate(wg_entry):
            _, m, _ = pb.pat_tile_info(int(ex["entry_tile"][e]))
            hp = int(ex["entry_heads_per_wg"][e])
            heads = min(hp, batch.num_kv_heads - (wg - wg_entry.index(e)) * hp) if m <= 16 else 1
            tokens = int(ex["item_kv_len"][ex["entry_item"][e]])
            rows.append((m, tokens, heads, float(t[wg, 1] - t[wg, 0]) * 10.0))        # 100 MHz ticks
    return rows


def fit(rows):
    """Least squares of ns = c0 + c1 * (tokens * heads), per tile (rows m = 128, 64, 16)."""
    res = {}
    for packed in (128, 64, 16):
        sel = [(tok * hd, ns) for m, tok, hd, ns in rows if m == packed]
        if len(sel) < 2:
            res[packed] = None
            continue
        x = np.array([s[0] for s in sel], float)
        y = np.array([s[1] for s in sel], float)
        A = np.stack([np.ones_like(x), x], 1)
        (c0, c1), *_ = np.linalg.lstsq(A, y, rcond=None)
        res[packed] = (float(c0), float(c1), float(np.sqrt(np.mean((A @ [c0, c1] - y) ** 2))), len(sel))
    return res


# ---- latency versus request size (the paper's Fig. 5a on this GPU) -----------------------------
def latency_curve(workgroups=(1, 256), loads=(1, 2, 4, 8, 16, 32), buffer_bytes=2 << 30, iters=64):
    """For every number of concurrent workgroups: [(request bytes, ns per request)], and the fit
    ns = L + bytes / B of the curve's ends (flat part = latency L, slope = 1 / bandwidth B per
    workgroup)."""
    from . import probe
    buf = torch.empty(buffer_bytes, dtype=torch.uint8, device="cuda")
    buf.fill_(1)
    out = {}
    for w in workgroups:
        pts = [(4096 * k, probe.request_latency_ns(buf, loads_per_thread=k, workgroups=w, iters=iters))
               for k in loads]
        x = np.array([p[0] for p in pts], float)
        y = np.array([p[1] for p in pts], float)
        (c0, c1), *_ = np.linalg.lstsq(np.stack([np.ones_like(x), x], 1), y, rcond=None)
        out[w] = {"points": pts, "latency_ns": float(c0),
                  "gbps_per_workgroup": float(1.0 / c1) if c1 > 0 else float("inf"),
                  "gbps_all": float(w / c1) if c1 > 0 else float("inf")}
    return out


# ---- feasible tiles under the hardware's constraints (the paper's constraints 1-3, restated) ----
CU = {"lds_bytes": 160 * 1024, "vgprs_per_simd": 512, "simds": 4, "cus": 256, "lane_bytes": 4}


def tile_solver(latency_ns=2500.0, hbm_gbps=6900.0, head_dim=128, elem=2, stages=2):
    """Feasible (m, n) for a 512-thread workgroup that owns a CU, m = query rows, n = KV tokens per
    pipeline stage, powers of two from 16:
      (1) LDS: `stages` staged K tiles (n x 272 B padded rows) and V^T tiles (128 x (2 n + 16) B) fit
          the CU's LDS -- only packed tiles (m > 16) stage V; 16-row tiles keep K per wavefront;
      (2) memory: the loads a CU keeps in flight, stages x n x 2 (K, V) x head_dim x elem, cover its
          share of latency x bandwidth (else the tile is latency-bound, however fast it computes);
      (3) registers: fp32 accumulators O[m x head_dim] and S[m x n / 2] (two token halves) spread over
          the workgroup's 512 lanes, plus Q operands and the in-flight ring, fit 256 VGPRs a lane.
    Returns a list of dicts, one per (m, n), with the three verdicts."""
    need_in_flight = latency_ns * 1e-9 * hbm_gbps * 1e9 / CU["cus"]           # bytes per CU
    out = []
    for m in (16, 32, 64, 128, 256):
        for n in (16, 32, 64, 128, 256):
            kv_stage = n * 2 * head_dim * elem
            if m <= 16:
                # eight wavefront streams per CU whatever n is: n / 32 of them work on one KV head
                # (n = 32: one wavefront per item, n = 128: four per head, two heads per workgroup);
                # a wavefront's stage is min(n, 32) tokens, its current and next stage are in flight
                w = min(n, 32)
                lds = 8 * w * (head_dim * elem + 16)
                in_flight = 8 * 2 * w * 2 * head_dim * elem
                acc = 16 * head_dim // 64 + 8 + 16 + 64 + 32   # O, S, Q, K/V load buffers, V copy
            else:
                lds = stages * (n * (head_dim * elem + 16) + head_dim * (n * elem + 16))
                in_flight = stages * kv_stage
                rows_per_wave = max(32, m // 4)
                acc = rows_per_wave * head_dim // 64 + rows_per_wave * (n // 2) // 64 \
                    + rows_per_wave * head_dim * elem // (64 * 4) + stages * kv_stage // (512 * 4) + 48
            out.append({"m": m, "n": n, "lds_bytes": lds, "lds_ok": lds <= CU["lds_bytes"],
                        "in_flight_bytes": in_flight, "memory_ok": in_flight >= 0.95 * need_in_flight,
                        "vgprs": acc, "registers_ok": acc <= 256,
                        "feasible": lds <= CU["lds_bytes"] and in_flight >= 0.95 * need_in_flight and acc <= 256})
    return out, need_in_flight


def built_tiles():
    out = []
    for t in range(pb.lib.pat_num_tiles()):
        rc, m, n = pb.pat_tile_info(t)
        if rc == pb.PAT_OK:
            out.append((t, m, n))
    return out


# ---- kernel-equivalence run (the paper's Fig. 5c-d / Fig. 6 on this GPU) -------------------------
def _time_forward(batch, copies, launches=20, replays=3, **plan_kw):
    plan = pb.plan_for_batch(batch, **plan_kw)
    dev, ws = pb.alloc_plan_buffers(plan)
    pb.pat_plan_upload(plan, dev)
    out = torch.empty_like(copies[0][0])
    lse = torch.empty(batch.num_requests, batch.num_q_heads, dtype=torch.float32, device="cuda")
    R = len(copies)

    def fwd(i):
        q, kp, vp, st = copies[i % R]
        pb.pat_decode_attention(plan, q, kp, vp, st, batch.softmax_scale, out, lse, ws)

    for i in range(3):
        fwd(i)
    torch.cuda.synchronize()
    times = []
    for _ in range(replays):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(launches):
            fwd(i)
        b.record()
        torch.cuda.synchronize()
        times.append(a.elapsed_time(b) * 1e3 / launches)
    return times, out, lse, plan


def kernel_equivalence(batch_size=512, kv_len=1024, num_q_heads=32, num_kv_heads=8, copies=2):
    """Every tile of the family on the SAME batch without any shared prefix (batch a multiple of the
    CU count, every request kv_len tokens): {tile id: (m, n, us min, us max, GB/s)} and the batch."""
    lens = np.full(batch_size, kv_len)
    b = wl.tree_batch([batch_size], [lambda rng, n: lens], num_q_heads=num_q_heads,
                      num_kv_heads=num_kv_heads, dtype="bf16", seed=7100, name="equivalence")
    tensors = [wl.make_tensors(b, seed=7100 + i, device="cuda") for i in range(copies)]
    res = {}
    for t, m, n in built_tiles():
        if m == 16 and n == 4 and batch_size * kv_len > (1 << 18):
            continue                                     # the VALU cross-check tile: small runs only
        times, out, lse, plan = _time_forward(b, tensors, force_tile=t)
        res[t] = {"m": m, "n": n, "us_min": min(times), "us_max": max(times),
                  "gbps": b.unique_kv_bytes() / min(times) / 1e3}
    return res, b, tensors


# ---- KV-length thresholds of the tile selector -------------------------------------------------
def sweep_kv(kv_lens=(16, 32, 48, 64, 96, 128, 192, 256, 384, 512, 1024), groups=256):
    """(a) 20 query rows (5 requests x GQA 4) over a shared node of kv tokens: one 64-row packed
    workgroup per KV head against two 16-row blocks; (b) unshared requests of kv tokens: the n = 128
    tile (four wavefronts per KV head) against the n = 32 tile (one wavefront per KV head).
    Returns two lists of (kv, us first option, us second option)."""
    shared, leaves = [], []
    for kv in kv_lens:
        b = wl.tree_batch([groups, groups * 5], [kv, 16], num_q_heads=32, num_kv_heads=8, dtype="bf16",
                          seed=7200 + kv, name=f"sweep{kv}")
        t = [wl.make_tensors(b, seed=i, device="cuda") for i in range(2)]
        packed, *_ = _time_forward(b, t, packed_min_tokens=1, split_policy=pb.PAT_SPLIT_NONE)
        blocks, *_ = _time_forward(b, t, packed_min_tokens=1 << 30, split_policy=pb.PAT_SPLIT_NONE)
        shared.append((kv, min(packed), min(blocks)))
        lens = np.full(groups * 8, kv)
        b = wl.tree_batch([groups * 8], [lambda rng, n: lens], num_q_heads=32, num_kv_heads=8, dtype="bf16",
                          seed=7300 + kv, name=f"leaf{kv}")
        t = [wl.make_tensors(b, seed=i, device="cuda") for i in range(2)]
        n128, *_ = _time_forward(b, t, split_policy=pb.PAT_SPLIT_NONE)
        n32, *_ = _time_forward(b, t, split_policy=pb.PAT_SPLIT_NONE, wave_kv_tokens=1 << 20)
        leaves.append((kv, min(n128), min(n32)))
    return shared, leaves


# ---- (B, L) trees x head settings x ablation modes (sec. "Kernel Performance", "Ablation Study") ---
# The paper's twenty (B, L) pairs are in a figure that its text does not carry; these trees are
# stand-ins in its notation: B = nodes per level (the last level is the batch), L = tokens per level.
GRID_TREES = (
    ([1, 16], [1024, 256]),
    ([1, 64], [4096, 128]),
    ([1, 256], [2048, 64]),
    ([1, 4, 16], [128, 256, 1024]),           # the example of sec. "Experiment Setup"
    ([1, 4, 64], [2048, 512, 128]),
    ([1, 8, 64], [64, 512, 512]),
    ([4, 64], [1024, 256]),
    ([1, 2, 8, 64], [512, 512, 512, 128]),
    ([16, 256], [2048, 64]),
    ([128], [1024]),                           # no shared prefix
)
GRID_HEADS = ((64, 8), (32, 8), (16, 8), (32, 32))     # the four head settings of the paper
GRID_MODES = (("pat", {}), ("naive", {"mode": pb.PAT_MODE_NAIVE_PER_NODE}),
              ("fixed64", {"force_tile": 3}), ("no-sharing", {"mode": pb.PAT_MODE_NO_SHARING}))


def grid(trees=GRID_TREES, heads=GRID_HEADS, modes=GRID_MODES, launches=20, copies=None, each=None):
    """us per step (forward + merge, the fastest of three runs of `launches` back-to-back steps over
    `copies` rotated KV pools; None: as many as make 1 GiB, at most 12, so that no step finds its KV
    in the 256 MB last-level cache) of every mode on every (tree, head setting), FP16 as in the paper.
    Returns [(B, L, (Hq, Hkv), unique MB, {mode: us}, max |out - out of the first mode|)];
    each(row) is called as the rows come."""
    rows = []
    for B, L in trees:
        for hq, hkv in heads:
            b = wl.tree_batch(list(B), list(L), num_q_heads=hq, num_kv_heads=hkv, dtype="fp16",
                              seed=7400 + 31 * len(rows), name="grid")
            n_copies = copies or max(1, min(12, (1 << 30) // b.unique_kv_bytes()))
            t = [wl.make_tensors(b, seed=7400 + i, device="cuda") for i in range(n_copies)]
            us, ref, dev = {}, None, 0.0
            _time_forward(b, t, launches=launches, replays=1, **modes[0][1])     # untimed: the first run
            for name, kw in modes:                                              # on new tensors is slow
                times, out, _, _ = _time_forward(b, t, launches=launches, **kw)
                us[name] = min(times)
                o = out.float()
                if ref is None:
                    ref = o.clone()
                else:
                    dev = max(dev, float((o - ref).abs().max()))
            rows.append((list(B), list(L), (hq, hkv), b.unique_kv_bytes() / 1e6, us, dev))
            if each:
                each(rows[-1])
            del t
        torch.cuda.empty_cache()
    return rows


# ---- per-workgroup timeline of one forward launch (the paper's Fig. 12 on this GPU) ---------------
def timeline(batch, warm=6, **plan_kw):
    """One traced forward launch (pat_debug_set_trace) after `warm` untraced steps, on KV pools the
    launch has not seen.  Returns a dict of numpy arrays per workgroup / wavefront item, in launch order:
    start, end (us from the first start), tile, kv_len, xcc, cu (a CU's id within the chip), and the
    four marks (us since the record's start, nan where the tile takes none); plus the plan's stats."""
    plan = pb.plan_for_batch(batch, **plan_kw)
    st = plan.stats()
    dev, ws = pb.alloc_plan_buffers(plan)
    pb.pat_plan_upload(plan, dev)
    R = max(2, min(20, (1 << 30) // max(1, batch.unique_kv_bytes())))
    copies = [wl.make_tensors(batch, seed=i, device="cuda") for i in range(R)]
    out = torch.empty_like(copies[0][0])
    lse = torch.empty(batch.num_requests, batch.num_q_heads, dtype=torch.float32, device="cuda")
    rec = torch.zeros((int(st.num_workgroups) + int(st.num_wave_items) + 8) * 8, dtype=torch.int64, device="cuda")
    for i in range(warm):
        q, kp, vp, sd = copies[i % R]
        pb.pat_decode_attention(plan, q, kp, vp, sd, batch.softmax_scale, out, lse, ws)
    torch.cuda.synchronize()
    pb.pat_debug_set_trace(rec)
    try:
        q, kp, vp, sd = copies[warm % R]
        pb.pat_forward(plan, q, kp, vp, sd, batch.softmax_scale, out, lse, ws)
        torch.cuda.synchronize()
    finally:
        pb.pat_debug_set_trace(None)
    t = rec.cpu().numpy().reshape(-1, 8)
    t = t[t[:, 0] > 0]
    t0 = t[:, 0].min()
    hw = t[:, 2] & 0xFFFFFFFF
    xcc = (t[:, 2] >> 32) & 0xF
    marks = np.where(t[:, 4:8] > 0, (t[:, 4:8] - t[:, 0:1]) / 100.0, np.nan)
    return {"start": (t[:, 0] - t0) / 100.0, "end": (t[:, 1] - t0) / 100.0, "tile": t[:, 3] >> 32,
            "kv_len": t[:, 3] & 0xFFFFFFFF, "xcc": xcc,
            "cu": xcc * 1000 + ((hw >> 13) & 7) * 100 + ((hw >> 12) & 1) * 20 + ((hw >> 8) & 0xF),
            "marks": marks, "stats": st}


def timeline_report(name, tl, out=print):
    start, end, tile = tl["start"], tl["end"], tl["tile"]
    span = float(end.max())
    st = tl["stats"]
    out(f"{name}: {len(start)} records, launch span {span:.1f} us, {int(st.num_workgroups)} workgroups, "
        f"{int(st.num_wave_items)} wavefront items, tiles {list(st.tile_histogram)[:pb.lib.pat_num_tiles()]}")
    names = {t: f"tile {t} (m = {m}, n = {n})" for t, m, n in built_tiles()}
    for tid in np.unique(tile):
        m = tile == tid
        d = end[m] - start[m]
        out(f"  {names.get(int(tid), tid)}: {int(m.sum())} records, kv {int(tl['kv_len'][m].min())}..{int(tl['kv_len'][m].max())}; "
            f"start {start[m].min():.1f} / {np.median(start[m]):.1f} / {start[m].max():.1f} us (min / median / max); "
            f"duration {d.min():.1f} / {np.median(d):.1f} / {d.max():.1f}; last end {end[m].max():.1f}")
        for k, what in enumerate(("mark 0", "mark 1", "mark 2", "mark 3")):
            v = tl["marks"][m, k]
            v = v[~np.isnan(v)]
            if len(v):
                out(f"      {what} after start: {v.min():.2f} / {np.median(v):.2f} / {v.max():.2f} us")
    grid_t = np.linspace(0.0, span, 21)
    out("  records running at 0 %, 5 %, ... 100 % of the span: "
        + " ".join(str(int(((start <= x) & (end > x)).sum())) for x in grid_t))
    cus = np.unique(tl["cu"])
    busy = np.array([(end[tl["cu"] == c] - start[tl["cu"] == c]).sum() for c in cus])
    last = np.array([end[tl["cu"] == c].max() for c in cus])
    out(f"  {len(cus)} CUs took work; busy {busy.mean() / span * 100:.0f} % of the span on average "
        f"(least busy {busy.min() / span * 100:.0f} %); a CU's last end: {last.min():.1f} / {np.median(last):.1f} / {last.max():.1f} us")
    per_xcc = [float((end[tl["xcc"] == x] - start[tl["xcc"] == x]).sum()) for x in range(8)]
    out("  busy time per XCD (us): " + " ".join(f"{v:.0f}" for v in per_xcc))


def run_model():
    rows = []
    for b in _one_round_batches():
        rows += workgroup_times(b)
    for b in _one_round_batches(num_q_heads=16):        # 64 rows per KV head: the 64-row packed tile
        rows += [r for r in workgroup_times(b) if r[0] == 64]
    res = fit(rows)
    for m, name in ((128, "128-row packed workgroup"), (64, "64-row packed workgroup"), (16, "16-row workgroup")):
        if res[m] is None:
            print(f"{name}: no samples", file=sys.stderr)
            continue
        c0, c1, rms, n = res[m]
        unit = "token x KV head" if m == 16 else "token"
        print(f"{name}: {c0:8.0f} ns + {c1:6.2f} ns per {unit}   (rms {rms:.0f} ns over {n} workgroups)",
              file=sys.stderr)
    if res[128] and res[16]:
        # the planner derives the 64-row tile's constants from the 128-row tile's (0.73, 0.90)
        model = [max(0, round(res[128][0])), max(1, round(res[128][1])),
                 max(0, round(res[16][0])), max(1, round(res[16][1]))]
        out = {"model_ns": model}
        if res[64]:
            out["ratio_64_row_tile"] = [round(res[64][0] / res[128][0], 2), round(res[64][1] / res[128][1], 2)]
        print(json.dumps(out))


def main(argv=None):
    argv = sys.argv[1:] if argv is None else argv
    what = argv[0] if argv else "model"
    if what == "solver":
        tiles, need = tile_solver()
        built = {(m, n) for _, m, n in built_tiles()}
        print(f"bytes a CU must keep in flight: {need / 1024:.0f} KiB (latency x bandwidth / CUs)")
        print("   m    n   LDS KiB  in flight KiB  VGPRs  feasible  built")
        for t in tiles:
            print(f"{t['m']:4d} {t['n']:4d} {t['lds_bytes'] / 1024:8.1f} {t['in_flight_bytes'] / 1024:13.0f} "
                  f"{t['vgprs']:6d}  {'yes' if t['feasible'] else 'no ':8s} {'*' if (t['m'], t['n']) in built else ''}")
        return
    if not torch.cuda.is_available():
        sys.exit("calibrate: needs the GPU")
    if what == "latency":
        for w, r in latency_curve().items():
            print(f"{w} workgroups at once: " + ", ".join(f"{b >> 10} KiB {ns:.0f} ns" for b, ns in r["points"]))
            print(f"   fit: latency {r['latency_ns']:.0f} ns, {r['gbps_per_workgroup']:.1f} GB/s per workgroup, "
                  f"{r['gbps_all']:.0f} GB/s in all")
    elif what == "equivalence":
        res, b, _ = kernel_equivalence()
        print(f"no shared prefix: {b.num_requests} requests x 1024 tokens, {b.unique_kv_bytes() / 1e6:.0f} MB")
        for t, r in res.items():
            print(f"tile {t} (m = {r['m']}, n = {r['n']}): {r['us_min']:.1f} .. {r['us_max']:.1f} us/step, "
                  f"{r['gbps']:.0f} GB/s")
    elif what == "sweep-kv":
        shared, leaves = sweep_kv()
        print("20 rows over a shared node:   kv   64-row packed   two 16-row blocks   (us/step)")
        for kv, a, c in shared:
            print(f"{kv:34d} {a:14.1f} {c:19.1f}   {'packed' if a < c else 'blocks'}")
        print("unshared requests:            kv   n = 128 (4 wavefronts)   n = 32 (1 wavefront)")
        for kv, a, c in leaves:
            print(f"{kv:34d} {a:22.1f} {c:22.1f}   {'n=128' if a < c else 'n=32'}")
    elif what == "timeline":
        for name in (argv[1:] or ["C2", "C3", "C4"]):
            b = wl.config(name) if name in wl.CONFIG_NAMES else wl.extra_config(name)
            timeline_report(name, timeline(b))
    elif what == "grid":
        names = [n for n, _ in GRID_MODES]
        print("us per step (forward + merge), FP16, head dim 128; speed-up = no-sharing / pat")
        print(f"{'B':>16s} {'L':>22s} {'heads':>6s} {'MB':>7s} " + " ".join(f"{n:>10s}" for n in names)
              + "  speed-up  GB/s(pat)", flush=True)

        def show(row):
            B, L, (hq, hkv), mb, us, dev = row
            print(f"{str(B):>16s} {str(L):>22s} {hq:3d}/{hkv:<2d} {mb:7.1f} "
                  + " ".join(f"{us[n]:10.1f}" for n in names)
                  + f"  {us['no-sharing'] / us['pat']:8.2f}  {mb / us['pat'] * 1e3:9.0f}", flush=True)

        rows = grid(each=show)
        print(f"largest difference between the modes' outputs: {max(r[5] for r in rows):.2e}")
    else:
        run_model()


if __name__ == "__main__":
    main()
