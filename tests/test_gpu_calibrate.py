"""The calibration module on the GPU at small size: the latency-versus-size probe gives a sane
latency and bandwidth, and the kernel-equivalence batch (no shared prefix) gives the oracle's
attention through every tile of the family."""
import numpy as np
import pytest

from paper_2511_22333_amd import calibrate
from paper_2511_22333_amd import binding as pb
from paper_2511_22333_amd import workloads as wl

from gpu_util import compare, run_oracle

pytestmark = pytest.mark.gpu


def test_latency_curve_is_flat_then_linear():
    print("case latency probe", flush=True)
    res = calibrate.latency_curve(workgroups=(1, 256), loads=(1, 4, 16), buffer_bytes=1 << 30, iters=32)
    for w, r in res.items():
        ns = [p[1] for p in r["points"]]
        print(f"  {w} workgroups: {[(b >> 10, round(t)) for b, t in r['points']]} -> "
              f"L = {r['latency_ns']:.0f} ns, {r['gbps_all']:.0f} GB/s", flush=True)
        assert all(200.0 < t < 200000.0 for t in ns)          # between an L2 hit and far too slow
        assert ns[-1] >= ns[0] * 0.8                          # 64 KiB cannot be much faster than 4 KiB
    # a lone workgroup is latency-bound; 256 of them move far more in total
    assert res[256]["gbps_all"] > 4 * res[1]["gbps_all"]


def test_kernel_equivalence_batch_matches_the_oracle_through_every_tile():
    print("case kernel equivalence", flush=True)
    res, b, tensors = calibrate.kernel_equivalence(batch_size=256, kv_len=200, num_q_heads=16,
                                                   num_kv_heads=4, copies=1)
    assert set(res) == {t for t, _, _ in calibrate.built_tiles()}
    q, kp, vp, st = tensors[0]
    want, want_lse = run_oracle(b, (q.cpu(), kp.cpu(), vp.cpu(), st))
    for t in res:
        _, out, lse, plan = calibrate._time_forward(b, tensors, launches=1, replays=1, force_tile=t)
        err, lerr = compare(b, out, lse, want, want_lse)
        print(f"  tile {t}: {res[t]['us_min']:.1f} us, {res[t]['gbps']:.0f} GB/s, err {err:.1e}", flush=True)
        assert list(plan.stats().tile_histogram)[t] == plan.stats().num_entries


def test_kv_sweep_runs():
    print("case kv sweep", flush=True)
    shared, leaves = calibrate.sweep_kv(kv_lens=(64, 512), groups=32)
    assert len(shared) == 2 and len(leaves) == 2
    assert all(a > 0 and c > 0 for _, a, c in shared + leaves)


def test_grid_of_trees_gives_one_result_in_every_mode():
    print("case grid", flush=True)
    rows = calibrate.grid(trees=(([1, 4, 16], [128, 256, 100]), ([24], [300])), heads=((32, 8), (4, 4)),
                          launches=2, copies=1)
    assert len(rows) == 4
    for B, L, heads, mb, us, dev in rows:
        print(f"  {B} {L} {heads}: {us}, modes differ by {dev:.1e}", flush=True)
        assert set(us) == {n for n, _ in calibrate.GRID_MODES} and all(v > 0 for v in us.values())
        assert dev < 4e-3                                       # one attention, four schedules (fp16 output)


def test_timeline_of_a_launch_accounts_for_every_workgroup():
    print("case timeline", flush=True)
    b = wl.tree_batch([1, 4, 40], [256, 128, lambda rng, n: rng.integers(1, 300, n)], num_q_heads=16, num_kv_heads=4,
                      dtype="bf16", seed=21)
    tl = calibrate.timeline(b, warm=2)
    st = tl["stats"]
    assert len(tl["start"]) == st.num_workgroups + st.num_wave_items
    assert (tl["end"] > tl["start"]).all() and tl["end"].max() < 10000.0          # microseconds, one launch
    hist = np.bincount(tl["tile"].astype(int), minlength=8)
    calibrate.timeline_report("timeline test", tl, out=lambda line: print("  " + line, flush=True))
    assert hist.sum() == len(tl["start"]) and len(np.unique(tl["cu"])) <= 256
