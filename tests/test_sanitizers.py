"""AddressSanitizer + UBSan builds (CPU only) of the planner and of the C oracle, run over the
cases the planner's output is followed unclamped by the kernels for: random forests, the benchmark
shapes, every packing mode and split policy, the wavefront-item schedule, the two-kernel order,
decode-step sequences through the lazy update, and inputs the planner must refuse.  The drivers
are separate executables (the sanitizer runtime has to be the first thing in its process)."""
import dataclasses
import os
import subprocess

import numpy as np
import pytest

from paper_2511_22333_amd import binding as pb
from paper_2511_22333_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2511_22333_amd", "csrc")
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
       "-fno-omit-frame-pointer", "-static-libasan", "-static-libubsan"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", LD_PRELOAD="")


@pytest.fixture(scope="session")
def drivers(tmp_path_factory):
    out = tmp_path_factory.mktemp("san")
    plan = str(out / "plan_driver")
    subprocess.check_call(["g++", "-std=c++17", *SAN, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                           os.path.join(ROOT, "tests", "sanitize", "plan_driver.cpp"),
                           os.path.join(CSRC, "pat_plan.cpp"), "-o", plan])
    orc = str(out / "oracle_driver")
    subprocess.check_call(["gcc", "-std=c99", *SAN, "-fopenmp",
                           os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
                           os.path.join(ROOT, "oracle", "pat_oracle.c"), "-o", orc, "-lm"])
    cache = str(out / "cache_driver")
    subprocess.check_call(["g++", "-std=c++17", *SAN, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                           os.path.join(ROOT, "tests", "sanitize", "cache_driver.cpp"),
                           os.path.join(CSRC, "pat_cache.cpp"), os.path.join(CSRC, "pat_plan.cpp"), "-o", cache])
    return plan, orc, out, cache


def _run(exe, path):
    r = subprocess.run([exe, path], env=ENV, stdout=subprocess.PIPE, stderr=subprocess.PIPE, timeout=300)
    err = r.stderr.decode(errors="replace")
    assert r.returncode == 0 and "Sanitizer" not in err and "runtime error" not in err, \
        f"{os.path.basename(exe)} rc={r.returncode}\n{err[-3000:]}"
    return r.stdout.decode()


def _plan_case(path, batch, *, mode=0, split=0, target=0, force_tile=-1, num_cus=0, wave_kv=0, dual=0,
               merge_factor=0, steps=(), want_rc=0, step_rcs=None):
    bt = np.ascontiguousarray(batch.block_tables, np.int32)
    head = [batch.num_requests, bt.shape[1], batch.page_size, batch.num_pages, batch.num_q_heads,
            batch.num_kv_heads, pb.DTYPES[batch.dtype], mode, split, target, force_tile, num_cus,
            wave_kv, dual, merge_factor, len(steps), want_rc]
    parts = [np.array(head, np.int32), bt.ravel(), np.ascontiguousarray(batch.kv_lens, np.int32)]
    for k, b2 in enumerate(steps):
        bt2 = np.ascontiguousarray(b2.block_tables, np.int32)
        parts += [np.array([bt2.shape[1], 0 if step_rcs is None else step_rcs[k]], np.int32), bt2.ravel(),
                  np.ascontiguousarray(b2.kv_lens, np.int32)]
    np.concatenate(parts).tofile(path)
    return path


def test_planner_under_sanitizers_random_forests(drivers):
    exe, _, out, _ = drivers
    for seed in range(30):
        b = wl.random_forest_batch(seed, max_requests=24, max_node_tokens=200,
                                   duplicate_rows=(seed % 3 == 0))
        for k, kw in enumerate([dict(), dict(mode=1, split=1), dict(mode=2, split=2),
                                dict(split=3, target=16), dict(force_tile=2), dict(wave_kv=32, num_cus=3),
                                dict(dual=1), dict(force_tile=4, merge_factor=16), dict(num_cus=1)]):
            _run(exe, _plan_case(str(out / f"f{seed}_{k}.bin"), b, **kw))


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5", "T3", "PK"])
def test_planner_under_sanitizers_benchmark_shapes(drivers, name):
    exe, _, out, _ = drivers
    b = wl.config(name)
    for k, kw in enumerate([dict(), dict(mode=2), dict(split=1), dict(wave_kv=256), dict(dual=1)]):
        _run(exe, _plan_case(str(out / f"{name}_{k}.bin"), b, **kw))


def test_planner_under_sanitizers_batches_of_a_few_rounds(drivers):
    # the cut searched with the simulated launch, with and without wavefront items for very short leaves
    exe, _, out, _ = drivers
    for k, (B, L, hq, hkv) in enumerate([([1, 256], [2048, 64], 64, 8), ([1, 256], [2048, 64], 32, 32),
                                         ([1, 64], [4096, 128], 32, 8), ([1, 4, 64], [2048, 512, 128], 16, 8),
                                         ([16, 256], [2048, 64], 32, 8), ([1, 2, 8, 64], [512, 512, 512, 128], 64, 8)]):
        b = wl.tree_batch(B, L, num_q_heads=hq, num_kv_heads=hkv, dtype="fp16", seed=50 + k)
        for j, kw in enumerate([dict(), dict(wave_kv=-1), dict(num_cus=64)]):
            assert "ok" in _run(exe, _plan_case(str(out / f"few{k}_{j}.bin"), b, **kw))


def test_plan_cache_under_sanitizers(drivers):
    *_, cache = drivers
    r = subprocess.run([cache], env=ENV, stdout=subprocess.PIPE, stderr=subprocess.PIPE, timeout=300)
    err = r.stderr.decode(errors="replace")
    assert r.returncode == 0 and "Sanitizer" not in err and "runtime error" not in err, err[-3000:]
    assert r.stdout.decode().strip() == "ok"


def test_lazy_update_under_sanitizers(drivers):
    exe, _, out, _ = drivers
    for seed in range(8):
        b = wl.random_forest_batch(300 + seed, max_requests=12, max_node_tokens=150)
        b = dataclasses.replace(b, num_pages=b.num_pages + 4096)
        last = {}
        for r in range(b.num_requests):
            n = -(-int(b.kv_lens[r]) // b.page_size)
            last.setdefault(int(b.block_tables[r, n - 1]), []).append(r)
        if any(len(v) > 1 for v in last.values()):
            continue
        steps, cur = [], b
        for n in (1, 1, 7, 16, 40):
            cur = wl.decode_steps(cur, n)
            steps.append(cur)
        # 16 reserve pages per request: 65 steps fit (at most 5 new pages)
        _run(exe, _plan_case(str(out / f"adv{seed}.bin"), b, steps=steps))
        _run(exe, _plan_case(str(out / f"advw{seed}.bin"), b, steps=steps, wave_kv=48, num_cus=2))
    # a request that shrinks is refused, nothing is touched
    b = wl.tree_batch([1, 4], [64, lambda rng, n: rng.integers(20, 60, n)], num_q_heads=8, num_kv_heads=2)
    shrunk = dataclasses.replace(b, kv_lens=b.kv_lens - 1)
    _run(exe, _plan_case(str(out / "shrink.bin"), b, steps=[shrunk], step_rcs=[pb.PAT_ERR_PLAN_STALE]))


def test_planner_refuses_bad_input_under_sanitizers(drivers):
    exe, _, out, _ = drivers
    b = wl.config("C1")
    bad = dataclasses.replace(b, block_tables=b.block_tables.copy())
    bad.block_tables[2, 1] = b.num_pages + 5
    _run(exe, _plan_case(str(out / "badpage.bin"), bad, want_rc=pb.PAT_ERR_BAD_PAGE_ID))
    bad = dataclasses.replace(b, kv_lens=b.kv_lens.copy())
    bad.kv_lens[0] = 0
    _run(exe, _plan_case(str(out / "badlen.bin"), bad, want_rc=pb.PAT_ERR_BAD_KV_LEN))
    bad = dataclasses.replace(b, kv_lens=b.kv_lens.copy())
    bad.kv_lens[1] = b.page_size * b.block_tables.shape[1] + 1
    _run(exe, _plan_case(str(out / "toolong.bin"), bad, want_rc=pb.PAT_ERR_BAD_KV_LEN))
    _run(exe, _plan_case(str(out / "badtile.bin"), b, force_tile=9, want_rc=pb.PAT_ERR_INVALID_ARG))


def test_oracle_under_sanitizers(drivers):
    _, exe, out, _ = drivers
    for seed, layout in ((1, "NHD"), (2, "HND"), (3, "NHD")):
        b = wl.random_forest_batch(seed, max_requests=6, max_node_tokens=60, num_q_heads=4, num_kv_heads=2,
                                   dtype="bf16" if seed % 2 else "fp16")
        q, kp, vp, st = wl.make_tensors(b, poison=True, layout=layout)
        import torch
        raw = lambda t: t.contiguous().view(torch.int16).numpy().view(np.uint16).ravel()
        head = np.array([b.num_requests, b.block_tables.shape[1], b.page_size, b.num_pages, b.num_q_heads,
                         b.num_kv_heads, 128, pb.DTYPES[b.dtype], st[0], st[1], st[2], 0], np.int32)
        path = str(out / f"oracle{seed}.bin")
        with open(path, "wb") as f:
            head.tofile(f)
            np.ascontiguousarray(b.block_tables, np.int32).tofile(f)
            np.ascontiguousarray(b.kv_lens, np.int32).tofile(f)
            raw(q).tofile(f)
            raw(kp).tofile(f)
            raw(vp).tofile(f)
        assert _run(exe, path).startswith("ok")
