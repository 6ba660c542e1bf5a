"""The entry point that allocates nothing (pat_decode_attention_static_ws) against
pat_decode_attention on the same plan and tensors: same kernels, the workspace is the library's
own fixed device array instead of a caller's buffer.  Two calls in a row, the second on a
smaller batch (the array still holds the first call's partials); a plan that needs more than the
array is refused."""
import numpy as np
import pytest
import torch

from paper_2511_22333_amd import binding as pb
from paper_2511_22333_amd import workloads as wl

from gpu_util import TOL, compare, run_oracle, to_gpu

pytestmark = pytest.mark.gpu


def _both_ways(batch, **plan_kw):
    cpu = wl.make_tensors(batch, poison=True)
    q, kp, vp, st = to_gpu(cpu)
    plan = pb.plan_for_batch(batch, **plan_kw)
    stats = plan.stats()
    assert stats.num_slots > 0, "the case must use the workspace"
    assert stats.workspace_bytes <= pb.PAT_STATIC_WORKSPACE_BYTES
    dev, ws = pb.alloc_plan_buffers(plan)
    pb.pat_plan_upload(plan, dev)
    res = []
    for static in (False, True):
        out = torch.full_like(q, float("nan"))
        lse = torch.full((batch.num_requests, batch.num_q_heads), float("nan"),
                         dtype=torch.float32, device="cuda")
        if static:
            pb.pat_decode_attention_static_ws(plan, q, kp, vp, st, batch.softmax_scale, out, lse)
        else:
            ws.fill_(0xFF)
            pb.pat_decode_attention(plan, q, kp, vp, st, batch.softmax_scale, out, lse, ws)
        torch.cuda.synchronize()
        res.append((out, lse))
    # same kernels on the same inputs: the two agree bit for bit, and with the oracle
    assert torch.equal(res[0][0], res[1][0]) and torch.equal(res[0][1], res[1][1])
    want, want_lse = run_oracle(batch, cpu)
    return compare(batch, res[1][0], res[1][1], want, want_lse)


def test_static_workspace_two_calls_second_smaller():
    print("case static workspace: large then small", flush=True)
    big = wl.tree_batch([1, 4, 24], [512, 192, lambda rng, n: rng.integers(1, 400, n)],
                        num_q_heads=32, num_kv_heads=8, dtype="bf16", seed=77)
    small = wl.tree_batch([1, 5], [64, lambda rng, n: rng.integers(1, 60, n)],
                          num_q_heads=8, num_kv_heads=2, dtype="fp16", seed=78)
    e1 = _both_ways(big)
    e2 = _both_ways(small)
    print(f"static workspace: err {e1[0]:.2e} / {e2[0]:.2e} (tol {TOL['bf16']}, {TOL['fp16']})", flush=True)


def test_static_workspace_refuses_a_plan_that_does_not_fit():
    print("case static workspace: too large", flush=True)
    # 96 unshared requests of 64 heads, cut into 16-token parts: far more partials than fit
    lens = np.full(96, 800)
    b = wl.tree_batch([96], [lambda rng, n: lens], num_q_heads=64, num_kv_heads=8, dtype="bf16", seed=79)
    plan = pb.plan_for_batch(b, split_policy=pb.PAT_SPLIT_TARGET, split_target_tokens=16)
    assert plan.stats().workspace_bytes > pb.PAT_STATIC_WORKSPACE_BYTES
    dev = torch.empty(int(plan.stats().plan_device_bytes), dtype=torch.uint8, device="cuda")
    pb.pat_plan_upload(plan, dev)
    q, kp, vp, st = wl.make_tensors(b, device="cuda")
    out = torch.zeros_like(q)
    with pytest.raises(pb.PatError) as ei:
        pb.pat_decode_attention_static_ws(plan, q, kp, vp, st, b.softmax_scale, out, None)
    assert ei.value.status == pb.PAT_ERR_WORKSPACE_TOO_SMALL
    torch.cuda.synchronize()
    assert int(out.abs().sum()) == 0                       # nothing was launched
