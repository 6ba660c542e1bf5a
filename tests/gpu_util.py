"""Helpers of the GPU parity tests: run the HIP path through the C ABI and the fp64 oracle on
the same seeded tensors."""
import numpy as np
import torch

from oracle import attention as oa
from paper_2511_22333_amd import binding as pb
from paper_2511_22333_amd import workloads as wl

TOL = {"fp16": 2e-3, "bf16": 1e-2}      # max-abs error of out against the fp64 oracle
# ... except where the output's own 16-bit rounding is coarser than that: half a unit in the last
# place is |x| * 2^-9 (bf16, 8 significant bits) or |x| * 2^-12 (fp16).  Three of them are allowed
# for outputs that large (one for the softmax weights, which are rounded to the element type
# before the second product and do not average out over two or three tokens, one for the output's
# own rounding, one for everything in fp32); that exceeds the absolute bound from |x| = 1.7 (bf16) on
HALF_ULP = {"fp16": 2.0 ** -12, "bf16": 2.0 ** -9}
# lse: the scores are fp32 sums of exact 16-bit products and the sum of exponentials is fp32, so
# the error is a few fp32 roundings of the score itself: 1e-4 absolute up to |lse| = 32, and in
# proportion beyond (keys made 30-40 times louder push |lse| into the hundreds)
LSE_TOL = 1e-4


def lse_tol(want_lse):
    return LSE_TOL * np.maximum(1.0, np.abs(want_lse) / 32.0)


def run_hip(batch, tensors, *, with_lse=True, separate_stages=False, **plan_kw):
    """tensors = (q, k_pool, v_pool, strides) on the GPU.  Returns (out, lse, plan)."""
    q, kp, vp, strides = tensors
    plan = pb.plan_for_batch(batch, **plan_kw)
    dev, ws = pb.alloc_plan_buffers(plan)
    pb.pat_plan_upload(plan, dev)
    out = torch.full_like(q, float("nan"))
    lse = torch.full((batch.num_requests, batch.num_q_heads), float("nan"), dtype=torch.float32,
                     device=q.device) if with_lse else None
    ws.fill_(0xFF)                            # NaN pattern: unwritten partials would show
    if separate_stages:
        pb.pat_forward(plan, q, kp, vp, strides, batch.softmax_scale, out, lse, ws)
        pb.pat_merge(plan, out, lse, ws)
    else:
        pb.pat_decode_attention(plan, q, kp, vp, strides, batch.softmax_scale, out, lse, ws)
    torch.cuda.synchronize()
    return out, lse, plan


def run_oracle(batch, cpu_tensors, req_ids=None):
    q, kp, vp, strides = cpu_tensors
    return oa.decode_attention(q, kp, vp, batch.block_tables, batch.kv_lens,
                               page_size=batch.page_size, num_kv_heads=batch.num_kv_heads,
                               dtype=batch.dtype, scale=batch.softmax_scale, strides=strides,
                               num_pages=batch.num_pages, req_ids=req_ids)


def to_gpu(cpu_tensors):
    q, kp, vp, strides = cpu_tensors
    return q.cuda(), kp.cuda(), vp.cuda(), strides


def compare(batch, out, lse, want, want_lse, req_ids=None):
    got = out.double().cpu().numpy()
    if req_ids is not None:
        got = got[np.asarray(req_ids)]
    assert np.isfinite(got).all(), "non-finite output (poison leaked or partial unwritten)"
    diff = np.abs(got - want)
    err = diff.max()
    tol = np.maximum(TOL[batch.dtype], 3 * HALF_ULP[batch.dtype] * np.abs(want))
    assert (diff <= tol).all(), f"max-abs error {err} > {TOL[batch.dtype]} (|out| up to {np.abs(want).max():.2f})"
    lerr = 0.0
    if lse is not None:
        gl = lse.double().cpu().numpy()
        if req_ids is not None:
            gl = gl[np.asarray(req_ids)]
        assert np.isfinite(gl).all()
        diff = np.abs(gl - want_lse)
        lerr = diff.max()
        assert (diff <= lse_tol(want_lse)).all(), f"lse error {lerr} (|lse| up to {np.abs(want_lse).max():.1f})"
    return float(err), float(lerr)


def compare_all_requests_in_groups(batch, out, lse, gpu_tensors, group=32):
    """Every request of a batch whose pools live on the GPU against the oracle: the pages of
    `group` requests at a time are gathered to the host (bounded host memory), the oracle attends
    those requests one by one, and out/lse are compared element by element."""
    q, kp, vp, st = gpu_tensors
    qc = q.cpu()
    P = batch.page_size
    worst, worst_l = 0.0, 0.0
    for g0 in range(0, batch.num_requests, group):
        ids = list(range(g0, min(batch.num_requests, g0 + group)))
        pages = np.unique(np.concatenate(
            [batch.block_tables[r, : -(-int(batch.kv_lens[r]) // P)] for r in ids]))
        remap = np.full(batch.num_pages, -1, np.int64)
        remap[pages] = np.arange(len(pages))
        idx = torch.from_numpy(pages.astype(np.int64)).to(kp.device)
        bt = np.where(batch.block_tables >= 0, remap[np.maximum(batch.block_tables, 0)], -1)
        sub = wl.DecodeBatch(batch.name, batch.num_requests, batch.num_q_heads,
                             batch.num_kv_heads, batch.head_dim, P, batch.dtype,
                             bt.astype(np.int32), batch.kv_lens, len(pages))
        want, want_lse = run_oracle(sub, (qc, kp[idx].cpu(), vp[idx].cpu(), st), req_ids=ids)
        e, l = compare(batch, out, lse, want, want_lse, req_ids=ids)
        worst, worst_l = max(worst, e), max(worst_l, l)
    return worst, worst_l


def parity(batch, *, layout="NHD", poison=True, seed=None, **plan_kw):
    cpu = wl.make_tensors(batch, seed=seed, poison=poison, layout=layout)
    want, want_lse = run_oracle(batch, cpu)
    out, lse, plan = run_hip(batch, to_gpu(cpu), **plan_kw)
    return compare(batch, out, lse, want, want_lse), plan
