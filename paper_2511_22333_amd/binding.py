"""ctypes binding of ``libpat.so``: argument marshalling only.

Function names mirror ``include/pat.h``.  Device buffers are torch tensors (device memory and
streams are all torch is used for); every step of the path runs inside the library.  There is
no CPU or PyTorch fallback: if the library is missing the import fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np
# torch ships its own HIP runtime (same soname as the system one).  It has to be in the process
# before libpat.so is loaded, so that the library binds to that runtime and device pointers,
# streams and kernels all live in one HIP context.
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpat.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2511_22333_amd.build` "
        "(there is no fallback path)")

lib = C.CDLL(LIB_PATH)

PAT_OK = 0
(PAT_ERR_INVALID_ARG, PAT_ERR_BAD_PAGE_ID, PAT_ERR_BAD_KV_LEN, PAT_ERR_UNSUPPORTED,
 PAT_ERR_WORKSPACE_TOO_SMALL, PAT_ERR_PLAN_NOT_UPLOADED, PAT_ERR_HIP, PAT_ERR_OUT_OF_MEMORY,
 PAT_ERR_BAD_TREE, PAT_ERR_PLAN_STALE) = range(-1, -11, -1)
PAT_F16, PAT_BF16 = 0, 1
PAT_MODE_PAT, PAT_MODE_NAIVE_PER_NODE, PAT_MODE_NO_SHARING = 0, 1, 2
PAT_SPLIT_AUTO, PAT_SPLIT_MEAN, PAT_SPLIT_NONE, PAT_SPLIT_TARGET = 0, 1, 2, 3
DTYPES = {"fp16": PAT_F16, "bf16": PAT_BF16}

_i32p = C.POINTER(C.c_int32)


class pat_batch_desc(C.Structure):
    _fields_ = [("num_requests", C.c_int32), ("max_pages_per_req", C.c_int32),
                ("block_tables", _i32p), ("kv_lens", _i32p),
                ("page_size", C.c_int32), ("num_pages", C.c_int32),
                ("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("dtype", C.c_int32),
                ("num_nodes", C.c_int32), ("node_parent", _i32p),
                ("node_num_pages", _i32p), ("req_leaf_node", _i32p)]


class pat_plan_opts(C.Structure):
    _fields_ = [("mode", C.c_int32), ("merge_factor", C.c_int32), ("split_policy", C.c_int32),
                ("split_target_tokens", C.c_int32), ("force_tile", C.c_int32),
                ("num_cus", C.c_int32), ("tail_reserve_pages", C.c_int32),
                ("model_ns", C.c_int32 * 4), ("wave_kv_tokens", C.c_int32),
                ("wave_max_tokens", C.c_int32), ("dual_launch", C.c_int32),
                ("fused_merge", C.c_int32), ("packed_min_tokens", C.c_int32), ("reserved", C.c_int32 * 1)]


class pat_plan_stats(C.Structure):
    _fields_ = [("num_nodes", C.c_int32), ("num_packs", C.c_int32),
                ("num_merged_children", C.c_int32), ("num_items", C.c_int32),
                ("num_entries", C.c_int32), ("num_workgroups", C.c_int32),
                ("num_slots", C.c_int32), ("num_merge_requests", C.c_int32),
                ("unique_kv_tokens", C.c_int64), ("total_kv_tokens", C.c_int64),
                ("plan_device_bytes", C.c_int64), ("workspace_bytes", C.c_int64),
                ("num_wave_items", C.c_int32), ("num_workers", C.c_int32),
                ("fused_merge", C.c_int32), ("pad0", C.c_int32),
                ("tile_histogram", C.c_int32 * 16)]


class pat_plan_view(C.Structure):
    _fields_ = [("num_items", C.c_int32), ("num_entries", C.c_int32),
                ("num_requests", C.c_int32), ("num_slots", C.c_int32)] + \
               [(n, _i32p) for n in (
                   "item_req_off", "item_req_ids", "item_req_slot", "item_page_off",
                   "item_page_ids", "item_page_start", "item_kv_len", "req_slot_off",
                   "req_slot_ids", "entry_item", "entry_row_begin", "entry_num_rows",
                   "entry_tile", "entry_heads_per_wg")]


EXPORTED = ("pat_plan", "pat_plan_destroy", "pat_plan_get_stats", "pat_plan_export",
            "pat_plan_upload", "pat_num_tiles", "pat_tile_info", "pat_forward", "pat_merge",
            "pat_decode_attention", "pat_strerror", "pat_version", "pat_debug_set_trace",
            "pat_plan_advance", "pat_plan_start", "pat_plan_finish",
            "pat_decode_attention_static_ws", "pat_debug_set_spin_limit", "pat_plan_cache_create",
            "pat_plan_cache_destroy", "pat_plan_cache_get")
PAT_STATIC_WORKSPACE_BYTES = 32 << 20

lib.pat_plan.argtypes = [C.POINTER(pat_batch_desc), C.POINTER(pat_plan_opts),
                         C.POINTER(C.c_void_p)]
lib.pat_plan.restype = C.c_int
lib.pat_plan_destroy.argtypes = [C.c_void_p]
lib.pat_plan_destroy.restype = None
lib.pat_plan_get_stats.argtypes = [C.c_void_p, C.POINTER(pat_plan_stats)]
lib.pat_plan_export.argtypes = [C.c_void_p, C.POINTER(pat_plan_view)]
lib.pat_plan_upload.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
lib.pat_plan_advance.argtypes = [C.c_void_p, _i32p, _i32p, C.c_int32]
lib.pat_plan_start.argtypes = [C.POINTER(pat_batch_desc), C.POINTER(pat_plan_opts),
                               C.POINTER(C.c_void_p)]
lib.pat_plan_start.restype = C.c_int
lib.pat_plan_finish.argtypes = [C.c_void_p, C.POINTER(C.c_void_p)]
lib.pat_plan_finish.restype = C.c_int
lib.pat_plan_advance.restype = C.c_int
lib.pat_plan_cache_create.argtypes = [C.c_int32, C.POINTER(C.c_void_p)]
lib.pat_plan_cache_destroy.argtypes = [C.c_void_p]
lib.pat_plan_cache_destroy.restype = None
lib.pat_plan_cache_get.argtypes = [C.c_void_p, C.POINTER(pat_batch_desc), C.POINTER(pat_plan_opts),
                                   C.POINTER(C.c_void_p), C.POINTER(C.c_int32)]
lib.pat_num_tiles.restype = C.c_int
lib.pat_tile_info.argtypes = [C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int)]
_fwd_args = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64,
             C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
lib.pat_forward.argtypes = _fwd_args
lib.pat_decode_attention.argtypes = _fwd_args
lib.pat_decode_attention_static_ws.argtypes = _fwd_args[:10] + [C.c_void_p]
lib.pat_merge.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                          C.c_void_p]
lib.pat_debug_set_trace.argtypes = [C.c_void_p, C.c_size_t]
lib.pat_debug_set_spin_limit.argtypes = [C.c_int]
lib.pat_strerror.argtypes = [C.c_int]
lib.pat_strerror.restype = C.c_char_p
lib.pat_version.restype = C.c_char_p


class PatError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib.pat_strerror(status).decode()} ({status})")


def _check(status: int, where: str):
    if status != PAT_OK:
        raise PatError(status, where)


def pat_strerror(status: int) -> str:
    return lib.pat_strerror(status).decode()


def pat_version() -> str:
    return lib.pat_version().decode()


def pat_tile_info(tile_id: int):
    m, n = C.c_int(), C.c_int()
    rc = lib.pat_tile_info(tile_id, C.byref(m), C.byref(n))
    return rc, m.value, n.value


def _ptr(a: Optional[np.ndarray]):
    return a.ctypes.data_as(_i32p) if a is not None else None


class Plan:
    """Owner of one pat_plan_t handle."""

    def __init__(self, handle: int, keep):
        self._h = C.c_void_p(handle)
        self._keep = keep
        self.device_buf = None

    def __del__(self):
        self.destroy()

    def destroy(self):
        # `lib` is already gone when the interpreter shuts down; the process ends anyway
        if getattr(self, "_h", None) is not None and self._h and lib is not None:
            if not getattr(self, "_borrowed", False):
                lib.pat_plan_destroy(self._h)
            self._h = None

    @property
    def handle(self):
        return self._h

    def stats(self) -> pat_plan_stats:
        s = pat_plan_stats()
        _check(lib.pat_plan_get_stats(self._h, C.byref(s)), "pat_plan_get_stats")
        return s

    def export(self) -> dict:
        v = pat_plan_view()
        _check(lib.pat_plan_export(self._h, C.byref(v)), "pat_plan_export")

        def arr(p, n):
            return np.ctypeslib.as_array(p, shape=(n,)).copy() if n > 0 else np.zeros(0, np.int32)

        out = {"num_items": v.num_items, "num_entries": v.num_entries,
               "num_requests": v.num_requests, "num_slots": v.num_slots}
        out["item_req_off"] = arr(v.item_req_off, v.num_items + 1)
        n_req = int(out["item_req_off"][-1])
        out["item_req_ids"] = arr(v.item_req_ids, n_req)
        out["item_req_slot"] = arr(v.item_req_slot, n_req)
        out["item_page_off"] = arr(v.item_page_off, v.num_items + 1)
        out["item_page_ids"] = arr(v.item_page_ids, int(out["item_page_off"][-1]))
        out["item_page_start"] = arr(v.item_page_start, v.num_items)
        out["item_kv_len"] = arr(v.item_kv_len, v.num_items)
        out["req_slot_off"] = arr(v.req_slot_off, v.num_requests + 1)
        out["req_slot_ids"] = arr(v.req_slot_ids, int(out["req_slot_off"][-1]))
        for k in ("entry_item", "entry_row_begin", "entry_num_rows", "entry_tile",
                  "entry_heads_per_wg"):
            out[k] = arr(getattr(v, k), v.num_entries)
        return out


def _desc_and_opts(block_tables, kv_lens, *, page_size, num_pages, num_q_heads, num_kv_heads, head_dim,
                   dtype, mode=PAT_MODE_PAT, merge_factor=0, split_policy=PAT_SPLIT_AUTO,
                   split_target_tokens=0, force_tile=-1, num_cus=0, tail_reserve_pages=0, model_ns=None,
                   wave_kv_tokens=0, wave_max_tokens=0, dual_launch=0, packed_min_tokens=0, fused_merge=0,
                   node_parent=None, node_num_pages=None, req_leaf_node=None):
    bt = np.ascontiguousarray(block_tables, dtype=np.int32)
    kl = np.ascontiguousarray(kv_lens, dtype=np.int32)
    d = pat_batch_desc()
    d.num_requests, d.max_pages_per_req = int(bt.shape[0]), int(bt.shape[1])
    d.block_tables, d.kv_lens = _ptr(bt), _ptr(kl)
    d.page_size, d.num_pages = int(page_size), int(num_pages)
    d.num_q_heads, d.num_kv_heads, d.head_dim = int(num_q_heads), int(num_kv_heads), int(head_dim)
    d.dtype = DTYPES[dtype] if isinstance(dtype, str) else int(dtype)
    keep = [bt, kl]
    if node_parent is not None:
        npar = np.ascontiguousarray(node_parent, dtype=np.int32)
        npg = np.ascontiguousarray(node_num_pages, dtype=np.int32)
        leaf = np.ascontiguousarray(req_leaf_node, dtype=np.int32)
        d.num_nodes = len(npar)
        d.node_parent, d.node_num_pages, d.req_leaf_node = _ptr(npar), _ptr(npg), _ptr(leaf)
        keep += [npar, npg, leaf]
    o = pat_plan_opts()
    o.mode, o.merge_factor, o.split_policy = int(mode), int(merge_factor), int(split_policy)
    o.split_target_tokens, o.force_tile, o.num_cus = (int(split_target_tokens), int(force_tile),
                                                      int(num_cus))
    o.tail_reserve_pages = int(tail_reserve_pages)
    o.wave_kv_tokens, o.wave_max_tokens = int(wave_kv_tokens), int(wave_max_tokens)
    o.dual_launch = int(dual_launch)
    o.packed_min_tokens = int(packed_min_tokens)
    o.fused_merge = int(fused_merge)
    if model_ns is not None:
        for i, x in enumerate(model_ns):
            o.model_ns[i] = int(x)
    return d, o, keep


def pat_plan(block_tables: np.ndarray, kv_lens: np.ndarray, *, background: bool = False, **kw) -> Plan:
    """pat_plan (or pat_plan_start with background=True); keywords: the fields of pat_batch_desc
    (page_size, num_pages, num_q_heads, num_kv_heads, head_dim, dtype, optional tree) and of
    pat_plan_opts."""
    d, o, keep = _desc_and_opts(block_tables, kv_lens, **kw)
    if background:
        job = C.c_void_p()
        _check(lib.pat_plan_start(C.byref(d), C.byref(o), C.byref(job)), "pat_plan_start")
        return PlanJob(job.value)
    h = C.c_void_p()
    _check(lib.pat_plan(C.byref(d), C.byref(o), C.byref(h)), "pat_plan")
    return Plan(h.value, keep)


class PlanCache:
    """Owner of one pat_plan_cache_t.  get() returns (Plan, how); the Plan objects do not own their
    handles (the cache does) and are valid until evicted or the cache is closed."""

    def __init__(self, capacity: int):
        h = C.c_void_p()
        _check(lib.pat_plan_cache_create(int(capacity), C.byref(h)), "pat_plan_cache_create")
        self._h = h

    def get(self, batch, **kw):
        d, o, _ = _desc_and_opts(batch.block_tables, batch.kv_lens, page_size=batch.page_size,
                                 num_pages=batch.num_pages, num_q_heads=batch.num_q_heads,
                                 num_kv_heads=batch.num_kv_heads, head_dim=batch.head_dim,
                                 dtype=batch.dtype, **kw)
        h, how = C.c_void_p(), C.c_int32(-1)
        _check(lib.pat_plan_cache_get(self._h, C.byref(d), C.byref(o), C.byref(h), C.byref(how)),
               "pat_plan_cache_get")
        p = Plan.__new__(Plan)
        p._h, p._keep, p.device_buf, p._borrowed = C.c_void_p(h.value), None, None, True
        return p, how.value

    def close(self):
        if getattr(self, "_h", None) is not None and self._h and lib is not None:
            lib.pat_plan_cache_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()


class PlanJob:
    """A plan being made on the library's worker thread (pat_plan_start); finish() waits for it."""

    def __init__(self, handle: int):
        self._h = handle

    def finish(self) -> Plan:
        if self._h is None:
            raise RuntimeError("PlanJob.finish() called twice")
        h, job = C.c_void_p(), self._h
        self._h = None
        _check(lib.pat_plan_finish(job, C.byref(h)), "pat_plan_finish")
        return Plan(h.value, [])

    def __del__(self):
        if getattr(self, "_h", None) is not None and lib is not None:
            lib.pat_plan_finish(self._h, None)      # discard
            self._h = None


def plan_for_batch(batch, **kw) -> Plan:
    """pat_plan for a workloads.DecodeBatch."""
    return pat_plan(batch.block_tables, batch.kv_lens, page_size=batch.page_size,
                    num_pages=batch.num_pages, num_q_heads=batch.num_q_heads,
                    num_kv_heads=batch.num_kv_heads, head_dim=batch.head_dim, dtype=batch.dtype,
                    **kw)


def pat_plan_advance(plan: Plan, new_kv_lens: np.ndarray, block_tables: np.ndarray):
    """Lazy update after decode steps; raises PatError(PAT_ERR_PLAN_STALE) when a new plan is
    needed.  Upload the plan again before the next forward."""
    bt = np.ascontiguousarray(block_tables, dtype=np.int32)
    kl = np.ascontiguousarray(new_kv_lens, dtype=np.int32)
    _check(lib.pat_plan_advance(plan.handle, _ptr(kl), _ptr(bt), int(bt.shape[1])),
           "pat_plan_advance")
    plan.device_buf = None


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def pat_plan_upload(plan: Plan, device_buf, stream=None):
    """device_buf: uint8 torch tensor on the GPU, >= stats.plan_device_bytes."""
    _check(lib.pat_plan_upload(plan.handle, device_buf.data_ptr(), device_buf.numel(),
                               _stream_ptr(stream)), "pat_plan_upload")
    plan.device_buf = device_buf            # keep the memory alive as long as the plan


def _fwd_call(fn, name, plan, q, k_pool, v_pool, strides, scale, out, lse, workspace, stream):
    _check(fn(plan.handle, q.data_ptr(), k_pool.data_ptr(), v_pool.data_ptr(),
              int(strides[0]), int(strides[1]), int(strides[2]), float(scale), out.data_ptr(),
              lse.data_ptr() if lse is not None else None, workspace.data_ptr(),
              workspace.numel() * workspace.element_size(), _stream_ptr(stream)), name)


def pat_forward(plan, q, k_pool, v_pool, strides, scale, out, lse, workspace, stream=None):
    _fwd_call(lib.pat_forward, "pat_forward", plan, q, k_pool, v_pool, strides, scale, out, lse,
              workspace, stream)


def pat_decode_attention(plan, q, k_pool, v_pool, strides, scale, out, lse, workspace,
                         stream=None):
    _fwd_call(lib.pat_decode_attention, "pat_decode_attention", plan, q, k_pool, v_pool, strides,
              scale, out, lse, workspace, stream)


def pat_decode_attention_static_ws(plan, q, k_pool, v_pool, strides, scale, out, lse, stream=None):
    _check(lib.pat_decode_attention_static_ws(
        plan.handle, q.data_ptr(), k_pool.data_ptr(), v_pool.data_ptr(), int(strides[0]),
        int(strides[1]), int(strides[2]), float(scale), out.data_ptr(),
        lse.data_ptr() if lse is not None else None, _stream_ptr(stream)),
        "pat_decode_attention_static_ws")


def pat_merge(plan, out, lse, workspace, stream=None):
    _check(lib.pat_merge(plan.handle, out.data_ptr(),
                         lse.data_ptr() if lse is not None else None, workspace.data_ptr(),
                         workspace.numel() * workspace.element_size(), _stream_ptr(stream)),
           "pat_merge")


def pat_debug_set_trace(buf=None):
    """buf: int64 torch tensor on the GPU with 4 entries per workgroup, or None to switch off."""
    if buf is None:
        _check(lib.pat_debug_set_trace(None, 0), "pat_debug_set_trace")
    else:
        _check(lib.pat_debug_set_trace(buf.data_ptr(), buf.numel() * buf.element_size()),
               "pat_debug_set_trace")


def pat_debug_set_spin_limit(polls: int):
    _check(lib.pat_debug_set_spin_limit(int(polls)), "pat_debug_set_spin_limit")


def alloc_plan_buffers(plan: Plan, device="cuda"):
    """Device buffers a plan needs: (plan image buffer, workspace), both uint8 tensors."""
    import torch
    s = plan.stats()
    dev = torch.empty(int(s.plan_device_bytes), dtype=torch.uint8, device=device)
    ws = torch.empty(int(s.workspace_bytes), dtype=torch.uint8, device=device)
    return dev, ws
