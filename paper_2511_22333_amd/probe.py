"""ctypes door to ``libpat_probe.so``: plain memory kernels that measure what the GPU's memory
system delivers (a streaming read and a latency-versus-request-size probe).  Used by ``bench.py``
(read ceiling next to every bandwidth figure) and by ``calibrate.py``; the attention path does
not depend on it."""
from __future__ import annotations

import ctypes as C
import os

import torch  # noqa: F401  (one HIP runtime in the process, loaded before the library)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpat_probe.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2511_22333_amd.build`")
lib = C.CDLL(LIB_PATH)
lib.pat_probe_read.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_int, C.c_void_p,
                               C.POINTER(C.c_size_t), C.c_void_p]
lib.pat_probe_read.restype = C.c_int
lib.pat_probe_latency.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_int, C.c_int, C.c_int,
                                  C.c_void_p, C.c_void_p, C.c_void_p]
lib.pat_probe_latency.restype = C.c_int


def _stream():
    return torch.cuda.current_stream().cuda_stream


def read_bandwidth(buf, *, nontemporal=True, workgroups=512, repeats=5):
    """GB/s of one pass over `buf` (uint8 GPU tensor), median of `repeats` launches timed with HIP
    events on the current stream."""
    sink = torch.zeros(4, dtype=torch.uint8, device=buf.device)
    done = C.c_size_t(0)

    def launch():
        rc = lib.pat_probe_read(buf.data_ptr(), buf.numel(), int(nontemporal), workgroups,
                                sink.data_ptr(), C.byref(done), _stream())
        if rc != 0:
            raise RuntimeError(f"pat_probe_read failed ({rc})")

    launch()
    torch.cuda.synchronize()
    times = []
    for _ in range(repeats):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        launch()
        b.record()
        torch.cuda.synchronize()
        times.append(a.elapsed_time(b) * 1e-3)
    times.sort()
    return done.value / times[len(times) // 2] / 1e9


def read_ceiling(buf):
    """Best streaming-read rate over a few launch shapes: (GB/s plain, GB/s non-temporal)."""
    plain = max(read_bandwidth(buf, nontemporal=False, workgroups=w) for w in (256, 512, 1024))
    nt = max(read_bandwidth(buf, nontemporal=True, workgroups=w) for w in (256, 512, 1024))
    return plain, nt


def request_latency_ns(buf, *, loads_per_thread, workgroups, iters=64):
    """Mean time (ns) of one request of 4096 * loads_per_thread bytes per workgroup, over
    `workgroups` workgroups making such requests at the same time."""
    ns = torch.zeros(workgroups, dtype=torch.float32, device=buf.device)
    sink = torch.zeros(4, dtype=torch.uint8, device=buf.device)
    for seed in range(2):                            # the first launch warms up; other addresses each time
        rc = lib.pat_probe_latency(buf.data_ptr(), buf.numel(), loads_per_thread, workgroups, iters,
                                   seed + 1, ns.data_ptr(), sink.data_ptr(), _stream())
        if rc != 0:
            raise RuntimeError(f"pat_probe_latency failed ({rc})")
        torch.cuda.synchronize()
    return float(ns.mean())
