"""ctypes binding of libsprnn_probe.so: the device microbenchmarks behind the stated roofline
(``include/sprnn_probe.h``).  Argument marshalling only."""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsprnn_probe.so")
EXPORTS = ["sprnn_probe_lds_gather", "sprnn_probe_lds_gather_offsets", "sprnn_probe_handoff", "sprnn_probe_fill"]
_lib = None


def load_library() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libsprnn_probe.so is missing: build it with `python -m paper_1804_10223_amd.build`")
        from .binding import load_with_one_runtime
        lib = load_with_one_runtime(LIB_PATH)   # one HIP runtime per process
        ci, dp = ctypes.c_int, ctypes.POINTER(ctypes.c_double)
        lib.sprnn_probe_lds_gather.restype = ci
        lib.sprnn_probe_lds_gather.argtypes = [ci, ci, ci, ci, ci, dp]
        lib.sprnn_probe_lds_gather_offsets.restype = ci
        lib.sprnn_probe_lds_gather_offsets.argtypes = [ci, ci, ci, ci, ci, ctypes.POINTER(ctypes.c_uint32), dp]
        lib.sprnn_probe_handoff.restype = ci
        lib.sprnn_probe_handoff.argtypes = [ci, ci, ci, dp, ctypes.POINTER(ci * 2)]
        lib.sprnn_probe_fill.restype = ci
        lib.sprnn_probe_fill.argtypes = [ci, ci, ci, ci, ci, dp]
        _lib = lib
    return _lib


def lds_gather(workgroups: int, threads: int, width_bytes: int, pattern: int = 0, device: int = 0) -> float:
    """Aggregate LDS gather rate in bytes/s (pattern 0 conflict free, 1 random columns)."""
    out = ctypes.c_double()
    rc = load_library().sprnn_probe_lds_gather(device, workgroups, threads, width_bytes, pattern, ctypes.byref(out))
    if rc:
        raise RuntimeError("sprnn_probe_lds_gather failed (%d)" % rc)
    return out.value


def lds_gather_offsets(offsets, width_bytes: int, workgroups: int = 256, device: int = 0, bare: bool = False) -> float:
    """Aggregate LDS gather rate in bytes/s for the caller's pattern: offsets is uint32 [16, threads] (byte offsets);
    bare leaves only the reads in the timed loop."""
    import numpy as np
    offsets = np.ascontiguousarray(offsets, dtype=np.uint32)
    assert offsets.ndim == 2 and offsets.shape[0] == 16
    out = ctypes.c_double()
    rc = load_library().sprnn_probe_lds_gather_offsets(device, workgroups, int(offsets.shape[1]), width_bytes, 1 if bare else 0,
                                                       offsets.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)), ctypes.byref(out))
    if rc:
        raise RuntimeError("sprnn_probe_lds_gather_offsets failed (%d)" % rc)
    return out.value


def handoff_ns(same_xcd: bool, rounds: int = 2000, device: int = 0):
    """(one-way store->observe latency in ns, (xcc of producer, xcc of consumer))."""
    out = ctypes.c_double()
    xcc = (ctypes.c_int * 2)()
    rc = load_library().sprnn_probe_handoff(device, 1 if same_xcd else 0, rounds, ctypes.byref(out), ctypes.byref(xcc))
    if rc:
        raise RuntimeError("sprnn_probe_handoff failed (%d)" % rc)
    return out.value, (xcc[0], xcc[1])


def fill_seconds(workgroups: int, threads: int, nbytes: int, rounds: int = 200, device: int = 0) -> float:
    """Seconds for one workgroup to copy ``nbytes`` of coherent global memory into LDS, all workgroups at once."""
    out = ctypes.c_double()
    rc = load_library().sprnn_probe_fill(device, workgroups, threads, nbytes, rounds, ctypes.byref(out))
    if rc:
        raise RuntimeError("sprnn_probe_fill failed (%d)" % rc)
    return out.value


def lds_peak(width_bytes: int, workgroups: int = 256, threads: int = 1024, device: int = 0) -> float:
    """Conflict-free LDS read rate in bytes/s with nothing but the reads in the timed loop: every wavefront reads 64
    consecutive pieces of ``width_bytes`` (16 different ones per thread), the pattern the banks serve at full rate."""
    import numpy as np
    t = np.arange(threads)
    offs = np.stack([(((t % 64) + 64 * ((t // 64 + k) % 16)) * width_bytes) % 65536 for k in range(16)]).astype(np.uint32)
    return lds_gather_offsets(offs, width_bytes, workgroups=workgroups, device=device, bare=True)


def handoff_ns_best(same_xcd: bool, launches: int = 5, rounds: int = 2000, device: int = 0, warm=None):
    """Smallest one-way store->observe latency over several probe launches (a latency floor is a minimum, and single
    launches differ by tens of per cent with where the two workgroups land).  `warm`, if given, is called before every
    launch: two lone workgroups do not keep the chip's clocks up by themselves, and on an idle device the same probe
    reads up to 1.6 times longer than right after a busy kernel."""
    best, where = None, None
    for _ in range(max(1, launches)):
        if warm is not None:
            warm()
        ns, xcc = handoff_ns(same_xcd, rounds, device)
        if best is None or ns < best:
            best, where = ns, xcc
    return best, where


def fill_fit(sizes=(16384, 36864, 65536), workgroups: int = 256, threads: int = 1024, device: int = 0):
    """Least-squares line through the copy times of several sizes: (seconds per byte, seconds at zero bytes, times).
    The slope is the marginal rate at which one CU brings coherent memory into LDS while every CU does the same; the
    intercept is the latency of the first piece, which the hand-off latency already accounts for."""
    import numpy as np
    times = [fill_seconds(workgroups, threads, int(n), device=device) for n in sizes]
    slope, intercept = np.polyfit(np.asarray(sizes, dtype=np.float64), np.asarray(times, dtype=np.float64), 1)
    return float(slope), float(intercept), dict(zip([int(n) for n in sizes], times))
